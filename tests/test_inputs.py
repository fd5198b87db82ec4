"""Pins for the seeded input generators (mixture data, grown forests)."""
import numpy as np
import pytest

import rfx_inputs as ri


def test_config_shapes_match_the_workload_table():
    shapes = {k: (c.N, c.M, c.C, c.B, c.mtry) for k, c in ri.CONFIGS.items()}
    assert shapes == {1: (178, 13, 3, 100, 3), 2: (10_000, 20, 5, 500, 4), 3: (50_000, 50, 10, 500, 7),
                      4: (100_000, 100, 10, 1000, 10), 5: (500_000, 64, 20, 1000, 8)}
    for c in ri.CONFIGS.values():
        assert c.mtry == int(np.floor(np.sqrt(c.M)))


def test_mixture_is_seeded_and_shaped(cfg1):
    c = cfg1["c"]
    X2, y2 = ri.gaussian_mixture(c)
    assert X2.dtype == np.float32 and X2.shape == (178, 13) and X2.flags.c_contiguous
    np.testing.assert_array_equal(X2, cfg1["X"])
    np.testing.assert_array_equal(y2, cfg1["y"])
    assert sorted(np.bincount(y2).tolist()) == [48, 59, 71]


def test_label_noise_rate():
    c = ri.CONFIGS[2]
    X, y = ri.gaussian_mixture(c)
    assert np.bincount(y, minlength=5).min() > 1500
    # nearest-class-mean labels disagree with y for roughly the flipped share
    mu = np.stack([X[y == k].mean(0) for k in range(c.C)])
    near = np.argmin(((X[:, None, :] - mu[None]) ** 2).sum(-1), axis=1)
    assert 0.07 < (near != y).mean() < 0.16


def _mt_bootstrap(seed, N):
    """In-bag counts from the 32-bit Mersenne Twister seeded the standard way (init_genrand),
    mapped to [0, N) by multiply-shift with rejection; written with numpy's generator, which is
    independent of the C++ library's."""
    bg = np.random.MT19937()
    bg._legacy_seeding(seed)
    raw = bg.random_raw
    cnt = np.zeros(N, np.int64)
    thresh = ((1 << 32) - N) % N
    for _ in range(N):
        while True:
            m = int(raw()) * N
            if (m & 0xFFFFFFFF) >= thresh:
                break
        cnt[m >> 32] += 1
    return cnt


def test_bootstrap_counts_follow_mt19937_seeded_iseed_plus_tree(cfg1):
    F = cfg1["F"]
    for b in (0, 1, 57, 99):
        np.testing.assert_array_equal(F.inbag[b].astype(np.int64), _mt_bootstrap(ri.mixture.FOREST_ISEED + b, 178))


def test_bootstrap_sums_and_oob_fraction(cfg1, small2):
    for d in (cfg1, small2):
        F = d["F"]
        N = F.inbag.shape[1]
        assert (F.inbag.sum(axis=1) == N).all()
        oob = (F.inbag == 0).mean()
        assert abs(oob - (1 - 1 / N) ** N) < 0.01      # "roughly one-third" of rows are out-of-bag


def _check_structure(F):
    for b in range(F.n_trees):
        s, e = int(F.node_offset[b]), int(F.node_offset[b + 1])
        feat, l, r, lid = F.feature[s:e], F.left[s:e], F.right[s:e], F.leaf_id[s:e]
        internal = feat >= 0
        assert ((l >= 0) == internal).all() and ((r >= 0) == internal).all()
        assert ((lid >= 0) == ~internal).all()
        assert sorted(lid[~internal].tolist()) == list(range(int(F.n_leaves[b])))
        kids = np.concatenate([l[internal], r[internal]])
        assert sorted(kids.tolist()) == list(range(1, e - s))   # every non-root node has exactly one parent
        assert (e - s) == 2 * int(F.n_leaves[b]) - 1
        assert (feat[internal] < F.n_features).all()


def test_tree_structure(cfg1, small2):
    _check_structure(cfg1["F"])
    _check_structure(small2["F"])


def test_leaves_are_pure_over_inbag_rows(cfg1, small2):
    for d in (cfg1, small2):
        F, y = d["F"], d["y"]
        for b in range(F.n_trees):
            tl = F.train_leaf[b]
            inb = F.inbag[b] > 0
            assert ((tl >= 0) == inb).all()
            for l in range(int(F.n_leaves[b])):
                assert len(set(y[tl == l].tolist())) == 1


def test_thresholds_are_observed_values(cfg1):
    F, X = cfg1["F"], cfg1["X"]
    internal = F.feature >= 0
    for f, t in zip(F.feature[internal][:200], F.threshold[internal][:200]):
        assert t in X[:, f]


def test_growth_is_deterministic_and_thread_independent(cfg1):
    c = cfg1["c"]
    F1 = ri.grow_forest(cfg1["X"], cfg1["y"], c.C, 12, c.mtry, n_threads=1)
    F2 = ri.grow_forest(cfg1["X"], cfg1["y"], c.C, 12, c.mtry, n_threads=4)
    for f in ("node_offset", "feature", "threshold", "left", "right", "leaf_id", "inbag", "train_leaf"):
        np.testing.assert_array_equal(getattr(F1, f), getattr(F2, f))
        np.testing.assert_array_equal(getattr(F1, f), getattr(cfg1["F"].subset(12), f))


def test_first_split_maximises_gini_decrease(cfg1):
    """Brute-force check of the root split of tree 0: among all thresholds of the chosen feature
    no candidate has a larger weighted Gini decrease."""
    F, X, y = cfg1["F"], cfg1["X"], cfg1["y"]
    w = F.inbag[0].astype(np.float64)
    f, tau = int(F.feature[0]), float(F.threshold[0])

    def gini(mask):
        n = w[mask].sum()
        if n == 0:
            return 0.0, 0.0
        p = np.array([w[mask & (y == k)].sum() for k in range(3)]) / n
        return 1 - (p ** 2).sum(), n

    allm = w > 0
    gp, n = gini(allm)

    def gain(t):
        gl, nl = gini(allm & (X[:, f] <= t))
        gr, nr = gini(allm & (X[:, f] > t))
        return gp - nl / n * gl - nr / n * gr

    vals = np.unique(X[allm, f])[:-1]
    gains = np.array([gain(t) for t in vals])
    assert gain(tau) >= gains.max() - 1e-12
    assert tau == vals[np.argmax(gains >= gains.max() - 1e-15)] or gain(tau) == pytest.approx(gains.max(), abs=1e-12)


def _exact_scores(X, y, w, rows, f, C):
    """Exact score of every candidate threshold of feature f in a node: maximising the paper's Gini decrease
    dI = I(parent) - nL/n I(left) - nR/n I(right) is maximising sum_c wL_c^2/nL + sum_c wR_c^2/nR, a fraction
    of integers when the weights are in-bag counts.  Returns [(Fraction score, threshold)] over the node's
    distinct values except the largest."""
    from fractions import Fraction
    order = sorted(rows, key=lambda i: X[i, f])
    tot = [0] * C
    for i in order:
        tot[y[i]] += int(w[i])
    n = sum(tot)
    left = [0] * C
    out = []
    for p, i in enumerate(order[:-1]):
        left[y[i]] += int(w[i])
        if X[order[p + 1], f] == X[i, f]:
            continue
        nL = sum(left)
        nR = n - nL
        a = sum(v * v for v in left)
        c = sum((t - v) * (t - v) for t, v in zip(tot, left))
        out.append((Fraction(a, nL) + Fraction(c, nR), X[i, f]))
    return out


def _walk_nodes(F, b, X):
    """Yields (node, rows) for every node of tree b, rows = the in-bag rows that reach it under x <= tau."""
    s = int(F.node_offset[b])
    stack = [(0, [i for i in range(X.shape[0]) if F.inbag[b][i] > 0])]
    while stack:
        v, rows = stack.pop()
        yield v, rows
        f = int(F.feature[s + v])
        if f >= 0:
            t = F.threshold[s + v]
            stack.append((int(F.left[s + v]), [i for i in rows if X[i, f] <= t]))
            stack.append((int(F.right[s + v]), [i for i in rows if X[i, f] > t]))


def test_every_interior_split_maximises_the_gini_decrease(cfg1):
    """Every internal node of the generator's trees, not only the root: the stored threshold attains the
    exact maximum of the Gini decrease over all thresholds of the stored feature (fractions of integers, so
    the check does not share the generator's floating-point gain).  Where two candidates tie exactly the
    lower threshold must have been kept (first best)."""
    F, X, y = cfg1["F"], cfg1["X"], cfg1["y"]
    checked = 0
    for b in (0, 3, 41, 99):
        s = int(F.node_offset[b])
        for v, rows in _walk_nodes(F, b, X):
            f = int(F.feature[s + v])
            if f < 0:
                assert len({int(y[i]) for i in rows}) == 1
                continue
            cands = _exact_scores(X, y, F.inbag[b], rows, f, 3)
            best = max(sc for sc, _ in cands)
            first = min(t for sc, t in cands if sc == best)
            assert F.threshold[s + v] == first, (b, v)
            checked += 1
    assert checked > 30


def test_every_split_is_the_global_best_when_all_features_are_offered(cfg1):
    """With mtry = M the feature draw offers every feature at every node, so the split must be a global
    maximiser of the Gini decrease over all (feature, threshold) pairs, at every depth."""
    X, y, c = cfg1["X"], cfg1["y"], cfg1["c"]
    F = ri.grow_forest(X, y, c.C, 3, c.M, iseed=4321)
    for b in range(3):
        s = int(F.node_offset[b])
        for v, rows in _walk_nodes(F, b, X):
            f = int(F.feature[s + v])
            if f < 0:
                continue
            per_feature = {g: _exact_scores(X, y, F.inbag[b], rows, g, c.C) for g in range(c.M)}
            best = max(sc for cands in per_feature.values() for sc, _ in cands)
            chosen = [sc for sc, t in per_feature[f] if t == F.threshold[s + v]]
            assert chosen and chosen[0] == best, (b, v)
