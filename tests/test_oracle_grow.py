"""Pins for the oracle's tree growth: the counter-based draws, the bootstrap, the tree structure,
growth-time partition = traversal, purity, and the chosen splits against exact brute force."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import rfx_inputs as ri

MASK = (1 << 64) - 1
K = 0x9E3779B97F4A7C15


def _mix(z):
    z = (z + K) & MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
    return z ^ (z >> 31)


def _draw(seed, tree, a, b):
    return _mix(_mix(_mix(seed ^ (((tree + 1) * K) & MASK)) ^ a) ^ b)


def _bounded(r, n):
    return ((r >> 32) * n) >> 32


def _forest(g):
    z = np.zeros_like(g["feature"])
    return ri.Forest(g["n_trees"], g["n_features"], g["node_offset"], g["feature"], g["threshold"], g["left"], g["right"],
                     g["leaf_id"], g["depth"], g["n_leaves"], g["inbag"], g["train_leaf"])


def test_draws_follow_splitmix64():
    # published first outputs of splitmix64 started at state 0
    assert _mix(0) == 0xE220A8397B1DCDAF and _mix(K) == 0x6E789E6AA1B965F4
    rng = np.random.default_rng(0)
    for _ in range(50):
        s, t, a, b = (int(v) for v in rng.integers(0, 2 ** 62, size=4))
        assert oracle.draw(s, t % 1000, a, b) == _draw(s, t % 1000, a, b)


def test_bootstrap_counts():
    N, seed = 5000, 99
    X = np.random.default_rng(1).standard_normal((N, 3)).astype(np.float32)
    y = (X[:, 0] > 0).astype(np.int32)
    g = oracle.grow(X, y, 2, 3, 1, seed, first_tree=7)
    for b in range(3):
        want = np.bincount([_bounded(_draw(seed, 7 + b, 0, t), N) for t in range(N)], minlength=N)
        np.testing.assert_array_equal(g["inbag"][b], want)
        assert g["inbag"][b].sum() == N
    assert abs((g["inbag"] == 0).mean() - np.exp(-1)) < 0.02      # about one third of the rows are out-of-bag


def test_structure_partition_and_purity(cfg1):
    X, y = cfg1["X"], cfg1["y"]
    B = 30
    g = oracle.grow(X, y, 3, B, 3, 2024)
    F = _forest(g)
    leaf, _ = oracle.leaf_assign(F, X)          # the independent traversal
    for b in range(B):
        s, e = int(g["node_offset"][b]), int(g["node_offset"][b + 1])
        feat, left, right, lid, depth = (g[k][s:e] for k in ("feature", "left", "right", "leaf_id", "depth"))
        inner = np.nonzero(feat >= 0)[0]
        # children are created in pairs, in the order in which their parents are split, breadth first
        np.testing.assert_array_equal(left[inner], 1 + 2 * np.arange(inner.size))
        np.testing.assert_array_equal(right[inner], left[inner] + 1)
        assert (depth[left[inner]] == depth[inner] + 1).all() and (np.diff(depth) >= 0).all() and depth[0] == 0
        leaves = np.nonzero(feat < 0)[0]
        np.testing.assert_array_equal(lid[leaves], np.arange(leaves.size))
        assert leaves.size == g["n_leaves"][b] == inner.size + 1 and (lid[inner] == -1).all()
        # every in-bag row is found again, by traversal, in the leaf it occupied when growth stopped
        rows = np.nonzero(g["inbag"][b] > 0)[0]
        np.testing.assert_array_equal(leaf[b][rows], g["train_leaf"][b][rows])
        assert (g["train_leaf"][b][g["inbag"][b] == 0] == -1).all()
        # pure leaves, labelled with their class
        np.testing.assert_array_equal(g["leaf_class"][b][leaf[b][rows]], y[rows])
        assert (g["leaf_class"][b][g["n_leaves"][b]:] == -1).all()


def _gini(w):
    n = sum(w)
    return 1 - sum(Fraction(v * v, n * n) for v in w)


def _brute_split(X, y, w, rows, feats, C):
    """First-best maximiser of the impurity decrease, the paper's formula in exact fractions."""
    best = None
    parent = [sum(int(w[i]) for i in rows if y[i] == c) for c in range(C)]
    n = sum(parent)
    for f in feats:
        vals = sorted(set(float(X[i, f]) for i in rows))
        for tau in vals[:-1]:
            L = [sum(int(w[i]) for i in rows if y[i] == c and X[i, f] <= tau) for c in range(C)]
            R = [p - l for p, l in zip(parent, L)]
            gain = _gini(parent) - Fraction(sum(L), n) * _gini(L) - Fraction(sum(R), n) * _gini(R)
            if best is None or gain > best[0]:
                best = (gain, f, tau)
    return best


def test_every_split_is_the_exact_first_best(cfg1):
    X, y = cfg1["X"], cfg1["y"]
    N, M = X.shape
    seed, mtry, C = 5, 3, 3
    g = oracle.grow(X, y, C, 4, mtry, seed, first_tree=11)
    for b in range(4):
        s, e = int(g["node_offset"][b]), int(g["node_offset"][b + 1])
        feat, thr, left, right = (g[k][s:e] for k in ("feature", "threshold", "left", "right"))
        w = g["inbag"][b]
        members = {0: [i for i in range(N) if w[i] > 0]}
        for v in range(e - s):
            rows = members[v]
            if feat[v] < 0:
                continue
            perm = list(range(M))
            for q in range(mtry):
                j = q + _bounded(_draw(seed, 11 + b, 1 + v, q), M - q)
                perm[q], perm[j] = perm[j], perm[q]
            gain, f, tau = _brute_split(X, y, w, rows, perm[:mtry], C)
            assert (f, np.float32(tau)) == (int(feat[v]), thr[v]), (b, v)
            members[int(left[v])] = [i for i in rows if X[i, f] <= tau]
            members[int(right[v])] = [i for i in rows if X[i, f] > tau]


def test_fallback_features_and_impure_leaves():
    rng = np.random.default_rng(3)
    N = 60
    X = np.zeros((N, 5), np.float32)
    X[:, 3] = rng.integers(0, 4, N)             # the only feature that varies
    y = (X[:, 3] >= 2).astype(np.int32)
    y[:6] = 1 - y[:6]                           # rows that no split can separate from their duplicates
    g = oracle.grow(X, y, 2, 8, 1, 17)
    F = _forest(g)
    leaf, _ = oracle.leaf_assign(F, X)
    for b in range(8):
        s, e = int(g["node_offset"][b]), int(g["node_offset"][b + 1])
        feat = g["feature"][s:e]
        assert set(feat[feat >= 0].tolist()) <= {3}          # constant features can never be chosen
        rows = np.nonzero(g["inbag"][b] > 0)[0]
        np.testing.assert_array_equal(leaf[b][rows], g["train_leaf"][b][rows])
        # a leaf holds one value of feature 3 or is pure; its label is the heaviest class, lowest on ties
        for l in range(g["n_leaves"][b]):
            mem = rows[leaf[b][rows] == l]
            wts = np.bincount(y[mem], weights=g["inbag"][b][mem], minlength=2)
            assert np.unique(X[mem, 3]).size == 1 or (wts > 0).sum() == 1
            assert g["leaf_class"][b][l] == int(np.argmax(wts))


def test_root_split_agrees_with_a_library_tree(small2):
    """With every feature offered (mtry = M) the root split is the plain best Gini split of the weighted
    bootstrap sample: the same partition as scikit-learn's tree finds with those sample weights."""
    from sklearn.tree import DecisionTreeClassifier
    X, y = small2["X"], small2["y"]
    N, M = X.shape
    g = oracle.grow(X, y, 5, 3, M, 1234)
    for b in range(3):
        w = g["inbag"][b].astype(np.float64)
        rows = w > 0
        t = DecisionTreeClassifier(criterion="gini", max_depth=1, random_state=0).fit(X[rows], y[rows], sample_weight=w[rows])
        f_lib, thr_lib = int(t.tree_.feature[0]), float(t.tree_.threshold[0])
        s = int(g["node_offset"][b])
        assert int(g["feature"][s]) == f_lib
        np.testing.assert_array_equal(X[rows, f_lib] <= g["threshold"][s], X[rows, f_lib] <= thr_lib)
