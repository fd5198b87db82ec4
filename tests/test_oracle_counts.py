"""Pins for the oracle's leaf assignment, co-occurrence counts and out-of-bag variant."""
from pathlib import Path

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import rfx_inputs as ri
from conftest import brute_counts


def _hand_forest():
    """Two hand-built trees on 2 features.
    Tree 0 (3 nodes): root splits f0 at 0.5 -> leaf 0 (left), leaf 1 (right).
    Tree 1 (7 nodes): root f1 @ 1.0; left child f0 @ -1.0 -> leaves 0, 1; right child f0 @ 2.0 -> leaves 2, 3.
    """
    feature = np.array([0, -1, -1, 1, 0, 0, -1, -1, -1, -1], np.int32)
    thr = np.array([0.5, 0, 0, 1.0, -1.0, 2.0, 0, 0, 0, 0], np.float32)
    left = np.array([1, -1, -1, 1, 3, 5, -1, -1, -1, -1], np.int32)
    right = np.array([2, -1, -1, 2, 4, 6, -1, -1, -1, -1], np.int32)
    leaf_id = np.array([-1, 0, 1, -1, -1, -1, 0, 1, 2, 3], np.int32)
    z = np.zeros(10, np.int32)
    return ri.Forest(2, 2, np.array([0, 3, 10], np.int64), feature, thr, left, right, leaf_id, z,
                     np.array([2, 4], np.int32), np.zeros((2, 6), np.uint16), np.zeros((2, 6), np.int32))


def test_hand_built_trees():
    F = _hand_forest()
    X = np.array([[0.5, 1.0],      # t0: 0.5<=0.5 left -> 0 ; t1: 1.0<=1.0 left, 0.5<=-1 no -> leaf 1
                  [0.6, 1.0],      # t0: right -> 1        ; t1: left, right -> 1
                  [-1.0, 0.0],     # t0: 0                 ; t1: left, -1<=-1 left -> 0
                  [2.0, 1.5],      # t0: 1                 ; t1: right, 2<=2 left -> 2
                  [2.5, 1.5],      # t0: 1                 ; t1: right, right -> 3
                  [np.nan, np.nan]], np.float32)   # comparisons with NaN are false -> always right
    leaf, plen = oracle.leaf_assign(F, X)
    np.testing.assert_array_equal(leaf, [[0, 1, 0, 1, 1, 1], [1, 1, 0, 2, 3, 3]])
    assert plen == 6 * 1 + 6 * 2
    cnt = oracle.counts_full(leaf)
    expect = np.array([[2, 1, 1, 0, 0, 0],
                       [1, 2, 0, 1, 1, 1],
                       [1, 0, 2, 0, 0, 0],
                       [0, 1, 0, 2, 1, 1],
                       [0, 1, 0, 1, 2, 2],
                       [0, 1, 0, 1, 2, 2]], np.uint32)
    np.testing.assert_array_equal(cnt, expect)


def test_malformed_forest_is_rejected():
    F = _hand_forest()
    F.left = F.left.copy()
    F.left[0] = 7     # outside tree 0's three nodes
    with pytest.raises(ValueError):
        oracle.leaf_assign(F, np.zeros((1, 2), np.float32))


def test_traversal_reproduces_the_growth_time_partition(cfg1, small2):
    """Every in-bag row must land in the leaf it occupied when the tree stopped growing."""
    for d in (cfg1, small2):
        tl, leaf = d["F"].train_leaf, d["leaf"]
        m = tl >= 0
        np.testing.assert_array_equal(leaf[m], tl[m].astype(np.uint32))
        assert (leaf < d["F"].n_leaves[:, None].astype(np.uint32)).all()


def test_leaf_assign_matches_python_walk(cfg1):
    F, X = cfg1["F"], cfg1["X"]
    for b in (0, 13, 99):
        off = int(F.node_offset[b])
        for i in range(0, 178, 7):
            n = 0
            while F.feature[off + n] >= 0:
                n = F.left[off + n] if X[i, F.feature[off + n]] <= F.threshold[off + n] else F.right[off + n]
            assert cfg1["leaf"][b, i] == F.leaf_id[off + n]


def test_counts_match_brute_force_on_tiny_forests(cfg1):
    leaf = cfg1["leaf"][:7, :40]
    np.testing.assert_array_equal(oracle.counts_full(np.ascontiguousarray(leaf)), brute_counts(leaf))
    rng = np.random.default_rng(3)
    leaf = rng.integers(0, 4, size=(5, 23)).astype(np.uint32)
    np.testing.assert_array_equal(oracle.counts_full(leaf), brute_counts(leaf))
    np.testing.assert_array_equal(oracle.counts_rows(leaf, 5, 9), brute_counts(leaf)[5:9])


def test_count_invariants(cfg1, small2):
    for d in (cfg1, small2):
        leaf = d["leaf"]
        B, N = leaf.shape
        cnt = oracle.counts_full(leaf)
        assert (np.diag(cnt) == B).all()                    # a sample always shares its own leaf
        np.testing.assert_array_equal(cnt, cnt.T)           # symmetric
        assert cnt.max() <= B
        # per tree, the number of co-occurring ordered pairs is the sum of squared leaf sizes
        total = sum(int((np.bincount(leaf[b]).astype(np.int64) ** 2).sum()) for b in range(B))
        assert int(cnt.astype(np.int64).sum()) == total
        P = oracle.normalise(cnt, B)
        assert P.dtype == np.float32 and P.min() >= 0.0 and P.max() == 1.0 and (np.diag(P) == 1.0).all()


def test_counts_equal_sparse_one_hot_gram(small2):
    """B*P = Z Z^T with Z = [Z_1 ... Z_B] the one-hot leaf-membership matrices (library product)."""
    leaf = small2["leaf"]
    B, N = leaf.shape
    nl = leaf.max(axis=1).astype(np.int64) + 1
    col = leaf.astype(np.int64) + np.concatenate([[0], np.cumsum(nl)[:-1]])[:, None]
    Z = sp.csr_matrix((np.ones(B * N, np.int32), (np.tile(np.arange(N), B), col.ravel())), shape=(N, int(nl.sum())))
    np.testing.assert_array_equal((Z @ Z.T).toarray().astype(np.uint32), oracle.counts_full(leaf))


def test_sparse_upper_triplets(small2):
    """Thresholded strict-upper coordinate form against the library sparse product and closed forms."""
    leaf = small2["leaf"]
    B, N = leaf.shape
    nl = leaf.max(axis=1).astype(np.int64) + 1
    col = leaf.astype(np.int64) + np.concatenate([[0], np.cumsum(nl)[:-1]])[:, None]
    Z = sp.csr_matrix((np.ones(B * N, np.int32), (np.tile(np.arange(N), B), col.ravel())), shape=(N, int(nl.sum())))
    U = sp.triu(Z @ Z.T, k=1).tocoo()
    for min_count in (1, 2, 7, B):
        r, c, v = oracle.sparse_upper(leaf, min_count)
        keep = U.data >= min_count
        want = sorted(zip(U.row[keep].tolist(), U.col[keep].tolist(), U.data[keep].tolist()))
        assert list(zip(r.tolist(), c.tolist(), v.tolist())) == want
        assert (r < c).all() and (v >= min_count).all() and (v <= B).all()
    r, c, v = oracle.sparse_upper(leaf, 1)
    # every co-occurring pair exactly once: 2 * sum + N B = sum over trees and leaves of (leaf size)^2
    total = sum(int((np.bincount(leaf[b]).astype(np.int64) ** 2).sum()) for b in range(B))
    assert 2 * int(v.astype(np.int64).sum()) + N * B == total
    assert oracle.sparse_upper(leaf, B + 1)[0].size == 0
    # a row range returns exactly that range's triplets
    r2, c2, v2 = oracle.sparse_upper(leaf, 1, 100, 400)
    sel = (r >= 100) & (r < 400)
    np.testing.assert_array_equal(r2, r[sel]); np.testing.assert_array_equal(c2, c[sel]); np.testing.assert_array_equal(v2, v[sel])
    # one tree: the pairs inside each leaf, all with count 1
    r1, c1, v1 = oracle.sparse_upper(leaf[:1], 1)
    s = np.bincount(leaf[0]).astype(np.int64)
    assert r1.size == int((s * (s - 1) // 2).sum()) and (v1 == 1).all() and (leaf[0][r1] == leaf[0][c1]).all()


def test_count_special_cases():
    N, B = 9, 4
    np.testing.assert_array_equal(oracle.counts_full(np.zeros((B, N), np.uint32)), np.full((N, N), B))
    ident = np.tile(np.arange(N, dtype=np.uint32), (B, 1))
    np.testing.assert_array_equal(oracle.counts_full(ident), B * np.eye(N, dtype=np.uint32))
    # one tree: an equivalence relation (0/1, transitive)
    rng = np.random.default_rng(0)
    one = rng.integers(0, 3, size=(1, N)).astype(np.uint32)
    c = oracle.counts_full(one).astype(np.int64)
    assert set(np.unique(c)) <= {0, 1}
    assert ((c @ c > 0) == (c > 0)).all()


def _brute_oob(leaf, inbag):
    B, N = leaf.shape
    num = np.zeros((N, N), np.uint32)
    den = np.zeros((N, N), np.uint32)
    for i in range(N):
        for j in range(N):
            for b in range(B):
                if inbag[b, i] == 0 and inbag[b, j] == 0:
                    den[i, j] += 1
                    if leaf[b, i] == leaf[b, j]:
                        num[i, j] += 1
    return num, den


def test_oob_variant(cfg1):
    leaf, inbag = cfg1["leaf"], cfg1["F"].inbag
    B, N = leaf.shape
    sub_l, sub_c = np.ascontiguousarray(leaf[:9, :30]), np.ascontiguousarray(inbag[:9, :30])
    num, den = oracle.oob_rows(sub_l, sub_c, 0, 30)
    bn, bd = _brute_oob(sub_l, sub_c)
    np.testing.assert_array_equal(num, bn)
    np.testing.assert_array_equal(den, bd)

    num, den = oracle.oob_rows(leaf, inbag, 0, N)
    cnt = oracle.counts_full(leaf)
    O = (inbag == 0).astype(np.int64)
    np.testing.assert_array_equal(den, (O.T @ O).astype(np.uint32))      # library product
    np.testing.assert_array_equal(np.diag(den), O.sum(axis=0))           # trees where i is out-of-bag
    assert (num <= np.minimum(cnt, den)).all()
    np.testing.assert_array_equal(num, num.T)
    np.testing.assert_array_equal(np.diag(num), np.diag(den))
    # with nobody in-bag the variant is the plain proximity
    n0, d0 = oracle.oob_rows(leaf, np.zeros_like(inbag), 3, 40)
    np.testing.assert_array_equal(n0, cnt[3:40])
    assert (d0 == B).all()
    # with everybody in-bag there is nothing to count; proximity rows are 0 with a unit diagonal
    n1, d1 = oracle.oob_rows(leaf, np.ones_like(inbag), 0, N)
    assert n1.max() == 0 and d1.max() == 0
    np.testing.assert_array_equal(oracle.prox_oob_rows(n1, d1, 0), np.eye(N, dtype=np.float32))
    p = oracle.prox_oob_rows(num[5:20], den[5:20], 5)
    assert p.dtype == np.float32 and p.min() >= 0 and p.max() <= 1 and (p[np.arange(15), 5 + np.arange(15)] == 1).all()


def test_packed_upper_layout():
    N = 7
    full = np.arange(N * N).reshape(N, N)
    packed = oracle.pack_upper(full)
    assert packed.shape == (N * (N - 1) // 2,)
    for i in range(N):
        for j in range(i + 1, N):
            assert packed[i * N - i * (i + 1) // 2 + (j - i - 1)] == full[i, j]


def test_paper_closed_forms():
    """Storage figures printed in the paper (tests/golden/paper_closed_forms.txt)."""
    unit = {"MB": 1e6, "GB": 1e9}
    for line in (Path(__file__).parent / "golden" / "paper_closed_forms.txt").read_text().splitlines():
        line = line.split(";")[0].strip()
        if not line or line.startswith("#"):
            continue
        key, n, r, bpe, val, u = line.split()
        n, r, bpe, val = int(n), int(r), int(bpe), float(val)
        if key == "full_fp64":
            got = bpe * n * n
            # the paper mixes decimal and binary units; accept either reading of the printed figure
            assert min(abs(got / unit[u] - val), abs(got / 2 ** (20 if u == "MB" else 30) - val)) / val < 0.06
        else:
            got = 2 * n * r * bpe           # two n x r factors
            assert got / unit[u] == pytest.approx(val, rel=1e-9)
    # this build keeps one symmetric factor: n*k INT8 codes, 6.4 MB at n = 100k, k = 64
    Q, s = oracle.quantise_int8(np.ones((10, 64), np.float32), np.ones(64, np.float32))
    assert Q.nbytes * 10_000 == 6_400_000 and s.shape == (64,)
