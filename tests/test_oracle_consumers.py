"""Pins for the oracle's proximity consumers: the two outlier measures and the out-of-bag vote."""
import numpy as np
import pytest

import oracle
import rfx_inputs as ri


def test_outlier_closed_forms():
    B = 8
    # every sample in one leaf of every tree: p = 1 everywhere
    n = 7
    cnt = np.full((n, n), B, np.uint32)
    np.testing.assert_allclose(oracle.outlier_printed(cnt, B), 1.0, rtol=1e-15)
    np.testing.assert_allclose(oracle.outlier_classic(cnt, B), n / (n - 1), rtol=1e-15)
    # every sample alone: no proximity to anyone
    cnt = np.diag(np.full(n, B)).astype(np.uint32)
    assert (oracle.outlier_printed(cnt, B) == 0).all() and np.isinf(oracle.outlier_classic(cnt, B)).all()
    # two blocks of sizes 3 and 5 that never meet
    cnt = np.zeros((8, 8), np.uint32)
    cnt[:3, :3] = B
    cnt[3:, 3:] = B
    np.testing.assert_allclose(oracle.outlier_printed(cnt, B), [2 / 7] * 3 + [4 / 7] * 5, rtol=1e-15)
    np.testing.assert_allclose(oracle.outlier_classic(cnt, B), [8 / 2] * 3 + [8 / 4] * 5, rtol=1e-15)
    # hand example, 3 samples, B = 4: p01 = 1/2, p02 = 1/4, p12 = 0
    cnt = np.array([[4, 2, 1], [2, 4, 0], [1, 0, 4]], np.uint32)
    np.testing.assert_allclose(oracle.outlier_printed(cnt, 4), [(4 + 16) / 2, 4 / 2, 16 / 2], rtol=1e-15)
    np.testing.assert_allclose(oracle.outlier_classic(cnt, 4), [3 / (1 / 4 + 1 / 16), 3 / (1 / 4), 3 / (1 / 16)], rtol=1e-15)
    # labels restrict the classic measure to the own class
    lab = np.array([0, 0, 1])
    np.testing.assert_allclose(oracle.outlier_classic(cnt, 4, lab), [3 / (1 / 4), 3 / (1 / 4), np.inf], rtol=1e-15)


def test_outlier_on_a_grown_forest(cfg1):
    leaf, y = cfg1["leaf"], cfg1["y"]
    B, N = leaf.shape
    cnt = oracle.counts_full(leaf)
    P = cnt.astype(np.float64) / B
    off = ~np.eye(N, dtype=bool)
    pr = oracle.outlier_printed(cnt, B)
    cl = oracle.outlier_classic(cnt, B)
    # vectorised restatement through the matrix
    with np.errstate(divide="ignore"):
        inv = np.where((P > 0) & off, 1.0 / P ** 2, 0.0)
    np.testing.assert_allclose(pr, inv.sum(axis=1) / (N - 1), rtol=1e-12)
    np.testing.assert_allclose(cl, N / (np.where(off, P, 0.0) ** 2).sum(axis=1), rtol=1e-12)
    # Cauchy-Schwarz over the m_i non-zero pairs of a sample: (sum 1/p^2)(sum p^2) >= m_i^2
    m = ((P > 0) & off).sum(axis=1)
    assert (pr * (N - 1) * (N / cl) >= m.astype(np.float64) ** 2 * (1 - 1e-12)).all()
    # every term of the printed sum is at least 1, and at most B^2
    assert (pr * (N - 1) >= m - 1e-9).all() and (pr * (N - 1) <= m * float(B) ** 2 + 1e-6).all()
    # the class-restricted measure is never below the unrestricted one (fewer terms in the denominator)
    assert (oracle.outlier_classic(cnt, B, y) >= cl * (1 - 1e-12)).all()


def test_oob_vote(cfg1):
    # hand example: 2 trees, 3 samples, 2 classes
    leaf = np.array([[0, 1, 1], [1, 0, 1]], np.uint32)
    inbag = np.array([[0, 1, 0], [0, 0, 2]], np.uint16)
    leaf_class = np.array([[1, 0], [0, 1]], np.int32)
    votes, pred = oracle.oob_vote(leaf, inbag, leaf_class, 2)
    # sample 0: tree 0 leaf 0 -> class 1, tree 1 leaf 1 -> class 1; sample 1: tree 1 leaf 0 -> class 0; sample 2: tree 0 leaf 1 -> class 0
    np.testing.assert_array_equal(votes, [[0, 2], [1, 0], [1, 0]])
    np.testing.assert_array_equal(pred, [1, 0, 0])
    assert oracle.oob_error(pred, np.array([1, 1, 0])) == (1, 3)
    # ties go to the lowest class; never out-of-bag gives -1
    leaf_class = np.array([[1, 0], [0, 0]], np.int32)
    inbag = np.array([[0, 1, 1], [0, 1, 0]], np.uint16)
    votes, pred = oracle.oob_vote(leaf, inbag, leaf_class, 2)
    np.testing.assert_array_equal(votes, [[1, 1], [0, 0], [1, 0]])
    np.testing.assert_array_equal(pred, [0, -1, 0])
    assert oracle.oob_error(pred, np.array([0, 0, 1])) == (1, 2)

    # grown forest: leaf classes of purity-grown trees are the (single) class of their in-bag rows
    F, X, y, leaf = cfg1["F"], cfg1["X"], cfg1["y"], cfg1["leaf"]
    C = int(y.max()) + 1
    lc = ri.leaf_classes(F, y, C)
    B, N = leaf.shape
    for b in range(0, B, 17):
        rows = np.nonzero(F.inbag[b] > 0)[0]
        np.testing.assert_array_equal(lc[b][leaf[b][rows]], y[rows])
        assert (lc[b][: F.n_leaves[b]] >= 0).all() and (lc[b][F.n_leaves[b]:] == -1).all()
    votes, pred = oracle.oob_vote(leaf, F.inbag, lc, C)
    # vectorised restatement: one-hot of the leaf classes masked by the out-of-bag indicator
    cls = np.take_along_axis(lc, leaf.astype(np.int64), axis=1)
    want = np.stack([((cls == c) & (F.inbag == 0)).sum(axis=0) for c in range(C)], axis=1)
    np.testing.assert_array_equal(votes, want)
    np.testing.assert_array_equal(votes.sum(axis=1), (F.inbag == 0).sum(axis=0))
    wrong, voted = oracle.oob_error(pred, y)
    assert voted == N and wrong / voted < 0.2          # a separable 3-class mixture
    # using every tree (in-bag ones included) can only look better on the training rows
    all_votes, all_pred = oracle.oob_vote(leaf, np.zeros_like(F.inbag), lc, C)
    assert oracle.oob_error(all_pred, y)[0] <= wrong
