"""GPU parity for forest growth: the library's trees against the oracle's, array by array (all integer
decisions, so everything is compared bit-exactly, thresholds included)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

KEYS = ("node_offset", "feature", "threshold", "left", "right", "leaf_id", "depth", "n_leaves", "inbag", "leaf_class")


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _compare(torch, X, y, C, B, mtry, seed, first_tree=0):
    import oracle
    import paper_2511_19493_amd as rfx
    print(f"grow N={X.shape[0]} M={X.shape[1]} C={C} B={B} mtry={mtry} seed={seed} first={first_tree}", flush=True)
    got = rfx.forest_grow(torch.from_numpy(np.ascontiguousarray(X, np.float32)).cuda(),
                          torch.from_numpy(np.ascontiguousarray(y, np.int32)).cuda(), C, B, mtry, seed, first_tree)
    ref = oracle.grow(X, y, C, B, mtry, seed, first_tree)
    for k in KEYS:
        if k == "threshold":
            np.testing.assert_array_equal(got[k].view(np.uint32), ref[k].view(np.uint32), err_msg=k)
        else:
            np.testing.assert_array_equal(got[k], ref[k], err_msg=k)
    # level passes: one per depth that holds an impure node (the last one may only turn nodes into impure leaves)
    assert got["levels"] in (int(ref["depth"].max()), int(ref["depth"].max()) + 1)
    return got


def test_growth_on_the_small_workloads(torch_cuda, cfg1, small2):
    _compare(torch_cuda, cfg1["X"], cfg1["y"], 3, 100, 3, 12345)
    _compare(torch_cuda, cfg1["X"], cfg1["y"], 3, 7, 13, 1, first_tree=1000)        # every feature offered
    _compare(torch_cuda, small2["X"], small2["y"], 5, 64, 4, 2024)                  # 10 % label noise: deep trees


def test_growth_on_degenerate_inputs(torch_cuda):
    rng = np.random.default_rng(5)
    # one row; two rows of one class; one class only
    _compare(torch_cuda, np.zeros((1, 2), np.float32), np.zeros(1, np.int32), 1, 3, 1, 9)
    _compare(torch_cuda, rng.standard_normal((2, 3)).astype(np.float32), np.array([1, 1], np.int32), 2, 4, 2, 9)
    _compare(torch_cuda, rng.standard_normal((50, 3)).astype(np.float32), np.zeros(50, np.int32), 1, 4, 2, 9)
    # constant features, few distinct values, rows that no split can separate: fallback features and impure leaves
    N = 300
    X = np.zeros((N, 6), np.float32)
    X[:, 4] = rng.integers(0, 5, N)
    X[:, 1] = rng.integers(0, 2, N)
    y = ((X[:, 4] >= 2) ^ (X[:, 1] > 0)).astype(np.int32)
    y[:30] = rng.integers(0, 2, 30)
    _compare(torch_cuda, X, y, 2, 24, 1, 77)
    _compare(torch_cuda, X, y, 2, 24, 2, 78)
    # signed zeros and ties between features
    X = rng.integers(-1, 2, size=(200, 4)).astype(np.float32) * np.float32(0.0) + rng.integers(-1, 2, size=(200, 4)).astype(np.float32)
    X[::7, 0] = -0.0
    y = rng.integers(0, 3, 200).astype(np.int32)
    _compare(torch_cuda, X, y, 3, 16, 2, 79)
    # many classes
    X = rng.standard_normal((500, 5)).astype(np.float32)
    y = rng.integers(0, 64, 500).astype(np.int32)
    _compare(torch_cuda, X, y, 64, 8, 2, 80)


def test_growth_with_long_segments_of_few_values(torch_cuda):
    """Segments far longer than the sorting networks take, whose values are a handful of distinct numbers (every pair of a
    segment lands in a few buckets that stay long through both bucket passes), next to continuous features and one whose
    values all share sign and exponent (spread over the buckets only by the second pass)."""
    rng = np.random.default_rng(21)
    N = 30000
    X = np.empty((N, 6), np.float32)
    X[:, 0] = rng.integers(0, 3, N)                       # three values
    X[:, 1] = 7.0                                         # one value
    X[:, 2] = rng.standard_normal(N)
    X[:, 3] = 1.0 + rng.random(N)                         # all in [1, 2): one exponent
    X[:, 4] = np.round(rng.standard_normal(N) * 2.0) * 0.5
    X[:, 5] = rng.standard_normal(N) * 1e-3
    y = ((X[:, 0] > 0) + (X[:, 2] > 0.3) + (X[:, 3] > 1.5)).astype(np.int32)
    y[::17] = rng.integers(0, 4, len(y[::17]))
    _compare(torch_cuda, X, y, 4, 6, 3, 4242)
    _compare(torch_cuda, X, y, 4, 3, 6, 4243)


def test_growth_with_the_largest_feature_subsets(torch_cuda):
    rng = np.random.default_rng(11)
    for M, mtry in ((64, 64), (70, 64), (200, 64), (1000, 31)):
        X = rng.standard_normal((400, M)).astype(np.float32)
        X[:, ::3] = np.round(X[:, ::3])                   # many ties inside a third of the features
        y = rng.integers(0, 4, 400).astype(np.int32)
        _compare(torch_cuda, X, y, 4, 6, mtry, 1000 + M)


def test_growth_medium(torch_cuda):
    import rfx_inputs as ri
    c = ri.CONFIGS[2]
    X, y = ri.gaussian_mixture(c)                       # 10,000 x 20, 5 classes, 10 % label noise
    g = _compare(torch_cuda, X, y, c.C, 24, c.mtry, 31337)
    # the grown forest drives the rest of the library
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    F = rfx.Forest(g["n_features"], g["node_offset"], g["feature"], g["threshold"], g["left"], g["right"], g["leaf_id"], g["n_leaves"])
    leaf = rfx.leaf_assign(F, torch.from_numpy(X).cuda())
    votes, pred, wrong, voted = rfx.oob_vote(leaf, torch.from_numpy(g["inbag"].view(np.int16)).cuda(),
                                             torch.from_numpy(g["leaf_class"]).cuda(), c.C, torch.from_numpy(y.astype(np.int32)).cuda())
    print(f"out-of-bag error of the grown forest: {wrong}/{voted}", flush=True)
    assert voted == X.shape[0] and 0.05 < wrong / voted < 0.25      # 10 % of the labels are noise


def test_growth_argument_errors(torch_cuda):
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    X = torch.zeros((4, 3), dtype=torch.float32, device="cuda")
    y = torch.zeros(4, dtype=torch.int32, device="cuda")
    for kw in (dict(n_classes=65), dict(mtry=4), dict(mtry=0), dict(n_trees=0)):
        a = dict(n_classes=2, n_trees=2, mtry=1, seed=1)
        a.update(kw)
        with pytest.raises(rfx.RfxError) as e:
            rfx.forest_grow(X, y, **a)
        assert e.value.code == rfx.ERR_INVALID_ARG
