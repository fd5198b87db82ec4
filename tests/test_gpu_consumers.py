"""GPU parity for the proximity consumers: outlier measures and the out-of-bag vote."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _dev(torch, leaf):
    return torch.from_numpy(np.ascontiguousarray(leaf).view(np.int32)).cuda()


def _check_outlier(torch, leaf, bound, labels):
    import oracle
    import paper_2511_19493_amd as rfx
    B, N = leaf.shape
    cnt = oracle.counts_full(leaf)
    dl = torch.from_numpy(labels.astype(np.int32)).cuda() if labels is not None else None
    printed, classic = rfx.prox_outlier(_dev(torch, leaf), bound, dl)
    # float64 sums in a different order: 1e-12 relative (N terms of rounding 1e-16 each); inf must match exactly
    np.testing.assert_allclose(printed.cpu().numpy(), oracle.outlier_printed(cnt, B), rtol=1e-12, atol=0)
    ref = oracle.outlier_classic(cnt, B, labels)
    got = classic.cpu().numpy()
    np.testing.assert_array_equal(np.isinf(got), np.isinf(ref))
    fin = ~np.isinf(ref)
    np.testing.assert_allclose(got[fin], ref[fin], rtol=1e-12, atol=0)
    # one output at a time gives the same values
    only_p, none = rfx.prox_outlier(_dev(torch, leaf), bound, dl, want_classic=False)
    assert none is None
    np.testing.assert_allclose(only_p.cpu().numpy(), printed.cpu().numpy(), rtol=1e-13)
    none, only_c = rfx.prox_outlier(_dev(torch, leaf), bound, dl, want_printed=False)
    assert torch.equal(only_c, classic)       # integer sums: bit-identical


@pytest.mark.parametrize("N,B,bound", [(2, 1, 2), (5, 3, 2), (255, 31, 40), (257, 33, 40), (515, 65, 2), (300, 97, 1),
                                       (700, 40, 3000)])
def test_outlier_on_boundary_shapes(torch_cuda, N, B, bound):
    print(f"outlier boundary shapes N={N} B={B} bound={bound}", flush=True)
    rng = np.random.default_rng(9000 * N + B)
    leaf = rng.integers(0, bound, size=(B, N)).astype(np.uint32)
    _check_outlier(torch_cuda, leaf, bound, None)
    _check_outlier(torch_cuda, leaf, bound, rng.integers(0, 3, size=N))


def test_outlier_on_grown_forests(torch_cuda, cfg1, small2):
    for name, w in (("cfg1", cfg1), ("small2", small2)):
        print(f"outlier {name}", flush=True)
        leaf = w["leaf"]
        _check_outlier(torch_cuda, leaf, int(leaf.max()) + 1, w["y"])
        _check_outlier(torch_cuda, leaf, int(leaf.max()) + 1, None)


def test_outlier_argument_errors(torch_cuda):
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    one = torch.zeros((3, 1), dtype=torch.int32, device="cuda")
    with pytest.raises(rfx.RfxError) as e:
        rfx.prox_outlier(one, 1)
    assert e.value.code == rfx.ERR_INVALID_ARG
    two = torch.zeros((3, 2), dtype=torch.int32, device="cuda")
    with pytest.raises(rfx.RfxError) as e:
        rfx.prox_outlier(two, 1, want_printed=False, want_classic=False)
    assert e.value.code == rfx.ERR_NULL


def _check_vote(torch, leaf, inbag, leaf_class, C, y):
    import oracle
    import paper_2511_19493_amd as rfx
    votes, pred, wrong, voted = rfx.oob_vote(_dev(torch, leaf), torch.from_numpy(inbag.view(np.int16)).cuda(),
                                             torch.from_numpy(np.ascontiguousarray(leaf_class, np.int32)).cuda(), C,
                                             torch.from_numpy(y.astype(np.int32)).cuda())
    rv, rp = oracle.oob_vote(leaf, inbag, leaf_class, C)
    np.testing.assert_array_equal(votes.cpu().numpy().view(np.uint32), rv)
    np.testing.assert_array_equal(pred.cpu().numpy(), rp)
    assert (wrong, voted) == oracle.oob_error(rp, y)
    # without labels and without the vote table
    v2, p2, w2, n2 = rfx.oob_vote(_dev(torch, leaf), torch.from_numpy(inbag.view(np.int16)).cuda(),
                                  torch.from_numpy(np.ascontiguousarray(leaf_class, np.int32)).cuda(), C, want_votes=False)
    assert v2 is None and w2 is None and n2 == voted and torch.equal(p2, pred)


@pytest.mark.parametrize("N,B,L,C", [(1, 1, 1, 1), (3, 2, 2, 2), (255, 7, 5, 3), (257, 64, 300, 20), (1000, 33, 17, 128),
                                     (513, 5, 9, 65)])
def test_oob_vote_on_random_inputs(torch_cuda, N, B, L, C):
    print(f"oob vote N={N} B={B} L={L} C={C}", flush=True)
    rng = np.random.default_rng(31 * N + B)
    leaf = rng.integers(0, L, size=(B, N)).astype(np.uint32)
    inbag = rng.integers(0, 3, size=(B, N)).astype(np.uint16)
    inbag[:, N // 2] = 1                                  # a sample that is never out-of-bag
    leaf_class = rng.integers(0, C, size=(B, L)).astype(np.int32)
    y = rng.integers(0, C, size=N)
    _check_vote(torch_cuda, leaf, inbag, leaf_class, C, y)


def test_oob_vote_on_grown_forests(torch_cuda, cfg1, small2):
    import rfx_inputs as ri
    for name, w in (("cfg1", cfg1), ("small2", small2)):
        print(f"oob vote {name}", flush=True)
        C = int(w["y"].max()) + 1
        lc = ri.leaf_classes(w["F"], w["y"], C)
        _check_vote(torch_cuda, w["leaf"], w["F"].inbag, lc, C, w["y"])
    # all in-bag: nobody votes
    leaf, F = cfg1["leaf"], cfg1["F"]
    C = int(cfg1["y"].max()) + 1
    _check_vote(torch_cuda, leaf, np.ones_like(F.inbag), ri.leaf_classes(F, cfg1["y"], C), C, cfg1["y"])


def test_oob_vote_argument_errors(torch_cuda):
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    leaf = torch.zeros((2, 4), dtype=torch.int32, device="cuda")
    inbag = torch.zeros((2, 4), dtype=torch.int16, device="cuda")
    lc = torch.zeros((2, 1), dtype=torch.int32, device="cuda")
    with pytest.raises(rfx.RfxError) as e:
        rfx.oob_vote(leaf, inbag, lc, 129)
    assert e.value.code == rfx.ERR_INVALID_ARG
    with pytest.raises(rfx.RfxError) as e:
        rfx.oob_vote(leaf, inbag, lc, 0)
    assert e.value.code == rfx.ERR_INVALID_ARG
