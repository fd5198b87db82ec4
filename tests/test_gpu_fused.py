"""GPU parity for the fused plain + out-of-bag proximity pass (rfx_prox_dense_oob)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _u(t):
    a = t.cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a.view(np.uint32)


def _check(torch, leaf, inbag, bound):
    import oracle
    import paper_2511_19493_amd as rfx
    B, N = leaf.shape
    dl = torch.from_numpy(np.ascontiguousarray(leaf).view(np.int32)).cuda()
    di = torch.from_numpy(np.ascontiguousarray(inbag).view(np.int16)).cuda()
    cnt = oracle.counts_full(leaf)
    rn, rd = oracle.oob_rows(leaf, inbag, 0, N)
    rp, rpo = oracle.normalise(cnt, B), oracle.prox_oob_rows(rn, rd, 0)
    for dtype, npdt in ((rfx.U32, np.uint32), (rfx.U16, np.uint16)):
        c, p, n, d, po = rfx.prox_dense_oob(dl, di, bound, dtype, rfx.FULL, rfx.FULL)
        np.testing.assert_array_equal(_u(c), cnt.astype(npdt))
        np.testing.assert_array_equal(p.cpu().numpy(), rp)
        np.testing.assert_array_equal(_u(n), rn.astype(npdt))
        np.testing.assert_array_equal(_u(d), rd.astype(npdt))
        np.testing.assert_array_equal(po.cpu().numpy(), rpo)
        if N > 1:
            c, p, n, d, po = rfx.prox_dense_oob(dl, di, bound, dtype, rfx.FULL, rfx.UPPER_PACKED)    # as bench.py uses it
            np.testing.assert_array_equal(_u(c), cnt.astype(npdt))
            np.testing.assert_array_equal(p.cpu().numpy(), rp)
            np.testing.assert_array_equal(_u(n), oracle.pack_upper(rn).astype(npdt))
            np.testing.assert_array_equal(_u(d), oracle.pack_upper(rd).astype(npdt))
            np.testing.assert_array_equal(po.cpu().numpy(), oracle.pack_upper(rpo))
            c, p, n, d, po = rfx.prox_dense_oob(dl, di, bound, dtype, rfx.UPPER_PACKED, rfx.FULL, want_num_den=False)
            assert n is None and d is None
            np.testing.assert_array_equal(_u(c), oracle.pack_upper(cnt).astype(npdt))
            np.testing.assert_array_equal(p.cpu().numpy(), oracle.pack_upper(rp))
            np.testing.assert_array_equal(po.cpu().numpy(), rpo)


@pytest.mark.parametrize("N,B,bound", [(1, 3, 5), (2, 1, 2), (255, 31, 40), (256, 32, 40), (257, 33, 40), (260, 64, 300),
                                       (515, 65, 2), (300, 97, 1), (130, 1023, 7)])
def test_fused_on_boundary_shapes(torch_cuda, N, B, bound):
    print(f"fused boundary shapes N={N} B={B} bound={bound}", flush=True)
    rng = np.random.default_rng(500 * N + B)
    leaf = rng.integers(0, bound, size=(B, N)).astype(np.uint32)
    inbag = rng.integers(0, 3, size=(B, N)).astype(np.uint16)
    _check(torch_cuda, leaf, inbag, bound)


def test_fused_field_limits(torch_cuda):
    """All three 10-bit fields at their maximum: one leaf, everything out-of-bag, 1023 trees."""
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    N, B = 70, 1023
    _check(torch, np.zeros((B, N), np.uint32), np.zeros((B, N), np.uint16), 1)
    # every pair mismatches in every tree: the mismatch field reaches 1023
    leaf = np.tile(np.arange(N, dtype=np.uint32), (B, 1))
    _check(torch, leaf, np.zeros((B, N), np.uint16), N)
    with pytest.raises(rfx.RfxError) as e:
        rfx.prox_dense_oob(torch.zeros((1024, 4), dtype=torch.int32, device="cuda"),
                           torch.zeros((1024, 4), dtype=torch.int16, device="cuda"), 1)
    assert e.value.code == rfx.ERR_UNSUPPORTED


def test_fused_on_grown_forests(torch_cuda, cfg1, small2):
    for name, w in (("cfg1", cfg1), ("small2", small2)):
        print(f"fused {name}", flush=True)
        _check(torch_cuda, w["leaf"], w["F"].inbag, int(w["leaf"].max()) + 1)
