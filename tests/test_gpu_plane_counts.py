"""Every bit-plane count the tile kernel is instantiated for (8..16, 18, 20, 22, 24), in every mode: plain,
out-of-bag, fused, sparse and outlier, against the oracle.  The ids come from a small set spread over the whole
range below the bound, so that pairs match and pairs differ in any single bit position, the high ones included."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

BOUNDS = [200, 400, 1000, 2000, 4000, 8000, 16000, 30000, 60000, 200000, 1000000, 3000000, 1 << 24]


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    return torch


def _u(t):
    a = t.cpu().numpy()
    return a.view({np.dtype(np.int32): np.uint32, np.dtype(np.int16): np.uint16}.get(a.dtype, a.dtype))


def _ids(rng, bound, B, N):
    base = rng.integers(0, bound, size=6, dtype=np.int64)
    hot = [base]
    bit = 1
    while bit < bound:                       # neighbours of the base ids that differ in exactly one bit
        hot.append(base ^ bit)
        bit <<= 1
    hot = np.unique(np.concatenate(hot + [np.array([0, bound - 1])]))
    hot = hot[hot < bound]
    return hot[rng.integers(0, hot.size, size=(B, N))].astype(np.uint32)


@pytest.mark.parametrize("bound", BOUNDS)
def test_every_plane_count_in_every_mode(torch_cuda, bound):
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    N, B = 300, 45
    rng = np.random.default_rng(bound)
    leaf = _ids(rng, bound, B, N)
    inbag = rng.integers(0, 3, size=(B, N)).astype(np.uint16)
    labels = rng.integers(0, 3, size=N).astype(np.int32)
    print(f"plane counts: bound={bound} distinct ids={np.unique(leaf).size}", flush=True)
    dl = torch.from_numpy(leaf.view(np.int32)).cuda()
    di = torch.from_numpy(inbag.view(np.int16)).cuda()
    cnt = oracle.counts_full(leaf)
    rn, rd = oracle.oob_rows(leaf, inbag, 0, N)
    # plain
    c, p = rfx.prox_dense(dl, bound, rfx.U32, rfx.FULL)
    np.testing.assert_array_equal(_u(c), cnt)
    np.testing.assert_array_equal(p.cpu().numpy(), oracle.normalise(cnt, B))
    # out-of-bag
    num, den, po = rfx.prox_oob(dl, di, bound, rfx.U32, rfx.FULL)
    np.testing.assert_array_equal(_u(num), rn)
    np.testing.assert_array_equal(_u(den), rd)
    np.testing.assert_array_equal(po.cpu().numpy(), oracle.prox_oob_rows(rn, rd, 0))
    # fused
    c, p, n, d, po = rfx.prox_dense_oob(dl, di, bound, rfx.U32, rfx.FULL, rfx.UPPER_PACKED)
    np.testing.assert_array_equal(_u(c), cnt)
    np.testing.assert_array_equal(_u(n), oracle.pack_upper(rn))
    np.testing.assert_array_equal(_u(d), oracle.pack_upper(rd))
    np.testing.assert_array_equal(po.cpu().numpy(), oracle.pack_upper(oracle.prox_oob_rows(rn, rd, 0)))
    # sparse
    rr, rc, rv = oracle.sparse_upper(leaf, 2)
    assert rfx.prox_sparse_count(dl, bound, 2) == rr.size
    rows, cols, counts, _ = rfx.prox_sparse(dl, bound, 2)
    got = np.stack([rows.cpu().numpy().astype(np.int64), cols.cpu().numpy().astype(np.int64),
                    _u(counts).astype(np.int64)], axis=1)
    got = got[np.lexsort((got[:, 1], got[:, 0]))]
    np.testing.assert_array_equal(got, np.stack([rr, rc, rv], axis=1).astype(np.int64))
    # outlier sums
    printed, classic = rfx.prox_outlier(dl, bound, torch.from_numpy(labels).cuda())
    np.testing.assert_allclose(printed.cpu().numpy(), oracle.outlier_printed(cnt, B), rtol=1e-12, atol=0)
    ref, got = oracle.outlier_classic(cnt, B, labels), classic.cpu().numpy()
    np.testing.assert_array_equal(np.isinf(got), np.isinf(ref))
    np.testing.assert_allclose(got[~np.isinf(ref)], ref[~np.isinf(ref)], rtol=1e-12, atol=0)
