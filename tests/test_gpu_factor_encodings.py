"""GPU parity for the FP32 / FP16 / NF4 factor encodings, scaling from any encoding, and the
correlation between embeddings from compressed factors and from the full proximity matrix."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _codes_to_numpy(codes, encoding, N, k):
    import paper_2511_19493_amd as rfx
    raw = codes.cpu().numpy()
    if encoding == rfx.ENC_INT8:
        return raw.view(np.int8).reshape(N, k)
    if encoding == rfx.ENC_FP16:
        return raw.view(np.float16).reshape(N, k)
    if encoding == rfx.ENC_FP32:
        return raw.view(np.float32).reshape(N, k)
    return raw.reshape((N + 1) // 2, k)


@pytest.mark.parametrize("N,k", [(301, 5), (178, 16), (4096, 64), (1000, 100)])
def test_encodings_bit_exact(torch_cuda, N, k):
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    print(f"factor encodings N={N} k={k}", flush=True)
    rng = np.random.default_rng(N + k)
    V = rng.standard_normal((N, k)).astype(np.float32)
    V[:, 0] = 0.0                                     # an all-zero column
    if N > 200:
        V[64:128, 1] = 0.0                            # an all-zero NF4 block
    lam = rng.uniform(0.0, 40.0, k).astype(np.float32)
    lam[-1] = -1.0                                    # a non-positive Ritz value contributes nothing
    dV, dl = torch.from_numpy(V).cuda(), torch.from_numpy(lam).cuda()
    for enc, oenc in ((rfx.ENC_INT8, oracle.ENC_INT8), (rfx.ENC_FP16, oracle.ENC_FP16), (rfx.ENC_NF4, oracle.ENC_NF4),
                      (rfx.ENC_FP32, oracle.ENC_FP32)):
        codes, scales = rfx.quantise_factor(dV, dl, enc)
        rc, rs = oracle.quantise_factor(V, lam, oenc)
        got = _codes_to_numpy(codes, enc, N, k)
        np.testing.assert_array_equal(got, rc)          # floating-point codes compare by value: the sign of a zero is not fixed
        np.testing.assert_array_equal(scales.cpu().numpy().reshape(rs.shape), rs)
        A = rfx.dequantise_factor(codes, scales, N, k, enc)
        np.testing.assert_array_equal(A.cpu().numpy(), oracle.dequantise_factor(rc, rs, oenc, N))
        cb, ns = rfx.factor_sizes(enc, N, k)
        assert cb == rc.nbytes and ns == rs.size


def test_nf4_level_table_of_the_library_equals_the_oracles(torch_cuda):
    """Every one of the 16 codes decoded on the GPU with unit scales gives the oracle's level bit for bit
    (the oracle's table is pinned to the normal-quantile construction by a CPU test), and the decision
    thresholds (midpoints of adjacent levels) agree: values just below, at and just above every midpoint
    encode to the same codes on both sides."""
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    N, k = 64, 1
    code = (np.arange(N) % 16).astype(np.uint8).reshape(N, 1)
    packed = (code[0::2] | (code[1::2] << 4)).astype(np.uint8)
    ones = np.ones((1, 1), np.float32)
    A = rfx.dequantise_factor(torch.from_numpy(packed).cuda(), torch.from_numpy(ones).cuda(), N, k, rfx.ENC_NF4)
    np.testing.assert_array_equal(A.cpu().numpy()[:16, 0], oracle.NF4_LEVELS)
    np.testing.assert_array_equal(A.cpu().numpy(), oracle.dequantise_factor(packed, ones, oracle.ENC_NF4, N))
    # one block whose maximum is exactly 1, so the normalised values are the values themselves
    lv = oracle.NF4_LEVELS
    mid = ((lv[:-1] + lv[1:]) * np.float32(0.5)).astype(np.float32)
    vals = np.concatenate([[1.0], np.nextafter(mid, np.float32(-2)), mid, np.nextafter(mid, np.float32(2)), lv[1:-1]])
    V = np.zeros((64, 1), np.float32)
    V[:vals.size, 0] = vals.astype(np.float32)
    lam = np.ones(1, np.float32)
    codes, scales = rfx.quantise_factor(torch.from_numpy(V).cuda(), torch.from_numpy(lam).cuda(), rfx.ENC_NF4)
    rc, rs = oracle.quantise_factor(V, lam, oracle.ENC_NF4)
    np.testing.assert_array_equal(codes.cpu().numpy().reshape(rc.shape), rc)
    np.testing.assert_array_equal(scales.cpu().numpy().reshape(rs.shape), rs)


def test_scaling_from_every_encoding_and_correlation_with_the_full_matrix(torch_cuda, small2):
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    leaf = small2["leaf"]
    B, N = leaf.shape
    k = 32
    dleaf = torch.from_numpy(leaf.view(np.int32)).cuda()
    lam, V, Q, s = rfx.prox_lowrank(dleaf, int(leaf.max()) + 1, torch.from_numpy(ri.start_block(N, k)).cuda(), 20)
    P = oracle.counts_full(leaf).astype(np.float64) / B
    full, _ = oracle.mds3d_from_dense_proximity(P)                 # the paper's full-matrix pathway
    x0 = torch.from_numpy(ri.start_block(N, 12, seed=778)).cuda()
    rho = {}
    for name, enc, oenc in (("fp32", rfx.ENC_FP32, oracle.ENC_FP32), ("fp16", rfx.ENC_FP16, oracle.ENC_FP16),
                            ("int8", rfx.ENC_INT8, oracle.ENC_INT8), ("nf4", rfx.ENC_NF4, oracle.ENC_NF4)):
        codes, scales = rfx.quantise_factor(V, lam, enc)
        A = rfx.dequantise_factor(codes, scales, N, k, enc)
        coords, ev, iters = rfx.mds3d_factor(A, x0, rfx.MDS_SQUARED, max_iters=500, tol=1e-7)
        ref, ev_ref = oracle.mds3d_from_factor(A.cpu().numpy())
        np.testing.assert_allclose(ev.cpu().numpy(), ev_ref, rtol=1e-4)
        c = coords.cpu().numpy().astype(np.float64)
        if (np.abs(np.diff(ev_ref)) / ev_ref[0]).min() <= 1e-2:
            U, _, Vt = np.linalg.svd(c.T @ ref)
            c = c @ (U @ Vt)
        assert np.linalg.norm(c - ref) / np.linalg.norm(ref) <= 1e-3
        rho[name] = oracle.mds_correlation(coords.cpu().numpy(), full)
    print("correlation of pairwise distances with the full-matrix embedding:", {n: round(v, 4) for n, v in rho.items()}, flush=True)
    assert rho["fp32"] > 0.9 and abs(rho["fp16"] - rho["fp32"]) < 1e-3 and abs(rho["int8"] - rho["fp32"]) < 1e-2
    assert rho["nf4"] > rho["fp32"] - 0.1
    # INT8 path of rfx_mds3d agrees with the generic one
    coords8, ev8, _ = rfx.mds3d(Q, s, x0, rfx.MDS_SQUARED, max_iters=500, tol=1e-7)
    A8 = rfx.dequantise_factor(Q.view(torch.uint8).reshape(-1), s, N, k, rfx.ENC_INT8)
    coordsg, evg, _ = rfx.mds3d_factor(A8, x0, rfx.MDS_SQUARED, max_iters=500, tol=1e-7)
    assert torch.equal(coords8, coordsg) and torch.equal(ev8, evg)
