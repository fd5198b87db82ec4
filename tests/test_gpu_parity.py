"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _forest(F):
    import paper_2511_19493_amd as rfx
    return rfx.Forest(F.n_features, F.node_offset, F.feature, F.threshold, F.left, F.right, F.leaf_id, F.n_leaves)


def _u(t):
    """Counts come back as int16/int32 tensors holding unsigned bits."""
    a = t.cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a.view(np.uint32)


def _dev_leaf(torch, leaf):
    return torch.from_numpy(leaf.view(np.int32)).cuda()


@pytest.mark.parametrize("which", ["cfg1", "small2"])
def test_leaf_assign_bit_exact(torch_cuda, request, which):
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    d = request.getfixturevalue(which)
    print(f"leaf_assign {which} N={d['X'].shape[0]} B={d['F'].n_trees}", flush=True)
    gf = _forest(d["F"])
    assert gf.leaf_bound == int(d["F"].n_leaves.max())
    leaf = rfx.leaf_assign(gf, torch.from_numpy(d["X"]).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(_u(leaf), d["leaf"])


def test_leaf_assign_nan_goes_right_and_bad_forest_is_rejected(torch_cuda, cfg1):
    import paper_2511_19493_amd as rfx
    import oracle
    torch = torch_cuda
    X = cfg1["X"].copy()
    X[::5, ::3] = np.nan
    ref, _ = oracle.leaf_assign(cfg1["F"], X)
    leaf = rfx.leaf_assign(_forest(cfg1["F"]), torch.from_numpy(X).cuda())
    np.testing.assert_array_equal(_u(leaf), ref)
    F = cfg1["F"]
    bad_left = F.left.copy()
    bad_left[0] = 10_000
    with pytest.raises(rfx.RfxError) as ei:
        rfx.Forest(F.n_features, F.node_offset, F.feature, F.threshold, bad_left, F.right, F.leaf_id, F.n_leaves)
    assert ei.value.code == -7


def test_prox_dense_full_u32_cfg1(torch_cuda, cfg1):
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    leaf = cfg1["leaf"]
    B, N = leaf.shape
    print(f"prox_dense full u32 N={N} B={B}", flush=True)
    cnt, prox = rfx.prox_dense(_dev_leaf(torch, leaf), int(leaf.max()) + 1, rfx.U32, rfx.FULL)
    torch.cuda.synchronize()
    ref = oracle.counts_full(leaf)
    np.testing.assert_array_equal(_u(cnt), ref)
    np.testing.assert_array_equal(prox.cpu().numpy(), oracle.normalise(ref, B))   # same IEEE division


def test_prox_dense_packed_u16_ragged(torch_cuda, small2):
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    leaf = small2["leaf"]
    B, N = leaf.shape                      # N = 1500: several tiles and a ragged tail
    print(f"prox_dense packed u16 N={N} B={B}", flush=True)
    cnt, prox = rfx.prox_dense(_dev_leaf(torch, leaf), int(leaf.max()) + 1, rfx.U16, rfx.UPPER_PACKED)
    torch.cuda.synchronize()
    ref = oracle.counts_full(leaf)
    np.testing.assert_array_equal(_u(cnt), oracle.pack_upper(ref).astype(np.uint16))
    np.testing.assert_allclose(prox.cpu().numpy(), oracle.pack_upper(oracle.normalise(ref, B)), rtol=1e-6)
    # full layout on the same input, counts only
    cnt2, none = rfx.prox_dense(_dev_leaf(torch, leaf), int(leaf.max()) + 1, rfx.U32, rfx.FULL, want_prox=False)
    assert none is None
    np.testing.assert_array_equal(_u(cnt2), ref)
    # full layout with N a multiple of 4 takes the vector-store path: uint16 counts and float32 quotients
    cnt3, prox3 = rfx.prox_dense(_dev_leaf(torch, leaf), int(leaf.max()) + 1, rfx.U16, rfx.FULL)
    np.testing.assert_array_equal(_u(cnt3), ref.astype(np.uint16))
    np.testing.assert_array_equal(prox3.cpu().numpy(), oracle.normalise(ref, B))
    # out-of-bag variant, full layout, same path
    inbag = small2["F"].inbag
    num, den, poob = rfx.prox_oob(_dev_leaf(torch, leaf), torch.from_numpy(inbag.view(np.int16)).cuda(),
                                  int(leaf.max()) + 1, rfx.U16, rfx.FULL)
    rn, rd = oracle.oob_rows(leaf, inbag, 0, N)
    np.testing.assert_array_equal(_u(num), rn.astype(np.uint16))
    np.testing.assert_array_equal(_u(den), rd.astype(np.uint16))
    np.testing.assert_array_equal(poob.cpu().numpy(), oracle.prox_oob_rows(rn, rd, 0))


@pytest.mark.parametrize("bound", [1, 2, 3, 17, 300, 70000])
def test_prox_dense_any_leaf_id_width(torch_cuda, bound):
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    rng = np.random.default_rng(bound)
    # ids drawn from a small pool inside [0, bound) so that matches occur at every width
    pool = rng.integers(0, bound, size=min(bound, 6))
    leaf = pool[rng.integers(0, len(pool), size=(37, 300))].astype(np.uint32)
    cnt, _ = rfx.prox_dense(_dev_leaf(torch, leaf), bound, rfx.U32, rfx.FULL, want_prox=False)
    np.testing.assert_array_equal(_u(cnt), oracle.counts_full(leaf))


@pytest.mark.parametrize("which,layout", [("cfg1", "full"), ("small2", "packed")])
def test_prox_oob(torch_cuda, request, which, layout):
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    d = request.getfixturevalue(which)
    leaf, inbag = d["leaf"], d["F"].inbag
    B, N = leaf.shape
    print(f"prox_oob {which} {layout} N={N} B={B}", flush=True)
    lay = rfx.FULL if layout == "full" else rfx.UPPER_PACKED
    num, den, prox = rfx.prox_oob(_dev_leaf(torch, leaf), torch.from_numpy(inbag.view(np.int16)).cuda(),
                                  int(leaf.max()) + 1, rfx.U32, lay)
    torch.cuda.synchronize()
    rn, rd = oracle.oob_rows(leaf, inbag, 0, N)
    rp = oracle.prox_oob_rows(rn, rd, 0)
    if layout == "packed":
        rn, rd, rp = oracle.pack_upper(rn), oracle.pack_upper(rd), oracle.pack_upper(rp)
    np.testing.assert_array_equal(_u(num), rn)
    np.testing.assert_array_equal(_u(den), rd)
    np.testing.assert_array_equal(prox.cpu().numpy(), rp)


@pytest.mark.parametrize("which,k", [("cfg1", 16), ("small2", 32), ("small2", 64), ("cfg1", 5), ("small2", 100)])
def test_matvec(torch_cuda, request, which, k):
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    d = request.getfixturevalue(which)
    leaf = d["leaf"]
    B, N = leaf.shape
    print(f"matvec {which} N={N} B={B} k={k}", flush=True)
    V = ri.start_block(N, k)
    ref = oracle.pv_implicit(leaf, V.astype(np.float64))
    Y = rfx.prox_matvec(_dev_leaf(torch, leaf), int(leaf.max()) + 1, torch.from_numpy(V).cuda())
    torch.cuda.synchronize()
    err = np.linalg.norm(Y.cpu().numpy().astype(np.float64) - ref) / np.linalg.norm(ref)
    assert err <= 1e-5, err
    # plan reuse and run-to-run reproducibility
    plan = rfx.PvPlan(_dev_leaf(torch, leaf), int(leaf.max()) + 1)
    Y1 = plan.apply(torch.from_numpy(V).cuda())
    Y2 = plan.apply(torch.from_numpy(V).cuda())
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2) and torch.equal(Y1, Y)
    plan.close()


def test_matvec_rejects_leaf_ids_beyond_the_bound(torch_cuda, cfg1):
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    leaf = cfg1["leaf"]
    with pytest.raises(rfx.RfxError):
        rfx.PvPlan(_dev_leaf(torch, leaf), int(leaf.max()))     # bound one too small


@pytest.mark.parametrize("which,k,T", [("cfg1", 16, 20), ("small2", 32, 20)])
def test_lowrank_against_the_same_iteration_in_float64(torch_cuda, request, which, k, T):
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    d = request.getfixturevalue(which)
    leaf = d["leaf"]
    B, N = leaf.shape
    print(f"lowrank {which} N={N} B={B} k={k} T={T}", flush=True)
    V0 = ri.start_block(N, k)
    lam_ref, V_ref = oracle.block_iteration(leaf, V0, T)
    lam, V, Q, s = rfx.prox_lowrank(_dev_leaf(torch, leaf), int(leaf.max()) + 1, torch.from_numpy(V0).cuda(), T)
    torch.cuda.synchronize()
    lam, V = lam.cpu().numpy(), V.cpu().numpy()
    np.testing.assert_allclose(lam, lam_ref, rtol=1e-4)
    assert oracle.principal_angle(V, V_ref) < 1e-3
    np.testing.assert_allclose(V.astype(np.float64).T @ V.astype(np.float64), np.eye(k), atol=5e-6)
    # sign convention: largest-magnitude entry of each column is positive
    assert (V[np.argmax(np.abs(V), axis=0), np.arange(k)] > 0).all()
    # the quantiser takes its rounding decisions in float32 on both sides: codes are bit-exact
    Qr, sr = oracle.quantise_int8(V, lam)
    np.testing.assert_array_equal(s.cpu().numpy(), sr)
    np.testing.assert_array_equal(Q.cpu().numpy(), Qr)
    Q2, s2 = rfx.quantise_int8(torch.from_numpy(V).cuda(), torch.from_numpy(lam).cuda())
    assert torch.equal(Q2, Q) and torch.equal(s2, s)
    # INT8-dequantised P.V on the converged block against the float64 product
    A = oracle.dequantise(Q.cpu().numpy(), s.cpu().numpy())
    Xb = V_ref
    PX = oracle.pv_implicit(leaf, Xb)
    err = np.linalg.norm(A @ (A.T @ Xb) - PX) / np.linalg.norm(PX)
    assert err <= 2e-2, err


@pytest.mark.parametrize("which,k", [("cfg1", 16), ("small2", 32)])
def test_reported_layer_against_the_dense_eigendecomposition(torch_cuda, request, which, k):
    """The binding check compares the library with the oracle running the same T = 20 applications in float64.
    This is the reported layer: the library's Ritz pairs against LAPACK's eigendecomposition of the materialised
    P.  After 20 applications only the leading, well-separated pairs have converged to 1e-4 (Ritz value j
    converges like (lambda_{k+1} / lambda_j)^(2T)); the test prints the longest converged prefix j*, the
    spectrum around it and the residuals, and requires that the prefix is not empty and that no library Ritz
    value exceeds its eigenvalue (Ritz values of a positive semi-definite matrix approach from below)."""
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    from conftest import converged_prefix
    torch = torch_cuda
    d = request.getfixturevalue(which)
    leaf = d["leaf"]
    B, N = leaf.shape
    T = 20
    Lb = int(d["F"].n_leaves.max())
    V0 = ri.start_block(N, k)
    lam, V, _, _ = rfx.prox_lowrank(torch.from_numpy(leaf.view(np.int32)).cuda(), Lb, torch.from_numpy(V0).cuda(), T,
                                    quantise=False)
    lam, V = lam.cpu().numpy().astype(np.float64), V.cpu().numpy().astype(np.float64)
    P = oracle.counts_full(leaf).astype(np.float64) / B
    lam_d, U_d = oracle.dense_eig(P, min(N, k + 8))
    j = converged_prefix(lam, V, lam_d, U_d)
    res = np.linalg.norm(P @ V - V * lam[None, :], axis=0) / lam
    rel = np.abs(lam - lam_d[:k]) / lam_d[:k]
    print(f"reported layer {which} N={N} B={B} k={k} T={T}: converged prefix j*={j}; "
          f"rel. eigenvalue error at j*, j*+1, k: {rel[max(j - 1, 0)]:.1e}, {rel[min(j, k - 1)]:.1e}, {rel[k - 1]:.1e}; "
          f"residuals at 1, j*, k: {res[0]:.1e}, {res[max(j - 1, 0)]:.1e}, {res[k - 1]:.1e}; "
          f"lambda_1={lam_d[0]:.3f} lambda_j*={lam_d[max(j - 1, 0)]:.3f} lambda_k={lam_d[k - 1]:.3f} "
          f"lambda_k+1={lam_d[k]:.3f} (ratio^2T={(lam_d[k] / lam_d[k - 1]) ** (2 * T):.1e})", flush=True)
    assert j >= 1
    assert (lam <= lam_d[:k] * (1 + 1e-5)).all()
    assert res[0] <= 1e-3
    # the library is as close to the dense spectrum as the float64 iteration is: same prefix
    lam_o, V_o = oracle.block_iteration(leaf, V0, T)
    assert abs(converged_prefix(lam_o, V_o, lam_d, U_d) - j) <= 1


def _align(coords, ref, lam):
    """Ritz vectors of (nearly) equal eigenvalues are defined up to a rotation inside their
    eigenspace; align with orthogonal Procrustes in that case, otherwise compare as is."""
    gaps = np.abs(np.diff(lam)) / np.abs(lam[0])
    if gaps.min() > 1e-2:
        return coords
    U, _, Vt = np.linalg.svd(coords.T @ ref)
    return coords @ (U @ Vt)


@pytest.mark.parametrize("which,k,mode", [("cfg1", 16, "squared"), ("cfg1", 16, "linear"), ("small2", 32, "squared"),
                                          ("small2", 48, "squared"), ("small2", 64, "squared"), ("small2", 64, "linear"),
                                          ("small2", 100, "squared")])
def test_mds3d_against_dense_torgerson_scaling(torch_cuda, request, which, k, mode):
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    d = request.getfixturevalue(which)
    leaf = d["leaf"]
    B, N = leaf.shape
    print(f"mds3d {which} N={N} k={k} {mode}", flush=True)
    # factors from the oracle so that this test isolates the scaling step
    lam, V = oracle.block_iteration(leaf, ri.start_block(N, k), 8)
    Qh, sh = oracle.quantise_int8(V, lam)
    omode = oracle.SQUARED if mode == "squared" else oracle.LINEAR
    gmode = rfx.MDS_SQUARED if mode == "squared" else rfx.MDS_LINEAR
    ref, ev_ref = oracle.mds3d_dense(Qh, sh, omode)
    m = 12
    x0 = ri.start_block(N, m, seed=778)
    coords, ev, iters = rfx.mds3d(torch.from_numpy(Qh).cuda(), torch.from_numpy(sh).cuda(), torch.from_numpy(x0).cuda(),
                                  gmode, max_iters=500, tol=1e-7)
    torch.cuda.synchronize()
    coords, ev = coords.cpu().numpy().astype(np.float64), ev.cpu().numpy().astype(np.float64)
    print(f"  iterations={iters} eig={ev} ref={ev_ref}", flush=True)
    assert iters < 500
    np.testing.assert_allclose(ev, ev_ref, rtol=1e-4)
    err = np.linalg.norm(_align(coords, ref, ev_ref) - ref) / np.linalg.norm(ref)
    assert err <= 1e-3, err
    # invariants of classical scaling: centred, mutually orthogonal columns with |col|^2 = lambda
    assert np.abs(coords.sum(axis=0)).max() <= 1e-3 * np.abs(coords).max() * np.sqrt(N)
    np.testing.assert_allclose(coords.T @ coords, np.diag(ev), atol=2e-4 * ev[0])
    # without a start block the library begins from the leading columns of the factor: the same answer, and it gets
    # there in no more applications than from the random block
    c2, ev2, it2 = rfx.mds3d(torch.from_numpy(Qh).cuda(), torch.from_numpy(sh).cuda(), None, gmode, max_iters=500, tol=1e-7, m=m)
    c2, ev2 = c2.cpu().numpy().astype(np.float64), ev2.cpu().numpy().astype(np.float64)
    print(f"  own start block: iterations={it2} eig={ev2}", flush=True)
    assert it2 <= iters
    np.testing.assert_allclose(ev2, ev_ref, rtol=1e-4)
    assert np.linalg.norm(_align(c2, ref, ev_ref) - ref) / np.linalg.norm(ref) <= 1e-3


def test_mds3d_own_start_block_wider_than_the_factor(torch_cuda, cfg1):
    """m > k: the start block is the k columns of the factor filled up with the library's fixed pseudo-random columns;
    the result is the dense scaling's, the same on every call."""
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    leaf = cfg1["leaf"]
    B, N = leaf.shape
    k, m = 4, 12
    lam, V = oracle.block_iteration(leaf, ri.start_block(N, k), 8)
    Qh, sh = oracle.quantise_int8(V, lam)
    ref, ev_ref = oracle.mds3d_dense(Qh, sh, oracle.SQUARED)
    dQ, ds = torch.from_numpy(Qh).cuda(), torch.from_numpy(sh).cuda()
    c1, ev1, it1 = rfx.mds3d(dQ, ds, None, rfx.MDS_SQUARED, max_iters=500, tol=1e-7, m=m)
    c2, ev2, it2 = rfx.mds3d(dQ, ds, None, rfx.MDS_SQUARED, max_iters=500, tol=1e-7, m=m)
    assert it1 == it2 < 500 and torch.equal(c1, c2) and torch.equal(ev1, ev2)
    c1, ev1 = c1.cpu().numpy().astype(np.float64), ev1.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(ev1, ev_ref, rtol=1e-4)
    assert np.linalg.norm(_align(c1, ref, ev_ref) - ref) / np.linalg.norm(ref) <= 1e-3
