"""GPU parity on degenerate and boundary shapes: single sample, single tree, one leaf, tile and
tree-group boundaries, count-type limits, all-in-bag / all-out-of-bag, extreme ranks."""
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


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int32) if a.dtype == np.uint32 else np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("N,B,bound", [(1, 3, 5), (2, 1, 2), (5, 1, 5), (255, 31, 40), (256, 32, 40), (257, 33, 40),
                                       (260, 64, 300), (515, 65, 2), (300, 97, 1)])
def test_dense_and_oob_on_boundary_shapes(torch_cuda, N, B, bound):
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    print(f"boundary shapes N={N} B={B} bound={bound}", flush=True)
    rng = np.random.default_rng(1000 * N + B)
    leaf = rng.integers(0, bound, size=(B, N)).astype(np.uint32)
    inbag = rng.integers(0, 3, size=(B, N)).astype(np.uint16)
    ref = oracle.counts_full(leaf)
    for dtype, npdt in ((rfx.U32, np.uint32), (rfx.U16, np.uint16)):
        cnt, prox = rfx.prox_dense(_dev(torch, leaf), bound, dtype, rfx.FULL)
        np.testing.assert_array_equal(_u(cnt), ref.astype(npdt))
        np.testing.assert_array_equal(prox.cpu().numpy(), oracle.normalise(ref, B))
        if N > 1:
            cnt, prox = rfx.prox_dense(_dev(torch, leaf), bound, dtype, rfx.UPPER_PACKED)
            np.testing.assert_array_equal(_u(cnt), oracle.pack_upper(ref).astype(npdt))
            np.testing.assert_array_equal(prox.cpu().numpy(), oracle.pack_upper(oracle.normalise(ref, B)))
    rn, rd = oracle.oob_rows(leaf, inbag, 0, N)
    num, den, prox = rfx.prox_oob(_dev(torch, leaf), torch.from_numpy(inbag.view(np.int16)).cuda(), bound, rfx.U32, rfx.FULL)
    np.testing.assert_array_equal(_u(num), rn)
    np.testing.assert_array_equal(_u(den), rd)
    np.testing.assert_array_equal(prox.cpu().numpy(), oracle.prox_oob_rows(rn, rd, 0))


def test_degenerate_forests(torch_cuda):
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    N, B = 70, 9
    # every sample in one leaf: all counts B, proximity all ones
    one = np.zeros((B, N), np.uint32)
    cnt, prox = rfx.prox_dense(_dev(torch, one), 1, rfx.U32, rfx.FULL)
    assert (_u(cnt) == B).all() and (prox.cpu().numpy() == 1.0).all()
    # every sample alone in its leaf: B on the diagonal only
    alone = np.tile(np.arange(N, dtype=np.uint32), (B, 1))
    cnt, prox = rfx.prox_dense(_dev(torch, alone), N, rfx.U32, rfx.FULL)
    np.testing.assert_array_equal(_u(cnt), B * np.eye(N, dtype=np.uint32))
    # out-of-bag variant: nobody in-bag -> the plain proximity; everybody in-bag -> identity
    rng = np.random.default_rng(4)
    leaf = rng.integers(0, 6, size=(B, N)).astype(np.uint32)
    ref = oracle.counts_full(leaf)
    num, den, prox = rfx.prox_oob(_dev(torch, leaf), torch.zeros((B, N), dtype=torch.int16).cuda(), 6)
    np.testing.assert_array_equal(_u(num), ref)
    assert (_u(den) == B).all()
    np.testing.assert_array_equal(prox.cpu().numpy(), oracle.normalise(ref, B))
    num, den, prox = rfx.prox_oob(_dev(torch, leaf), torch.ones((B, N), dtype=torch.int16).cuda(), 6)
    assert _u(num).max() == 0 and _u(den).max() == 0
    np.testing.assert_array_equal(prox.cpu().numpy(), np.eye(N, dtype=np.float32))


def test_count_type_limits(torch_cuda):
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    N, B = 6, 65535                      # the most trees uint16 counts (and the out-of-bag counters) can hold
    leaf = np.zeros((B, N), np.uint32)
    leaf[:, 3] = 1                       # sample 3 never shares a leaf with the others
    cnt, _ = rfx.prox_dense(_dev(torch, leaf), 2, rfx.U16, rfx.FULL, want_prox=False)
    c = _u(cnt)
    assert c[0, 1] == 65535 and c[3, 3] == 65535 and c[0, 3] == 0
    num, den, prox = rfx.prox_oob(_dev(torch, leaf), torch.zeros((B, N), dtype=torch.int16).cuda(), 2, rfx.U32, rfx.FULL)
    assert _u(num)[0, 1] == 65535 and _u(den)[0, 3] == 65535 and _u(num)[0, 3] == 0
    assert float(prox[0, 1]) == 1.0 and float(prox[0, 3]) == 0.0
    lib = rfx.load()
    big = torch.zeros((8,), dtype=torch.int32).cuda()
    assert lib.rfx_prox_dense(big.data_ptr(), 2, 65536, 2, rfx.U16, rfx.FULL, big.data_ptr(), None, None) == -3
    assert lib.rfx_prox_oob(big.data_ptr(), big.data_ptr(), 2, 65536, 2, rfx.U32, rfx.FULL, big.data_ptr(), None, None, None) == -6
    assert lib.rfx_prox_dense(big.data_ptr(), 0, 4, 2, rfx.U32, rfx.FULL, big.data_ptr(), None, None) == -1   # empty input


@pytest.mark.parametrize("k", [1, 3, 17, 33, 128, 200, 256])
def test_matvec_any_rank(torch_cuda, small2, k):
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    leaf = small2["leaf"]
    B, N = leaf.shape
    V = ri.start_block(N, k, seed=5 + k)
    ref = oracle.pv_implicit(leaf, V.astype(np.float64))
    Y = rfx.prox_matvec(_dev(torch, leaf), int(leaf.max()) + 1, torch.from_numpy(V).cuda())
    err = np.linalg.norm(Y.cpu().numpy().astype(np.float64) - ref) / np.linalg.norm(ref)
    assert err <= 1e-5, err


def test_matvec_tiny_and_single_tree(torch_cuda):
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    for N, B, bound in ((1, 1, 1), (3, 2, 2), (40, 1, 7)):
        rng = np.random.default_rng(N + B)
        leaf = rng.integers(0, bound, size=(B, N)).astype(np.uint32)
        V = rng.standard_normal((N, 4)).astype(np.float32)
        ref = oracle.pv_implicit(leaf, V.astype(np.float64))
        Y = rfx.prox_matvec(_dev(torch, leaf), bound, torch.from_numpy(V).cuda())
        np.testing.assert_allclose(Y.cpu().numpy(), ref, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("N,bound", [(40000, 30001), (40000, 65536), (70000, 70000), (70000, 20000)])
def test_matvec_with_many_leaves(torch_cuda, N, bound):
    """Leaf bounds above what a 32-bit LDS histogram holds: 16-bit counter pairs in LDS (bound <= 65,536 and parts
    below 65,536 samples) and global counters (beyond); most leaves hold one or two samples, a few are skipped."""
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    B = 3
    rng = np.random.default_rng(N + bound)
    leaf = rng.integers(0, bound, size=(B, N)).astype(np.uint32)
    leaf[0, :9000] = bound - 1            # one big leaf at the last id
    leaf[1] = rng.permutation(N).astype(np.uint32) % np.uint32(bound)
    V = rng.standard_normal((N, 8)).astype(np.float32)
    ref = oracle.pv_implicit(leaf, V.astype(np.float64))
    Y = rfx.prox_matvec(_dev(torch, leaf), bound, torch.from_numpy(V).cuda())
    err = np.linalg.norm(Y.cpu().numpy().astype(np.float64) - ref) / np.linalg.norm(ref)
    assert err <= 1e-5, err


def test_matvec_with_one_huge_leaf(torch_cuda):
    """A leaf far above the big-leaf threshold next to many singletons (workgroup-per-leaf path)."""
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    N, B = 5000, 5
    rng = np.random.default_rng(8)
    leaf = np.zeros((B, N), np.uint32)
    for b in range(B):
        rest = rng.permutation(N)[: 700 + 13 * b]
        leaf[b, rest] = 1 + np.arange(len(rest), dtype=np.uint32)
    V = rng.standard_normal((N, 64)).astype(np.float32)
    ref = oracle.pv_implicit(leaf, V.astype(np.float64))
    Y = rfx.prox_matvec(_dev(torch, leaf), int(leaf.max()) + 1, torch.from_numpy(V).cuda())
    err = np.linalg.norm(Y.cpu().numpy().astype(np.float64) - ref) / np.linalg.norm(ref)
    assert err <= 1e-5, err


def test_lowrank_extreme_ranks(torch_cuda, small2):
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    leaf = small2["leaf"]
    B, N = leaf.shape
    for k, T in ((1, 30), (40, 6), (80, 6), (88, 6), (96, 6), (112, 6), (128, 6)):   # 40, 80: not multiples of 16; 80..128: beyond one 64-column tile
        V0 = ri.start_block(N, k, seed=21 + k)
        lam_ref, V_ref = oracle.block_iteration(leaf, V0, T)
        lam, V, Q, s = rfx.prox_lowrank(_dev(torch, leaf), int(leaf.max()) + 1, torch.from_numpy(V0).cuda(), T)
        np.testing.assert_allclose(lam.cpu().numpy(), lam_ref, rtol=1e-4)
        assert oracle.principal_angle(V.cpu().numpy(), V_ref) < 1e-3
        Qr, sr = oracle.quantise_int8(V.cpu().numpy(), lam.cpu().numpy())
        np.testing.assert_array_equal(Q.cpu().numpy(), Qr)
    # a block wider than the rank of P cannot be orthonormalised: reported, not silently wrong
    ident = np.zeros((3, 40), np.uint32)                 # P = all-ones matrix, rank 1
    V0 = ri.start_block(40, 4)
    with pytest.raises(rfx.RfxError):
        rfx.prox_lowrank(_dev(torch, ident), 1, torch.from_numpy(V0).cuda(), 3)


def test_quantise_special_columns(torch_cuda):
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    V = np.array([[127.0, 0.0, -2.0], [0.5, 0.0, 1.0], [1.5, 0.0, 0.25], [2.5, 0.0, 0.0], [-0.5, 0.0, 0.5],
                  [-3.5, 0.0, 2.0]], np.float32)
    lam = np.array([1.0, 3.0, 1.0], np.float32)
    Q, s = rfx.quantise_int8(torch.from_numpy(V).cuda(), torch.from_numpy(lam).cuda())
    Qr, sr = oracle.quantise_int8(V, lam)
    np.testing.assert_array_equal(Q.cpu().numpy(), Qr)         # ties to even, +-127 at the column maximum
    np.testing.assert_array_equal(s.cpu().numpy(), sr)         # all-zero column: scale 1, codes 0
    lam_neg = np.array([1.0, -1.0, 4.0], np.float32)           # a non-positive Ritz value contributes nothing
    Q, s = rfx.quantise_int8(torch.from_numpy(V).cuda(), torch.from_numpy(lam_neg).cuda())
    Qr, sr = oracle.quantise_int8(V, lam_neg)
    np.testing.assert_array_equal(Q.cpu().numpy(), Qr)
    np.testing.assert_array_equal(s.cpu().numpy(), sr)


def test_leaf_assign_wide_rows_and_single_node_trees(torch_cuda):
    """More features than fit the LDS row tile (global-memory rows) and trees that are a single leaf."""
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    rng = np.random.default_rng(6)
    N, M = 300, 700
    X = rng.standard_normal((N, M)).astype(np.float32)
    y = (X[:, 5] + X[:, 600] > 0).astype(np.int32)
    F = ri.grow_forest(X, y, 2, 7, 26)
    ref, _ = oracle.leaf_assign(F, X)
    gf = rfx.Forest(F.n_features, F.node_offset, F.feature, F.threshold, F.left, F.right, F.leaf_id, F.n_leaves)
    np.testing.assert_array_equal(_u(rfx.leaf_assign(gf, torch.from_numpy(X).cuda())), ref)
    # all labels equal: every tree is one leaf
    F1 = ri.grow_forest(X[:, :9].copy(), np.zeros(N, np.int32), 1, 5, 3)
    assert (np.diff(F1.node_offset) == 1).all()
    g1 = rfx.Forest(F1.n_features, F1.node_offset, F1.feature, F1.threshold, F1.left, F1.right, F1.leaf_id, F1.n_leaves)
    assert g1.leaf_bound == 1
    assert int(rfx.leaf_assign(g1, torch.from_numpy(X[:, :9].copy()).cuda()).abs().max()) == 0


def test_mds_small_blocks_and_linear_rank(torch_cuda, cfg1):
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    leaf = cfg1["leaf"]
    N = leaf.shape[1]
    lam, V = oracle.block_iteration(leaf, ri.start_block(N, 8), 10)
    Qh, sh = oracle.quantise_int8(V, lam)
    for m, mode, omode in ((3, rfx.MDS_SQUARED, oracle.SQUARED), (8, rfx.MDS_LINEAR, oracle.LINEAR),
                           (32, rfx.MDS_SQUARED, oracle.SQUARED)):
        ref, ev_ref = oracle.mds3d_dense(Qh, sh, omode)
        x0 = ri.start_block(N, m, seed=779)
        coords, ev, iters = rfx.mds3d(torch.from_numpy(Qh).cuda(), torch.from_numpy(sh).cuda(), torch.from_numpy(x0).cuda(),
                                      mode, max_iters=3000, tol=1e-9)
        np.testing.assert_allclose(ev.cpu().numpy(), ev_ref, rtol=1e-4)
        err = np.linalg.norm(coords.cpu().numpy() - ref) / np.linalg.norm(ref)
        assert err <= 1e-3, (m, err, iters)
    lib = rfx.load()
    q = torch.from_numpy(Qh).cuda()
    assert lib.rfx_mds3d(q.data_ptr(), q.data_ptr(), N, 8, 0, 2, 10, 1e-6, q.data_ptr(), q.data_ptr(), q.data_ptr(), None,
                         None) == -1   # block narrower than 3


@pytest.mark.parametrize("N,k,spread,m,seed", [(400, 4, 1.5, 8, 31), (500, 8, 1.0, 12, 32), (300, 3, 2.0, 6, 33)])
def test_mds_on_a_gram_matrix_dominated_by_negative_eigenvalues(torch_cuda, N, k, spread, m, seed):
    """The squared-dissimilarity Gram matrix of these synthetic factors has at least m negative eigenvalues larger in
    magnitude than its third-largest eigenvalue (checked on the CPU in tests/test_oracle_factors.py): only an
    iteration that converges to the algebraically largest eigenvalues matches the dense reference."""
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    print(f"indefinite scaling N={N} k={k} spread={spread} m={m}", flush=True)
    Q, s = ri.random_int8_factor(N, k, spread, seed)
    ref, ev_ref = oracle.mds3d_dense(Q, s, oracle.SQUARED)
    x0 = ri.start_block(N, m, seed=780)
    coords, ev, iters = rfx.mds3d(torch.from_numpy(Q).cuda(), torch.from_numpy(s).cuda(), torch.from_numpy(x0).cuda(),
                                  rfx.MDS_SQUARED, max_iters=4000, tol=1e-9)
    coords, ev = coords.cpu().numpy().astype(np.float64), ev.cpu().numpy().astype(np.float64)
    print(f"  iterations={iters} eig={ev} ref={ev_ref}", flush=True)
    np.testing.assert_allclose(ev, ev_ref, rtol=1e-4)
    gaps = np.abs(np.diff(ev_ref)) / ev_ref[0]
    if gaps.min() < 1e-2:
        U, _, Vt = np.linalg.svd(coords.T @ ref)
        coords = coords @ (U @ Vt)
    err = np.linalg.norm(coords - ref) / np.linalg.norm(ref)
    assert err <= 1e-3, (err, iters)


def test_mds_of_a_factor_of_rank_below_the_block_width(torch_cuda):
    """LINEAR mode with k = 2 and a block of 8 vectors: G has rank 2, the block cannot keep full rank, and that is
    not an error: the third eigenvalue is (numerically) zero and the third coordinate vanishes, as in the dense
    reference.  The same with a start block that has two equal columns."""
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    N, k, m = 200, 2, 8
    Q, s = ri.random_int8_factor(N, k, 0.3, 34)
    ref, ev_ref = oracle.mds3d_dense(Q, s, oracle.LINEAR)
    for dup in (False, True):
        x0 = ri.start_block(N, m, seed=781)
        if dup:
            x0[:, 4] = x0[:, 1]
        coords, ev, iters = rfx.mds3d(torch.from_numpy(Q).cuda(), torch.from_numpy(s).cuda(), torch.from_numpy(x0).cuda(),
                                      rfx.MDS_LINEAR, max_iters=200, tol=1e-9)
        coords, ev = coords.cpu().numpy().astype(np.float64), ev.cpu().numpy().astype(np.float64)
        print(f"rank-2 scaling dup={dup}: iterations={iters} eig={ev} ref={ev_ref}", flush=True)
        np.testing.assert_allclose(ev[:2], ev_ref[:2], rtol=1e-4)
        assert abs(ev[2]) <= 1e-5 * ev_ref[0]
        err = np.linalg.norm(coords[:, :2] - ref[:, :2]) / np.linalg.norm(ref[:, :2])
        assert err <= 1e-3, err
        assert np.abs(coords[:, 2]).max() <= 3e-3 * np.abs(ref[:, 0]).max()
