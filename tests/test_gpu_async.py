"""The asynchronous forms of the boundary: scratch from a caller workspace, no wait inside the calls.

One stream carries leaf assignment, the fused dense pass, the factorisation on an existing plan and the
scaling, with a single synchronisation at the end; every result is then compared with the oracle.  The
other tests check that each *_ws call writes what its synchronous convenience writes."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def test_whole_path_on_one_stream_with_a_single_synchronisation(torch_cuda, small2):
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    F, X, leaf_ref = small2["F"], small2["X"], small2["leaf"]
    B, N = leaf_ref.shape
    k, T, m, mds_iters = 16, 20, 12, 60
    dev = torch.device("cuda:0")
    print(f"async path N={N} B={B} k={k}", flush=True)
    gf = rfx.Forest(F.n_features, F.node_offset, F.feature, F.threshold, F.left, F.right, F.leaf_id, F.n_leaves)
    Lb = gf.leaf_bound
    # everything that allocates or waits happens before the stream section: inputs, outputs, workspaces, the plan
    # (its creation needs leaf ids, so the plan is built from a first leaf assignment and reused below)
    dX = torch.from_numpy(X).to(dev)
    d_inbag = torch.from_numpy(F.inbag.view(np.int16)).to(dev)
    leaf = torch.empty((B, N), dtype=torch.int32, device=dev)
    plan = rfx.PvPlan(rfx.leaf_assign(gf, dX), Lb)
    rfx.pv_plan_reserve(plan, k)
    assert rfx.pv_plan_info(plan) == (N, B, k)
    ws_prox = rfx.new_workspace(rfx.prox_workspace_bytes(N, B, Lb))
    ws_lr = rfx.new_workspace(rfx.lowrank_workspace_bytes(N, k))
    ws_mds = rfx.new_workspace(rfx.mds3d_workspace_bytes(N, k, m, rfx.MDS_SQUARED))
    cnt = torch.empty((N, N), dtype=torch.int32, device=dev)
    prox = torch.empty((N, N), dtype=torch.float32, device=dev)
    npk = N * (N - 1) // 2
    num = torch.empty(npk, dtype=torch.int32, device=dev)
    den = torch.empty(npk, dtype=torch.int32, device=dev)
    poob = torch.empty(npk, dtype=torch.float32, device=dev)
    dV0 = torch.from_numpy(ri.start_block(N, k)).to(dev)
    dx0 = torch.from_numpy(ri.start_block(N, m, seed=778)).to(dev)
    lam = torch.empty(k, dtype=torch.float32, device=dev)
    V = torch.empty((N, k), dtype=torch.float32, device=dev)
    Q = torch.empty((N, k), dtype=torch.int8, device=dev)
    s = torch.empty(k, dtype=torch.float32, device=dev)
    status = torch.full((1,), -1, dtype=torch.int32, device=dev)
    coords = torch.empty((N, 3), dtype=torch.float32, device=dev)
    ev = torch.empty(3, dtype=torch.float32, device=dev)
    rel = torch.empty(1, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        rfx.leaf_assign(gf, dX, leaf)
        rfx.prox_dense_oob_ws(leaf, d_inbag, Lb, ws_prox, rfx.U32, rfx.FULL, rfx.UPPER_PACKED, counts=cnt, prox=prox, num=num,
                              den=den, prox_oob=poob)
        rfx.prox_lowrank_plan(plan, dV0, T, ws_lr, lam, V, Q, s, status)
        rfx.mds3d_ws(Q, s, dx0, mds_iters, ws_mds, coords, ev, rel)
    stream.synchronize()                                    # the only wait

    np.testing.assert_array_equal(leaf.cpu().numpy().view(np.uint32), leaf_ref)
    ref_cnt = oracle.counts_full(leaf_ref)
    np.testing.assert_array_equal(cnt.cpu().numpy().view(np.uint32), ref_cnt)
    np.testing.assert_array_equal(prox.cpu().numpy(), oracle.normalise(ref_cnt, B))
    rn, rd = oracle.oob_rows(leaf_ref, F.inbag, 0, N)
    iu = np.triu_indices(N, 1)
    np.testing.assert_array_equal(num.cpu().numpy().view(np.uint32), rn[iu])
    np.testing.assert_array_equal(den.cpu().numpy().view(np.uint32), rd[iu])
    assert int(status[0]) == 0
    lam_ref, V_ref = oracle.block_iteration(leaf_ref, ri.start_block(N, k), T)
    np.testing.assert_allclose(lam.cpu().numpy(), lam_ref, rtol=1e-4)
    assert oracle.principal_angle(V.cpu().numpy(), V_ref) < 1e-3
    Qr, sr = oracle.quantise_int8(V.cpu().numpy(), lam.cpu().numpy())
    np.testing.assert_array_equal(Q.cpu().numpy(), Qr)
    np.testing.assert_array_equal(s.cpu().numpy(), sr)
    ref_c, ev_ref = oracle.mds3d_dense(Qr, sr, oracle.SQUARED)
    print(f"  mds rel change after {mds_iters} applications: {float(rel[0]):.2e}; eig={ev.cpu().numpy()} ref={ev_ref}", flush=True)
    assert float(rel[0]) < 1e-5
    np.testing.assert_allclose(ev.cpu().numpy(), ev_ref, rtol=1e-4)
    err = np.linalg.norm(coords.cpu().numpy() - ref_c) / np.linalg.norm(ref_c)
    assert err <= 1e-3, err


def test_workspace_forms_write_what_the_conveniences_write(torch_cuda, small2):
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    F, leaf_ref, y = small2["F"], small2["leaf"], small2["y"]
    B, N = leaf_ref.shape
    dev = torch.device("cuda:0")
    leaf = torch.from_numpy(leaf_ref.view(np.int32)).to(dev)
    inbag = torch.from_numpy(F.inbag.view(np.int16)).to(dev)
    Lb = int(F.n_leaves.max())
    need = rfx.prox_workspace_bytes(N, B, Lb)
    ws = rfx.new_workspace(need)
    ws.fill_(0xAB)                                           # stale contents must not matter
    # dense, packed uint16
    c0, p0 = rfx.prox_dense(leaf, Lb, rfx.U16, rfx.UPPER_PACKED)
    c1, p1 = torch.empty_like(c0), torch.empty_like(p0)
    rfx.prox_dense_ws(leaf, Lb, ws, rfx.U16, rfx.UPPER_PACKED, counts=c1, prox=p1)
    torch.cuda.synchronize()
    assert torch.equal(c0, c1) and torch.equal(p0, p1)
    # out-of-bag, full
    n0, d0, q0 = rfx.prox_oob(leaf, inbag, Lb)
    n1, d1, q1 = torch.empty_like(n0), torch.empty_like(d0), torch.empty_like(q0)
    rfx.prox_oob_ws(leaf, inbag, Lb, ws, num=n1, den=d1, prox=q1)
    torch.cuda.synchronize()
    assert torch.equal(n0, n1) and torch.equal(d0, d1) and torch.equal(q0, q1)
    # sparse: same set of triplets, count on the device
    r0, s0, v0, _ = rfx.prox_sparse(leaf, Lb, min_count=2)
    nnz = torch.full((1,), -5, dtype=torch.int64, device=dev)
    r1 = torch.empty(r0.numel() + 7, dtype=torch.int32, device=dev)
    s1, v1 = torch.empty_like(r1), torch.empty_like(r1)
    rfx.prox_sparse_ws(leaf, Lb, ws, nnz, r1, s1, v1, min_count=2)
    torch.cuda.synchronize()
    n = int(nnz[0])
    assert n == r0.numel()
    key0 = (r0.long() * N + s0.long()) * (B + 1) + v0.long()
    key1 = (r1[:n].long() * N + s1[:n].long()) * (B + 1) + v1[:n].long()
    assert torch.equal(key0.sort().values, key1.sort().values)
    # counting only
    nnz.fill_(123)
    rfx.prox_sparse_ws(leaf, Lb, ws, nnz, min_count=2)
    torch.cuda.synchronize()
    assert int(nnz[0]) == n
    # outlier sums
    labels = torch.from_numpy(y.astype(np.int32)).to(dev)
    a0, b0 = rfx.prox_outlier(leaf, Lb, labels)
    a1, b1 = torch.empty_like(a0), torch.empty_like(b0)
    ws.fill_(0xCD)
    rfx.prox_outlier_ws(leaf, Lb, ws, labels, a1, b1)
    torch.cuda.synchronize()
    assert torch.allclose(a0, a1, rtol=1e-12, atol=0) and torch.equal(b0, b1)
    # a workspace that is too small, misaligned or missing is refused before anything is launched
    lib = rfx.load()
    small = rfx.new_workspace(need - 256)
    with pytest.raises(rfx.RfxError) as e:
        rfx.prox_dense_ws(leaf, Lb, small, counts=torch.empty((N, N), dtype=torch.int32, device=dev))
    assert e.value.code == rfx.ERR_CAPACITY
    assert lib.rfx_prox_dense_ws(leaf.data_ptr(), N, B, Lb, rfx.U32, rfx.FULL, c0.data_ptr(), None, ws.data_ptr() + 64, need, None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_prox_dense_ws(leaf.data_ptr(), N, B, Lb, rfx.U32, rfx.FULL, c0.data_ptr(), None, None, need, None) == rfx.ERR_NULL


def test_lowrank_on_a_plan_equals_the_one_shot_call_and_reports_lost_rank(torch_cuda, small2):
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    leaf_ref = small2["leaf"]
    B, N = leaf_ref.shape
    dev = torch.device("cuda:0")
    leaf = torch.from_numpy(leaf_ref.view(np.int32)).to(dev)
    Lb = int(small2["F"].n_leaves.max())
    k, T = 24, 6
    V0 = torch.from_numpy(ri.start_block(N, k)).to(dev)
    lam0, Vr0, Q0, s0 = rfx.prox_lowrank(leaf, Lb, V0, T)
    plan = rfx.PvPlan(leaf, Lb)
    ws = rfx.new_workspace(rfx.lowrank_workspace_bytes(N, k))
    lam, V = torch.empty_like(lam0), torch.empty_like(Vr0)
    Q, s = torch.empty_like(Q0), torch.empty_like(s0)
    status = torch.full((1,), 9, dtype=torch.int32, device=dev)
    with pytest.raises(rfx.RfxError):                      # the sums are not reserved yet
        rfx.prox_lowrank_plan(plan, V0, T, ws, lam, V, Q, s, status)
    rfx.pv_plan_reserve(plan, 32)
    rfx.prox_lowrank_plan(plan, V0, T, ws, lam, V, Q, s, status)
    torch.cuda.synchronize()
    assert int(status[0]) == 0
    assert torch.equal(lam, lam0) and torch.equal(V, Vr0) and torch.equal(Q, Q0) and torch.equal(s, s0)
    # a start block with a zero column loses rank: reported in the status word, not by an exception
    bad = V0.clone()
    bad[:, 5] = 0.0
    rfx.prox_lowrank_plan(plan, bad, T, ws, lam, V, Q, s, status)
    torch.cuda.synchronize()
    assert int(status[0]) == 1
    with pytest.raises(rfx.RfxError):
        rfx.prox_lowrank(leaf, Lb, bad, T)


def test_plan_rebuilt_for_other_leaf_ids_equals_a_fresh_plan(torch_cuda, small2):
    """rfx_pv_plan_rebuild regroups an existing plan without allocating: the product it then applies is bit-identical
    to the product of a plan created from the same leaf ids, and a rebuild with an id out of range is refused and
    leaves the plan unusable until a good rebuild."""
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    leaf_ref = small2["leaf"]
    B, N = leaf_ref.shape
    dev = torch.device("cuda:0")
    Lb = int(small2["F"].n_leaves.max())
    leaf_a = torch.from_numpy(leaf_ref.view(np.int32)).to(dev)
    leaf_b = leaf_a.flip(0).contiguous()                     # the same trees in reverse order: other slots everywhere
    leaf_c = (leaf_a * 7 + 3) % Lb                           # other ids altogether
    V = torch.from_numpy(ri.start_block(N, 24)).to(dev)
    plan = rfx.PvPlan(leaf_a, Lb)
    Ya = plan.apply(V).clone()
    for other in (leaf_b, leaf_c, leaf_a):
        before = torch.cuda.memory_allocated()
        rfx.pv_plan_rebuild(plan, other)
        got = plan.apply(V)
        fresh = rfx.PvPlan(other, Lb)
        want = fresh.apply(V)
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        fresh.close()
        del got, want
        assert torch.cuda.memory_allocated() <= before + V.numel() * 4 * 2
    assert torch.equal(plan.apply(V), Ya)
    bad = leaf_a.clone()
    bad[3, 5] = Lb
    with pytest.raises(rfx.RfxError):
        rfx.pv_plan_rebuild(plan, bad)
    with pytest.raises(rfx.RfxError):
        plan.apply(V)
    rfx.pv_plan_rebuild(plan, leaf_a)
    assert torch.equal(plan.apply(V), Ya)
