"""The asynchronous calls under HIP graph capture: they allocate nothing, clear their scratch with kernels and never wait,
so a caller can record them once and replay them.  Every replay is checked against the eager results, with the program's own
eager work and synchronisations between the replays (outputs cleared, another eager call on the same plan)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def test_whole_path_recorded_once_and_replayed(torch_cuda, small2):
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    F, X = small2["F"], small2["X"]
    B, N = small2["leaf"].shape
    k, T, m, mds_iters = 16, 20, 12, 40
    dev = torch.device("cuda:0")
    print(f"graph replay of the whole path N={N} B={B} k={k}", flush=True)
    gf = rfx.Forest(F.n_features, F.node_offset, F.feature, F.threshold, F.left, F.right, F.leaf_id, F.n_leaves)
    Lb = gf.leaf_bound
    dX = torch.from_numpy(X).to(dev)
    d_inbag = torch.from_numpy(F.inbag.view(np.int16)).to(dev)
    leaf = torch.empty((B, N), dtype=torch.int32, device=dev)
    plan = rfx.PvPlan(rfx.leaf_assign(gf, dX), Lb)
    rfx.pv_plan_reserve(plan, k)
    ws_prox = rfx.new_workspace(rfx.prox_workspace_bytes(N, B, Lb))
    ws_lr = rfx.new_workspace(rfx.lowrank_workspace_bytes(N, k))
    ws_mds = rfx.new_workspace(rfx.mds3d_workspace_bytes(N, k, m, rfx.MDS_SQUARED))
    npk = N * (N - 1) // 2
    out = dict(cnt=torch.empty((N, N), dtype=torch.int32, device=dev), prox=torch.empty((N, N), dtype=torch.float32, device=dev),
               num=torch.empty(npk, dtype=torch.int32, device=dev), den=torch.empty(npk, dtype=torch.int32, device=dev),
               poob=torch.empty(npk, dtype=torch.float32, device=dev), lam=torch.empty(k, dtype=torch.float32, device=dev),
               V=torch.empty((N, k), dtype=torch.float32, device=dev), Q=torch.empty((N, k), dtype=torch.int8, device=dev),
               s=torch.empty(k, dtype=torch.float32, device=dev), status=torch.full((1,), -1, dtype=torch.int32, device=dev),
               coords=torch.empty((N, 3), dtype=torch.float32, device=dev), ev=torch.empty(3, dtype=torch.float32, device=dev),
               rel=torch.empty(1, dtype=torch.float32, device=dev), leaf=leaf)
    dV0 = torch.from_numpy(ri.start_block(N, k)).to(dev)
    dx0 = torch.from_numpy(ri.start_block(N, m, seed=778)).to(dev)

    def run():
        rfx.leaf_assign(gf, dX, leaf)
        rfx.prox_dense_oob_ws(leaf, d_inbag, Lb, ws_prox, rfx.U32, rfx.FULL, rfx.UPPER_PACKED, counts=out["cnt"], prox=out["prox"],
                              num=out["num"], den=out["den"], prox_oob=out["poob"])
        rfx.prox_lowrank_plan(plan, dV0, T, ws_lr, out["lam"], out["V"], out["Q"], out["s"], out["status"])
        rfx.mds3d_ws(out["Q"], out["s"], dx0, mds_iters, ws_mds, out["coords"], out["ev"], out["rel"])

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        run()                                   # eager, on the stream that will be captured
    stream.synchronize()
    eager = {n: t.clone() for n, t in out.items()}
    assert int(eager["status"][0]) == 0
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        run()
    for replay in range(3):
        for t in out.values():
            t.zero_()                           # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, t in out.items():
            assert torch.equal(t, eager[n]), f"replay {replay}: {n} differs from the eager run"
        print(f"replay {replay}: every output equals the eager run's", flush=True)
    plan.close()


def test_product_in_groups_of_trees_recorded_and_replayed(torch_cuda):
    """Large enough (B N >= 10^7, B >= 64) for the product to run in four groups of trees with the gather of a group on the
    plan's second stream: the fork to that stream and the join back are part of the recording."""
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    N, B, bound, k = 160000, 64, 3000, 32
    print(f"graph replay of the product N={N} B={B} k={k}", flush=True)
    rng = np.random.default_rng(77)
    leaf = torch.from_numpy(rng.integers(0, bound, size=(B, N)).astype(np.int32)).cuda()
    plan = rfx.PvPlan(leaf, bound)
    rfx.pv_plan_reserve(plan, k)
    V = torch.from_numpy(ri.start_block(N, k)).cuda()
    Y = torch.empty_like(V)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        plan.apply(V, Y)
    stream.synchronize()
    eager = Y.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        plan.apply(V, Y)
    for replay in range(3):
        Y.zero_()
        W = plan.apply(eager)                   # an eager application on the same plan between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, eager), f"replay {replay}"
        assert bool(torch.isfinite(W).all())
    plan.close()
