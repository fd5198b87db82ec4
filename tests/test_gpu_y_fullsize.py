"""GPU parity at the workloads' full sizes, in the launch configurations bench.py times.

Workload 2 is compared entry by entry; workloads 3 and 4 on sampled rows the oracle computes one
by one plus properties that hold at any size; workload 5 with its full row count and a reduced
number of trees (growing 1,000 trees on 500,000 rows takes the CPU grower tens of minutes).
Each test prints its own progress lines.
"""
import time

import numpy as np
import pytest

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]


def say(*a):
    print("[fullsize]", *a, flush=True)


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _forest(F):
    import paper_2511_19493_amd as rfx
    return rfx.Forest(F.n_features, F.node_offset, F.feature, F.threshold, F.left, F.right, F.leaf_id, F.n_leaves)


def _load(cfg, B=None):
    import torch
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    assert torch.cuda.is_available()
    c = ri.CONFIGS[cfg]
    t0 = time.time()
    X, y, F = ri.load_or_grow(c, B=B)
    say(f"cfg{cfg}: N={c.N} M={c.M} B={F.n_trees}: inputs in {time.time() - t0:.0f}s, {F.total_nodes} nodes, "
        f"max leaves {int(F.n_leaves.max())}, max depth {int(F.depth.max())}")
    t0 = time.time()
    ref_leaf, plen = oracle.leaf_assign(F, X)
    say(f"oracle leaf assignment in {time.time() - t0:.0f}s, mean path {plen / ref_leaf.size:.2f}")
    gf = _forest(F)
    leaf = rfx.leaf_assign(gf, torch.from_numpy(X).cuda())
    torch.cuda.synchronize()
    return dict(c=c, X=X, F=F, ref_leaf=ref_leaf, gf=gf, leaf=leaf, Lb=gf.leaf_bound)


@pytest.fixture(scope="module")
def w2():
    return _load(2)


@pytest.fixture(scope="module")
def w3():
    return _load(3)


@pytest.fixture(scope="module")
def w4():
    return _load(4)


@pytest.fixture(scope="module")
def w5_reduced():
    return _load(5, B=32)


def _sample_rows(N, n, seed):
    rng = np.random.default_rng(seed)
    rows = set(rng.integers(0, N, size=n).tolist()) | {0, 1, N - 1, N - 2, N // 2, 255, 256, 257}
    return sorted(r for r in rows if 0 <= r < N)


# ------------------------------------------------------------------------------------------ workload 2
def test_cfg2_everything_entry_by_entry(w2):
    import torch
    import oracle
    import paper_2511_19493_amd as rfx
    d = w2
    B, N = d["ref_leaf"].shape
    np.testing.assert_array_equal(_u32(d["leaf"]), d["ref_leaf"])
    say("cfg2 leaf ids bit-exact")
    t0 = time.time()
    ref = oracle.counts_full(d["ref_leaf"])
    say(f"oracle counts in {time.time() - t0:.0f}s")
    cnt, _ = rfx.prox_dense(d["leaf"], d["Lb"], rfx.U16, rfx.UPPER_PACKED, want_prox=False)
    np.testing.assert_array_equal(cnt.cpu().numpy().view(np.uint16), oracle.pack_upper(ref).astype(np.uint16))
    say("cfg2 packed uint16 counts bit-exact")
    inbag = d["F"].inbag
    num, den, prox = rfx.prox_oob(d["leaf"], torch.from_numpy(inbag.view(np.int16)).cuda(), d["Lb"], rfx.U32, rfx.FULL)
    t0 = time.time()
    rn, rd = oracle.oob_rows(d["ref_leaf"], inbag, 0, N)
    say(f"oracle out-of-bag counts in {time.time() - t0:.0f}s")
    np.testing.assert_array_equal(_u32(num), rn)
    np.testing.assert_array_equal(_u32(den), rd)
    np.testing.assert_array_equal(prox.cpu().numpy(), oracle.prox_oob_rows(rn, rd, 0))
    say("cfg2 out-of-bag numerator, denominator, proximity bit-exact")


# ------------------------------------------------------------------------------------------ workloads 3, 4
def _check_leaf(d):
    np.testing.assert_array_equal(_u32(d["leaf"]), d["ref_leaf"])


def _check_dense(d, n_rows):
    import torch
    import oracle
    import paper_2511_19493_amd as rfx
    B, N = d["ref_leaf"].shape
    prox = torch.empty((N, N), dtype=torch.float32, device="cuda")
    rfx.prox_dense(d["leaf"], d["Lb"], rfx.U32, rfx.FULL, prox=prox, want_counts=False)   # as bench.py launches it
    torch.cuda.synchronize()
    say("dense proximity computed")
    rows = _sample_rows(N, n_rows, 11)
    for i in rows:
        ref = oracle.normalise(oracle.counts_rows(d["ref_leaf"], i, i + 1)[0], B)
        np.testing.assert_array_equal(prox[i].cpu().numpy(), ref, err_msg=f"row {i}")
        np.testing.assert_array_equal(prox[:, i].cpu().numpy(), ref, err_msg=f"column {i}")
    say(f"{len(rows)} sampled rows and columns bit-exact")
    # properties at full size: unit diagonal, range, and sum_ij cnt = sum_b sum_leaf size^2
    assert bool((torch.diagonal(prox) == 1.0).all())
    assert float(prox.min()) >= 0.0 and float(prox.max()) == 1.0
    total = 0.0
    for s in range(0, N, 8192):
        total += float(prox[s:s + 8192].sum(dtype=torch.float64))
    expect = sum(int((np.bincount(d["ref_leaf"][b]).astype(np.int64) ** 2).sum()) for b in range(B)) / B
    assert abs(total - expect) <= 1e-6 * expect, (total, expect)
    say("diagonal, range and total-sum identity hold")
    return prox


def _check_fused(d, n_rows):
    """The fused plain + out-of-bag pass in the configuration bench.py times: full float32 plain output,
    packed float32 out-of-bag output; sampled rows of both against the oracle."""
    import torch
    import oracle
    import paper_2511_19493_amd as rfx
    B, N = d["ref_leaf"].shape
    inbag = d["F"].inbag
    prox = torch.empty((N, N), dtype=torch.float32, device="cuda")
    poob = torch.empty((N * (N - 1) // 2,), dtype=torch.float32, device="cuda")
    rfx._check(rfx.load().rfx_prox_dense_oob(d["leaf"].data_ptr(), torch.from_numpy(inbag.view(np.int16)).cuda().data_ptr(), N, B,
                                             d["Lb"], rfx.U32, rfx.FULL, 0, prox.data_ptr(), rfx.UPPER_PACKED, 0, 0,
                                             poob.data_ptr(), torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    rows = [i for i in _sample_rows(N, n_rows, 17) if i < N - 1]
    for i in rows:
        ref = oracle.normalise(oracle.counts_rows(d["ref_leaf"], i, i + 1)[0], B)
        np.testing.assert_array_equal(prox[i].cpu().numpy(), ref, err_msg=f"row {i}")
        np.testing.assert_array_equal(prox[:, i].cpu().numpy(), ref, err_msg=f"column {i}")
        rn, rd = oracle.oob_rows(d["ref_leaf"], inbag, i, i + 1)
        ref = oracle.prox_oob_rows(rn, rd, i)[0, i + 1:]
        st = i * N - i * (i + 1) // 2
        np.testing.assert_array_equal(poob[st:st + N - i - 1].cpu().numpy(), ref, err_msg=f"out-of-bag row {i}")
    say(f"fused pass: {len(rows)} sampled rows of both outputs bit-exact")


def _check_oob(d, n_rows):
    import torch
    import oracle
    import paper_2511_19493_amd as rfx
    B, N = d["ref_leaf"].shape
    inbag = d["F"].inbag
    lib = rfx.load()
    out = torch.empty((N * (N - 1) // 2,), dtype=torch.float32, device="cuda")
    rfx._check(lib.rfx_prox_oob(d["leaf"].data_ptr(), torch.from_numpy(inbag.view(np.int16)).cuda().data_ptr(), N, B,
                                d["Lb"], rfx.U32, rfx.UPPER_PACKED, 0, 0, out.data_ptr(),
                                torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    rows = [i for i in _sample_rows(N, n_rows, 12) if i < N - 1]
    for i in rows:
        rn, rd = oracle.oob_rows(d["ref_leaf"], inbag, i, i + 1)
        ref = oracle.prox_oob_rows(rn, rd, i)[0, i + 1:]
        st = i * N - i * (i + 1) // 2
        np.testing.assert_array_equal(out[st:st + N - i - 1].cpu().numpy(), ref, err_msg=f"row {i}")
    say(f"out-of-bag packed proximity: {len(rows)} sampled rows bit-exact")


def _check_sparse(d, n_rows, budget_bytes=40e9):
    """Thresholded sparse proximity at full size: sampled rows and columns against the oracle, and
    for min_count = 1 the exact identity 2 * sum(counts) + N B = sum over trees and leaves of size^2."""
    import torch
    import oracle
    import paper_2511_19493_amd as rfx
    B, N = d["ref_leaf"].shape
    min_count = 1
    while True:
        t0 = time.time()
        nnz = rfx.prox_sparse_count(d["leaf"], d["Lb"], min_count)
        say(f"sparse: {nnz} pairs with count >= {min_count} ({nnz / (N * (N - 1) / 2):.2%} of the triangle), counted in {time.time() - t0:.3f}s")
        if nnz * 12 <= budget_bytes:
            break
        min_count += 1
    t0 = time.time()
    rows, cols, counts, _ = rfx.prox_sparse(d["leaf"], d["Lb"], min_count, capacity=max(nnz, 1), count_dtype=rfx.U32)
    torch.cuda.synchronize()
    say(f"sparse: list of {rows.numel()} triplets written in {time.time() - t0:.3f}s")
    assert rows.numel() == nnz
    assert bool((rows < cols).all()) and bool((rows >= 0).all()) and int(cols.max()) < N and int(counts.min()) >= min_count
    if min_count == 1:
        expect = sum(int((np.bincount(d["ref_leaf"][b]).astype(np.int64) ** 2).sum()) for b in range(B))
        assert 2 * int(counts.sum(dtype=torch.int64)) + N * B == expect
        say("sparse: sum identity holds exactly")
    for i in _sample_rows(N, n_rows, 14):
        ref = oracle.counts_rows(d["ref_leaf"], i, i + 1)[0]
        for own, other, lo, hi in ((rows, cols, i + 1, N), (cols, rows, 0, i)):
            m = own == i
            j = other[m].cpu().numpy().astype(np.int64)
            v = counts[m].cpu().numpy().view(np.uint32)
            order = np.argsort(j)
            want_j = np.nonzero(ref[lo:hi] >= min_count)[0] + lo
            np.testing.assert_array_equal(j[order], want_j, err_msg=f"sample {i}")
            np.testing.assert_array_equal(v[order], ref[want_j], err_msg=f"sample {i}")
    say(f"sparse: {n_rows}+ sampled rows and columns exact")


def _check_consumers(d, n_rows):
    """Outlier measures and out-of-bag vote at full size, on sampled samples the oracle computes one by one."""
    import torch
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    B, N = d["ref_leaf"].shape
    _, y = ri.gaussian_mixture(d["c"])
    C = d["c"].C
    dy = torch.from_numpy(y.astype(np.int32)).cuda()
    t0 = time.time()
    printed, classic = rfx.prox_outlier(d["leaf"], d["Lb"], dy)
    torch.cuda.synchronize()
    say(f"outlier measures in {time.time() - t0:.3f}s")
    rows = _sample_rows(N, n_rows, 15)
    cnt = np.concatenate([oracle.counts_rows(d["ref_leaf"], i, i + 1) for i in rows])
    np.testing.assert_allclose(printed.cpu().numpy()[rows], oracle.outlier_printed(cnt, B, rows), rtol=1e-12)
    np.testing.assert_allclose(classic.cpu().numpy()[rows], oracle.outlier_classic(cnt, B, y, rows), rtol=1e-12)
    say(f"outlier measures: {len(rows)} sampled samples within 1e-12")
    lc = ri.leaf_classes(d["F"], y, C)
    t0 = time.time()
    votes, pred, wrong, voted = rfx.oob_vote(d["leaf"], torch.from_numpy(d["F"].inbag.view(np.int16)).cuda(),
                                             torch.from_numpy(lc).cuda(), C, dy)
    say(f"out-of-bag vote in {time.time() - t0:.3f}s: error {wrong}/{voted} = {wrong / max(voted, 1):.4f}")
    cols = np.array(_sample_rows(N, 200, 16))
    rv, rp = oracle.oob_vote(d["ref_leaf"][:, cols], d["F"].inbag[:, cols], lc, C)
    np.testing.assert_array_equal(votes.cpu().numpy().view(np.uint32)[cols], rv)
    np.testing.assert_array_equal(pred.cpu().numpy()[cols], rp)
    # whole-array properties: votes per sample = number of trees that missed it; tallies agree with the predictions
    np.testing.assert_array_equal(votes.sum(dim=1).cpu().numpy(), (d["F"].inbag == 0).sum(axis=0))
    p = pred.cpu().numpy()
    assert voted == int((p >= 0).sum()) and wrong == int(((p != y) & (p >= 0)).sum())
    say(f"out-of-bag vote: {cols.size} sampled samples exact, tallies consistent")


def _check_matvec(d, k, n_rows, prox=None):
    import torch
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    B, N = d["ref_leaf"].shape
    V = ri.start_block(N, k)
    plan = rfx.PvPlan(d["leaf"], d["Lb"])
    dV = torch.from_numpy(V).cuda()
    Y = plan.apply(dV)
    torch.cuda.synchronize()
    rows = _sample_rows(N, n_rows, 13)
    Yh = Y.cpu().numpy().astype(np.float64)
    num = den = 0.0
    for i in rows:
        ref = oracle.pv_rows(d["ref_leaf"], V.astype(np.float64), i, i + 1)[0]
        num += float(((Yh[i] - ref) ** 2).sum())
        den += float((ref ** 2).sum())
    err = np.sqrt(num / den)
    say(f"P.V k={k}: relative error on {len(rows)} sampled rows {err:.2e}")
    assert err <= 1e-5
    # P.1: B * y_i is the summed size of the leaves holding sample i
    ones = torch.ones((N, 1), dtype=torch.float32, device="cuda")
    y1 = plan.apply(ones).cpu().numpy()[:, 0].astype(np.float64) * B
    sizes = np.zeros(N, np.int64)
    for b in range(B):
        sizes += np.bincount(d["ref_leaf"][b])[d["ref_leaf"][b]]
    assert np.abs(y1 - sizes).max() <= 2e-6 * sizes.max()
    say("P.1 equals the summed leaf sizes")
    if prox is not None:
        # the materialised dense matrix times V (float64 library product, row blocks) against the implicit product
        worst = 0.0
        Vd = dV.double()
        for s in range(0, N, 4096):
            ref = prox[s:s + 4096].double() @ Vd
            worst = max(worst, float((ref - Y[s:s + 4096].double()).norm() / ref.norm()))
        say(f"dense P times V vs implicit product: worst row-block relative error {worst:.2e}")
        assert worst <= 1e-5
    plan.close()


def _check_lowrank_and_mds(d, k, T, mds_reference="arpack", reported_pairs=0):
    import torch
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    B, N = d["ref_leaf"].shape
    V0 = ri.start_block(N, k)
    lam, V, Q, s = rfx.prox_lowrank(d["leaf"], d["Lb"], torch.from_numpy(V0).cuda(), T)
    torch.cuda.synchronize()
    say("library block iteration done; running the float64 iteration on the CPU ...")
    t0 = time.time()
    lam_ref, V_ref = oracle.block_iteration(d["ref_leaf"], V0, T)
    say(f"oracle block iteration ({T} applications, k={k}) in {time.time() - t0:.0f}s")
    lam, V = lam.cpu().numpy(), V.cpu().numpy()
    rel = np.abs(lam - lam_ref) / lam_ref
    ang = oracle.principal_angle(V, V_ref)
    say(f"Ritz values: max relative difference {rel.max():.2e}; largest principal angle {ang:.2e} rad")
    assert rel.max() <= 1e-4 and ang < 1e-3
    if reported_pairs:
        # the reported layer: the library's Ritz pairs against the eigendecomposition itself (ARPACK on the float64
        # operator, P being too large for LAPACK): longest converged prefix, spectrum around it, residuals
        from conftest import converged_prefix
        t0 = time.time()
        lam_e, U_e = oracle.implicit_eig(d["ref_leaf"], reported_pairs, tol=1e-10)
        j = converged_prefix(lam.astype(np.float64), V.astype(np.float64), lam_e, U_e)
        PV = oracle.pv_implicit(d["ref_leaf"], V.astype(np.float64))
        res = np.linalg.norm(PV - V * lam[None, :], axis=0) / lam
        rel_e = np.abs(lam[:reported_pairs] - lam_e) / lam_e
        say(f"reported layer: top {reported_pairs} eigenpairs by ARPACK in {time.time() - t0:.0f}s; converged prefix j*={j}; "
            f"relative eigenvalue errors {np.array2string(rel_e, precision=1)}; residuals of pairs 1, j*, k: {res[0]:.1e}, "
            f"{res[max(j - 1, 0)]:.1e}, {res[k - 1]:.1e}; eigenvalues {np.array2string(lam_e, precision=2)}; Ritz values "
            f"{k - 1}, {k}: {lam[k - 2]:.3f}, {lam[k - 1]:.3f}")
        assert j >= 1 and (lam[:reported_pairs] <= lam_e * (1 + 1e-5)).all()
    Qr, sr = oracle.quantise_int8(V, lam)
    np.testing.assert_array_equal(s.cpu().numpy(), sr)
    np.testing.assert_array_equal(Q.cpu().numpy(), Qr)
    say("INT8 codes and scales bit-exact")
    A = oracle.dequantise(Qr, sr)
    PX = oracle.pv_implicit(d["ref_leaf"], V_ref)
    err = np.linalg.norm(A @ (A.T @ V_ref) - PX) / np.linalg.norm(PX)
    say(f"INT8-dequantised P.V on the converged block: relative Frobenius error {err:.2e}")
    assert err <= 2e-2
    assert Q.numel() == N * k      # one byte per code: N*k bytes of factor storage

    m = 16
    x0 = ri.start_block(N, m, seed=778)
    coords, ev, iters = rfx.mds3d(Q, s, torch.from_numpy(x0).cuda(), rfx.MDS_SQUARED, max_iters=300, tol=1e-7)
    torch.cuda.synchronize()
    coords, ev = coords.cpu().numpy().astype(np.float64), ev.cpu().numpy().astype(np.float64)
    assert np.abs(coords.sum(axis=0)).max() <= 1e-3 * np.abs(coords).max() * np.sqrt(N)
    np.testing.assert_allclose(coords.T @ coords, np.diag(ev), atol=2e-4 * ev[0])
    if mds_reference == "arpack":
        t0 = time.time()
        ref_c, ref_ev = oracle.mds3d_implicit(Qr, sr, oracle.SQUARED)
        say(f"oracle implicit scaling (ARPACK, float64) in {time.time() - t0:.0f}s; library took {iters} iterations")
        say(f"scaling eigenvalues {ev} vs {ref_ev}")
        np.testing.assert_allclose(ev, ref_ev, rtol=1e-4)
        gaps = np.abs(np.diff(ref_ev)) / ref_ev[0]
        if gaps.min() <= 1e-2:
            U, _, Vt = np.linalg.svd(coords.T @ ref_c)
            coords = coords @ (U @ Vt)
        err = np.linalg.norm(coords - ref_c) / np.linalg.norm(ref_c)
        say(f"scaling coordinates: relative Frobenius difference {err:.2e}")
        assert err <= 1e-3
    else:
        # too large for an eigen-solver run in the test: check the pairs against the float64 operator itself
        op = oracle.mds_operator(oracle.dequantise(Qr, sr), oracle.SQUARED)
        Vn = coords / np.sqrt(ev)[None, :]
        GV = op(Vn)
        rq = (Vn * GV).sum(axis=0)
        res = np.linalg.norm(GV - Vn * ev[None, :], axis=0) / ev[0]
        say(f"library took {iters} iterations; eigenvalues {ev}; Rayleigh quotients {rq}; residuals {res}")
        np.testing.assert_allclose(rq, ev, rtol=1e-4)
        assert res.max() <= 5e-3


def test_cfg3_dense_and_rank32(w3):
    _check_leaf(w3)
    say("cfg3 leaf ids bit-exact")
    prox = _check_dense(w3, 24)
    _check_matvec(w3, 32, 24, prox)
    del prox
    _check_fused(w3, 12)
    _check_sparse(w3, 16)
    _check_consumers(w3, 12)
    _check_oob(w3, 12)
    _check_lowrank_and_mds(w3, 32, 20, reported_pairs=14)


def test_cfg4_leaf_and_dense(w4):
    _check_leaf(w4)
    say("cfg4 leaf ids bit-exact")
    prox = _check_dense(w4, 24)
    _check_matvec(w4, 64, 16, prox)
    del prox
    _check_fused(w4, 10)
    _check_sparse(w4, 12)
    _check_consumers(w4, 8)
    _check_oob(w4, 12)


def test_cfg4_rank64_factors_and_scaling(w4):
    _check_lowrank_and_mds(w4, 64, 20)


def test_cfg5_rows_with_reduced_trees(w5_reduced):
    """500,000 rows x 64 features, 20 classes; 32 of the 1,000 trees (deep trees, ~46k leaves each)."""
    _check_leaf(w5_reduced)
    say("cfg5 (32 trees) leaf ids bit-exact")
    _check_matvec(w5_reduced, 64, 8)
    _check_sparse(w5_reduced, 8)
    _check_lowrank_and_mds(w5_reduced, 64, 20, mds_reference="residual")


def test_cfg5_full_tree_count():
    """Workload 5 as bench.py runs it: 500,000 rows x 64 features, 20 classes, all 1,000 trees (about 90 M nodes,
    46k leaves per tree, 5e8 (tree, sample) slots).  The CPU input generator would need tens of minutes for this
    forest, so it is grown by rfx_forest_grow (bit-identical to the oracle's grower on the 8-tree check above; for
    everything downstream a forest is only an input).  Covered: leaf ids of all 5e8 walks bit-exact against the
    oracle's traversal; the sparse pass on sampled rows and columns plus its exact sum identity; one implicit product
    against the oracle's float64 product IN FULL (all N rows); the factorisation against the oracle's float64 block
    iteration from the same start block (Ritz values, subspace angle); INT8 codes bit-exact; INT8 product error; the
    scaling eigenpairs through the float64 operator.  Not covered at this size: the dense outputs (1 TB, they do not
    exist) and an eigen-solver reference for the scaling step (residuals instead)."""
    import torch
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    c = ri.CONFIGS[5]
    N, B, k, T = c.N, c.B, 64, 20
    X, y = ri.gaussian_mixture(c)
    dX, dy = torch.from_numpy(X).cuda(), torch.from_numpy(y.astype(np.int32)).cuda()
    t0 = time.time()
    g = rfx.forest_grow(dX, dy, c.C, B, c.mtry, ri.mixture.FOREST_ISEED)
    say(f"cfg5 at {B} trees: forest grown on the GPU in {time.time() - t0:.1f}s, {int(g['node_offset'][-1])} nodes, "
        f"most leaves {int(g['n_leaves'].max())}, deepest level {int(g['depth'].max())}")
    F = ri.Forest(B, c.M, g["node_offset"], g["feature"], g["threshold"], g["left"], g["right"], g["leaf_id"], g["depth"],
                  g["n_leaves"], g["inbag"], None)
    gf = _forest(F)
    Lb = gf.leaf_bound
    leaf = rfx.leaf_assign(gf, dX)
    torch.cuda.synchronize()
    t0 = time.time()
    ref_leaf, plen = oracle.leaf_assign(F, X)
    say(f"oracle leaf assignment of {B * N:.1e} walks in {time.time() - t0:.0f}s, mean path {plen / ref_leaf.size:.2f}")
    for b0 in range(0, B, 125):                            # 250 MB at a time
        np.testing.assert_array_equal(_u32(leaf[b0:b0 + 125]), ref_leaf[b0:b0 + 125])
    say("cfg5 leaf ids bit-exact (all trees, all samples)")
    d = dict(c=c, X=X, F=F, ref_leaf=ref_leaf, gf=gf, leaf=leaf, Lb=Lb)

    # sparse pass (the tile kernel bench.py times at this workload): count, sum identity, sampled rows and columns
    t0 = time.time()
    nnz = rfx.prox_sparse_count(leaf, Lb, 1)
    say(f"sparse: {nnz} non-zero pairs ({nnz / (N * (N - 1) / 2):.2%} of the triangle), counted in {time.time() - t0:.2f}s")
    sq = 0
    for b in range(B):
        sq += int((np.bincount(ref_leaf[b]).astype(np.int64) ** 2).sum())
    say(f"sum over trees and leaves of size^2 = {sq:.6e} = {sq / B:.4e} per tree, against N^2/2 = {N * N / 2:.3e} pair tests per tree "
        f"({N * N / 2 / (sq / B):.0f}x)")
    rows, cols, counts, _ = rfx.prox_sparse(leaf, Lb, 1, capacity=nnz, count_dtype=rfx.U16)
    torch.cuda.synchronize()
    assert rows.numel() == nnz and bool((rows < cols).all()) and int(cols.max()) < N
    total = 0
    for s0 in range(0, nnz, 1 << 28):
        total += int(counts[s0:s0 + (1 << 28)].to(torch.int32).bitwise_and(0xFFFF).sum(dtype=torch.int64))
    assert 2 * total + N * B == sq
    say("sparse: 2 sum(counts) + N B equals the summed squared leaf sizes exactly")
    for i in _sample_rows(N, 4, 14):
        ref = oracle.counts_rows(ref_leaf, i, i + 1)[0]
        for own, other, lo, hi in ((rows, cols, i + 1, N), (cols, rows, 0, i)):
            js, vs = [], []
            for s0 in range(0, nnz, 1 << 30):               # masks over more than 2^31 entries are taken in pieces
                at = (own[s0:s0 + (1 << 30)] == i).nonzero().flatten() + s0
                js.append(other[at].cpu().numpy().astype(np.int64))
                vs.append(counts[at].cpu().numpy().view(np.uint16).astype(np.uint32))
            j, v = np.concatenate(js), np.concatenate(vs)
            order = np.argsort(j)
            want_j = np.nonzero(ref[lo:hi] >= 1)[0] + lo
            np.testing.assert_array_equal(j[order], want_j, err_msg=f"sample {i}")
            np.testing.assert_array_equal(v[order], ref[want_j], err_msg=f"sample {i}")
    say("sparse: sampled rows and columns exact")
    del rows, cols, counts
    torch.cuda.empty_cache()

    # implicit product, in full, and the factorisation against the float64 iteration from the same start block
    V0 = ri.start_block(N, k)
    plan = rfx.PvPlan(leaf, Lb)
    # the row pass out of this plan first (count only; it marks the plan's member lists and takes the marks out again),
    # then the product from the same plan: the way bench.py's step uses the two at this workload
    ws = rfx.new_workspace(rfx.prox_sparse_plan_workspace_bytes(plan))
    nz = torch.zeros(1, dtype=torch.int64, device="cuda")
    rfx.prox_sparse_plan(plan, ws, nz)
    Y = plan.apply(torch.from_numpy(V0).cuda()).cpu().numpy().astype(np.float64)
    assert int(nz.item()) == nnz
    say("sparse: the row pass out of the product's plan counts the same pairs")
    del ws
    plan.close()
    t0 = time.time()
    Yref = oracle.pv_implicit(ref_leaf, V0.astype(np.float64))
    err = np.linalg.norm(Y - Yref) / np.linalg.norm(Yref)
    say(f"P.V k={k} against the oracle's float64 product on all {N} rows ({time.time() - t0:.0f}s): relative Frobenius error {err:.2e}")
    assert err <= 1e-5
    del Y, Yref
    lam, V, Q, s = rfx.prox_lowrank(leaf, Lb, torch.from_numpy(V0).cuda(), T)
    torch.cuda.synchronize()
    t0 = time.time()
    lam_ref, V_ref = oracle.block_iteration(ref_leaf, V0, T, progress=lambda t: say(f"  oracle block iteration: application {t}/{T} after {time.time() - t0:.0f}s"))
    lam_h, V_h = lam.cpu().numpy(), V.cpu().numpy()
    rel = np.abs(lam_h - lam_ref) / lam_ref
    ang = oracle.principal_angle(V_h, V_ref)
    say(f"Ritz values: max relative difference {rel.max():.2e}; largest principal angle {ang:.2e} rad")
    assert rel.max() <= 1e-4 and ang < 1e-3
    Qr, sr = oracle.quantise_int8(V_h, lam_h)
    np.testing.assert_array_equal(s.cpu().numpy(), sr)
    np.testing.assert_array_equal(Q.cpu().numpy(), Qr)
    say("INT8 codes and scales bit-exact")
    A = oracle.dequantise(Qr, sr)
    PX = oracle.pv_implicit(ref_leaf, V_ref)
    err = np.linalg.norm(A @ (A.T @ V_ref) - PX) / np.linalg.norm(PX)
    say(f"INT8-dequantised P.V on the converged block: relative Frobenius error {err:.2e}")
    assert err <= 2e-2
    del PX, V_ref

    m = 16
    x0 = ri.start_block(N, m, seed=778)
    coords, ev, iters = rfx.mds3d(Q, s, torch.from_numpy(x0).cuda(), rfx.MDS_SQUARED, max_iters=300, tol=1e-7)
    coords, ev = coords.cpu().numpy().astype(np.float64), ev.cpu().numpy().astype(np.float64)
    op = oracle.mds_operator(A, oracle.SQUARED)
    Vn = coords / np.sqrt(ev)[None, :]
    GV = op(Vn)
    rq = (Vn * GV).sum(axis=0)
    res = np.linalg.norm(GV - Vn * ev[None, :], axis=0) / ev[0]
    say(f"scaling: {iters} iterations; eigenvalues {ev}; Rayleigh quotients {rq}; residuals {res}")
    np.testing.assert_allclose(rq, ev, rtol=1e-4)
    assert res.max() <= 5e-3
    assert np.abs(coords.sum(axis=0)).max() <= 1e-3 * np.abs(coords).max() * np.sqrt(N)


# ------------------------------------------------------------------------------------------ forest growth
@pytest.mark.parametrize("cfg,trees", [(4, 128), (5, 8)])
def test_growth_at_full_row_counts(cfg, trees):
    """The library's forest against the oracle's at the workloads' full row counts (a reduced number of
    trees keeps the sequential oracle to about ten seconds); every array bit-exact."""
    import torch
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    c = ri.CONFIGS[cfg]
    X, y = ri.gaussian_mixture(c)
    dX, dy = torch.from_numpy(X).cuda(), torch.from_numpy(y.astype(np.int32)).cuda()
    rfx.forest_grow(dX, dy, c.C, 2, c.mtry, 99)                       # first call: allocator warm-up
    t0 = time.time()
    got = rfx.forest_grow(dX, dy, c.C, trees, c.mtry, 20251119, first_tree=3)
    t_gpu = time.time() - t0
    t0 = time.time()
    ref = oracle.grow(X, y, c.C, trees, c.mtry, 20251119, first_tree=3)
    t_cpu = time.time() - t0
    say(f"cfg{cfg}: {trees} trees on {c.N} rows: library {t_gpu:.2f}s, oracle {t_cpu:.1f}s; {int(ref['node_offset'][-1])} nodes, "
        f"deepest level {int(ref['depth'].max())}, most leaves {int(ref['n_leaves'].max())}")
    for k in ("node_offset", "feature", "left", "right", "leaf_id", "depth", "n_leaves", "inbag", "leaf_class"):
        np.testing.assert_array_equal(got[k], ref[k], err_msg=k)
    np.testing.assert_array_equal(got["threshold"].view(np.uint32), ref["threshold"].view(np.uint32))
    say("forest identical to the oracle's")
