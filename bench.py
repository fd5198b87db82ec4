#!/usr/bin/env python3
"""Benchmark of the random-forest proximity hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--cfg 4]

One step = one pass of the whole path over one synthetic workload, inputs resident in HBM:
leaf assignment -> dense proximity (full float32) -> out-of-bag proximity (packed upper float32)
-> rank-k block iteration with INT8 factors -> 3-D scaling from the factors.
Prints ONE JSON line (metric: leaf co-occurrence tests per second, N^2*B/2 per step), with the
roofline of the dominant kernel and the CPU oracle timed on a bounded sample of the same work.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

PEAK_VALU_LANE_OPS = 256 * 64 * 2.4e9   # 256 CUs x 64 lanes/clk x 2.4 GHz: plain 32-bit vector ops per second
FUSED_FETCH_KIB, FUSED_WRITE_KIB = 39202305.0, 63045597.1   # rocprofv3 per-launch counters of the fused kernel, workload 4
PEAK_HBM_BYTES = 8.0e12


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--cfg", type=int, default=4, help="workload 1..5 (default: N=100,000, B=1,000)")
    ap.add_argument("--trees", type=int, default=0, help="override the tree count (debugging only)")
    ap.add_argument("--rows", type=int, default=0, help="override the row count (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mds-block", type=int, default=16)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one 4 GiB device copy before the steps (reference for rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    rfx.load()          # fails loudly if librfx.so is missing: there is no fallback path
    dev = torch.device("cuda:0")
    c = ri.CONFIGS[args.cfg]
    N = args.rows or c.N
    B = args.trees or c.B
    k, T = c.k, c.T
    reduced = bool(args.rows or args.trees)

    # Workloads whose dense float32 output does not fit the GPU (workload 5: 1 TB) take the exact sparse list instead of
    # the dense passes, and their forest is grown on the GPU (the CPU input generator needs tens of minutes there).
    large = 4.0 * N * N > 120e9
    t0 = time.time()
    if large:
        X, y = ri.gaussian_mixture(c, N if args.rows else None)
        grown = rfx.forest_grow(torch.from_numpy(X).to(dev), torch.from_numpy(y.astype(np.int32)).to(dev), c.C, B, c.mtry,
                                ri.mixture.FOREST_ISEED)
        F = ri.Forest(B, c.M, grown["node_offset"], grown["feature"], grown["threshold"], grown["left"], grown["right"],
                      grown["leaf_id"], grown["depth"], grown["n_leaves"], grown["inbag"], np.zeros((B, 0), np.int32))
        large_leaf_class = grown["leaf_class"]
        del grown
    else:
        X, y, F = ri.load_or_grow(c, N=N if args.rows else None, B=B if args.trees else None)
    log(f"workload cfg{c.cfg}: N={N} M={c.M} B={B} k={k} T={T}; inputs ready in {time.time() - t0:.1f}s "
        f"(nodes={F.total_nodes}, max leaves/tree={int(F.n_leaves.max())}" + (", forest grown on the GPU)" if large else ")"))
    t0 = time.perf_counter()
    gf = rfx.Forest(F.n_features, F.node_offset, F.feature, F.threshold, F.left, F.right, F.leaf_id, F.n_leaves)
    forest_create_ms = (time.perf_counter() - t0) * 1e3     # host validation + re-layout + upload, once per forest
    Lb = gf.leaf_bound
    dX = torch.from_numpy(X).to(dev)
    d_inbag = torch.from_numpy(F.inbag.view(np.int16)).to(dev)
    dV0 = torch.from_numpy(ri.start_block(N, k)).to(dev)
    m = args.mds_block
    dx0 = torch.from_numpy(ri.start_block(N, m, seed=ri.mixture.START_SEED + 1)).to(dev)
    leaf = torch.empty((B, N), dtype=torch.int32, device=dev)
    n_ut = N * (N - 1) // 2
    if large:
        # capacity of the sparse list: one counting call on the leaf ids of this forest
        rfx.leaf_assign(gf, dX, leaf)
        sp_cap = max(rfx.prox_sparse_count(leaf, Lb, 1), 1)
        sp_rows = torch.empty(sp_cap, dtype=torch.int32, device=dev)
        sp_cols = torch.empty_like(sp_rows)
        sp_cnt = torch.empty(sp_cap, dtype=torch.int16, device=dev)
        sp_got = ctypes.c_int64(0)
    else:
        prox = torch.empty((N, N), dtype=torch.float32, device=dev)
        prox_oob = torch.empty((n_ut,), dtype=torch.float32, device=dev)

    lib = rfx.load()
    st = torch.cuda.current_stream().cuda_stream
    phase_ms = {}

    def timed(name, fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = fn()
        e1.record()
        phase_ms.setdefault(name, []).append((e0, e1))
        return out

    fused = B <= 1023 and not large   # plain and out-of-bag proximities from one pass over the trees

    def dense_and_oob_separately():
        timed("prox_dense", lambda: rfx.prox_dense(leaf, Lb, rfx.U32, rfx.FULL, prox=prox, want_counts=False))
        timed("prox_oob", lambda: rfx._check(lib.rfx_prox_oob(leaf.data_ptr(), d_inbag.data_ptr(), N, B, Lb, rfx.U32,
                                                               rfx.UPPER_PACKED, 0, 0, prox_oob.data_ptr(), st)))

    def step():
        timed("leaf_assign", lambda: rfx.leaf_assign(gf, dX, leaf))
        if large:
            timed("prox_sparse", lambda: rfx._check(lib.rfx_prox_sparse(leaf.data_ptr(), N, B, Lb, 1, rfx.U16, sp_cap,
                                                                         sp_rows.data_ptr(), sp_cols.data_ptr(), sp_cnt.data_ptr(),
                                                                         0, ctypes.byref(sp_got), st)))
        elif fused:
            timed("prox_dense_oob", lambda: rfx._check(lib.rfx_prox_dense_oob(
                leaf.data_ptr(), d_inbag.data_ptr(), N, B, Lb, rfx.U32, rfx.FULL, 0, prox.data_ptr(), rfx.UPPER_PACKED, 0, 0,
                prox_oob.data_ptr(), st)))
        else:
            dense_and_oob_separately()
        lam, V, Q, s = timed("prox_lowrank", lambda: rfx.prox_lowrank(leaf, Lb, dV0, T))
        res = timed("mds3d", lambda: rfx.mds3d(Q, s, dx0, rfx.MDS_SQUARED, max_iters=200, tol=1e-5))
        return lam, res

    if args.calibrate_copy:
        # a plain device-to-device copy of known size: calibrates the HBM byte counters of a --pmc run
        n_cal = 1 << 30
        src = torch.empty(n_cal, dtype=torch.int32, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        log(f"calibration copy: {4 * n_cal} bytes read and {4 * n_cal} bytes written by one elementwise copy kernel")
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    phase_ms.clear()
    rfx.timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        lam, (coords, ev, mds_iters) = step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    phases = {n: float(np.mean([a.elapsed_time(b) for a, b in evs])) for n, evs in phase_ms.items()}
    if fused:
        # the two passes the fused one replaces, outside the step, for their own kernel times
        for _ in range(2):
            dense_and_oob_separately()
        torch.cuda.synchronize()
        phases["separate_prox_dense"] = float(np.mean([a.elapsed_time(b) for a, b in phase_ms.pop("prox_dense")]))
        phases["separate_prox_oob"] = float(np.mean([a.elapsed_time(b) for a, b in phase_ms.pop("prox_oob")]))
    kern = {}
    for name in ("leaf_assign_kernel", "prox_tile_kernel_both", "prox_tile_kernel", "prox_tile_kernel_oob",
                 "prox_tile_kernel_sparse", "pv_leaf_sum_kernel", "pv_gather_kernel"):
        ms, n = rfx.timing_get(name)
        kern[name] = {"avg_ms": ms / max(n, 1), "launches": n}
    # outside the timed step: the thresholded sparse form of the same counts (every non-zero pair)
    if large:
        assert sp_got.value == sp_cap, "the sparse pass found a different number of pairs than the counting call"
        nnz = sp_cap
        sp_ms = kern["prox_tile_kernel_sparse"]["avg_ms"]
        rfx.timing_enable(True)
    else:
        nnz = rfx.prox_sparse_count(leaf, Lb, 1)
        sp_rows = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
        sp_cols = torch.empty_like(sp_rows)
        sp_cnt = torch.empty(max(nnz, 1), dtype=torch.int16, device=dev)
        got = ctypes.c_int64(0)
        rfx.timing_enable(True)
        for _ in range(2):
            rfx._check(lib.rfx_prox_sparse(leaf.data_ptr(), N, B, Lb, 1, rfx.U16, max(nnz, 1), sp_rows.data_ptr(),
                                           sp_cols.data_ptr(), sp_cnt.data_ptr(), 0, ctypes.byref(got), st))
        sp_ms, sp_n = rfx.timing_get("prox_tile_kernel_sparse")
        sp_ms /= max(sp_n, 1)
    del sp_rows, sp_cols, sp_cnt
    # consumers of the proximity rows, also outside the step
    d_y = torch.from_numpy(y.astype(np.int32)).to(dev)
    d_lc = torch.from_numpy(large_leaf_class if large else ri.leaf_classes(F, y, c.C)).to(dev)
    for _ in range(2):
        rfx.prox_outlier(leaf, Lb, d_y)
        _, _, oob_wrong, oob_voted = rfx.oob_vote(leaf, d_inbag, d_lc, c.C, d_y, want_votes=False)
    ol_ms, ol_n = rfx.timing_get("prox_tile_kernel_outlier")
    ov_ms, ov_n = rfx.timing_get("oob_vote_kernel")
    consumers = {"note": "not part of the step",
                 "outlier_avg_launch_ms": ol_ms / max(ol_n, 1), "oob_vote_avg_launch_ms": ov_ms / max(ov_n, 1),
                 "oob_vote_GBps": (6.0 * N * B + 8.0 * N) / (ov_ms / max(ov_n, 1) * 1e-3) / 1e9 if ov_ms > 0 else 0.0,
                 "oob_error": oob_wrong / max(oob_voted, 1)}
    rfx.timing_enable(False)
    # once-per-forest grouping of samples by leaf for the implicit product (inside every prox_lowrank call above)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan = rfx.PvPlan(leaf, Lb)
    torch.cuda.synchronize()
    pv_plan_ms = (time.perf_counter() - t0) * 1e3
    plan.close()
    # growth of the same forest shape on the GPU (outside the step; the step's forest comes from the input generator)
    torch.cuda.synchronize()
    rfx.forest_grow(dX, d_y, c.C, min(B, 8), c.mtry, 1)                      # warm-up
    t0 = time.perf_counter()
    grown = rfx.forest_grow(dX, d_y, c.C, B if not large else min(B, 128), c.mtry, ri.mixture.FOREST_ISEED)
    grow_s = time.perf_counter() - t0
    grown_trees = B if not large else min(B, 128)
    growth = {"note": "not part of the step", "trees": grown_trees, "seconds": grow_s, "trees_per_s": grown_trees / grow_s,
              "nodes": int(grown["node_offset"][-1]), "level_passes": grown["levels"], "sorted_pairs": grown["sorted_pairs"],
              "pairs_per_s": grown["sorted_pairs"] / grow_s}
    del grown
    # practical ceilings of this GPU next to the published peaks
    valu_rate = rfx.probe_valu(4096)
    copy_rate = rfx.probe_copy(1 << 32)

    tests = N * N * B / 2.0
    P = int(np.ceil(np.log2(max(Lb, 2))))
    P = 8 if P < 8 else (P if P <= 16 else (P + 1) & ~1)   # plane count the library uses for this bound
    # dominant kernel: bit-plane compare-and-count.  One launch covers the tile pairs on and below the
    # diagonal of the (padded) N x N grid; per 32 trees and pair, P + 1 vector ops for the plain count, P + 7 for the
    # fused pass that also yields the out-of-bag numerator and denominator: algorithmic lane-ops per launch
    dom = "prox_tile_kernel_sparse" if large else ("prox_tile_kernel_both" if fused else "prox_tile_kernel")
    ops_per_test = (P + 7) / 32.0 if fused else (P + 1) / 32.0
    ops_per_launch = tests * ops_per_test
    tile_ms = kern[dom]["avg_ms"]
    achieved = ops_per_launch / (tile_ms * 1e-3) if tile_ms > 0 else 0.0
    # HBM-side bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    # (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 KiB, calibrated on a 4 GiB copy); measured for workload 4 only
    traffic = None
    if c.cfg == 4 and not reduced:
        traffic = (FUSED_FETCH_KIB * 2.0 + FUSED_WRITE_KIB) * 1024.0 if fused else (39087769.4 * 2.0 + 42359959.7) * 1024.0
    plain_ms = kern["prox_tile_kernel"]["avg_ms"]
    roofline = {"kernel": dom, "bound": "alu", "achieved": achieved / 1e12, "peak": PEAK_VALU_LANE_OPS / 1e12,
                "unit": "T lane-ops/s", "frac": achieved / PEAK_VALU_LANE_OPS, "traffic": traffic,
                "traffic_source": "profiles/bench_cfg4_pmc_fetch_write.txt (L2-to-fabric bytes; outputs are 4*N*N + 2*N*(N-1))",
                "ops_per_test": ops_per_test, "avg_launch_ms": tile_ms,
                # the plain compare-and-count kernel on its own (P + 1 ops per 32 trees), run outside the step
                "plain_kernel": {"avg_launch_ms": plain_ms, "ops_per_test": (P + 1) / 32.0,
                                 "frac": tests * (P + 1) / 32.0 / (plain_ms * 1e-3) / PEAK_VALU_LANE_OPS} if plain_ms > 0 else None,
                "tests_per_s": tests / (tile_ms * 1e-3) if tile_ms > 0 else 0.0,
                # the same rate against the roof of a plain compare-and-add loop (2 lane-ops per test: 19.7 T tests/s),
                # which does not depend on this kernel's own op count (above 1 = faster than a perfect such loop),
                # and against the rate a dependency-free loop of the same two instructions reaches on this GPU
                "ratio_to_2op_roof": (tests / (tile_ms * 1e-3)) / (PEAK_VALU_LANE_OPS / 2.0) if tile_ms > 0 else 0.0,
                "measured_valu_lane_ops_per_s": valu_rate, "frac_of_measured_valu": achieved / valu_rate if valu_rate > 0 else 0.0}
    # implicit product: algorithmic bytes per application = B*N*(2*4k + 4) + 2*4*N*k
    w_pv = B * N * (2 * 4 * k + 4) + 2 * 4 * N * k
    pv_ms = kern["pv_leaf_sum_kernel"]["avg_ms"] + kern["pv_gather_kernel"]["avg_ms"]
    pv = {"bytes_per_application": w_pv, "avg_ms": pv_ms, "GBps": w_pv / (pv_ms * 1e-3) / 1e9 if pv_ms > 0 else 0.0,
          "frac_of_hbm_peak": (w_pv / (pv_ms * 1e-3)) / PEAK_HBM_BYTES if pv_ms > 0 else 0.0,
          "leaf_sum_ms": kern["pv_leaf_sum_kernel"]["avg_ms"], "gather_ms": kern["pv_gather_kernel"]["avg_ms"],
          "compulsory_floor_bytes": 4 * N * B + 8 * N * k,
          # rocprofv3 FETCH_SIZE x 2 + WRITE_SIZE of the three kernels of one application (workload 4 only)
          "measured_fabric_bytes": ((7119809.3 + 3330050.5 + 2570010.1) * 2.0 + 827637.2 + 25000.0) * 1024.0
          if (c.cfg == 4 and not reduced) else None,
          "measured_copy_bytes_per_s": copy_rate,
          "frac_of_measured_copy": (w_pv / (pv_ms * 1e-3)) / copy_rate if pv_ms > 0 and copy_rate > 0 else 0.0,
          "valu_bound_ms": 2.0 * B * N * k / PEAK_VALU_LANE_OPS * 1e3, "plan_build_ms": pv_plan_ms,
          "note": "above 100 % of the HBM peak = cache-assisted: V and the per-tree sums are served by L2 / Infinity Cache"}

    # leaf assignment: one 8-byte node record and one 4-byte feature value per visited internal node,
    # plus the leaf-id write and X read once
    depth_tab = np.zeros((B, Lb), np.int32)
    for b in range(B):
        s, e = int(F.node_offset[b]), int(F.node_offset[b + 1])
        lid = F.leaf_id[s:e]
        depth_tab[b, lid[lid >= 0]] = F.depth[s:e][lid >= 0]
    d_depth = torch.from_numpy(depth_tab).to(dev)
    path_total = int(sum(int(d_depth[b0:b0 + 50].gather(1, leaf[b0:b0 + 50].long()).sum()) for b0 in range(0, B, 50)))
    w_la = path_total * (8 + 4) + 4 * N * B + 4 * N * c.M
    la_ms = kern["leaf_assign_kernel"]["avg_ms"]
    la = {"bytes_model": w_la, "mean_path": path_total / (N * B), "avg_ms": la_ms,
          "GBps": w_la / (la_ms * 1e-3) / 1e9 if la_ms > 0 else 0.0,
          "frac_of_hbm_peak": (w_la / (la_ms * 1e-3)) / PEAK_HBM_BYTES if la_ms > 0 else 0.0,
          "compulsory_floor_bytes": 4 * N * c.M + 8 * int(F.total_nodes) + 4 * N * B,
          "measured_fabric_bytes": (970263.7 * 2.0 + 390625.0) * 1024.0 if (c.cfg == 4 and not reduced) else None,
          "forest_create_ms": forest_create_ms,
          "note": "gather-latency bound; nodes and X are cache / LDS resident, so the byte model is not HBM traffic"}

    out = {
        "metric": "leaf co-occurrence tests/s (N^2*B/2 per pass of the whole proximity path)",
        "value": tests / (ms_per_step * 1e-3),
        "unit": "tests/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": f"cfg{c.cfg}: N={N} M={c.M} B={B} trees to purity, mtry={c.mtry}, k={k}, T={T}"
                               + (" (REDUCED, debugging)" if reduced else "")
                               + (" (dense outputs do not fit: exact sparse list instead; forest grown by rfx_forest_grow)" if large else ""),
                   "leaf_bound": Lb, "bit_planes": P, "mds_block": m, "mds_iters": mds_iters},
        "phases_ms": phases,
        "mds": {"iterations": mds_iters, "ms_per_iteration": phases["mds3d"] / max(mds_iters, 1),
                "factor_GBps": N * k * mds_iters / (phases["mds3d"] * 1e-3) / 1e9},
        "dense_tests_per_s": tests / (phases["prox_sparse" if large else ("prox_dense_oob" if fused else "prox_dense")] * 1e-3),
        "pv": pv,
        "leaf_assign": la,
        "kernels": kern,
        "roofline": roofline,
        "consumers": consumers,
        "growth": growth,
        "sparse": {"note": "not part of the step: strict-upper (i, j, count) triplets of every non-zero pair",
                   "min_count": 1, "pairs": nnz, "fraction_of_triangle": nnz / max(N * (N - 1) / 2.0, 1.0),
                   "bytes_out": 10 * nnz, "avg_launch_ms": sp_ms,
                   "tests_per_s": tests / (sp_ms * 1e-3) if sp_ms > 0 else 0.0,
                   "frac_of_alu_peak": (tests * (P + 1) / 32.0 / (sp_ms * 1e-3)) / PEAK_VALU_LANE_OPS if sp_ms > 0 else 0.0},
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(leaf, N, B, X, F, k, y, c)
    print(json.dumps(out))


def cpu_baseline(leaf_dev, N, B, X, F, k, y, c):
    """The oracle as it stands, on the host cores, on bounded samples of the same workload: naive pair
    counting on a block of rows (the metric's unit), plus leaf assignment and one float64 implicit P.V
    on the first trees of the forest."""
    import oracle
    leaf = leaf_dev.cpu().numpy().view(np.uint32)
    cores = len(os.sched_getaffinity(0))
    try:
        cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    except ValueError:
        pass
    rows = min(N, 8)
    t0 = time.perf_counter()
    oracle.counts_rows(leaf, 0, rows)
    dt = time.perf_counter() - t0
    # size the sample for roughly 10 s of work
    rows2 = int(min(N, max(rows, rows * 10.0 / max(dt, 1e-3))))
    t0 = time.perf_counter()
    oracle.counts_rows(leaf, 0, rows2)
    dt = time.perf_counter() - t0
    tests = rows2 * N * B
    out = {"value": tests / dt, "unit": "tests/s", "cores": cores, "kind": "oracle",
           "sample": f"orc_counts_rows on rows 0..{rows2 - 1} x all {N} columns x {B} trees ({tests:.3g} tests, {dt:.1f}s)"}
    # the same routine on one core, on a proportionally smaller block of rows (about 3 s)
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        before = gomp.omp_get_max_threads()
        gomp.omp_set_num_threads(1)
        rows1 = max(1, int(rows2 * 3.0 / max(dt, 1e-3) / max(cores, 1)))
        t0 = time.perf_counter()
        oracle.counts_rows(leaf, 0, rows1)
        dt1 = time.perf_counter() - t0
        gomp.omp_set_num_threads(before)
        out["one_core"] = {"value": rows1 * N * B / dt1, "unit": "tests/s",
                           "sample": f"rows 0..{rows1 - 1} ({dt1:.1f}s), extrapolates to {N * N * B / 2.0 / (rows1 * N * B / dt1) / 3600:.1f} h for the whole triangle"}
    except OSError:
        pass
    # other phases, on the first Bs trees (context; same byte models as the GPU figures)
    Bs = min(B, 64)
    Fs = F.subset(Bs)
    t0 = time.perf_counter()
    sub_leaf, plen = oracle.leaf_assign(Fs, X)
    dt_la = time.perf_counter() - t0
    w_la = plen * 12 + 4 * N * Bs + 4 * N * X.shape[1]
    rng = np.random.default_rng(1)
    V = rng.standard_normal((N, k))
    t0 = time.perf_counter()
    oracle.pv_implicit(sub_leaf, V)
    dt_pv = time.perf_counter() - t0
    w_pv = Bs * N * (2 * 4 * k + 4) + 2 * 4 * N * k      # the float32 byte model, for comparison with the GPU figure
    t0 = time.perf_counter()
    n_grow = min(B, cores)
    oracle.grow(X, y, c.C, n_grow, c.mtry, 1)
    dt_grow = time.perf_counter() - t0
    out["phases"] = {
        "growth": {"trees": n_grow, "seconds": dt_grow, "trees_per_s": n_grow / dt_grow},
        "leaf_assign": {"trees": Bs, "seconds": dt_la, "walks_per_s": N * Bs / dt_la, "model_GBps": w_la / dt_la / 1e9},
        "pv_implicit_f64": {"trees": Bs, "k": k, "seconds": dt_pv, "model_GBps": w_pv / dt_pv / 1e9},
    }
    return out


if __name__ == "__main__":
    main()
