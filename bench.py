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
# rocprofv3 --pmc per-launch counters (KiB) at workload 4, from the committed summaries under profiles/
FUSED_FETCH_KIB, FUSED_WRITE_KIB = 39202305.0, 63045597.1      # fused plain + out-of-bag tile kernel
PLAIN_FETCH_KIB, PLAIN_WRITE_KIB = 39087769.4, 42359959.7      # plain tile kernel
PV_FETCH_KIB, PV_WRITE_KIB = (7119809.3, 3330050.5, 2570010.1), (827637.2, 25000.0)   # the kernels of one P.V application
LEAF_FETCH_KIB, LEAF_WRITE_KIB = 970263.7, 390625.0            # leaf assignment
PEAK_HBM_BYTES = 8.0e12


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def parse_args():
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
    return args


class Workload:
    """One synthetic workload resident in HBM: data, forest, start blocks and the output buffers of the step."""

    def __init__(self, args, torch, rfx, ri):
        self.torch, self.rfx, self.ri = torch, rfx, ri
        self.dev = dev = torch.device("cuda:0")
        self.c = c = ri.CONFIGS[args.cfg]
        self.N = N = args.rows or c.N
        self.B = B = args.trees or c.B
        self.k, self.T, self.m = c.k, c.T, args.mds_block
        self.reduced = bool(args.rows or args.trees)
        # Workloads whose dense float32 output does not fit the GPU (workload 5: 1 TB) take the exact sparse list instead
        # of the dense passes, and their forest is grown on the GPU (the CPU input generator needs tens of minutes there).
        self.large = large = 4.0 * N * N > 120e9
        # plain and out-of-bag proximities from one pass over the trees (three 10-bit fields per counter)
        self.fused = B <= 1023 and not large
        t0 = time.time()
        if large:
            X, y = ri.gaussian_mixture(c, N if args.rows else None)
            grown = rfx.forest_grow(torch.from_numpy(X).to(dev), torch.from_numpy(y.astype(np.int32)).to(dev), c.C, B,
                                    c.mtry, ri.mixture.FOREST_ISEED)
            F = ri.Forest(B, c.M, grown["node_offset"], grown["feature"], grown["threshold"], grown["left"],
                          grown["right"], grown["leaf_id"], grown["depth"], grown["n_leaves"], grown["inbag"],
                          np.zeros((B, 0), np.int32))
            leaf_class = grown["leaf_class"]
            del grown
        else:
            X, y, F = ri.load_or_grow(c, N=N if args.rows else None, B=B if args.trees else None)
            leaf_class = ri.leaf_classes(F, y, c.C)
        self.X, self.y, self.F = X, y, F
        log(f"workload cfg{c.cfg}: N={N} M={c.M} B={B} k={self.k} T={self.T}; inputs ready in {time.time() - t0:.1f}s "
            f"(nodes={F.total_nodes}, max leaves/tree={int(F.n_leaves.max())}"
            + (", forest grown on the GPU)" if large else ")"))
        t0 = time.perf_counter()
        self.gf = rfx.Forest(F.n_features, F.node_offset, F.feature, F.threshold, F.left, F.right, F.leaf_id, F.n_leaves)
        self.forest_create_ms = (time.perf_counter() - t0) * 1e3   # host validation + re-layout + upload, once per forest
        self.Lb = self.gf.leaf_bound
        P = int(np.ceil(np.log2(max(self.Lb, 2))))
        self.P = 8 if P < 8 else (P if P <= 16 else (P + 1) & ~1)   # plane count the library uses for this bound
        self.tests = N * N * B / 2.0
        self.dX = torch.from_numpy(X).to(dev)
        self.d_y = torch.from_numpy(y.astype(np.int32)).to(dev)
        self.d_leaf_class = torch.from_numpy(leaf_class).to(dev)
        self.d_inbag = torch.from_numpy(F.inbag.view(np.int16)).to(dev)
        self.dV0 = torch.from_numpy(ri.start_block(N, self.k)).to(dev)
        self.dx0 = torch.from_numpy(ri.start_block(N, self.m, seed=ri.mixture.START_SEED + 1)).to(dev)
        self.leaf = torch.empty((B, N), dtype=torch.int32, device=dev)
        self.lib = rfx.load()
        self.stream = torch.cuda.current_stream().cuda_stream
        self.phase_events = {}
        if large:
            # capacity of the sparse list: one counting call on the leaf ids of this forest
            rfx.leaf_assign(self.gf, self.dX, self.leaf)
            self.sp_cap = max(rfx.prox_sparse_count(self.leaf, self.Lb, 1), 1)
            self.sp_got = ctypes.c_int64(0)
            self.alloc_sparse(self.sp_cap)
        else:
            self.prox = torch.empty((N, N), dtype=torch.float32, device=dev)
            self.prox_oob = torch.empty((N * (N - 1) // 2,), dtype=torch.float32, device=dev)

    def alloc_sparse(self, cap):
        torch = self.torch
        self.sp_rows = torch.empty(cap, dtype=torch.int32, device=self.dev)
        self.sp_cols = torch.empty_like(self.sp_rows)
        self.sp_cnt = torch.empty(cap, dtype=torch.int16, device=self.dev)

    def free_sparse(self):
        del self.sp_rows, self.sp_cols, self.sp_cnt

    def timed(self, name, fn):
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = fn()
        e1.record()
        self.phase_events.setdefault(name, []).append((e0, e1))
        return out

    def phase_means(self, names=None):
        """Mean milliseconds per phase from the recorded event pairs (after a synchronize); removes what it reports."""
        names = list(self.phase_events) if names is None else names
        return {n: float(np.mean([a.elapsed_time(b) for a, b in self.phase_events.pop(n)])) for n in names}

    def sparse_pass(self, cap, got):
        rfx = self.rfx
        rfx._check(self.lib.rfx_prox_sparse(self.leaf.data_ptr(), self.N, self.B, self.Lb, 1, rfx.U16, cap,
                                            self.sp_rows.data_ptr(), self.sp_cols.data_ptr(), self.sp_cnt.data_ptr(),
                                            0, ctypes.byref(got), self.stream))

    def dense_and_oob_separately(self):
        rfx = self.rfx
        self.timed("prox_dense", lambda: rfx.prox_dense(self.leaf, self.Lb, rfx.U32, rfx.FULL, prox=self.prox,
                                                        want_counts=False))
        self.timed("prox_oob", lambda: rfx._check(self.lib.rfx_prox_oob(
            self.leaf.data_ptr(), self.d_inbag.data_ptr(), self.N, self.B, self.Lb, rfx.U32, rfx.UPPER_PACKED, 0, 0,
            self.prox_oob.data_ptr(), self.stream)))

    def step(self):
        """One pass of the whole path."""
        rfx = self.rfx
        self.timed("leaf_assign", lambda: rfx.leaf_assign(self.gf, self.dX, self.leaf))
        if self.large:
            self.timed("prox_sparse", lambda: self.sparse_pass(self.sp_cap, self.sp_got))
        elif self.fused:
            self.timed("prox_dense_oob", lambda: rfx._check(self.lib.rfx_prox_dense_oob(
                self.leaf.data_ptr(), self.d_inbag.data_ptr(), self.N, self.B, self.Lb, rfx.U32, rfx.FULL, 0,
                self.prox.data_ptr(), rfx.UPPER_PACKED, 0, 0, self.prox_oob.data_ptr(), self.stream)))
        else:
            self.dense_and_oob_separately()
        lam, V, Q, s = self.timed("prox_lowrank", lambda: rfx.prox_lowrank(self.leaf, self.Lb, self.dV0, self.T))
        res = self.timed("mds3d", lambda: rfx.mds3d(Q, s, self.dx0, rfx.MDS_SQUARED, max_iters=200, tol=1e-5))
        return lam, res


def calibration_copy(w):
    """A plain device-to-device copy of known size: calibrates the HBM byte counters of a --pmc run."""
    torch = w.torch
    n_cal = 1 << 30
    src = torch.empty(n_cal, dtype=torch.int32, device=w.dev).fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    log(f"calibration copy: {4 * n_cal} bytes read and {4 * n_cal} bytes written by one elementwise copy kernel")


def measure_sparse(w, kern):
    """The thresholded sparse form of the same counts (every non-zero pair); outside the step unless the workload is large."""
    rfx = w.rfx
    if w.large:
        assert w.sp_got.value == w.sp_cap, "the sparse pass found a different number of pairs than the counting call"
        nnz, sp_ms = w.sp_cap, kern["prox_tile_kernel_sparse"]["avg_ms"]
    else:
        nnz = rfx.prox_sparse_count(w.leaf, w.Lb, 1)
        w.alloc_sparse(max(nnz, 1))
        got = ctypes.c_int64(0)
        rfx.timing_enable(True)          # also clears the kernel timers
        for _ in range(2):
            w.sparse_pass(max(nnz, 1), got)
        sp_ms, sp_n = rfx.timing_get("prox_tile_kernel_sparse")
        sp_ms /= max(sp_n, 1)
    w.free_sparse()
    N, tests = w.N, w.tests
    return {"note": ("part of the step" if w.large else "not part of the step")
                    + ": strict-upper (i, j, count) triplets of every non-zero pair",
            "min_count": 1, "pairs": nnz, "fraction_of_triangle": nnz / max(N * (N - 1) / 2.0, 1.0),
            "bytes_out": 10 * nnz, "avg_launch_ms": sp_ms,
            "tests_per_s": tests / (sp_ms * 1e-3) if sp_ms > 0 else 0.0,
            "frac_of_alu_peak": (tests * (w.P + 1) / 32.0 / (sp_ms * 1e-3)) / PEAK_VALU_LANE_OPS if sp_ms > 0 else 0.0}


def measure_consumers(w):
    """Consumers of the proximity rows (outlier scores, out-of-bag vote), outside the step."""
    rfx, N, B = w.rfx, w.N, w.B
    rfx.timing_enable(True)
    for _ in range(2):
        rfx.prox_outlier(w.leaf, w.Lb, w.d_y)
        _, _, oob_wrong, oob_voted = rfx.oob_vote(w.leaf, w.d_inbag, w.d_leaf_class, w.c.C, w.d_y, want_votes=False)
    ol_ms, ol_n = rfx.timing_get("prox_tile_kernel_outlier")
    ov_ms, ov_n = rfx.timing_get("oob_vote_kernel")
    rfx.timing_enable(False)
    ov_avg = ov_ms / max(ov_n, 1)
    return {"note": "not part of the step",
            "outlier_avg_launch_ms": ol_ms / max(ol_n, 1), "oob_vote_avg_launch_ms": ov_avg,
            "oob_vote_GBps": (6.0 * N * B + 8.0 * N) / (ov_avg * 1e-3) / 1e9 if ov_avg > 0 else 0.0,
            "oob_error": oob_wrong / max(oob_voted, 1)}


def measure_plan_build(w):
    """Once-per-forest grouping of samples by leaf for the implicit product (inside every prox_lowrank call of the step)."""
    torch = w.torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan = w.rfx.PvPlan(w.leaf, w.Lb)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3
    plan.close()
    return ms


def measure_growth(w):
    """Growth of the same forest shape on the GPU, outside the step."""
    rfx, c = w.rfx, w.c
    w.torch.cuda.synchronize()
    rfx.forest_grow(w.dX, w.d_y, c.C, min(w.B, 8), c.mtry, 1)                      # warm-up
    trees = w.B if not w.large else min(w.B, 128)
    t0 = time.perf_counter()
    grown = rfx.forest_grow(w.dX, w.d_y, c.C, trees, c.mtry, w.ri.mixture.FOREST_ISEED)
    grow_s = time.perf_counter() - t0
    return {"note": "not part of the step", "trees": trees, "seconds": grow_s, "trees_per_s": trees / grow_s,
            "nodes": int(grown["node_offset"][-1]), "level_passes": grown["levels"], "sorted_pairs": grown["sorted_pairs"],
            "pairs_per_s": grown["sorted_pairs"] / grow_s}


def roofline_of_tile_kernel(w, kern, valu_rate):
    """Dominant kernel: bit-plane compare-and-count.  One launch covers the tile pairs on and below the diagonal of the
    (padded) N x N grid; per 32 trees and pair, P + 1 vector ops for the plain count, P + 7 for the fused pass that also
    yields the out-of-bag numerator and denominator."""
    tests, P = w.tests, w.P
    dom = "prox_tile_kernel_sparse" if w.large else ("prox_tile_kernel_both" if w.fused else "prox_tile_kernel")
    ops_per_test = (P + 7) / 32.0 if w.fused else (P + 1) / 32.0
    tile_ms = kern[dom]["avg_ms"]
    achieved = tests * ops_per_test / (tile_ms * 1e-3) if tile_ms > 0 else 0.0
    # HBM-side bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 KiB,
    # calibrated on a 4 GiB copy); measured for workload 4 only
    traffic = None
    if w.c.cfg == 4 and not w.reduced:
        fetch_kib, write_kib = (FUSED_FETCH_KIB, FUSED_WRITE_KIB) if w.fused else (PLAIN_FETCH_KIB, PLAIN_WRITE_KIB)
        traffic = (fetch_kib * 2.0 + write_kib) * 1024.0
    plain_ms = kern["prox_tile_kernel"]["avg_ms"]
    return {"kernel": dom, "bound": "alu", "achieved": achieved / 1e12, "peak": PEAK_VALU_LANE_OPS / 1e12,
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


def pv_figures(w, kern, copy_rate, plan_ms):
    """Implicit product: algorithmic bytes per application = B*N*(2*4k + 4) + 2*4*N*k.  One application (`pv_apply`: a
    bracket on the caller's stream around the whole call) runs in groups of trees, the gather of a group on a second
    stream next to the leaf sums of the following one, so the two kernel figures overlap and add up to more."""
    N, B, k = w.N, w.B, w.k
    w_pv = B * N * (2 * 4 * k + 4) + 2 * 4 * N * k
    applications = kern["pv_apply"]["launches"]
    if applications:
        pv_ms = kern["pv_apply"]["avg_ms"]
    else:                                         # one group of trees: the two kernel brackets are the application
        applications = max(kern["pv_gather_kernel"]["launches"], 1)
        pv_ms = (kern["pv_leaf_sum_kernel"]["total_ms"] + kern["pv_gather_kernel"]["total_ms"]) / applications
    rate = w_pv / (pv_ms * 1e-3) if pv_ms > 0 else 0.0
    return {"bytes_per_application": w_pv, "avg_ms": pv_ms, "GBps": rate / 1e9, "frac_of_hbm_peak": rate / PEAK_HBM_BYTES,
            "leaf_sum_ms": kern["pv_leaf_sum_kernel"]["total_ms"] / applications,
            "gather_ms": kern["pv_gather_kernel"]["total_ms"] / applications,
            "tree_groups": kern["pv_gather_kernel"]["launches"] // applications,
            "compulsory_floor_bytes": 4 * N * B + 8 * N * k,
            # rocprofv3 FETCH_SIZE x 2 + WRITE_SIZE of the three kernels of one application (workload 4 only)
            "measured_fabric_bytes": (sum(PV_FETCH_KIB) * 2.0 + sum(PV_WRITE_KIB)) * 1024.0
            if (w.c.cfg == 4 and not w.reduced) else None,
            "measured_copy_bytes_per_s": copy_rate, "frac_of_measured_copy": rate / copy_rate if copy_rate > 0 else 0.0,
            "valu_bound_ms": 2.0 * B * N * k / PEAK_VALU_LANE_OPS * 1e3, "plan_build_ms": plan_ms,
            "note": "above 100 % of the HBM peak = cache-assisted: V and the per-tree sums are served by L2 / Infinity Cache"}


def leaf_assign_figures(w, kern):
    """Leaf assignment: one 8-byte node record and one 4-byte feature value per visited internal node, plus the leaf-id
    write and X read once."""
    torch, F, N, B = w.torch, w.F, w.N, w.B
    depth_tab = np.zeros((B, w.Lb), np.int32)
    for b in range(B):
        s, e = int(F.node_offset[b]), int(F.node_offset[b + 1])
        lid = F.leaf_id[s:e]
        depth_tab[b, lid[lid >= 0]] = F.depth[s:e][lid >= 0]
    d_depth = torch.from_numpy(depth_tab).to(w.dev)
    path_total = int(sum(int(d_depth[b0:b0 + 50].gather(1, w.leaf[b0:b0 + 50].long()).sum()) for b0 in range(0, B, 50)))
    w_la = path_total * (8 + 4) + 4 * N * B + 4 * N * w.c.M
    la_ms = kern["leaf_assign_kernel"]["avg_ms"]
    rate = w_la / (la_ms * 1e-3) if la_ms > 0 else 0.0
    return {"bytes_model": w_la, "mean_path": path_total / (N * B), "avg_ms": la_ms, "GBps": rate / 1e9,
            "frac_of_hbm_peak": rate / PEAK_HBM_BYTES,
            "compulsory_floor_bytes": 4 * N * w.c.M + 8 * int(F.total_nodes) + 4 * N * B,
            "measured_fabric_bytes": (LEAF_FETCH_KIB * 2.0 + LEAF_WRITE_KIB) * 1024.0
            if (w.c.cfg == 4 and not w.reduced) else None,
            "forest_create_ms": w.forest_create_ms,
            "note": "gather-latency bound; nodes and X are cache / LDS resident, so the byte model is not HBM traffic"}


def main():
    args = parse_args()
    import torch
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    rfx.load()          # fails loudly if librfx.so is missing: there is no fallback path
    w = Workload(args, torch, rfx, ri)
    if args.calibrate_copy:
        calibration_copy(w)

    for _ in range(args.warmup):
        w.step()
    torch.cuda.synchronize()
    w.phase_events.clear()
    rfx.timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        lam, (coords, ev, mds_iters) = w.step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    phases = w.phase_means()
    if w.fused:
        # the two passes the fused one replaces, outside the step, for their own kernel times
        for _ in range(2):
            w.dense_and_oob_separately()
        torch.cuda.synchronize()
        sep = w.phase_means(["prox_dense", "prox_oob"])
        phases["separate_prox_dense"], phases["separate_prox_oob"] = sep["prox_dense"], sep["prox_oob"]
    kern = {}
    for name in ("leaf_assign_kernel", "prox_tile_kernel_both", "prox_tile_kernel", "prox_tile_kernel_oob",
                 "prox_tile_kernel_sparse", "pv_apply", "pv_leaf_sum_kernel", "pv_gather_kernel"):
        ms, n = rfx.timing_get(name)
        kern[name] = {"avg_ms": ms / max(n, 1), "launches": n, "total_ms": ms}

    sparse = measure_sparse(w, kern)
    consumers = measure_consumers(w)
    plan_ms = measure_plan_build(w)
    growth = measure_growth(w)
    # practical ceilings of this GPU next to the published peaks
    valu_rate = rfx.probe_valu(4096)
    copy_rate = rfx.probe_copy(1 << 32)

    c, N, B, tests = w.c, w.N, w.B, w.tests
    dense_phase = "prox_sparse" if w.large else ("prox_dense_oob" if w.fused else "prox_dense")
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
        "config": {"workload": f"cfg{c.cfg}: N={N} M={c.M} B={B} trees to purity, mtry={c.mtry}, k={w.k}, T={w.T}"
                               + (" (REDUCED, debugging)" if w.reduced else "")
                               + (" (dense outputs do not fit: exact sparse list instead; forest grown by rfx_forest_grow)"
                                  if w.large else ""),
                   "leaf_bound": w.Lb, "bit_planes": w.P, "mds_block": w.m, "mds_iters": mds_iters},
        "phases_ms": phases,
        "mds": {"iterations": mds_iters, "ms_per_iteration": phases["mds3d"] / max(mds_iters, 1),
                "factor_GBps": N * w.k * mds_iters / (phases["mds3d"] * 1e-3) / 1e9},
        "dense_tests_per_s": tests / (phases[dense_phase] * 1e-3),
        "pv": pv_figures(w, kern, copy_rate, plan_ms),
        "leaf_assign": leaf_assign_figures(w, kern),
        "kernels": kern,
        "roofline": roofline_of_tile_kernel(w, kern, valu_rate),
        "consumers": consumers,
        "growth": growth,
        "sparse": sparse,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w.leaf, N, B, w.X, w.F, w.k, w.y, c)
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
