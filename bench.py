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
PEAK_HBM_BYTES = 8.0e12
ROOT = os.path.dirname(os.path.abspath(__file__))
MDS_TOL = 1e-5


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--cfg", type=int, default=4, help="workload 1..5 (default: N=100,000, B=1,000)")
    ap.add_argument("--trees", type=int, default=0, help="override the tree count (debugging only)")
    ap.add_argument("--rows", type=int, default=0, help="override the row count (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mds-block", type=int, default=16)
    ap.add_argument("--profile", action="store_true",
                    help="a run under rocprofv3: leaves out the one measurement that launches the step's kernels on a reduced input "
                         "(the phases of the implicit product one after the other), so that the per-dispatch averages of the profile "
                         "hold launches of the full workload only")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one 4 GiB device copy before the steps (reference for rocprofv3 --pmc byte counters)")
    ap.add_argument("--summarise-kernel-trace", metavar="CSV",
                    help="print the per-kernel table of a rocprofv3 --kernel-trace csv (kernel_trace.csv) and exit")
    ap.add_argument("--summarise-pmc", nargs="+", metavar="CSV",
                    help="print the per-kernel averages of rocprofv3 --pmc counter_collection.csv files and exit")
    args = ap.parse_args()
    if args.summarise_kernel_trace or args.summarise_pmc:
        return args
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
        self.profile_run = bool(getattr(args, "profile", False))
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
        self.leaf = torch.empty((B, N), dtype=torch.int32, device=dev)
        self.lib = rfx.load()
        self.stream = torch.cuda.current_stream().cuda_stream
        self.phase_events = {}
        # Everything the step needs is allocated here, once: the step itself calls the asynchronous forms of the
        # boundary with these workspaces and allocates nothing.
        k, m = self.k, self.m
        rfx.leaf_assign(self.gf, self.dX, self.leaf)
        self.ws_prox = rfx.new_workspace(rfx.prox_workspace_bytes(N, B, self.Lb))
        self.ws_lr = rfx.new_workspace(rfx.lowrank_workspace_bytes(N, k))
        self.ws_mds = rfx.new_workspace(rfx.mds3d_workspace_bytes(N, k, m, rfx.MDS_SQUARED))
        self.plan = rfx.PvPlan(self.leaf, self.Lb)          # regrouped inside every step (rfx_pv_plan_rebuild)
        rfx.pv_plan_reserve(self.plan, k)
        self.lam = torch.empty(k, dtype=torch.float32, device=dev)
        self.V = torch.empty((N, k), dtype=torch.float32, device=dev)
        self.Q = torch.empty((N, k), dtype=torch.int8, device=dev)
        self.scales = torch.empty(k, dtype=torch.float32, device=dev)
        self.status = torch.zeros(1, dtype=torch.int32, device=dev)
        self.coords = torch.empty((N, 3), dtype=torch.float32, device=dev)
        self.ev = torch.empty(3, dtype=torch.float32, device=dev)
        self.mds_rel = torch.zeros(1, dtype=torch.float32, device=dev)
        self.mds_iters = 0           # fixed by the first warm-up step: the count the tolerance-driven call needs
        if large:
            # capacity of the sparse list: one counting call on the leaf ids of this forest
            self.sp_cap = max(rfx.prox_sparse_count(self.leaf, self.Lb, 1), 1)
            self.sp_nnz = torch.zeros(1, dtype=torch.int64, device=dev)
            # the row pass works from the grouping the factorisation needs anyway (4 B N bytes of scratch of its own)
            self.ws_sparse = rfx.new_workspace(rfx.prox_sparse_plan_workspace_bytes(self.plan)) if B <= 4096 else None
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

    def phase_stats(self, names=None):
        """Per phase, from the recorded event pairs (after a synchronize): mean, median, min in milliseconds and the
        number of samples; removes what it reports."""
        names = list(self.phase_events) if names is None else names
        out = {}
        for n in names:
            t = np.array([a.elapsed_time(b) for a, b in self.phase_events.pop(n)], np.float64)
            out[n] = {"mean": float(t.mean()), "median": float(np.median(t)), "min": float(t.min()), "n": int(t.size)}
        return out

    def sparse_pass(self):
        """Every non-zero pair as (i, j, count).  Large workloads count row by row from the samples grouped by leaf, out of
        the grouping this step has just built for the implicit product (asynchronous, nothing allocated; beyond 4,096
        trees the synchronous call, which picks the cheaper of the two algorithms and builds a grouping of its own); the
        others time the asynchronous tile pass."""
        rfx = self.rfx
        if self.large and self.ws_sparse is not None:
            rfx.prox_sparse_plan(self.plan, self.ws_sparse, self.sp_nnz, self.sp_rows, self.sp_cols, self.sp_cnt, min_count=1,
                                 count_dtype=rfx.U16)
        elif self.large:
            got = ctypes.c_int64(0)
            rfx._check(self.lib.rfx_prox_sparse(self.leaf.data_ptr(), self.N, self.B, self.Lb, 1, rfx.U16, self.sp_cap,
                                                self.sp_rows.data_ptr(), self.sp_cols.data_ptr(), self.sp_cnt.data_ptr(), 0,
                                                ctypes.byref(got), self.stream))
            self.sp_nnz[0] = got.value
        else:
            rfx.prox_sparse_ws(self.leaf, self.Lb, self.ws_prox, self.sp_nnz, self.sp_rows, self.sp_cols, self.sp_cnt,
                               min_count=1, count_dtype=rfx.U16)

    def dense_and_oob_separately(self):
        rfx = self.rfx
        self.timed("prox_dense", lambda: rfx.prox_dense_ws(self.leaf, self.Lb, self.ws_prox, rfx.U32, rfx.FULL, prox=self.prox))
        self.timed("prox_oob", lambda: rfx.prox_oob_ws(self.leaf, self.d_inbag, self.Lb, self.ws_prox, rfx.U32,
                                                       rfx.UPPER_PACKED, prox=self.prox_oob))

    def step(self):
        """One pass of the whole path, enqueued on one stream: traversal, the dense pass (fused plain + out-of-bag), the
        grouping of the samples by leaf for the implicit product (it depends on this step's leaf ids; the only call that
        waits for the device: it reads the number of big leaves back), the factorisation with INT8 factors, the scaling.
        Where the dense outputs do not fit, the exact sparse list takes the place of the dense pass and is counted out of
        that grouping, which therefore comes first."""
        rfx = self.rfx
        self.timed("leaf_assign", lambda: rfx.leaf_assign(self.gf, self.dX, self.leaf))
        if self.large:
            # the sparse list is counted out of the grouping, so the grouping comes first here
            self.timed("pv_plan", lambda: rfx.pv_plan_rebuild(self.plan, self.leaf))
            self.timed("prox_sparse", self.sparse_pass)
        elif self.fused:
            self.timed("prox_dense_oob", lambda: rfx.prox_dense_oob_ws(
                self.leaf, self.d_inbag, self.Lb, self.ws_prox, rfx.U32, rfx.FULL, rfx.UPPER_PACKED, prox=self.prox,
                prox_oob=self.prox_oob))
        else:
            self.dense_and_oob_separately()
        if not self.large:
            self.timed("pv_plan", lambda: rfx.pv_plan_rebuild(self.plan, self.leaf))
        self.timed("prox_lowrank", lambda: rfx.prox_lowrank_plan(self.plan, self.dV0, self.T, self.ws_lr, self.lam, self.V,
                                                                 self.Q, self.scales, self.status))
        if self.mds_iters == 0:
            # first warm-up step: the tolerance-driven call fixes the number of applications for the timed steps
            _, _, self.mds_iters = rfx.mds3d(self.Q, self.scales, None, rfx.MDS_SQUARED, max_iters=200, tol=MDS_TOL, m=self.m)
        # no start block: the library begins from the leading columns of the factor
        self.timed("mds3d", lambda: rfx.mds3d_ws(self.Q, self.scales, None, self.mds_iters, self.ws_mds, self.coords,
                                                 self.ev, self.mds_rel, m=self.m))


def calibration_copy(w):
    """A plain device-to-device copy of known size by the library's copy kernel (copy_probe_kernel: 4 GiB read and 4 GiB
    written per dispatch): the row the HBM byte counters of a --pmc run are scaled by."""
    rate = w.rfx.probe_copy(1 << 32)
    log(f"calibration copy: 4 GiB read and 4 GiB written per dispatch of copy_probe_kernel ({rate / 1e12:.2f} TB/s)")


def measure_sparse(w, kern):
    """The thresholded sparse form of the same counts (every non-zero pair); outside the step unless the workload is large."""
    rfx, torch = w.rfx, w.torch
    if w.large:
        assert int(w.sp_nnz[0]) == w.sp_cap, "the sparse pass found a different number of pairs than the counting call"
        by_rows = kern["sparse_rows_kernel"]["launches"] > 0
        nnz, sp_ms = w.sp_cap, kern["sparse_rows_kernel" if by_rows else "prox_tile_kernel_sparse"]["avg_ms"]
    else:
        nnz = rfx.prox_sparse_count(w.leaf, w.Lb, 1)
        w.alloc_sparse(max(nnz, 1))
        w.sp_nnz = torch.zeros(1, dtype=torch.int64, device=w.dev)
        rfx.timing_enable(True)          # also clears the kernel timers
        for _ in range(2):
            w.sparse_pass()
        sp_ms, sp_n = rfx.timing_get("prox_tile_kernel_sparse")
        sp_ms /= max(sp_n, 1)
        assert int(w.sp_nnz[0]) == nnz
        by_rows = False
    w.free_sparse()
    N, tests = w.N, w.tests
    return {"note": ("part of the step" if w.large else "not part of the step")
                    + ": strict-upper (i, j, count) triplets of every non-zero pair",
            "algorithm": "row by row from the samples grouped by leaf (sparse_rows_kernel)" if by_rows
                         else "pair tests on bit planes (prox_tile_kernel_sparse)",
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


def measure_one_shot(w):
    """What the synchronous conveniences cost on top of the step's asynchronous calls (outside the step): a plan built
    from nothing (allocation included) and rfx_prox_lowrank, which builds and destroys its own plan and scratch."""
    torch, rfx = w.torch, w.rfx
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan = rfx.PvPlan(w.leaf, w.Lb)
    torch.cuda.synchronize()
    plan_ms = (time.perf_counter() - t0) * 1e3
    plan.close()
    t0 = time.perf_counter()
    rfx.prox_lowrank(w.leaf, w.Lb, w.dV0, w.T)
    torch.cuda.synchronize()
    return {"pv_plan_create_ms": plan_ms, "prox_lowrank_one_shot_ms": (time.perf_counter() - t0) * 1e3}


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


# ------------------------------------------------------------------------------------------------------------------
# rocprofv3 summaries.  The byte counters quoted in the line are read from the committed summary of a --pmc run of this
# file on the same workload (profiles/bench_cfg<c>_pmc_fetch_write.txt, written by --summarise-pmc below), never typed in.

def _short_kernel_name(name):
    import re
    name = name.replace("(anonymous namespace)::", "").replace("void ", "").strip().strip('"')
    name = re.sub(r"\(.*", "", name)
    return re.sub(r"\s+", "", name)


def summarise_kernel_trace(path):
    """Per-kernel table (calls, total, average, min, max in ms, share) of a rocprofv3 kernel_trace.csv."""
    import collections
    import csv
    agg = collections.OrderedDict()
    with open(path) as f:
        for r in csv.DictReader(f):
            d = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) * 1e-6
            agg.setdefault(_short_kernel_name(r["Kernel_Name"]), []).append(d)
    total = sum(sum(v) for v in agg.values())
    print(f"{'kernel':64s} {'calls':>6s} {'total_ms':>10s} {'avg_ms':>9s} {'min_ms':>9s} {'max_ms':>9s} {'%':>6s}")
    for n, v in sorted(agg.items(), key=lambda kv: -sum(kv[1])):
        print(f"{n[:64]:64s} {len(v):6d} {sum(v):10.3f} {sum(v) / len(v):9.4f} {min(v):9.4f} {max(v):9.4f} {100 * sum(v) / total:6.2f}")


def summarise_pmc(paths):
    """Per-kernel averages per dispatch of every counter found in rocprofv3 counter_collection.csv files (one run each)."""
    import collections
    import csv
    agg = collections.OrderedDict()
    counters = []
    for path in paths:
        with open(path) as f:
            for r in csv.DictReader(f):
                c = r["Counter_Name"]
                if c not in counters:
                    counters.append(c)
                a = agg.setdefault(_short_kernel_name(r["Kernel_Name"]), {}).setdefault(c, [0, 0.0])
                a[0] += 1
                a[1] += float(r["Counter_Value"])
    print("kernel".ljust(64) + " " + " ".join(f"{'disp':>6s} {c[:18]:>18s}" for c in counters))
    for n, cs in sorted(agg.items(), key=lambda kv: -max(v[1] for v in kv[1].values())):
        cells = []
        for c in counters:
            a = cs.get(c)
            cells.append(f"{a[0]:6d} {a[1] / a[0]:18.1f}" if a else f"{'-':>6s} {'-':>18s}")
        print(f"{n[:64]:64s} " + " ".join(cells))


def load_pmc_profile(cfg):
    """{kernel: {counter: (dispatches, average per dispatch)}} from the committed summary of this workload, the file's name and a
    hash of its contents; (None, None, None) when there is no summary."""
    import hashlib
    path = os.path.join(ROOT, "profiles", f"bench_cfg{cfg}_pmc_fetch_write.txt")
    if not os.path.exists(path):
        return None, None, None
    text = open(path).read()
    table, counters = {}, None
    for line in text.splitlines():
        if line.startswith("#") or not line.strip():
            continue
        parts = line.split()
        if parts[0] == "kernel":
            counters = [p for p in parts[1:] if p != "disp"]
            continue
        if counters is None or len(parts) != 1 + 2 * len(counters):
            continue
        row = {}
        for i, c in enumerate(counters):
            if parts[2 + 2 * i] != "-":
                row[c] = (int(parts[1 + 2 * i]), float(parts[2 + 2 * i]))     # dispatches, average per dispatch
        table[parts[0]] = row
    return table, os.path.relpath(path, ROOT), hashlib.sha256(text.encode()).hexdigest()[:16]


def fabric_bytes(profile, kernels, optional=()):
    """HBM-side bytes per launch of the named kernels from the profile: FETCH_SIZE and WRITE_SIZE (KiB per dispatch),
    each scaled by what the same counter reads for the library's plain copy kernel of known size (copy_probe_kernel:
    4 GiB read, 4 GiB written per dispatch).  None if a kernel or the calibration row is missing; the `optional` kernels
    (those a workload may or may not launch) are added where the profile has them."""
    if not profile or "copy_probe_kernel" not in profile:
        return None

    def average(prefix, counter):
        """Average per dispatch over all rows whose kernel name starts with prefix (template variants of one kernel)."""
        n = tot = 0
        for name, row in profile.items():
            if name.startswith(prefix) and counter in row:
                n += row[counter][0]
                tot += row[counter][0] * row[counter][1]
        return tot / n if n else None

    known_kib = float(1 << 32) / 1024.0
    cal_f, cal_w = average("copy_probe_kernel", "FETCH_SIZE"), average("copy_probe_kernel", "WRITE_SIZE")
    if not cal_f or not cal_w:
        return None
    total = 0.0
    for kname in kernels:
        f, wr = average(kname, "FETCH_SIZE"), average(kname, "WRITE_SIZE")
        if f is None or wr is None:
            return None
        total += (f * known_kib / cal_f + wr * known_kib / cal_w) * 1024.0
    for kname in optional:
        f, wr = average(kname, "FETCH_SIZE"), average(kname, "WRITE_SIZE")
        if f is not None and wr is not None:
            total += (f * known_kib / cal_f + wr * known_kib / cal_w) * 1024.0
    return total


def roofline_of_tile_kernel(w, kern, valu_rate, profile, profile_src):
    """Dominant kernel: bit-plane compare-and-count.  One launch covers the tile pairs on and below the diagonal of the
    (padded) N x N grid; per 32 trees and pair, P + 1 vector ops for the plain count, P + 7 for the fused pass that also
    yields the out-of-bag numerator and denominator."""
    tests, P = w.tests, w.P
    if w.large and kern["sparse_rows_kernel"]["launches"] > 0:
        # the row pass: its work is counter increments (LDS atomics), one per co-member pair and tree
        ms = kern["sparse_rows_kernel"]["avg_ms"]
        sizes_sq = 0
        for b0 in range(0, w.B, 50):
            for b in range(b0, min(b0 + 50, w.B)):
                cnt = w.torch.bincount(w.leaf[b].long(), minlength=w.Lb).double()
                sizes_sq += float((cnt * (cnt - 1) / 2).sum())
        peak = 256 * 32 * 2.4e9          # LDS atomic lanes per second: 256 CUs x 32 banks x 2.4 GHz
        return {"kernel": "sparse_rows_kernel", "bound": "lds", "achieved": sizes_sq / (ms * 1e-3) / 1e12, "peak": peak / 1e12,
                "unit": "T counter increments/s", "frac": sizes_sq / (ms * 1e-3) / peak, "traffic": None,
                "increments": sizes_sq, "avg_launch_ms": ms, "tests_per_s": tests / (ms * 1e-3),
                "note": "sum over trees and leaves of s (s - 1) / 2 increments instead of N^2 B / 2 pair tests; the pass is bound by "
                        "the instructions that fetch and place a leaf's members (cursor and address arithmetic per tree visit, one LDS atomic per member), "
                        "not by the rate of the LDS atomics, so the fraction against that rate is small by construction; "
                        "tests_per_s is the pair-test rate the same result would need"}
    mode = 2 if w.large else (4 if w.fused else 0)
    dom = "prox_tile_kernel_sparse" if w.large else ("prox_tile_kernel_both" if w.fused else "prox_tile_kernel")
    ops_per_test = (P + 7) / 32.0 if w.fused else (P + 1) / 32.0
    tile_ms = kern[dom]["avg_ms"]
    achieved = tests * ops_per_test / (tile_ms * 1e-3) if tile_ms > 0 else 0.0
    traffic = None if w.reduced else fabric_bytes(profile, [f"prox_tile_kernel<{P},16,{mode}>"])
    plain_ms = kern["prox_tile_kernel"]["avg_ms"]
    return {"kernel": dom, "bound": "alu", "achieved": achieved / 1e12, "peak": PEAK_VALU_LANE_OPS / 1e12,
            "unit": "T lane-ops/s", "frac": achieved / PEAK_VALU_LANE_OPS, "traffic": traffic,
            "traffic_source": (f"{profile_src[0]} (sha256 {profile_src[1]}): FETCH_SIZE and WRITE_SIZE per dispatch, each scaled by "
                               "the copy_probe_kernel row of the same file; L2-to-fabric bytes") if traffic is not None else None,
            "algorithmic_bytes": (4.0 * w.N * w.N + 2.0 * w.N * (w.N - 1) if w.fused else 4.0 * w.N * w.N) if not w.large else None,
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


def pv_phases_alone(w, ceil_v, ceil_s):
    """The two phases of the implicit product with nothing running next to them: a plan on the first trees only, few
    enough (B N below 10^7) that the library keeps them in one group, so the leaf sums and the gather run one after the
    other on one stream.  Same kernels, same leaf sizes per tree, same ceilings.  None where the whole forest is that small
    anyway (then the main figures are already of this kind)."""
    rfx, torch = w.rfx, w.torch
    N, B, k = w.N, w.B, w.k
    nb = int(min(B, 9_900_000 // N))
    if nb < 8 or nb >= B:
        return None
    plan = rfx.PvPlan(w.leaf[:nb].contiguous(), w.Lb)
    rfx.pv_plan_reserve(plan, k)
    Y = torch.empty_like(w.dV0)
    for _ in range(3):
        plan.apply(w.dV0, Y)
    torch.cuda.synchronize()
    rfx.timing_enable(True)          # also clears the kernel timers (the step's have been read by now)
    reps = 20
    for _ in range(reps):
        plan.apply(w.dV0, Y)
    torch.cuda.synchronize()
    sum_ms, n_sum = rfx.timing_get("pv_leaf_sum_kernel")
    gat_ms, n_gat = rfx.timing_get("pv_gather_kernel")
    plan.close()
    assert n_sum == reps and n_gat == reps, "the reduced plan ran in more than one group"
    rows_bytes = 4.0 * k * nb * N
    sum_rate, gat_rate = rows_bytes / (sum_ms / reps * 1e-3), rows_bytes / (gat_ms / reps * 1e-3)
    return {"trees": nb, "leaf_sum_ms_per_tree": sum_ms / reps / nb, "gather_ms_per_tree": gat_ms / reps / nb,
            "leaf_sums": {"achieved": sum_rate / 1e9, "ceiling": ceil_v / 1e9, "frac": sum_rate / ceil_v},
            "gather": {"achieved": gat_rate / 1e9, "ceiling": ceil_s / 1e9, "frac": gat_rate / ceil_s},
            "both": {"achieved": 2.0 * rows_bytes / ((sum_ms + gat_ms) / reps * 1e-3) / 1e9,
                     "ceiling": 2.0 / (1.0 / ceil_v + 1.0 / ceil_s) / 1e9,
                     "frac": 2.0 * rows_bytes / ((sum_ms + gat_ms) / reps * 1e-3) / (2.0 / (1.0 / ceil_v + 1.0 / ceil_s))}}


def pv_figures(w, kern, copy_rate, profile):
    """Implicit product: algorithmic bytes per application = B*N*(2*4k + 4) + 2*4*N*k.  One application (`pv_apply`: a
    bracket on the caller's stream around the whole call) runs in groups of trees, the gather of a group on a second
    stream next to the leaf sums of the following one, so the two kernel figures overlap and add up to more.

    The row reads of both phases come from the caches, not from HBM, so the ceiling they are held against is measured:
    rfx_probe_gather reads rows of k floats at random indices, eight loads in flight per wave, from a table the size of V
    (the leaf sums gather V rows) and from a table the size of one tree's leaf sums (the gather phase sweeps the trees
    in order, so that is what is live in L2)."""
    rfx = w.rfx
    N, B, k = w.N, w.B, w.k
    w_pv = B * N * (2 * 4 * k + 4) + 2 * 4 * N * k
    applications = kern["pv_apply"]["launches"]
    if applications:
        pv_ms = kern["pv_apply"]["avg_ms"]
    else:                                         # one group of trees: the two kernel brackets are the application
        applications = max(kern["pv_gather_kernel"]["launches"], 1)
        pv_ms = (kern["pv_leaf_sum_kernel"]["total_ms"] + kern["pv_gather_kernel"]["total_ms"]) / applications
    rate = w_pv / (pv_ms * 1e-3) if pv_ms > 0 else 0.0
    sum_ms = kern["pv_leaf_sum_kernel"]["total_ms"] / applications
    gat_ms = kern["pv_gather_kernel"]["total_ms"] / applications
    kp = 16 if k <= 16 else (32 if k <= 32 else 64 * ((k + 63) // 64))     # row width the probe supports
    leaves_per_tree = max(64, int(np.mean(w.F.n_leaves)))
    gathers = int(min(B * N, 1 << 27))
    ceil_v = rfx.probe_gather(max(N, 64), kp, gathers)                 # rows of V: table of N rows
    ceil_s = rfx.probe_gather(leaves_per_tree, kp, gathers)            # rows of one tree's leaf sums
    rows_bytes = 4.0 * k * B * N                                       # row bytes either phase reads
    sum_rate = rows_bytes / (sum_ms * 1e-3) if sum_ms > 0 else 0.0
    gat_rate = rows_bytes / (gat_ms * 1e-3) if gat_ms > 0 else 0.0
    ceil_both = 2.0 / (1.0 / ceil_v + 1.0 / ceil_s)                    # both phases one after the other, each at its ceiling
    both_rate = 2.0 * rows_bytes / ((sum_ms + gat_ms) * 1e-3) if sum_ms + gat_ms > 0 else 0.0
    alone = None if w.profile_run else pv_phases_alone(w, ceil_v, ceil_s)
    fabric = None if w.reduced else fabric_bytes(profile, ["pv_leaf_sum_kernel<", "pv_gather_kernel<"],
                                                  optional=["pv_leaf_sum_big_kernel<", "pv_leaf_sum_split_kernel<", "pv_combine_kernel"])
    if fabric is not None:
        # the profile's rows are per dispatch, one dispatch per group of trees
        fabric *= max(kern["pv_gather_kernel"]["launches"] // applications, 1)
    return {"bytes_per_application": w_pv, "avg_ms": pv_ms, "GBps": rate / 1e9, "frac_of_hbm_peak": rate / PEAK_HBM_BYTES,
            "leaf_sum_ms": sum_ms, "gather_ms": gat_ms,
            "tree_groups": kern["pv_gather_kernel"]["launches"] // applications,
            "compulsory_floor_bytes": 4 * N * B + 8 * N * k,
            "roofline": {"bound": "cache gather", "unit": "GB/s of row reads",
                         "achieved": both_rate / 1e9, "ceiling": ceil_both / 1e9, "frac": both_rate / ceil_both,
                         "leaf_sums": {"achieved": sum_rate / 1e9, "ceiling": ceil_v / 1e9, "frac": sum_rate / ceil_v,
                                       "ceiling_is": f"rfx_probe_gather on a table of {max(N, 64)} rows x {kp} floats (the size of V)"},
                         "gather": {"achieved": gat_rate / 1e9, "ceiling": ceil_s / 1e9, "frac": gat_rate / ceil_s,
                                    "ceiling_is": f"rfx_probe_gather on a table of {leaves_per_tree} rows x {kp} floats (one tree's leaf sums)"},
                         "note": "kernel times of the two phases added up (in the step they overlap on two streams: avg_ms), "
                                 "so each is slowed by the other; phases_alone has them one after the other",
                         "phases_alone": alone},
            "measured_fabric_bytes": fabric,
            "measured_fabric_frac_of_hbm_peak": fabric / (pv_ms * 1e-3) / PEAK_HBM_BYTES if fabric and pv_ms > 0 else None,
            "measured_copy_bytes_per_s": copy_rate, "frac_of_measured_copy": rate / copy_rate if copy_rate > 0 else 0.0,
            "valu_bound_ms": 2.0 * B * N * k / PEAK_VALU_LANE_OPS * 1e3,
            "note": "GBps is the byte model over the time; above 100 % of the HBM peak = cache-assisted: V and the per-tree sums are "
                    "served by L2 / Infinity Cache, which is why the roofline above uses a measured cache-gather ceiling"}


def leaf_assign_figures(w, kern, profile):
    """Leaf assignment: one 8-byte node record and one 4-byte feature value per visited internal node, plus the leaf-id
    write and X read once.  The walk is a chain of dependent loads, so the ceiling it is held against is measured:
    rfx_probe_chase advances chains of dependent 8-byte loads (a dependent LDS read between two of them, as the feature
    lookup) at the kernel's occupancy, through a table that stays in the first-level caches (every step a hit: no walk
    can be faster) and, for reference, through a table the size of the forest (no locality at all)."""
    torch, F, N, B, rfx = w.torch, w.F, w.N, w.B, w.rfx
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
    steps_rate = path_total / (la_ms * 1e-3) if la_ms > 0 else 0.0
    ceil_hit = rfx.probe_chase(16 << 10, 2, 2048, True)
    ceil_cold = rfx.probe_chase(max(8 * int(F.total_nodes), 4096), 2, 256, True)
    fabric = None if w.reduced else fabric_bytes(profile, ["leaf_assign_kernel<"])
    return {"bytes_model": w_la, "mean_path": path_total / (N * B), "avg_ms": la_ms, "GBps": rate / 1e9,
            "frac_of_hbm_peak": rate / PEAK_HBM_BYTES,
            "compulsory_floor_bytes": 4 * N * w.c.M + 8 * int(F.total_nodes) + 4 * N * B,
            "roofline": {"bound": "dependent load chain", "unit": "G node steps/s", "achieved": steps_rate / 1e9,
                         "ceiling": ceil_hit / 1e9, "frac": steps_rate / ceil_hit if ceil_hit > 0 else 0.0,
                         "ceiling_is": "rfx_probe_chase, 2 walks per thread, 16 KiB table (every step a first-level cache hit)",
                         "no_locality_reference": ceil_cold / 1e9,
                         "no_locality_is": f"the same chase through {8 * int(F.total_nodes)} bytes (the forest's node records)"},
            "measured_fabric_bytes": fabric,
            "measured_fabric_frac_of_hbm_peak": fabric / (la_ms * 1e-3) / PEAK_HBM_BYTES if fabric and la_ms > 0 else None,
            "forest_create_ms": w.forest_create_ms,
            "note": "gather-latency bound; nodes and X are cache / LDS resident, so the byte model is not HBM traffic"}


def main():
    args = parse_args()
    if args.summarise_kernel_trace:
        return summarise_kernel_trace(args.summarise_kernel_trace)
    if args.summarise_pmc:
        return summarise_pmc(args.summarise_pmc)
    import torch
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    rfx.load()          # fails loudly if librfx.so is missing: there is no fallback path
    w = Workload(args, torch, rfx, ri)
    if args.calibrate_copy:
        calibration_copy(w)

    for _ in range(max(args.warmup, 1)):      # the first warm-up step fixes the scaling step's iteration count
        w.step()
    torch.cuda.synchronize()
    w.phase_events.clear()
    rfx.timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        w.step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    mds_iters, mds_rel = w.mds_iters, float(w.mds_rel[0])
    assert int(w.status[0]) == 0, "the factorisation's block lost rank"
    assert mds_rel <= 10 * MDS_TOL, f"the scaling step has not converged after {mds_iters} applications ({mds_rel})"

    stats = w.phase_stats()
    if w.fused:
        # the two passes the fused one replaces, outside the step, for their own kernel times
        for _ in range(3):
            w.dense_and_oob_separately()
        torch.cuda.synchronize()
        sep = w.phase_stats(["prox_dense", "prox_oob"])
        stats["separate_prox_dense"], stats["separate_prox_oob"] = sep["prox_dense"], sep["prox_oob"]
    phases = {n: v["mean"] for n, v in stats.items()}
    kern = {}
    for name in ("leaf_assign_kernel", "prox_tile_kernel_both", "prox_tile_kernel", "prox_tile_kernel_oob",
                 "prox_tile_kernel_sparse", "sparse_rows_kernel", "pv_apply", "pv_leaf_sum_kernel", "pv_gather_kernel"):
        ms, n = rfx.timing_get(name)
        kern[name] = {"avg_ms": ms / max(n, 1), "launches": n, "total_ms": ms}

    sparse = measure_sparse(w, kern)
    consumers = measure_consumers(w)
    one_shot = measure_one_shot(w)
    growth = measure_growth(w)
    # practical ceilings of this GPU next to the published peaks
    valu_rate = rfx.probe_valu(4096)
    copy_rate = rfx.probe_copy(1 << 32)
    profile, prof_file, prof_hash = load_pmc_profile(w.c.cfg)

    c, N, B, tests = w.c, w.N, w.B, w.tests
    dense_phase = "prox_sparse" if w.large else ("prox_dense_oob" if w.fused else "prox_dense")
    pv = pv_figures(w, kern, copy_rate, profile)
    out = {
        "metric": "leaf co-occurrence tests/s: N^2*B/2 per pass of the whole proximity path (traversal, dense pass, "
                  "factorisation, scaling); the dense pass alone is dense_tests_per_s",
        "value": tests / (ms_per_step * 1e-3),
        "unit": "tests/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": max(args.warmup, 1),
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": f"cfg{c.cfg}: N={N} M={c.M} B={B} trees to purity, mtry={c.mtry}, k={w.k}, T={w.T}"
                               + (" (REDUCED, debugging)" if w.reduced else "")
                               + (" (dense outputs do not fit: exact sparse list instead; forest grown by rfx_forest_grow, "
                                  "checked against the oracle by tests/test_gpu_y_fullsize.py::test_cfg5_full_tree_count)"
                                  if w.large else ""),
                   "leaf_bound": w.Lb, "bit_planes": w.P, "mds_block": w.m, "mds_iters": mds_iters},
        "phases_ms": phases,
        "phases_median_ms": {n: v["median"] for n, v in stats.items()},
        "phases_min_ms": {n: v["min"] for n, v in stats.items()},
        "phases_samples": {n: v["n"] for n, v in stats.items()},
        "lowrank_outside_pv_ms": phases["prox_lowrank"] - w.T * pv["avg_ms"],
        "mds": {"iterations": mds_iters, "rel_change_last": mds_rel, "ms_per_iteration": phases["mds3d"] / max(mds_iters, 1),
                "factor_GBps": N * w.k * mds_iters / (phases["mds3d"] * 1e-3) / 1e9},
        "dense_tests_per_s": tests / (phases[dense_phase] * 1e-3),
        "pv": pv,
        "leaf_assign": leaf_assign_figures(w, kern, profile),
        "kernels": kern,
        "roofline": roofline_of_tile_kernel(w, kern, valu_rate, profile, (prof_file, prof_hash)),
        "one_shot_conveniences": one_shot,
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
