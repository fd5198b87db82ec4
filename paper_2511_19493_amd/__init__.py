"""Thin Python binding of librfx (random-forest proximity path, HIP kernels for gfx950).

Argument marshalling only: every computation runs in the library's kernels.  Tensors are
torch CUDA tensors used as device buffers; work is enqueued on torch's current stream.
Function names and arguments mirror include/rfx.h.  Importing the package does not load the
library; the first call does, and raises if it has not been built
(`python -m paper_2511_19493_amd.build`).
"""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional, Tuple

import numpy as np

_LIB_PATH = Path(__file__).resolve().parent / "lib" / "librfx.so"
_lib = None

U16, U32 = 0, 1
ERR_INVALID_ARG, ERR_NULL, ERR_OVERFLOW, ERR_OOM, ERR_HIP, ERR_UNSUPPORTED, ERR_FOREST, ERR_CAPACITY = -1, -2, -3, -4, -5, -6, -7, -8
FULL, UPPER_PACKED = 0, 1
MDS_SQUARED, MDS_LINEAR = 0, 1
ENC_INT8, ENC_FP16, ENC_NF4, ENC_FP32 = 0, 1, 2, 3

EXPORTS = (
    "rfx_last_error", "rfx_timing_enable", "rfx_timing_get", "rfx_probe_valu", "rfx_probe_copy", "rfx_probe_gather", "rfx_probe_chase", "rfx_forest_grow", "rfx_grown_sizes", "rfx_grown_export", "rfx_grown_destroy", "rfx_growth_draw", "rfx_forest_create", "rfx_forest_destroy", "rfx_forest_leaf_bound", "rfx_leaf_assign",
    "rfx_prox_dense", "rfx_prox_oob", "rfx_prox_dense_oob", "rfx_prox_sparse", "rfx_prox_sparse_rows", "rfx_prox_outlier", "rfx_oob_vote", "rfx_pv_plan_create", "rfx_pv_plan_destroy", "rfx_pv_apply",
    "rfx_prox_matvec", "rfx_prox_lowrank", "rfx_quantise_int8", "rfx_mds3d", "rfx_mds3d_factor",
    "rfx_factor_sizes", "rfx_quantise_factor", "rfx_dequantise_factor",
    "rfx_prox_workspace_bytes", "rfx_prox_dense_ws", "rfx_prox_oob_ws", "rfx_prox_dense_oob_ws", "rfx_prox_sparse_ws",
    "rfx_prox_outlier_ws", "rfx_pv_plan_reserve", "rfx_pv_plan_rebuild", "rfx_pv_plan_info", "rfx_lowrank_workspace_bytes", "rfx_prox_lowrank_plan",
    "rfx_mds3d_workspace_bytes", "rfx_mds3d_ws", "rfx_prox_dense_noalloc", "rfx_prox_sparse_plan_workspace_bytes", "rfx_prox_sparse_plan",
)


class RfxError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"librfx error {code}: {msg}")
        self.code = code


class _ForestDesc(ctypes.Structure):
    _fields_ = [("n_trees", ctypes.c_int32), ("n_features", ctypes.c_int32), ("node_offset", ctypes.c_void_p),
                ("feature", ctypes.c_void_p), ("threshold", ctypes.c_void_p), ("left", ctypes.c_void_p),
                ("right", ctypes.c_void_p), ("leaf_id", ctypes.c_void_p), ("n_leaves", ctypes.c_void_p)]


def lib_path() -> Path:
    return _LIB_PATH


def load():
    """Loads librfx.so; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise RuntimeError(f"{_LIB_PATH} not built: run `python -m paper_2511_19493_amd.build`")
        lib = ctypes.CDLL(str(_LIB_PATH))
        vp, i64, i32, ci, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int, ctypes.c_float
        lib.rfx_last_error.restype = ctypes.c_char_p
        lib.rfx_last_error.argtypes = []
        sigs = {
            "rfx_forest_create": [ctypes.POINTER(_ForestDesc), ctypes.POINTER(vp)],
            "rfx_forest_destroy": [vp],
            "rfx_timing_enable": [ci],
            "rfx_timing_get": [ctypes.c_char_p, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)],
            "rfx_probe_valu": [i32, ctypes.POINTER(ctypes.c_double), vp],
            "rfx_probe_copy": [i64, ctypes.POINTER(ctypes.c_double), vp],
            "rfx_probe_gather": [i64, i32, i64, i32, ctypes.POINTER(ctypes.c_double), vp],
            "rfx_probe_chase": [i64, i32, i32, i32, ctypes.POINTER(ctypes.c_double), vp],
            "rfx_forest_grow": [vp, vp, i64, i32, i32, i32, i32, i32, ctypes.c_uint64, ctypes.POINTER(vp), vp],
            "rfx_grown_sizes": [vp, ctypes.POINTER(i64), ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i64)],
            "rfx_grown_export": [vp] * 11,
            "rfx_grown_destroy": [vp],
            "rfx_leaf_assign": [vp, vp, i64, i32, vp, vp],
            "rfx_prox_dense": [vp, i64, i32, i32, ci, ci, vp, vp, vp],
            "rfx_prox_oob": [vp, vp, i64, i32, i32, ci, ci, vp, vp, vp, vp],
            "rfx_prox_dense_oob": [vp, vp, i64, i32, i32, ci, ci, vp, vp, ci, vp, vp, vp, vp],
            "rfx_prox_sparse": [vp, i64, i32, i32, i32, ci, i64, vp, vp, vp, vp, ctypes.POINTER(i64), vp],
            "rfx_prox_sparse_rows": [vp, i64, i32, i32, i32, ci, i64, vp, vp, vp, vp, ctypes.POINTER(i64), vp],
            "rfx_prox_outlier": [vp, i64, i32, i32, vp, vp, vp, vp],
            "rfx_oob_vote": [vp, vp, vp, i64, i32, i32, i32, vp, vp, vp, ctypes.POINTER(i64), ctypes.POINTER(i64), vp],
            "rfx_pv_plan_create": [vp, i64, i32, i32, ctypes.POINTER(vp), vp],
            "rfx_pv_plan_destroy": [vp],
            "rfx_pv_apply": [vp, vp, i32, vp, vp],
            "rfx_prox_matvec": [vp, i64, i32, i32, vp, i32, vp, vp],
            "rfx_prox_lowrank": [vp, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp],
            "rfx_quantise_int8": [vp, vp, i64, i32, vp, vp, vp],
            "rfx_mds3d": [vp, vp, i64, i32, ci, i32, i32, f32, vp, vp, vp, ctypes.POINTER(i32), vp],
            "rfx_mds3d_factor": [vp, i64, i32, ci, i32, i32, f32, vp, vp, vp, ctypes.POINTER(i32), vp],
            "rfx_factor_sizes": [ci, i64, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)],
            "rfx_quantise_factor": [vp, vp, i64, i32, ci, vp, vp, vp],
            "rfx_dequantise_factor": [vp, vp, i64, i32, ci, vp, vp],
            "rfx_prox_workspace_bytes": [i64, i32, i32, ctypes.POINTER(i64)],
            "rfx_prox_dense_ws": [vp, i64, i32, i32, ci, ci, vp, vp, vp, i64, vp],
            "rfx_prox_dense_noalloc": [vp, i64, i32, i32, ci, ci, vp, vp, vp],
            "rfx_prox_oob_ws": [vp, vp, i64, i32, i32, ci, ci, vp, vp, vp, vp, i64, vp],
            "rfx_prox_dense_oob_ws": [vp, vp, i64, i32, i32, ci, ci, vp, vp, ci, vp, vp, vp, vp, i64, vp],
            "rfx_prox_sparse_ws": [vp, i64, i32, i32, i32, ci, i64, vp, vp, vp, vp, vp, vp, i64, vp],
            "rfx_prox_outlier_ws": [vp, i64, i32, i32, vp, vp, vp, vp, i64, vp],
            "rfx_prox_sparse_plan_workspace_bytes": [vp, ctypes.POINTER(i64)],
            "rfx_prox_sparse_plan": [vp, i32, ci, i64, vp, vp, vp, vp, vp, vp, i64, vp],
            "rfx_pv_plan_reserve": [vp, i32],
            "rfx_pv_plan_rebuild": [vp, vp, vp],
            "rfx_pv_plan_info": [vp, ctypes.POINTER(i64), ctypes.POINTER(i32), ctypes.POINTER(i32)],
            "rfx_lowrank_workspace_bytes": [i64, i32, ctypes.POINTER(i64)],
            "rfx_prox_lowrank_plan": [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, i64, vp],
            "rfx_mds3d_workspace_bytes": [i64, i32, i32, ci, ctypes.POINTER(i64)],
            "rfx_mds3d_ws": [vp, vp, i64, i32, ci, i32, i32, vp, vp, vp, vp, vp, i64, vp],
        }
        for name, args in sigs.items():
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = args
        lib.rfx_growth_draw.restype = ctypes.c_uint64
        lib.rfx_growth_draw.argtypes = [ctypes.c_uint64] * 4
        lib.rfx_forest_leaf_bound.restype = ctypes.c_int32
        lib.rfx_forest_leaf_bound.argtypes = [vp]
        _lib = lib
    return _lib


def _check(rc: int):
    if rc != 0:
        raise RfxError(rc, load().rfx_last_error().decode())


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _dev(t, dtype, shape=None) -> int:
    """Device address of a contiguous CUDA tensor of the given dtype (and shape)."""
    if t is None:
        return 0
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise TypeError(f"expected a contiguous CUDA tensor of {dtype}, got {t.dtype} on {t.device}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr()


def timing_enable(on: bool = True):
    """rfx_timing_enable: per-kernel HIP-event timing inside the library (clears the totals)."""
    _check(load().rfx_timing_enable(1 if on else 0))


def timing_get(kernel: str):
    """rfx_timing_get: (total milliseconds, launches) of one kernel since timing was enabled."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
    _check(load().rfx_timing_get(kernel.encode(), ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value


def probe_valu(rounds: int = 4096) -> float:
    """rfx_probe_valu: lane-operations per second of a dependency-free integer vector loop."""
    r = ctypes.c_double(0.0)
    _check(load().rfx_probe_valu(rounds, ctypes.byref(r), _stream()))
    return r.value


def probe_copy(nbytes: int = 1 << 32) -> float:
    """rfx_probe_copy: bytes read + written per second by a plain device copy of nbytes."""
    r = ctypes.c_double(0.0)
    _check(load().rfx_probe_copy(nbytes, ctypes.byref(r), _stream()))
    return r.value


def probe_gather(table_rows: int, k: int = 64, gathers: int = 1 << 26, xcd_local: bool = False) -> float:
    """rfx_probe_gather: row bytes per second of pseudo-random row gathers from a table of table_rows x k floats."""
    r = ctypes.c_double(0.0)
    _check(load().rfx_probe_gather(table_rows, k, gathers, 1 if xcd_local else 0, ctypes.byref(r), _stream()))
    return r.value


def probe_chase(table_bytes: int, walks_per_thread: int = 2, steps: int = 256, with_lds: bool = True) -> float:
    """rfx_probe_chase: dependent-load chain steps per second through a table of table_bytes."""
    r = ctypes.c_double(0.0)
    _check(load().rfx_probe_chase(table_bytes, walks_per_thread, steps, 1 if with_lds else 0, ctypes.byref(r), _stream()))
    return r.value


def growth_draw(seed: int, tree: int, a: int, b: int) -> int:
    """rfx_growth_draw: the counter-based draw of the grower, on the host."""
    return int(load().rfx_growth_draw(seed, tree, a, b))


def forest_grow(X, y, n_classes: int, n_trees: int, mtry: int, seed: int, first_tree: int = 0) -> dict:
    """rfx_forest_grow + rfx_grown_export: grows the trees on the GPU and returns the host arrays
    node_offset, feature, threshold, left, right, leaf_id, depth, n_leaves, inbag, leaf_class
    (plus n_trees, n_features, levels, sorted_pairs)."""
    import torch
    N, M = X.shape
    lib = load()
    h = ctypes.c_void_p()
    _check(lib.rfx_forest_grow(_dev(X, torch.float32), _dev(y, torch.int32, (N,)), N, M, n_classes, first_tree, n_trees, mtry,
                               seed, ctypes.byref(h), _stream()))
    try:
        nn, ml, lv, sp = ctypes.c_int64(0), ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int64(0)
        _check(lib.rfx_grown_sizes(h, ctypes.byref(nn), ctypes.byref(ml), ctypes.byref(lv), ctypes.byref(sp)))
        nn, ml = nn.value, ml.value
        out = dict(node_offset=np.empty(n_trees + 1, np.int64), feature=np.empty(nn, np.int32),
                   threshold=np.empty(nn, np.float32), left=np.empty(nn, np.int32), right=np.empty(nn, np.int32),
                   leaf_id=np.empty(nn, np.int32), depth=np.empty(nn, np.int32), n_leaves=np.empty(n_trees, np.int32),
                   inbag=np.empty((n_trees, N), np.uint16), leaf_class=np.empty((n_trees, ml), np.int32))
        _check(lib.rfx_grown_export(h, *(out[k].ctypes.data for k in ("node_offset", "feature", "threshold", "left", "right",
                                                                        "leaf_id", "depth", "n_leaves", "inbag", "leaf_class"))))
    finally:
        lib.rfx_grown_destroy(h)
    out["n_trees"], out["n_features"], out["levels"], out["sorted_pairs"] = n_trees, M, lv.value, sp.value
    return out


class Forest:
    """Device-resident forest (rfx_forest_create / rfx_forest_destroy)."""

    def __init__(self, n_features: int, node_offset, feature, threshold, left, right, leaf_id, n_leaves):
        arrs = [np.ascontiguousarray(node_offset, np.int64), np.ascontiguousarray(feature, np.int32),
                np.ascontiguousarray(threshold, np.float32), np.ascontiguousarray(left, np.int32),
                np.ascontiguousarray(right, np.int32), np.ascontiguousarray(leaf_id, np.int32),
                np.ascontiguousarray(n_leaves, np.int32)]
        self.n_trees = len(arrs[6])
        self.n_features = int(n_features)
        d = _ForestDesc(self.n_trees, self.n_features, *(a.ctypes.data for a in arrs))
        h = ctypes.c_void_p()
        _check(load().rfx_forest_create(ctypes.byref(d), ctypes.byref(h)))
        self._h = h

    @property
    def leaf_bound(self) -> int:
        return int(load().rfx_forest_leaf_bound(self._h))

    def close(self):
        if getattr(self, "_h", None):
            load().rfx_forest_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def leaf_assign(forest: Forest, X, leaf=None):
    """rfx_leaf_assign: X float32 [N][M] -> leaf uint32 [B][N] (stored in an int32 tensor)."""
    import torch
    N, M = X.shape
    if leaf is None:
        leaf = torch.empty((forest.n_trees, N), dtype=torch.int32, device=X.device)
    _check(load().rfx_leaf_assign(forest._h, _dev(X, torch.float32), N, M,
                                  _dev(leaf, torch.int32, (forest.n_trees, N)), _stream()))
    return leaf


def _count_dtype(count_dtype):
    import torch
    return torch.int16 if count_dtype == U16 else torch.int32


def _sym_shape(N: int, layout: int):
    return (N, N) if layout == FULL else (N * (N - 1) // 2,)


def prox_dense(leaf, leaf_bound: int, count_dtype: int = U32, layout: int = FULL, counts=None, prox=None,
               want_counts: bool = True, want_prox: bool = True):
    """rfx_prox_dense.  Counts come back in int16 / int32 tensors holding the uint16 / uint32 bits."""
    import torch
    B, N = leaf.shape
    shp = _sym_shape(N, layout)
    if counts is None and want_counts:
        counts = torch.empty(shp, dtype=_count_dtype(count_dtype), device=leaf.device)
    if prox is None and want_prox:
        prox = torch.empty(shp, dtype=torch.float32, device=leaf.device)
    _check(load().rfx_prox_dense(_dev(leaf, torch.int32), N, B, leaf_bound, count_dtype, layout,
                                 _dev(counts, _count_dtype(count_dtype), shp) if counts is not None else 0,
                                 _dev(prox, torch.float32, shp) if prox is not None else 0, _stream()))
    return counts, prox


def prox_oob(leaf, inbag, leaf_bound: int, count_dtype: int = U32, layout: int = FULL, want_prox: bool = True):
    """rfx_prox_oob: returns (num, den, prox)."""
    import torch
    B, N = leaf.shape
    shp = _sym_shape(N, layout)
    num = torch.empty(shp, dtype=_count_dtype(count_dtype), device=leaf.device)
    den = torch.empty(shp, dtype=_count_dtype(count_dtype), device=leaf.device)
    prox = torch.empty(shp, dtype=torch.float32, device=leaf.device) if want_prox else None
    _check(load().rfx_prox_oob(_dev(leaf, torch.int32), _dev(inbag, torch.int16, (B, N)), N, B, leaf_bound,
                               count_dtype, layout, num.data_ptr(), den.data_ptr(),
                               prox.data_ptr() if prox is not None else 0, _stream()))
    return num, den, prox


def prox_dense_oob(leaf, inbag, leaf_bound: int, count_dtype: int = U32, layout: int = FULL, oob_layout: int = FULL,
                   want_counts: bool = True, want_prox: bool = True, want_num_den: bool = True, want_prox_oob: bool = True):
    """rfx_prox_dense_oob: returns (counts, prox, num, den, prox_oob); B <= 1023."""
    import torch
    B, N = leaf.shape
    cdt = _count_dtype(count_dtype)
    mk = lambda want, lay, dt: torch.empty(_sym_shape(N, lay), dtype=dt, device=leaf.device) if want else None
    counts, prox = mk(want_counts, layout, cdt), mk(want_prox, layout, torch.float32)
    num, den = mk(want_num_den, oob_layout, cdt), mk(want_num_den, oob_layout, cdt)
    prox_oob = mk(want_prox_oob, oob_layout, torch.float32)
    ptr = lambda t: t.data_ptr() if t is not None else 0
    _check(load().rfx_prox_dense_oob(_dev(leaf, torch.int32), _dev(inbag, torch.int16, (B, N)), N, B, leaf_bound, count_dtype,
                                     layout, ptr(counts), ptr(prox), oob_layout, ptr(num), ptr(den), ptr(prox_oob), _stream()))
    return counts, prox, num, den, prox_oob


def _sparse_fn(method: str):
    """rfx_prox_sparse ("auto": the library chooses; "tiles": not selectable from here, auto on shallow forests) or
    rfx_prox_sparse_rows ("rows")."""
    if method not in ("auto", "rows"):
        raise ValueError("method must be 'auto' or 'rows'")
    return load().rfx_prox_sparse if method == "auto" else load().rfx_prox_sparse_rows


def prox_sparse_count(leaf, leaf_bound: int, min_count: int = 1, method: str = "auto") -> int:
    """rfx_prox_sparse with capacity 0: the number of pairs i < j with cnt(i,j) >= min_count."""
    import torch
    B, N = leaf.shape
    nnz = ctypes.c_int64(0)
    _check(_sparse_fn(method)(_dev(leaf, torch.int32), N, B, leaf_bound, min_count, U32, 0, 0, 0, 0, 0,
                                  ctypes.byref(nnz), _stream()))
    return nnz.value


def prox_sparse(leaf, leaf_bound: int, min_count: int = 1, capacity: int = None, count_dtype: int = U32,
                want_counts: bool = True, want_prox: bool = False, method: str = "auto"):
    """rfx_prox_sparse: returns (rows, cols, counts, prox), each trimmed to the number of kept pairs.

    `capacity` None runs the counting call first and allocates exactly; a given capacity that is too
    small raises RfxError with code ERR_CAPACITY."""
    import torch
    B, N = leaf.shape
    if capacity is None:
        capacity = max(prox_sparse_count(leaf, leaf_bound, min_count, method), 1)
    rows = torch.empty(capacity, dtype=torch.int32, device=leaf.device)
    cols = torch.empty(capacity, dtype=torch.int32, device=leaf.device)
    counts = torch.empty(capacity, dtype=_count_dtype(count_dtype), device=leaf.device) if want_counts else None
    prox = torch.empty(capacity, dtype=torch.float32, device=leaf.device) if want_prox else None
    nnz = ctypes.c_int64(0)
    _check(_sparse_fn(method)(_dev(leaf, torch.int32), N, B, leaf_bound, min_count, count_dtype, capacity,
                                  rows.data_ptr(), cols.data_ptr(), counts.data_ptr() if counts is not None else 0,
                                  prox.data_ptr() if prox is not None else 0, ctypes.byref(nnz), _stream()))
    n = nnz.value
    return rows[:n], cols[:n], counts[:n] if counts is not None else None, prox[:n] if prox is not None else None


def prox_outlier(leaf, leaf_bound: int, labels=None, want_printed: bool = True, want_classic: bool = True):
    """rfx_prox_outlier: returns (printed, classic), float64 [N] each (None when not asked for)."""
    import torch
    B, N = leaf.shape
    printed = torch.empty(N, dtype=torch.float64, device=leaf.device) if want_printed else None
    classic = torch.empty(N, dtype=torch.float64, device=leaf.device) if want_classic else None
    _check(load().rfx_prox_outlier(_dev(leaf, torch.int32), N, B, leaf_bound, _dev(labels, torch.int32, (N,)),
                                   printed.data_ptr() if printed is not None else 0,
                                   classic.data_ptr() if classic is not None else 0, _stream()))
    return printed, classic


def oob_vote(leaf, inbag, leaf_class, n_classes: int, y=None, want_votes: bool = True):
    """rfx_oob_vote: returns (votes, pred, wrong, voted); wrong is None without labels."""
    import torch
    B, N = leaf.shape
    if leaf_class.dim() != 2 or leaf_class.shape[0] != B:
        raise ValueError("leaf_class must be [B][leaf_stride]")
    votes = torch.empty((N, n_classes), dtype=torch.int32, device=leaf.device) if want_votes else None
    pred = torch.empty(N, dtype=torch.int32, device=leaf.device)
    wrong, voted = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(load().rfx_oob_vote(_dev(leaf, torch.int32), _dev(inbag, torch.int16, (B, N)), _dev(leaf_class, torch.int32),
                               N, B, leaf_class.shape[1], n_classes, _dev(y, torch.int32, (N,)),
                               votes.data_ptr() if votes is not None else 0, pred.data_ptr(),
                               ctypes.byref(wrong) if y is not None else None, ctypes.byref(voted), _stream()))
    return votes, pred, (wrong.value if y is not None else None), voted.value


class PvPlan:
    """rfx_pv_plan_create / rfx_pv_apply / rfx_pv_plan_destroy."""

    def __init__(self, leaf, leaf_bound: int):
        import torch
        B, N = leaf.shape
        self.N, self.B = N, B
        h = ctypes.c_void_p()
        _check(load().rfx_pv_plan_create(_dev(leaf, torch.int32), N, B, leaf_bound, ctypes.byref(h), _stream()))
        self._h = h

    def apply(self, V, Y=None):
        import torch
        N, k = V.shape
        if N != self.N:
            raise ValueError("V has the wrong number of rows")
        if Y is None:
            Y = torch.empty_like(V)
        _check(load().rfx_pv_apply(self._h, _dev(V, torch.float32), k, _dev(Y, torch.float32, (N, k)), _stream()))
        return Y

    def close(self):
        if getattr(self, "_h", None):
            load().rfx_pv_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def prox_matvec(leaf, leaf_bound: int, V):
    """rfx_prox_matvec: one P.V without a persistent plan."""
    import torch
    B, N = leaf.shape
    k = V.shape[1]
    Y = torch.empty_like(V)
    _check(load().rfx_prox_matvec(_dev(leaf, torch.int32), N, B, leaf_bound, _dev(V, torch.float32, (N, k)), k,
                                  Y.data_ptr(), _stream()))
    return Y


def prox_lowrank(leaf, leaf_bound: int, V0, iters: int, quantise: bool = True):
    """rfx_prox_lowrank: returns (eigvals [k], V [N][k], Q int8 [N][k] or None, scales [k] or None)."""
    import torch
    B, N = leaf.shape
    k = V0.shape[1]
    dev = leaf.device
    eig = torch.empty(k, dtype=torch.float32, device=dev)
    V = torch.empty((N, k), dtype=torch.float32, device=dev)
    Q = torch.empty((N, k), dtype=torch.int8, device=dev) if quantise else None
    s = torch.empty(k, dtype=torch.float32, device=dev) if quantise else None
    _check(load().rfx_prox_lowrank(_dev(leaf, torch.int32), N, B, leaf_bound, k, iters,
                                   _dev(V0, torch.float32, (N, k)), eig.data_ptr(), V.data_ptr(),
                                   Q.data_ptr() if quantise else 0, s.data_ptr() if quantise else 0, _stream()))
    return eig, V, Q, s


def quantise_int8(V, eigvals):
    """rfx_quantise_int8: returns (Q int8 [N][k], scales float32 [k])."""
    import torch
    N, k = V.shape
    Q = torch.empty((N, k), dtype=torch.int8, device=V.device)
    s = torch.empty(k, dtype=torch.float32, device=V.device)
    _check(load().rfx_quantise_int8(_dev(V, torch.float32), _dev(eigvals, torch.float32, (k,)), N, k, Q.data_ptr(),
                                    s.data_ptr(), _stream()))
    return Q, s


def mds3d(Q, scales, x0=None, mode: int = MDS_SQUARED, max_iters: int = 300, tol: float = 1e-6, m: int = 16) -> Tuple:
    """rfx_mds3d: returns (coords float32 [N][3], eigvals float32 [3], iterations done).  x0 None: the library's own
    start block of width m (the leading columns of the factor)."""
    import torch
    N, k = Q.shape
    m = x0.shape[1] if x0 is not None else min(m, N)
    coords = torch.empty((N, 3), dtype=torch.float32, device=Q.device)
    ev = torch.empty(3, dtype=torch.float32, device=Q.device)
    it = ctypes.c_int32(0)
    _check(load().rfx_mds3d(_dev(Q, torch.int8), _dev(scales, torch.float32, (k,)), N, k, mode, m, max_iters, tol,
                            _dev(x0, torch.float32, (N, m)), coords.data_ptr(), ev.data_ptr(), ctypes.byref(it),
                            _stream()))
    return coords, ev, int(it.value)


def factor_sizes(encoding: int, N: int, k: int) -> Tuple[int, int]:
    """rfx_factor_sizes: (bytes of codes, floats of scales)."""
    cb, ns = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(load().rfx_factor_sizes(encoding, N, k, ctypes.byref(cb), ctypes.byref(ns)))
    return cb.value, ns.value


def quantise_factor(V, eigvals, encoding: int):
    """rfx_quantise_factor: returns (codes uint8 buffer of rfx_factor_sizes bytes, scales float32)."""
    import torch
    N, k = V.shape
    cb, ns = factor_sizes(encoding, N, k)
    codes = torch.empty(cb, dtype=torch.uint8, device=V.device)
    scales = torch.empty(max(ns, 1), dtype=torch.float32, device=V.device)
    _check(load().rfx_quantise_factor(_dev(V, torch.float32), _dev(eigvals, torch.float32, (k,)), N, k, encoding,
                                      codes.data_ptr(), scales.data_ptr(), _stream()))
    return codes, scales[:ns]


def dequantise_factor(codes, scales, N: int, k: int, encoding: int):
    """rfx_dequantise_factor: float32 [N][k]."""
    import torch
    A = torch.empty((N, k), dtype=torch.float32, device=codes.device)
    _check(load().rfx_dequantise_factor(codes.data_ptr(), scales.data_ptr() if scales is not None and scales.numel() else 0,
                                        N, k, encoding, A.data_ptr(), _stream()))
    return A


def mds3d_factor(A, x0=None, mode: int = MDS_SQUARED, max_iters: int = 300, tol: float = 1e-6, m: int = 16) -> Tuple:
    """rfx_mds3d_factor: as mds3d, from a float32 factor."""
    import torch
    N, k = A.shape
    m = x0.shape[1] if x0 is not None else min(m, N)
    coords = torch.empty((N, 3), dtype=torch.float32, device=A.device)
    ev = torch.empty(3, dtype=torch.float32, device=A.device)
    it = ctypes.c_int32(0)
    _check(load().rfx_mds3d_factor(_dev(A, torch.float32), N, k, mode, m, max_iters, tol, _dev(x0, torch.float32, (N, m)),
                                   coords.data_ptr(), ev.data_ptr(), ctypes.byref(it), _stream()))
    return coords, ev, int(it.value)


# ------------------------------------------------------------------------------ asynchronous forms
# Scratch comes from a caller-owned workspace tensor; nothing here waits for the device.

def _ws_ptr(workspace):
    import torch
    if workspace is None or not workspace.is_cuda or workspace.dtype != torch.uint8 or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous CUDA uint8 tensor")
    return workspace.data_ptr(), workspace.numel()


def prox_workspace_bytes(N: int, B: int, leaf_bound: int) -> int:
    """rfx_prox_workspace_bytes."""
    out = ctypes.c_int64(0)
    _check(load().rfx_prox_workspace_bytes(N, B, leaf_bound, ctypes.byref(out)))
    return out.value


def new_workspace(nbytes: int, device="cuda"):
    """A device buffer usable as `workspace` (torch allocations are at least 256-byte aligned)."""
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def prox_dense_ws(leaf, leaf_bound: int, workspace, count_dtype: int = U32, layout: int = FULL, counts=None, prox=None):
    """rfx_prox_dense_ws: writes the given outputs (at least one); asynchronous."""
    import torch
    B, N = leaf.shape
    shp = _sym_shape(N, layout)
    wp, wb = _ws_ptr(workspace)
    _check(load().rfx_prox_dense_ws(_dev(leaf, torch.int32), N, B, leaf_bound, count_dtype, layout,
                                    _dev(counts, _count_dtype(count_dtype), shp), _dev(prox, torch.float32, shp), wp, wb,
                                    _stream()))


def prox_oob_ws(leaf, inbag, leaf_bound: int, workspace, count_dtype: int = U32, layout: int = FULL, num=None, den=None,
                prox=None):
    """rfx_prox_oob_ws; asynchronous."""
    import torch
    B, N = leaf.shape
    shp = _sym_shape(N, layout)
    cdt = _count_dtype(count_dtype)
    wp, wb = _ws_ptr(workspace)
    _check(load().rfx_prox_oob_ws(_dev(leaf, torch.int32), _dev(inbag, torch.int16, (B, N)), N, B, leaf_bound, count_dtype,
                                  layout, _dev(num, cdt, shp), _dev(den, cdt, shp), _dev(prox, torch.float32, shp), wp, wb,
                                  _stream()))


def prox_dense_oob_ws(leaf, inbag, leaf_bound: int, workspace, count_dtype: int = U32, layout: int = FULL,
                      oob_layout: int = FULL, counts=None, prox=None, num=None, den=None, prox_oob=None):
    """rfx_prox_dense_oob_ws; asynchronous."""
    import torch
    B, N = leaf.shape
    cdt = _count_dtype(count_dtype)
    s1, s2 = _sym_shape(N, layout), _sym_shape(N, oob_layout)
    wp, wb = _ws_ptr(workspace)
    _check(load().rfx_prox_dense_oob_ws(_dev(leaf, torch.int32), _dev(inbag, torch.int16, (B, N)), N, B, leaf_bound,
                                        count_dtype, layout, _dev(counts, cdt, s1), _dev(prox, torch.float32, s1), oob_layout,
                                        _dev(num, cdt, s2), _dev(den, cdt, s2), _dev(prox_oob, torch.float32, s2), wp, wb,
                                        _stream()))


def prox_sparse_ws(leaf, leaf_bound: int, workspace, nnz, rows=None, cols=None, counts=None, prox=None, min_count: int = 1,
                   count_dtype: int = U32):
    """rfx_prox_sparse_ws: nnz is a CUDA int64 tensor of one element that receives the pair count; the
    capacity is the length of rows (0 without it: count only); asynchronous."""
    import torch
    B, N = leaf.shape
    cap = 0 if rows is None else rows.numel()
    wp, wb = _ws_ptr(workspace)
    _check(load().rfx_prox_sparse_ws(_dev(leaf, torch.int32), N, B, leaf_bound, min_count, count_dtype, cap,
                                     _dev(rows, torch.int32), _dev(cols, torch.int32, (cap,)) if cols is not None else 0,
                                     _dev(counts, _count_dtype(count_dtype), (cap,)) if counts is not None else 0,
                                     _dev(prox, torch.float32, (cap,)) if prox is not None else 0,
                                     _dev(nnz, torch.int64, (1,)), wp, wb, _stream()))


def prox_sparse_plan_workspace_bytes(plan: "PvPlan") -> int:
    """rfx_prox_sparse_plan_workspace_bytes."""
    out = ctypes.c_int64(0)
    _check(load().rfx_prox_sparse_plan_workspace_bytes(plan._h, ctypes.byref(out)))
    return out.value


def prox_sparse_plan(plan: "PvPlan", workspace, nnz, rows=None, cols=None, counts=None, prox=None, min_count: int = 1,
                     count_dtype: int = U32):
    """rfx_prox_sparse_plan: the row-by-row list from an existing plan; nnz is a CUDA int64 tensor of one element; the
    capacity is the length of rows (0 without it: count only); asynchronous."""
    import torch
    cap = 0 if rows is None else rows.numel()
    wp, wb = _ws_ptr(workspace)
    _check(load().rfx_prox_sparse_plan(plan._h, min_count, count_dtype, cap,
                                       _dev(rows, torch.int32), _dev(cols, torch.int32, (cap,)) if cols is not None else 0,
                                       _dev(counts, _count_dtype(count_dtype), (cap,)) if counts is not None else 0,
                                       _dev(prox, torch.float32, (cap,)) if prox is not None else 0,
                                       _dev(nnz, torch.int64, (1,)), wp, wb, _stream()))


def prox_outlier_ws(leaf, leaf_bound: int, workspace, labels=None, printed=None, classic=None):
    """rfx_prox_outlier_ws; asynchronous."""
    import torch
    B, N = leaf.shape
    wp, wb = _ws_ptr(workspace)
    _check(load().rfx_prox_outlier_ws(_dev(leaf, torch.int32), N, B, leaf_bound, _dev(labels, torch.int32, (N,)),
                                      _dev(printed, torch.float64, (N,)), _dev(classic, torch.float64, (N,)), wp, wb,
                                      _stream()))


def pv_plan_rebuild(plan: "PvPlan", leaf):
    """rfx_pv_plan_rebuild: regroup the plan for new leaf ids of the same shape, without allocating."""
    import torch
    _check(load().rfx_pv_plan_rebuild(plan._h, _dev(leaf, torch.int32, (plan.B, plan.N)), _stream()))


def pv_plan_reserve(plan: "PvPlan", k: int):
    """rfx_pv_plan_reserve."""
    _check(load().rfx_pv_plan_reserve(plan._h, k))


def pv_plan_info(plan: "PvPlan"):
    """rfx_pv_plan_info: (N, B, reserved rank)."""
    n, b, k = ctypes.c_int64(0), ctypes.c_int32(0), ctypes.c_int32(0)
    _check(load().rfx_pv_plan_info(plan._h, ctypes.byref(n), ctypes.byref(b), ctypes.byref(k)))
    return n.value, b.value, k.value


def lowrank_workspace_bytes(N: int, k: int) -> int:
    """rfx_lowrank_workspace_bytes."""
    out = ctypes.c_int64(0)
    _check(load().rfx_lowrank_workspace_bytes(N, k, ctypes.byref(out)))
    return out.value


def prox_lowrank_plan(plan: "PvPlan", V0, iters: int, workspace, eigvals, V, Q=None, scales=None, status=None):
    """rfx_prox_lowrank_plan: outputs are written into the given tensors; asynchronous."""
    import torch
    N, k = V0.shape
    wp, wb = _ws_ptr(workspace)
    _check(load().rfx_prox_lowrank_plan(plan._h, k, iters, _dev(V0, torch.float32, (N, k)), _dev(eigvals, torch.float32, (k,)),
                                        _dev(V, torch.float32, (N, k)), _dev(Q, torch.int8, (N, k)),
                                        _dev(scales, torch.float32, (k,)), _dev(status, torch.int32, (1,)), wp, wb, _stream()))


def mds3d_workspace_bytes(N: int, k: int, m: int, mode: int = MDS_SQUARED) -> int:
    """rfx_mds3d_workspace_bytes."""
    out = ctypes.c_int64(0)
    _check(load().rfx_mds3d_workspace_bytes(N, k, m, mode, ctypes.byref(out)))
    return out.value


def mds3d_ws(Q, scales, x0, iters: int, workspace, coords, eigvals, rel_change=None, mode: int = MDS_SQUARED, m: int = 16):
    """rfx_mds3d_ws: exactly `iters` applications of the Gram operator; asynchronous.  x0 None: the library's own start
    block of width m."""
    import torch
    N, k = Q.shape
    m = x0.shape[1] if x0 is not None else min(m, N)
    wp, wb = _ws_ptr(workspace)
    _check(load().rfx_mds3d_ws(_dev(Q, torch.int8), _dev(scales, torch.float32, (k,)), N, k, mode, m, iters,
                               _dev(x0, torch.float32, (N, m)), _dev(coords, torch.float32, (N, 3)),
                               _dev(eigvals, torch.float32, (3,)), _dev(rel_change, torch.float32, (1,)), wp, wb, _stream()))


def prox_dense_noalloc(leaf, leaf_bound: int, count_dtype: int = U32, layout: int = FULL, counts=None, prox=None):
    """rfx_prox_dense_noalloc: writes the given outputs (at least one) using the library's built-in scratch;
    allocates nothing; asynchronous."""
    import torch
    B, N = leaf.shape
    shp = _sym_shape(N, layout)
    _check(load().rfx_prox_dense_noalloc(_dev(leaf, torch.int32), N, B, leaf_bound, count_dtype, layout,
                                         _dev(counts, _count_dtype(count_dtype), shp), _dev(prox, torch.float32, shp),
                                         _stream()))
