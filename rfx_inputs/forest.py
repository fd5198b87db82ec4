"""Grown forests as flat arrays: ctypes wrapper around forest_grower.cpp, plus a disk cache."""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from pathlib import Path
from typing import Optional

import numpy as np

from .mixture import FOREST_ISEED, WorkloadConfig, gaussian_mixture

_HERE = Path(__file__).resolve().parent
# RFX_SANITIZE=1 selects a build with AddressSanitizer and UndefinedBehaviorSanitizer (its own file name); the process
# that loads it must have the sanitizer runtimes preloaded.
_SANITIZE = os.environ.get("RFX_SANITIZE", "") == "1"
_LIB_PATH = _HERE / ("libforest_grower_san.so" if _SANITIZE else "libforest_grower.so")
_lib = None


@dataclass
class Forest:
    """Flattened trees, concatenated over trees (tree b owns nodes [node_offset[b], node_offset[b+1]))."""

    n_trees: int
    n_features: int
    node_offset: np.ndarray   # int64 [B+1]
    feature: np.ndarray       # int32 [nodes], -1 at leaves
    threshold: np.ndarray     # float32 [nodes], go left iff x <= threshold
    left: np.ndarray          # int32 [nodes], tree-local child index, -1 at leaves
    right: np.ndarray         # int32 [nodes]
    leaf_id: np.ndarray       # int32 [nodes], dense 0..L_b-1 at leaves, -1 otherwise
    depth: np.ndarray         # int32 [nodes], root = 0
    n_leaves: np.ndarray      # int32 [B]
    inbag: np.ndarray         # uint16 [B][N] bootstrap in-bag counts
    train_leaf: np.ndarray    # int32 [B][N] leaf an in-bag row ended in while growing; -1 if out-of-bag

    @property
    def total_nodes(self) -> int:
        return int(self.node_offset[-1])

    def subset(self, n_trees: int) -> "Forest":
        """The first n_trees trees as a forest of their own."""
        e = int(self.node_offset[n_trees])
        return Forest(n_trees, self.n_features, self.node_offset[: n_trees + 1].copy(), self.feature[:e],
                      self.threshold[:e], self.left[:e], self.right[:e], self.leaf_id[:e], self.depth[:e],
                      self.n_leaves[:n_trees], self.inbag[:n_trees], self.train_leaf[:n_trees])


def build_grower(force: bool = False) -> Path:
    """Compiles forest_grower.cpp with g++ (in-tree)."""
    src = _HERE / "forest_grower.cpp"
    if force or not _LIB_PATH.exists() or _LIB_PATH.stat().st_mtime < src.stat().st_mtime:
        san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"] if _SANITIZE else []
        subprocess.run(["g++", "-O2", "-std=c++17", "-fopenmp", "-shared", "-fPIC", *san, str(src), "-o", str(_LIB_PATH)],
                       check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build_grower()
        lib = ctypes.CDLL(str(_LIB_PATH))
        lib.fg_grow.restype = ctypes.c_void_p
        lib.fg_grow.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
                                ctypes.c_int32, ctypes.c_int32, ctypes.c_uint32, ctypes.c_int32]
        lib.fg_total_nodes.restype = ctypes.c_int64
        lib.fg_total_nodes.argtypes = [ctypes.c_void_p]
        lib.fg_export.restype = None
        lib.fg_export.argtypes = [ctypes.c_void_p] * 11
        lib.fg_free.restype = None
        lib.fg_free.argtypes = [ctypes.c_void_p]
        _lib = lib
    return _lib


def grow_forest(X: np.ndarray, y: np.ndarray, n_classes: int, n_trees: int, mtry: int,
                iseed: int = FOREST_ISEED, n_threads: int = 0) -> Forest:
    """Grows n_trees purity-grown trees on (X, y); tree b uses seed iseed + b."""
    lib = _load()
    X = np.ascontiguousarray(X, dtype=np.float32)
    y = np.ascontiguousarray(y, dtype=np.int32)
    N, M = X.shape
    h = lib.fg_grow(X.ctypes.data, N, M, y.ctypes.data, n_classes, n_trees, mtry, iseed, n_threads)
    if not h:
        raise ValueError("fg_grow rejected its arguments")
    try:
        nn = lib.fg_total_nodes(h)
        off = np.empty(n_trees + 1, np.int64)
        feat, left, right, leaf, depth = (np.empty(nn, np.int32) for _ in range(5))
        thr = np.empty(nn, np.float32)
        nl = np.empty(n_trees, np.int32)
        inbag = np.empty((n_trees, N), np.uint16)
        tl = np.empty((n_trees, N), np.int32)
        lib.fg_export(h, *(a.ctypes.data for a in (off, feat, thr, left, right, leaf, depth, nl, inbag, tl)))
    finally:
        lib.fg_free(h)
    return Forest(n_trees, M, off, feat, thr, left, right, leaf, depth, nl, inbag, tl)


def leaf_classes(forest: Forest, y: np.ndarray, n_classes: int) -> np.ndarray:
    """Class label of every leaf: the class with the largest in-bag weight among the training rows that
    ended in it (lowest class on ties).  int32 [B][max leaves per tree], -1 past a tree's last leaf."""
    y = np.asarray(y, np.int64)
    out = np.full((forest.n_trees, int(forest.n_leaves.max())), -1, np.int32)
    for b in range(forest.n_trees):
        tl = forest.train_leaf[b]
        rows = np.nonzero(tl >= 0)[0]
        table = np.zeros((int(forest.n_leaves[b]), n_classes), np.int64)
        np.add.at(table, (tl[rows], y[rows]), forest.inbag[b][rows].astype(np.int64))
        out[b, : table.shape[0]] = table.argmax(axis=1)
    return out


def cache_dir() -> Path:
    return Path(os.environ.get("RFX_INPUT_CACHE", str(_HERE.parent / ".rfx_cache")))


_FIELDS = ("node_offset", "feature", "threshold", "left", "right", "leaf_id", "depth", "n_leaves", "inbag",
           "train_leaf")


def load_or_grow(c: WorkloadConfig, N: Optional[int] = None, B: Optional[int] = None, n_threads: int = 0,
                 use_cache: bool = True):
    """Returns (X, y, Forest) for a workload, growing the forest once and caching it on disk.

    `N` / `B` override the row and tree counts for reduced-size cases.
    """
    n = c.N if N is None else int(N)
    b = c.B if B is None else int(B)
    X, y = gaussian_mixture(c, None if N is None else n)
    path = cache_dir() / f"forest_cfg{c.cfg}_N{n}_B{b}_mtry{c.mtry}_seed{FOREST_ISEED}.npz"
    if use_cache and path.exists():
        try:
            with np.load(path) as z:
                return X, y, Forest(b, c.M, *(z[f] for f in _FIELDS))
        except Exception:
            path.unlink(missing_ok=True)
    F = grow_forest(X, y, c.C, b, c.mtry, FOREST_ISEED, n_threads)
    if use_cache:
        try:
            path.parent.mkdir(parents=True, exist_ok=True)
            tmp = path.with_suffix(".tmp.npz")
            np.savez(tmp, **{f: getattr(F, f) for f in _FIELDS})
            os.replace(tmp, path)
        except OSError:
            pass
    return X, y, F
