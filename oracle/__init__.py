"""CPU ORACLE -- TEST INFRASTRUCTURE ONLY.

Plain, slow reference implementations of the random-forest proximity path,
written from the paper's definitions.  Integer steps and the float64 products
live in oracle_core.c (loaded with ctypes); the dense linear-algebra steps are
numpy / scipy library calls in float64.  Nothing here is shared with the HIP
library.  Only tests, the smoke check and the benchmark's CPU-baseline leg may
import this package; the product path never does.

Parity status: every function below is pinned by tests/test_oracle_*.py
against brute force, closed forms, invariants or library routines.  The paper
prints no proximity, eigenvalue or MDS value for any worked example, so no
paper-printed numbers are involved; the paper's MDS-correlation table needs its
own data and forests and stays "parity unpinned" (context only).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path
from typing import Tuple

import numpy as np

_HERE = Path(__file__).resolve().parent
# RFX_SANITIZE=1 selects builds with AddressSanitizer and UndefinedBehaviorSanitizer (own file names, so both kinds
# can sit side by side); the process that loads them must have the sanitizer runtimes preloaded.
_SANITIZE = os.environ.get("RFX_SANITIZE", "") == "1"
_SAN_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]
_LIB_PATH = _HERE / ("liboracle_core_san.so" if _SANITIZE else "liboracle_core.so")
_lib = None

SQUARED = 0   # dissimilarity squared before double-centring (the paper's Step 1-2)
LINEAR = 1    # 1 - P itself taken as the squared distance


def build_core(force: bool = False) -> Path:
    """Compiles oracle_core.c with gcc (in-tree)."""
    src = _HERE / "oracle_core.c"
    if force or not _LIB_PATH.exists() or _LIB_PATH.stat().st_mtime < src.stat().st_mtime:
        subprocess.run(["gcc", "-O2", "-std=c99", "-fopenmp", "-Wall", "-shared", "-fPIC", *(_SAN_FLAGS if _SANITIZE else []),
                        str(src), "-o", str(_LIB_PATH)], check=True)
    return _LIB_PATH


_GROW_PATH = _HERE / ("liboracle_grow_san.so" if _SANITIZE else "liboracle_grow.so")
_grow_lib = None


def build_grow(force: bool = False) -> Path:
    """Compiles grow_core.c with gcc (in-tree)."""
    src = _HERE / "grow_core.c"
    if force or not _GROW_PATH.exists() or _GROW_PATH.stat().st_mtime < src.stat().st_mtime:
        subprocess.run(["gcc", "-O2", "-std=c99", "-fopenmp", "-Wall", "-shared", "-fPIC", *(_SAN_FLAGS if _SANITIZE else []),
                        str(src), "-o", str(_GROW_PATH)], check=True)
    return _GROW_PATH


def _grow():
    global _grow_lib
    if _grow_lib is None:
        build_grow()
        lib = ctypes.CDLL(str(_GROW_PATH))
        vp, i64, i32, u64 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64
        lib.orc_draw.restype = u64
        lib.orc_draw.argtypes = [u64, u64, u64, u64]
        lib.orc_grow.restype = vp
        lib.orc_grow.argtypes = [vp, i64, i32, vp, i32, i32, i32, i32, u64]
        lib.orc_grown_total_nodes.restype = i64
        lib.orc_grown_total_nodes.argtypes = [vp]
        lib.orc_grown_max_leaves.restype = i32
        lib.orc_grown_max_leaves.argtypes = [vp]
        lib.orc_grown_export.restype = None
        lib.orc_grown_export.argtypes = [vp] * 12
        lib.orc_grown_free.restype = None
        lib.orc_grown_free.argtypes = [vp]
        _grow_lib = lib
    return _grow_lib


def _core():
    global _lib
    if _lib is None:
        build_core()
        lib = ctypes.CDLL(str(_LIB_PATH))
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        lib.orc_leaf_assign.restype = ctypes.c_int
        lib.orc_leaf_assign.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, i64, i32, vp, vp]
        lib.orc_counts_rows.restype = None
        lib.orc_counts_rows.argtypes = [vp, i64, i32, i64, i64, vp]
        lib.orc_oob_rows.restype = None
        lib.orc_oob_rows.argtypes = [vp, vp, i64, i32, i64, i64, vp, vp]
        lib.orc_pv_implicit.restype = ctypes.c_int
        lib.orc_pv_implicit.argtypes = [vp, i64, i32, i64, vp, i32, vp]
        lib.orc_pv_rows.restype = None
        lib.orc_pv_rows.argtypes = [vp, i64, i32, i64, i64, vp, i32, vp]
        _lib = lib
    return _lib


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


# --------------------------------------------------------------------------- forest growth
def draw(seed: int, tree: int, a: int, b: int) -> int:
    """The counter-based 64-bit draw that the growth uses (see grow_core.c)."""
    return int(_grow().orc_draw(seed, tree, a, b))


def grow(X, y, n_classes: int, n_trees: int, mtry: int, seed: int, first_tree: int = 0):
    """Grows trees first_tree .. first_tree + n_trees - 1 to purity (Methodology: bootstrap sample,
    mtry random features per node, best Gini decrease over the values present in the node; the open
    points are fixed in grow_core.c's header).  Returns a dict of flat arrays: node_offset [B+1],
    feature, threshold, left, right, leaf_id, depth [nodes], n_leaves [B], inbag uint16 [B][N],
    train_leaf [B][N], leaf_class [B][max leaves]."""
    lib = _grow()
    X = _c(X, np.float32)
    y = _c(y, np.int32)
    N, M = X.shape
    h = lib.orc_grow(X.ctypes.data, N, M, y.ctypes.data, n_classes, first_tree, n_trees, mtry, seed)
    if not h:
        raise ValueError("orc_grow rejected its arguments")
    try:
        nn = lib.orc_grown_total_nodes(h)
        ml = lib.orc_grown_max_leaves(h)
        out = dict(node_offset=np.empty(n_trees + 1, np.int64), feature=np.empty(nn, np.int32),
                   threshold=np.empty(nn, np.float32), left=np.empty(nn, np.int32), right=np.empty(nn, np.int32),
                   leaf_id=np.empty(nn, np.int32), depth=np.empty(nn, np.int32), n_leaves=np.empty(n_trees, np.int32),
                   inbag=np.empty((n_trees, N), np.uint16), train_leaf=np.empty((n_trees, N), np.int32),
                   leaf_class=np.empty((n_trees, ml), np.int32))
        lib.orc_grown_export(h, *(out[k].ctypes.data for k in ("node_offset", "feature", "threshold", "left", "right",
                                                               "leaf_id", "depth", "n_leaves", "inbag", "train_leaf",
                                                               "leaf_class")))
    finally:
        lib.orc_grown_free(h)
    out["n_trees"], out["n_features"] = n_trees, M
    return out


# --------------------------------------------------------------------------- a1: leaf assignment
def leaf_assign(forest, X) -> Tuple[np.ndarray, int]:
    """Terminal node of every row of X in every tree (Methodology, "Threshold-based Splits":
    x <= tau goes left, x > tau goes right; every sample, in-bag or not, is dropped down every tree).

    Returns (leaf uint32 [B][N], summed path length over all (tree, row) pairs).
    """
    X = _c(X, np.float32)
    N, M = X.shape
    assert M == forest.n_features
    B = forest.n_trees
    leaf = np.empty((B, N), np.uint32)
    plen = ctypes.c_int64(0)
    rc = _core().orc_leaf_assign(B, _c(forest.node_offset, np.int64).ctypes.data,
                                 _c(forest.feature, np.int32).ctypes.data,
                                 _c(forest.threshold, np.float32).ctypes.data,
                                 _c(forest.left, np.int32).ctypes.data, _c(forest.right, np.int32).ctypes.data,
                                 _c(forest.leaf_id, np.int32).ctypes.data, X.ctypes.data, N, M, leaf.ctypes.data,
                                 ctypes.addressof(plen))
    if rc != 0:
        raise ValueError("malformed forest: a walk left its tree")
    return leaf, int(plen.value)


# --------------------------------------------------------------------------- a2-a4: counts and proximities
def counts_rows(leaf, i0: int, i1: int) -> np.ndarray:
    """Rows i0..i1-1 of cnt(i,j) = #{b : node_b(i) = node_b(j)} (proximity equation, numerator)."""
    leaf = _c(leaf, np.uint32)
    B, N = leaf.shape
    out = np.empty((i1 - i0, N), np.uint32)
    _core().orc_counts_rows(leaf.ctypes.data, N, B, i0, i1, out.ctypes.data)
    return out


def counts_full(leaf) -> np.ndarray:
    return counts_rows(leaf, 0, leaf.shape[1])


def oob_rows(leaf, inbag, i0: int, i1: int) -> Tuple[np.ndarray, np.ndarray]:
    """Rows i0..i1-1 of the out-of-bag-only numerator and denominator ("Case-wise Bootstrap Tracking":
    OOB_i is the set of trees whose bootstrap sample misses i; both samples must be out-of-bag)."""
    leaf = _c(leaf, np.uint32)
    inbag = _c(inbag, np.uint16)
    B, N = leaf.shape
    assert inbag.shape == (B, N)
    num = np.empty((i1 - i0, N), np.uint32)
    den = np.empty((i1 - i0, N), np.uint32)
    _core().orc_oob_rows(leaf.ctypes.data, inbag.ctypes.data, N, B, i0, i1, num.ctypes.data, den.ctypes.data)
    return num, den


def normalise(cnt, B: int) -> np.ndarray:
    """p = cnt / B in float32 IEEE division (proximity equation)."""
    return (cnt.astype(np.float32) / np.float32(B)).astype(np.float32)


def prox_oob_rows(num, den, i0: int) -> np.ndarray:
    """Out-of-bag proximity rows: num/den in float32, 0 where no tree has both samples out-of-bag,
    and 1 on the diagonal (row r of the block is sample i0 + r)."""
    p = np.zeros(num.shape, np.float32)
    m = den > 0
    p[m] = num[m].astype(np.float32) / den[m].astype(np.float32)
    r = np.arange(num.shape[0])
    p[r, i0 + r] = np.float32(1.0)
    return p


def pack_upper(full) -> np.ndarray:
    """Strict upper triangle, row-major: idx(i,j) = i*N - i(i+1)/2 + (j-i-1) for i < j
    (n(n-1)/2 elements, "Packed Upper Triangle Storage")."""
    N = full.shape[0]
    iu = np.triu_indices(N, 1)
    return np.ascontiguousarray(full[iu])


def sparse_upper(leaf, min_count: int = 1, i0: int = 0, i1: int = None):
    """Thresholded strict upper triangle as coordinate triplets ("CPU TriBlock Proximity": only pairs
    i < j are kept, and only those whose proximity reaches the threshold; the threshold is given as
    a count, p >= tau <=> cnt >= ceil(tau B), so the kept set is decided in integers).

    Returns (rows, cols, counts) of all pairs i0 <= i < i1, i < j with cnt(i,j) >= min_count, ordered
    by (i, j); counts are exact.  Computed row block by row block from the pair-by-pair counts."""
    leaf = _c(leaf, np.uint32)
    B, N = leaf.shape
    i1 = N if i1 is None else i1
    rows, cols, vals = [], [], []
    for r0 in range(i0, i1, 256):
        r1 = min(r0 + 256, i1)
        cnt = counts_rows(leaf, r0, r1)
        for i in range(r0, r1):
            c = cnt[i - r0, i + 1:]
            j = np.nonzero(c >= min_count)[0]
            rows.append(np.full(j.size, i, np.int64))
            cols.append(j + i + 1)
            vals.append(c[j])
    cat = lambda parts, dt: np.concatenate(parts).astype(dt) if parts else np.zeros(0, dt)
    return cat(rows, np.int64), cat(cols, np.int64), cat(vals, np.uint32)


# --------------------------------------------------------------------------- proximity consumers
def outlier_printed(cnt, B: int, rows=None) -> np.ndarray:
    """Case-wise outlier measure as the paper prints it ("Case-wise Proximity"):
    (1/(n-1)) sum_{j != i} 1 / p(i,j)^2, p = cnt / B in float64.  The term of a pair with p = 0 is
    undefined; such pairs are skipped (they are the implicit zeros of the paper's sparse storage).
    `cnt` holds the count rows of the samples `rows` (all samples, in order, when None)."""
    cnt = np.asarray(cnt)
    n = cnt.shape[1]
    rows = range(cnt.shape[0]) if rows is None else rows
    out = np.zeros(len(rows), np.float64)
    for r, i in enumerate(rows):
        for j in range(n):
            if j != i and cnt[r, j] > 0:
                p = float(cnt[r, j]) / float(B)
                out[r] += 1.0 / (p * p)
        out[r] /= (n - 1)
    return out


def outlier_classic(cnt, B: int, labels=None, rows=None) -> np.ndarray:
    """Breiman and Cutler's raw outlier measure, which the paper's section builds on: n divided by the
    sum of squared proximities to the other samples of the same class (all other samples when no
    labels are given).  A sample with no proximity to any of them gets +inf.  `cnt`, `rows` as in
    outlier_printed."""
    cnt = np.asarray(cnt)
    n = cnt.shape[1]
    rows = range(cnt.shape[0]) if rows is None else rows
    out = np.empty(len(rows), np.float64)
    for r, i in enumerate(rows):
        s = 0.0
        for j in range(n):
            if j != i and (labels is None or labels[j] == labels[i]):
                p = float(cnt[r, j]) / float(B)
                s += p * p
        out[r] = float(n) / s if s > 0 else np.inf
    return out


def oob_vote(leaf, inbag, leaf_class, n_classes: int):
    """Out-of-bag votes and prediction ("OOB Error Estimation"): for sample i only the trees whose
    bootstrap sample missed i vote, each with the class of the leaf i falls in; the prediction is the
    class with most votes (lowest class on ties), -1 for a sample that was never out-of-bag.
    Returns (votes uint32 [N][C], pred int32 [N])."""
    leaf = np.asarray(leaf)
    B, N = leaf.shape
    votes = np.zeros((N, n_classes), np.uint32)
    for b in range(B):
        for i in range(N):
            if inbag[b, i] == 0:
                votes[i, leaf_class[b, leaf[b, i]]] += 1
    pred = np.where(votes.sum(axis=1) > 0, votes.argmax(axis=1), -1).astype(np.int32)
    return votes, pred


def oob_error(pred, y):
    """(wrong, voted): samples whose out-of-bag prediction differs from the label, and samples that
    have a prediction; the error rate is wrong / voted (= the paper's (1/n) sum when every sample
    was out-of-bag at least once)."""
    pred = np.asarray(pred)
    voted = pred >= 0
    return int((pred[voted] != np.asarray(y)[voted]).sum()), int(voted.sum())


# --------------------------------------------------------------------------- a5: products
def pv_implicit(leaf, V) -> np.ndarray:
    """Y = P V = (1/B) sum_b Z_b (Z_b^T V) in float64 without forming P."""
    leaf = _c(leaf, np.uint32)
    V = _c(V, np.float64)
    B, N = leaf.shape
    assert V.shape[0] == N
    Y = np.empty_like(V)
    rc = _core().orc_pv_implicit(leaf.ctypes.data, N, B, int(leaf.max()) + 1, V.ctypes.data, V.shape[1],
                                 Y.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"orc_pv_implicit failed ({rc})")
    return Y


def pv_rows(leaf, V, i0: int, i1: int) -> np.ndarray:
    """Rows i0..i1-1 of the dense product (1/B) sum_j cnt(i,j) V[j,:] in float64."""
    leaf = _c(leaf, np.uint32)
    V = _c(V, np.float64)
    B, N = leaf.shape
    Y = np.empty((i1 - i0, V.shape[1]), np.float64)
    _core().orc_pv_rows(leaf.ctypes.data, N, B, i0, i1, V.ctypes.data, V.shape[1], Y.ctypes.data)
    return Y


# --------------------------------------------------------------------------- a6: block power iteration
def fix_signs(V) -> np.ndarray:
    """Makes the largest-magnitude entry of every column positive."""
    V = np.array(V, copy=True)
    idx = np.argmax(np.abs(V), axis=0)
    s = np.sign(V[idx, np.arange(V.shape[1])])
    s[s == 0] = 1.0
    return V * s


def block_iteration(leaf, V0, T: int, progress=None) -> Tuple[np.ndarray, np.ndarray]:
    """Top-k eigenpairs of P by block power iteration with exactly T applications of P, float64.

    V <- orth(V0); T-1 times V <- orth(P V); then Y = P V, H = sym(V^T Y), H = W diag(theta) W^T
    (descending), V <- V W.  orth is Householder QR.  P is symmetric positive semi-definite (a sum of
    Gram matrices Z_b Z_b^T), so P ~ V diag(theta) V^T is the symmetric form of the paper's
    low-rank factorisation P ~ Q U^T with Q = U = V diag(sqrt(theta)).
    Returns (theta [k] descending, V [N][k]) with the sign convention of fix_signs.
    `progress`, if given, is called with the number of applications done after each one (long runs
    report their own steps); it takes no part in the arithmetic.
    """
    V, _ = np.linalg.qr(np.asarray(V0, np.float64))
    for t in range(T - 1):
        V, _ = np.linalg.qr(pv_implicit(leaf, V))
        if progress:
            progress(t + 1)
    Y = pv_implicit(leaf, V)
    if progress:
        progress(T)
    H = V.T @ Y
    H = 0.5 * (H + H.T)
    theta, W = np.linalg.eigh(H)
    order = np.argsort(theta)[::-1]
    return theta[order], fix_signs(V @ W[:, order])


def dense_eig(P, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Top-k eigenpairs of a materialised symmetric P by LAPACK (descending)."""
    import scipy.linalg as sla
    P = np.asarray(P, np.float64)
    n = P.shape[0]
    lam, U = sla.eigh(P, subset_by_index=[n - k, n - 1])
    return lam[::-1].copy(), fix_signs(U[:, ::-1])


def implicit_eig(leaf, k: int, tol: float = 1e-12, seed: int = 4243) -> Tuple[np.ndarray, np.ndarray]:
    """Top-k eigenpairs of P (descending) from the float64 implicit operator with ARPACK, for N too large to
    materialise P; the dense eigendecomposition is the definition, this is the same spectrum to `tol`."""
    import scipy.sparse.linalg as spla
    leaf = np.asarray(leaf)
    n = leaf.shape[1]

    def mv(v):
        return pv_implicit(leaf, np.asarray(v, np.float64).reshape(n, -1)).reshape(np.shape(v))

    L = spla.LinearOperator((n, n), matvec=mv, matmat=mv, dtype=np.float64)
    rng = np.random.default_rng(seed)
    lam, U = spla.eigsh(L, k=k, which="LA", tol=tol, v0=rng.standard_normal(n))
    order = np.argsort(lam)[::-1]
    return lam[order], fix_signs(U[:, order])


def principal_angle(U, V) -> float:
    """Largest principal angle (rad) between the column spans of U and V."""
    Qu, _ = np.linalg.qr(np.asarray(U, np.float64))
    Qv, _ = np.linalg.qr(np.asarray(V, np.float64))
    # sin of the largest angle = norm of the part of Qu outside span(Qv); accurate for small angles
    R = Qu - Qv @ (Qv.T @ Qu)
    s = np.linalg.svd(R, compute_uv=False)
    return float(np.arcsin(min(1.0, s[0])))


# --------------------------------------------------------------------------- a7: INT8 factors
def quantise_int8(V, lam) -> Tuple[np.ndarray, np.ndarray]:
    """Per-column symmetric INT8 codes of A = V diag(sqrt(lam)), all arithmetic in float32.

    s_c = max_i |A_ic| / 127 (1 for an all-zero column); q = clamp(round-half-even(A / s_c), -127, 127).
    The paper only names the encoding "INT8 (8-bit)" ("Low-Rank Factorization and Quantization
    Trade-offs"); the per-column absmax scheme is this build's reading.
    """
    V = np.asarray(V, np.float32)
    lam = np.asarray(lam, np.float32)
    A = (V * np.sqrt(np.maximum(lam, np.float32(0.0)))[None, :]).astype(np.float32)
    amax = np.max(np.abs(A), axis=0).astype(np.float32)
    s = np.where(amax > 0, amax / np.float32(127.0), np.float32(1.0)).astype(np.float32)
    q = np.rint((A / s[None, :]).astype(np.float32))
    return np.clip(q, -127, 127).astype(np.int8), s


def dequantise(Q, s) -> np.ndarray:
    return Q.astype(np.float64) * np.asarray(s, np.float64)[None, :]


# --------------------------------------------------------------------------- a8: 3-D MDS from the factors
def double_centre(D2) -> np.ndarray:
    """G = -1/2 H D2 H with H = I - 11^T/n (paper, MDS Step 2)."""
    D2 = np.asarray(D2, np.float64)
    n = D2.shape[0]
    H = np.eye(n) - np.full((n, n), 1.0 / n)
    return -0.5 * (H @ D2 @ H)


def mds_gram_dense(A, mode: int = SQUARED) -> np.ndarray:
    """Gram matrix of the scaling from P^ = A A^T (paper, MDS Steps 1-2).

    D = max P - P with max P read as 1 (an exact proximity matrix has unit diagonal); SQUARED takes
    D2 = D o D as the paper does, LINEAR takes D2 = D.
    """
    A = np.asarray(A, np.float64)
    D = 1.0 - A @ A.T
    return double_centre(D * D if mode == SQUARED else D)


def mds_operator(A, mode: int = SQUARED):
    """v -> G v in float64 using only the factor A (paper, MDS Step 3: u = H v, z = D2 u, w = H z,
    G v = -w/2).  With p_ij = a_i . a_j and sum(u) = 0:
    SQUARED: (1 - p)^2 = 1 - 2p + p^2, so z = -2 A (A^T u) + rowquad(A, A^T diag(u) A);
    LINEAR:  z = -A (A^T u)."""
    A = np.asarray(A, np.float64)

    def apply(v):
        v = np.asarray(v, np.float64)
        u = v - v.mean(axis=0)
        if mode == SQUARED:
            if u.ndim == 1:
                Mq = A.T @ (u[:, None] * A)
                z = -2.0 * (A @ (A.T @ u)) + np.einsum("ik,kl,il->i", A, Mq, A)
            else:
                z = np.stack([-2.0 * (A @ (A.T @ u[:, c])) +
                              np.einsum("ik,kl,il->i", A, A.T @ (u[:, c, None] * A), A)
                              for c in range(u.shape[1])], axis=1)
        else:
            z = -(A @ (A.T @ u))
        w = z - z.mean(axis=0)
        return -0.5 * w

    return apply


def mds3d_dense(Q, s, mode: int = SQUARED, dims: int = 3) -> Tuple[np.ndarray, np.ndarray]:
    """Classical (Torgerson) scaling from the INT8 factors: top `dims` eigenpairs of G by algebraic
    value via LAPACK, coordinates x_i = sqrt(max(lam,0)) v_i (paper, MDS Step 4).  Small N only."""
    G = mds_gram_dense(dequantise(Q, s), mode)
    lam, U = np.linalg.eigh(0.5 * (G + G.T))
    lam = lam[::-1][:dims].copy()
    U = fix_signs(U[:, ::-1][:, :dims])
    return U * np.sqrt(np.maximum(lam, 0.0))[None, :], lam


def mds3d_implicit(Q, s, mode: int = SQUARED, dims: int = 3, tol: float = 1e-12) -> Tuple[np.ndarray, np.ndarray]:
    """Same eigenpairs from the float64 implicit operator with ARPACK; for N too large to form G."""
    import scipy.sparse.linalg as spla
    A = dequantise(Q, s)
    n = A.shape[0]
    op = mds_operator(A, mode)
    L = spla.LinearOperator((n, n), matvec=op, matmat=op, dtype=np.float64)
    rng = np.random.default_rng(4242)
    lam, U = spla.eigsh(L, k=dims, which="LA", tol=tol, v0=rng.standard_normal(n))
    order = np.argsort(lam)[::-1]
    lam = lam[order]
    U = fix_signs(U[:, order])
    return U * np.sqrt(np.maximum(lam, 0.0))[None, :], lam


# --------------------------------------------------------------------------- other factor encodings
# The paper lists four precisions for the low-rank factors: NF4 (4-bit), INT8, FP16 and FP32
# ("Low-Rank Factorization and Quantization Trade-offs").  INT8 is quantise_int8 above.  FP16 and
# FP32 store A = V diag(sqrt(lam)) rounded to nearest-even.  NF4 is the 4-bit NormalFloat type of
# the QLoRA paper the RFX paper cites: 16 fixed levels in [-1, 1] applied to values normalised by
# the absolute maximum of their block; this build's reading takes blocks of 64 consecutive rows of
# one column (the per-column scaling of the INT8 reading, refined to blocks), two codes per byte
# (even row in the low nibble), and decides "nearest level" in float32 by counting the midpoints
# between adjacent levels that lie below the normalised value.
ENC_INT8, ENC_FP16, ENC_NF4, ENC_FP32 = 0, 1, 2, 3
NF4_BLOCK = 64
NF4_LEVELS = np.array([-1.0, -0.6961928009986877, -0.5250730514526367, -0.39491748809814453,
                       -0.28444138169288635, -0.18477343022823334, -0.09105003625154495, 0.0,
                       0.07958029955625534, 0.16093020141124725, 0.24611230194568634, 0.33791524171829224,
                       0.44070982933044434, 0.5626170039176941, 0.7229568362236023, 1.0], dtype=np.float32)


def _factor(V, lam) -> np.ndarray:
    V = np.asarray(V, np.float32)
    lam = np.asarray(lam, np.float32)
    return (V * np.sqrt(np.maximum(lam, np.float32(0.0)))[None, :]).astype(np.float32)


def quantise_factor(V, lam, encoding: int):
    """Returns (codes, scales) of A = V diag(sqrt(lam)) in the given encoding (float32 arithmetic).

    INT8: int8 [N][k], scales float32 [k].  FP16: float16 [N][k], no scales.  FP32: float32 [N][k].
    NF4: uint8 [ceil(N/2)][k] (rows 2i and 2i+1 in the low and high nibble; a missing last row is the
    zero level), scales float32 [ceil(N/64)][k] = block maxima of |A| (1 for an all-zero block).
    """
    if encoding == ENC_INT8:
        return quantise_int8(V, lam)
    A = _factor(V, lam)
    N, k = A.shape
    if encoding == ENC_FP32:
        return A, np.zeros(0, np.float32)
    if encoding == ENC_FP16:
        return A.astype(np.float16), np.zeros(0, np.float32)
    if encoding != ENC_NF4:
        raise ValueError("unknown encoding")
    nb = (N + NF4_BLOCK - 1) // NF4_BLOCK
    pad = np.zeros((nb * NF4_BLOCK, k), np.float32)
    pad[:N] = A
    blocks = pad.reshape(nb, NF4_BLOCK, k)
    amax = np.abs(blocks).max(axis=1).astype(np.float32)
    scales = np.where(amax > 0, amax, np.float32(1.0)).astype(np.float32)
    x = (blocks / scales[:, None, :]).astype(np.float32).reshape(nb * NF4_BLOCK, k)[:N]
    mid = ((NF4_LEVELS[:-1] + NF4_LEVELS[1:]) * np.float32(0.5)).astype(np.float32)
    code = (x[:, :, None] > mid[None, None, :]).sum(axis=2).astype(np.uint8)
    if N % 2:
        code = np.concatenate([code, np.full((1, k), 7, np.uint8)], axis=0)
    packed = (code[0::2] | (code[1::2] << 4)).astype(np.uint8)
    return packed, scales


def dequantise_factor(codes, scales, encoding: int, N: int) -> np.ndarray:
    """float32 [N][k] factor represented by (codes, scales)."""
    if encoding == ENC_INT8:
        return (codes.astype(np.float32) * np.asarray(scales, np.float32)[None, :]).astype(np.float32)
    if encoding in (ENC_FP16, ENC_FP32):
        return codes.astype(np.float32)
    k = codes.shape[1]
    code = np.empty((2 * codes.shape[0], k), np.uint8)
    code[0::2] = codes & 0xF
    code[1::2] = codes >> 4
    vals = NF4_LEVELS[code[:N]]
    s = np.repeat(np.asarray(scales, np.float32), NF4_BLOCK, axis=0)[:N]
    return (vals * s).astype(np.float32)


def mds3d_from_factor(A, mode: int = SQUARED, dims: int = 3):
    """Dense Torgerson scaling from a float factor A (P^ = A A^T).  Small N only."""
    G = mds_gram_dense(np.asarray(A, np.float64), mode)
    lam, U = np.linalg.eigh(0.5 * (G + G.T))
    lam = lam[::-1][:dims].copy()
    U = fix_signs(U[:, ::-1][:, :dims])
    return U * np.sqrt(np.maximum(lam, 0.0))[None, :], lam


def mds3d_from_dense_proximity(P, mode: int = SQUARED, dims: int = 3):
    """Torgerson scaling of the full proximity matrix (the paper's "CPU full matrix" pathway)."""
    P = np.asarray(P, np.float64)
    D = 1.0 - P
    G = double_centre(D * D if mode == SQUARED else D)
    lam, U = np.linalg.eigh(0.5 * (G + G.T))
    lam = lam[::-1][:dims].copy()
    U = fix_signs(U[:, ::-1][:, :dims])
    return U * np.sqrt(np.maximum(lam, 0.0))[None, :], lam


def mds_correlation(X1, X2, max_pairs: int = 2_000_000, seed: int = 0) -> float:
    """Pearson correlation between the pairwise Euclidean distances of two embeddings (invariant to
    rotation, reflection and translation).  This is this build's reading of the paper's "MDS
    correlation" between compressed and full-matrix embeddings, which the paper does not define."""
    X1 = np.asarray(X1, np.float64)
    X2 = np.asarray(X2, np.float64)
    n = X1.shape[0]
    rng = np.random.default_rng(seed)
    if n * (n - 1) // 2 <= max_pairs:
        i, j = np.triu_indices(n, 1)
    else:
        i = rng.integers(0, n, size=max_pairs)
        j = rng.integers(0, n, size=max_pairs)
        keep = i != j
        i, j = i[keep], j[keep]
    d1 = np.linalg.norm(X1[i] - X1[j], axis=1)
    d2 = np.linalg.norm(X2[i] - X2[j], axis=1)
    return float(np.corrcoef(d1, d2)[0, 1])
