"""Gaussian-mixture sample matrices and random start blocks (seeded, synthetic)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import numpy as np

DATA_SEED_BASE = 20251119
FOREST_ISEED = 12345
START_SEED = 777


@dataclass(frozen=True)
class WorkloadConfig:
    """One synthetic workload: data shape, class structure, forest and rank."""

    cfg: int
    N: int
    M: int
    C: int
    B: int
    mtry: int
    mean_sd: float                      # class means ~ N(0, mean_sd^2) per feature
    var_range: Optional[Tuple[float, float]] = None  # per-class diagonal variances ~ U(a, b); None = unit
    label_noise: float = 0.0            # fraction of labels flipped to a different class
    class_sizes: Optional[Sequence[int]] = None      # None = balanced
    k: int = 0                          # rank of the low-rank factorisation (0 = not used)
    T: int = 0                          # applications of P in the block iteration

    @property
    def data_seed(self) -> int:
        return DATA_SEED_BASE + self.cfg


CONFIGS = {
    1: WorkloadConfig(1, 178, 13, 3, 100, 3, 2.0, class_sizes=(59, 71, 48), k=16, T=20),
    2: WorkloadConfig(2, 10_000, 20, 5, 500, 4, 1.5, label_noise=0.10, k=32, T=20),
    3: WorkloadConfig(3, 50_000, 50, 10, 500, 7, 1.0, var_range=(0.5, 2.0), k=32, T=20),
    4: WorkloadConfig(4, 100_000, 100, 10, 1000, 10, 1.0, var_range=(0.5, 2.0), k=64, T=20),
    5: WorkloadConfig(5, 500_000, 64, 20, 1000, 8, 1.0, label_noise=0.05, k=64, T=20),
}


def gaussian_mixture(c: WorkloadConfig, N: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (X float32 [N][M] row-major, y int32 [N]) for a workload.

    x = mu_c + sigma_c * eps with eps ~ N(0, I) drawn in float64 and rounded to
    float32; rows are randomly permuted; label noise replaces a label by a
    uniformly drawn different class.  `N` overrides the row count (class
    proportions kept) for reduced-size test cases.
    """
    rng = np.random.default_rng(c.data_seed)
    n = c.N if N is None else int(N)
    if c.class_sizes is not None and N is None:
        sizes = np.asarray(c.class_sizes, dtype=np.int64)
    else:
        frac = (np.asarray(c.class_sizes, dtype=np.float64) / sum(c.class_sizes)
                if c.class_sizes is not None else np.full(c.C, 1.0 / c.C))
        sizes = np.floor(frac * n).astype(np.int64)
        sizes[: n - int(sizes.sum())] += 1
    assert int(sizes.sum()) == n
    mu = rng.normal(0.0, c.mean_sd, size=(c.C, c.M))
    if c.var_range is None:
        sd = np.ones((c.C, c.M))
    else:
        sd = np.sqrt(rng.uniform(c.var_range[0], c.var_range[1], size=(c.C, c.M)))
    y = np.repeat(np.arange(c.C, dtype=np.int32), sizes)
    X = np.empty((n, c.M), dtype=np.float32)
    step = 1 << 16
    for s in range(0, n, step):
        ys = y[s:s + step]
        eps = rng.standard_normal((len(ys), c.M))
        X[s:s + step] = (mu[ys] + sd[ys] * eps).astype(np.float32)
    if c.label_noise > 0.0:
        flip = rng.random(n) < c.label_noise
        shift = rng.integers(1, c.C, size=n).astype(np.int32)
        y = np.where(flip, (y + shift) % c.C, y).astype(np.int32)
    perm = rng.permutation(n)
    return np.ascontiguousarray(X[perm]), np.ascontiguousarray(y[perm])


def start_block(N: int, k: int, seed: int = START_SEED) -> np.ndarray:
    """iid N(0,1) float32 [N][k] start block for the block iterations."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal((N, k)).astype(np.float32)


def random_int8_factor(N: int, k: int, spread: float, seed: int):
    """A synthetic INT8 factor that is not a proximity factor: codes round(127 z / max|z|) of iid N(0,1) draws z
    per column and scales spread * max|z| / 127, so that the rows of Q diag(scales) are about N(0, spread^2 I).
    With a spread of 1 or more the element-wise square of P^ = A A^T outweighs P^ itself, which makes the
    squared-dissimilarity Gram matrix of the scaling step strongly indefinite: the case a solver that
    converges to the largest magnitudes gets wrong.  Returns (Q int8 [N][k], scales float32 [k])."""
    rng = np.random.default_rng(seed)
    z = rng.standard_normal((N, k))
    top = np.abs(z).max(axis=0)
    Q = np.rint(127.0 * z / top[None, :]).astype(np.int8)
    scales = (spread * top / 127.0).astype(np.float32)
    return Q, scales


def workload(cfg: int) -> WorkloadConfig:
    return CONFIGS[cfg]
