import sys
from pathlib import Path

import numpy as np
import pytest

ROOT = Path(__file__).resolve().parents[1]
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def cfg1():
    """Workload 1 (178 x 13, 3 classes, 100 trees) with its grown forest and oracle leaf ids."""
    import oracle
    import rfx_inputs as ri

    c = ri.CONFIGS[1]
    X, y, F = ri.load_or_grow(c, use_cache=False)
    leaf, plen = oracle.leaf_assign(F, X)
    return dict(c=c, X=X, y=y, F=F, leaf=leaf, path_len=plen)


@pytest.fixture(scope="session")
def small2():
    """Reduced workload 2 (1,500 x 20, 5 classes, 10 % label noise, 64 trees)."""
    import oracle
    import rfx_inputs as ri

    c = ri.CONFIGS[2]
    X, y, F = ri.load_or_grow(c, N=1500, B=64, use_cache=False)
    leaf, plen = oracle.leaf_assign(F, X)
    return dict(c=c, X=X, y=y, F=F, leaf=leaf, path_len=plen)


def brute_counts(leaf):
    """Pure-Python triple loop over (i, j, b)."""
    B, N = leaf.shape
    out = np.zeros((N, N), np.uint32)
    L = leaf.tolist()
    for i in range(N):
        for j in range(N):
            c = 0
            for b in range(B):
                if L[b][i] == L[b][j]:
                    c += 1
            out[i, j] = c
    return out


def converged_prefix(lam, V, lam_ref, U_ref, rtol=1e-4, angle=1e-3):
    """The reported layer of the eigen check: the longest prefix j of Ritz pairs (lam, V) whose values are all
    within rtol (relative) of the reference eigenvalues and whose j-dimensional span is within `angle` radians
    of the span of the first j reference eigenvectors; and the residuals |P v - lam v| / lam cannot be formed
    here (no P), so the caller adds them.  Returns j (0 if not even the leading pair qualifies)."""
    import oracle
    kk = min(len(lam), len(lam_ref))
    rel = np.abs(np.asarray(lam[:kk], np.float64) - lam_ref[:kk]) / np.abs(lam_ref[:kk])
    j = 0
    while j < kk and rel[j] <= rtol:
        j += 1
    while j > 0 and oracle.principal_angle(V[:, :j], U_ref[:, :j]) >= angle:
        j -= 1
    return j
