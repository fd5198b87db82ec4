"""Pins for the oracle's products, block iteration, INT8 factors and 3-D scaling."""
import numpy as np
import pytest

import oracle
import rfx_inputs as ri


def test_implicit_product_equals_dense_product(cfg1, small2):
    for d, k in ((cfg1, 5), (small2, 8)):
        leaf = d["leaf"]
        B, N = leaf.shape
        V = ri.start_block(N, k).astype(np.float64)
        P = oracle.counts_full(leaf).astype(np.float64) / B
        ref = P @ V                                            # library product on the materialised matrix
        Y = oracle.pv_implicit(leaf, V)
        np.testing.assert_allclose(Y, ref, rtol=0, atol=1e-12 * np.abs(ref).max())
        rows = oracle.pv_rows(leaf, V, 10, 25)
        np.testing.assert_allclose(rows, ref[10:25], rtol=0, atol=1e-12 * np.abs(ref).max())


def test_product_with_ones_is_the_leaf_size_sum(small2):
    """B * (P 1)_i = sum_b |leaf_b(i)|, an exact integer."""
    leaf = small2["leaf"]
    B, N = leaf.shape
    Y = oracle.pv_implicit(leaf, np.ones((N, 1)))
    sizes = np.zeros(N, np.int64)
    for b in range(B):
        sizes += np.bincount(leaf[b])[leaf[b]]
    np.testing.assert_array_equal(np.rint(Y[:, 0] * B).astype(np.int64), sizes)
    assert np.abs(Y[:, 0] * B - sizes).max() < 1e-7


def test_product_is_linear_symmetric_psd(cfg1):
    leaf = cfg1["leaf"]
    N = leaf.shape[1]
    rng = np.random.default_rng(5)
    u, v = rng.standard_normal((N, 1)), rng.standard_normal((N, 1))
    Pu, Pv = oracle.pv_implicit(leaf, u), oracle.pv_implicit(leaf, v)
    np.testing.assert_allclose(oracle.pv_implicit(leaf, 2 * u - 3 * v), 2 * Pu - 3 * Pv, atol=1e-12)
    assert float((u * Pv).sum()) == pytest.approx(float((Pu * v).sum()), rel=1e-12)
    assert float((v * Pv).sum()) >= 0.0


def test_block_iteration_converges_to_lapack(cfg1):
    leaf = cfg1["leaf"]
    B, N = leaf.shape
    P = oracle.counts_full(leaf).astype(np.float64) / B
    lam_all = np.linalg.eigvalsh(P)[::-1]
    assert lam_all.sum() == pytest.approx(N, rel=1e-12)            # trace P = N
    assert lam_all.min() > -1e-10                                   # P is positive semi-definite
    assert lam_all[0] <= P.sum(axis=1).max() + 1e-9
    assert (lam_all ** 2).sum() == pytest.approx((P ** 2).sum(), rel=1e-12)

    k = 8
    lam_d, U_d = oracle.dense_eig(P, k)
    np.testing.assert_allclose(lam_d, lam_all[:k], rtol=1e-12)
    # enough applications of P that the leading three pairs have converged
    lam, V = oracle.block_iteration(leaf, ri.start_block(N, k), T=60)
    np.testing.assert_allclose(V.T @ V, np.eye(k), atol=1e-12)
    np.testing.assert_allclose(lam[:3], lam_d[:3], rtol=1e-9)
    assert oracle.principal_angle(V[:, :3], U_d[:, :3]) < 1e-4
    assert (lam <= lam_d + 1e-10).all()                              # Ritz values never exceed eigenvalues
    # a full-width block spans everything: Ritz values are the spectrum after one application
    lam_f, _ = oracle.block_iteration(leaf, ri.start_block(N, N), T=1)
    np.testing.assert_allclose(lam_f, lam_all, atol=1e-10)


def test_block_iteration_counts_applications(monkeypatch, cfg1):
    calls = []
    real = oracle.pv_implicit
    monkeypatch.setattr(oracle, "pv_implicit", lambda l, v: calls.append(1) or real(l, v))
    oracle.block_iteration(cfg1["leaf"], ri.start_block(178, 4), T=5)
    assert len(calls) == 5


def test_principal_angle():
    e = np.eye(4)
    assert oracle.principal_angle(e[:, :2], e[:, :2] @ np.array([[0, 1], [1, 0.0]])) < 1e-12
    t = 1e-4
    U = np.stack([e[:, 0], np.cos(t) * e[:, 1] + np.sin(t) * e[:, 2]], axis=1)
    assert oracle.principal_angle(e[:, :2], U) == pytest.approx(t, rel=1e-6)
    assert oracle.principal_angle(e[:, :1], e[:, 1:2]) == pytest.approx(np.pi / 2)


def test_int8_quantisation():
    # ties go to the even code; the column maximum maps to +-127
    V = np.array([[127.0, -2.0], [0.5, 1.0], [1.5, 0.25], [2.5, 0.0], [-0.5, 0.5], [-3.5, 2.0]], np.float32)
    Q, s = oracle.quantise_int8(V, np.ones(2, np.float32))
    assert s[0] == np.float32(1.0) and s[1] == np.float32(2.0) / np.float32(127.0)
    np.testing.assert_array_equal(Q[:, 0], [127, 0, 2, 2, 0, -4])
    assert Q[0, 1] == -127 and Q[5, 1] == 127
    # eigenvalue scaling: A = V sqrt(lam)
    Q2, s2 = oracle.quantise_int8(V, np.array([4.0, 0.0], np.float32))
    assert s2[0] == np.float32(2.0) and s2[1] == np.float32(1.0) and (Q2[:, 1] == 0).all()
    np.testing.assert_array_equal(Q2[:, 0], Q[:, 0])

    rng = np.random.default_rng(9)
    V = rng.standard_normal((1000, 6)).astype(np.float32)
    lam = rng.uniform(0.1, 50, 6).astype(np.float32)
    Q, s = oracle.quantise_int8(V, lam)
    A = V.astype(np.float64) * np.sqrt(lam.astype(np.float64))
    assert Q.dtype == np.int8 and (np.abs(Q).max(axis=0) == 127).all()
    assert (np.abs(oracle.dequantise(Q, s) - A) <= 0.5 * s * (1 + 1e-5)).all()


def test_double_centring_recovers_a_euclidean_configuration():
    """Torgerson scaling: for squared Euclidean distances, -1/2 H D2 H is the Gram matrix of the
    centred points, and the embedding reproduces every pairwise distance."""
    rng = np.random.default_rng(2)
    Xp = rng.standard_normal((40, 3)) * [3.0, 2.0, 0.5]
    D2 = ((Xp[:, None] - Xp[None]) ** 2).sum(-1)
    G = oracle.double_centre(D2)
    Xc = Xp - Xp.mean(0)
    np.testing.assert_allclose(G, Xc @ Xc.T, atol=1e-10)


def test_mds_linear_mode_embeds_factor_rows():
    # LINEAR: G = 1/2 H A A^T H = 1/2 (HA)(HA)^T, so with k = 3 the 3-D embedding is exact:
    # |x_i - x_j|^2 = |a_i - a_j|^2 / 2
    rng = np.random.default_rng(1)
    A = rng.standard_normal((60, 3))
    s = np.abs(A).max(axis=0) / 127
    Q = np.rint(A / s).astype(np.int8)
    Ah = oracle.dequantise(Q, s)
    coords, lam = oracle.mds3d_dense(Q, s, oracle.LINEAR)
    d_true = np.linalg.norm(Ah[:, None] - Ah[None], axis=-1) / np.sqrt(2.0)
    d_emb = np.linalg.norm(coords[:, None] - coords[None], axis=-1)
    np.testing.assert_allclose(d_emb, d_true, atol=1e-8)
    Ac = Ah - Ah.mean(0)
    np.testing.assert_allclose(lam, np.linalg.eigvalsh(0.5 * Ac.T @ Ac)[::-1], rtol=1e-10)


@pytest.mark.parametrize("mode", [oracle.SQUARED, oracle.LINEAR])
def test_mds_operator_and_invariants(cfg1, mode):
    leaf = cfg1["leaf"]
    N = leaf.shape[1]
    lam, V = oracle.block_iteration(leaf, ri.start_block(N, 12), T=20)
    Q, s = oracle.quantise_int8(V, lam)
    A = oracle.dequantise(Q, s)
    G = oracle.mds_gram_dense(A, mode)
    # brute-force entries of G from the definition
    D2 = (1 - A @ A.T) ** (2 if mode == oracle.SQUARED else 1)
    i, j = 3, 77
    g = -0.5 * (D2[i, j] - D2[i].mean() - D2[:, j].mean() + D2.mean())
    assert G[i, j] == pytest.approx(g, abs=1e-12)
    # the implicit operator is the dense matrix
    op = oracle.mds_operator(A, mode)
    Vt = np.random.default_rng(0).standard_normal((N, 4))
    np.testing.assert_allclose(op(Vt), G @ Vt, atol=1e-10)
    np.testing.assert_allclose(op(Vt[:, 0]), G @ Vt[:, 0], atol=1e-10)
    coords, ev = oracle.mds3d_dense(Q, s, mode)
    assert coords.shape == (N, 3)
    np.testing.assert_allclose(coords.sum(axis=0), 0, atol=1e-9)           # centred
    gram = coords.T @ coords
    np.testing.assert_allclose(gram, np.diag(ev), atol=1e-9)               # orthogonal, |col|^2 = lambda
    np.testing.assert_allclose(ev, np.linalg.eigvalsh(G)[::-1][:3], rtol=1e-12)
    c2, ev2 = oracle.mds3d_implicit(Q, s, mode)
    np.testing.assert_allclose(ev2, ev, rtol=1e-9)
    if min(ev[0] - ev[1], ev[1] - ev[2]) > 1e-3 * ev[0]:
        np.testing.assert_allclose(c2, coords, atol=1e-6 * np.abs(coords).max())
    if mode == oracle.LINEAR:
        assert np.linalg.eigvalsh(G).min() > -1e-10                         # 1/2 H P^ H is PSD


def test_nf4_levels_follow_the_normal_quantile_construction():
    """The 16 NormalFloat levels of the QLoRA paper (cited under "Low-Rank Factorization and Quantization
    Trade-offs") are quantiles of N(0,1): eight positive levels from 9 equally spaced probabilities between
    an offset and 1/2 (the 1/2 dropped), seven negative ones from 8 such probabilities, an exact zero, all
    divided by the largest magnitude; the offset is the mean of 1 - 1/30 and 1 - 1/32.  The stored table is
    rebuilt here from scipy's normal quantile function; a wrong digit in any level fails."""
    from scipy.stats import norm
    offset = 0.5 * ((1.0 - 1.0 / 30.0) + (1.0 - 1.0 / 32.0))
    pos = norm.ppf(np.linspace(offset, 0.5, 9))[:-1]
    neg = -norm.ppf(np.linspace(offset, 0.5, 8))[:-1]
    built = np.sort(np.concatenate([neg, [0.0], pos]))
    built /= np.abs(built).max()
    assert built.shape == (16,)
    np.testing.assert_allclose(oracle.NF4_LEVELS.astype(np.float64), built, rtol=0, atol=2.5e-7)
    # float32 neighbours of a level differ by up to 6e-8, adjacent levels by at least 0.079: no other
    # table of float32 values passes for a different level
    assert np.diff(built).min() > 0.079
    # asymmetric by construction: one more positive level than negative ones, and no level is mirrored
    assert (oracle.NF4_LEVELS > 0).sum() == 8 and (oracle.NF4_LEVELS < 0).sum() == 7
    assert not np.isclose(-oracle.NF4_LEVELS[1], oracle.NF4_LEVELS[14], atol=1e-3)


def test_nf4_levels_and_fp16_nf4_encodings():
    lv = oracle.NF4_LEVELS
    assert lv.shape == (16,) and lv[0] == -1.0 and lv[7] == 0.0 and lv[15] == 1.0 and (np.diff(lv) > 0).all()
    rng = np.random.default_rng(12)
    N, k = 301, 5                                      # odd row count: the last nibble is padding
    V = rng.standard_normal((N, k)).astype(np.float32)
    V[64:128, 2] = 0.0                                 # an all-zero block
    lam = rng.uniform(0.5, 30, k).astype(np.float32)
    A = (V * np.sqrt(lam)[None, :]).astype(np.float32)
    # FP32 / FP16: nearest representable value
    c32, s32 = oracle.quantise_factor(V, lam, oracle.ENC_FP32)
    np.testing.assert_array_equal(c32, A)
    c16, _ = oracle.quantise_factor(V, lam, oracle.ENC_FP16)
    assert c16.dtype == np.float16
    back = oracle.dequantise_factor(c16, None, oracle.ENC_FP16, N)
    assert (np.abs(back - A) <= np.abs(A) * 2.0 ** -11 + 2.0 ** -25).all()      # half an ulp of binary16
    exact = np.array([[1.0, -0.5, 1024.0, 0.0, 65504.0]], np.float32)
    np.testing.assert_array_equal(oracle.quantise_factor(exact, np.ones(5, np.float32), oracle.ENC_FP16)[0].astype(np.float32), exact)
    # NF4
    codes, scales = oracle.quantise_factor(V, lam, oracle.ENC_NF4)
    assert codes.dtype == np.uint8 and codes.shape == ((N + 1) // 2, k) and scales.shape == ((N + 63) // 64, k)
    assert codes.nbytes == ((N + 1) // 2) * k                                      # 4 bits per code
    assert scales[1, 2] == 1.0                                                     # zero block
    deq = oracle.dequantise_factor(codes, scales, oracle.ENC_NF4, N)
    assert (deq[64:128, 2] == 0).all()
    s_full = np.repeat(scales, 64, axis=0)[:N]
    half_gap = np.diff(lv).max() / 2
    assert (np.abs(deq - A) <= s_full * half_gap * (1 + 1e-6)).all()
    # nearest level, checked by brute force
    x = A / s_full
    nearest = np.abs(x[:, :, None].astype(np.float64) - lv[None, None, :].astype(np.float64)).argmin(axis=2)
    unp = np.empty((2 * codes.shape[0], k), np.uint8)
    unp[0::2], unp[1::2] = codes & 15, codes >> 4
    assert (unp[:N] == nearest).mean() > 0.9999 and (np.abs(unp[:N].astype(int) - nearest) <= 1).all()
    assert (unp[N:] == 7).all()
    # the element that sets a block's scale maps to -1 or +1
    blk = np.abs(A[:64, 0]).argmax()
    assert unp[blk, 0] in (0, 15)
    # storage closed forms the paper prints for two rank-32 factors at n = 100k: NF4 3.2 MB, INT8 6.4 MB
    assert 2 * 100_000 * 32 // 2 == 3_200_000 and 2 * 100_000 * 32 == 6_400_000


def test_mds_correlation_metric(cfg1):
    rng = np.random.default_rng(3)
    X = rng.standard_normal((50, 3))
    R, _ = np.linalg.qr(rng.standard_normal((3, 3)))
    assert oracle.mds_correlation(X, X @ R + 5.0) == pytest.approx(1.0, abs=1e-12)   # rigid motions do not matter
    Y = rng.standard_normal((50, 3))
    assert abs(oracle.mds_correlation(X, Y)) < 0.2
    from scipy.spatial.distance import pdist
    from scipy.stats import pearsonr
    assert oracle.mds_correlation(X, Y) == pytest.approx(pearsonr(pdist(X), pdist(Y))[0], abs=1e-12)
    assert oracle.mds_correlation(X, X + 0.3 * Y) < 1.0 - 1e-3
    # compressed factors reproduce the full-matrix embedding of workload 1
    leaf = cfg1["leaf"]
    B, N = leaf.shape
    P = oracle.counts_full(leaf).astype(np.float64) / B
    full, _ = oracle.mds3d_from_dense_proximity(P)
    lam, V = oracle.block_iteration(leaf, ri.start_block(N, 16), 20)
    rho = {}
    for name, enc in (("fp32", oracle.ENC_FP32), ("fp16", oracle.ENC_FP16), ("int8", oracle.ENC_INT8), ("nf4", oracle.ENC_NF4)):
        codes, scales = oracle.quantise_factor(V, lam, enc)
        emb, _ = oracle.mds3d_from_factor(oracle.dequantise_factor(codes, scales, enc, N))
        rho[name] = oracle.mds_correlation(emb, full)
    assert rho["fp32"] > 0.95 and rho["fp16"] > 0.95 and rho["int8"] > 0.95 and rho["nf4"] > 0.9, rho
    assert abs(rho["fp16"] - rho["fp32"]) < 1e-3 and abs(rho["int8"] - rho["fp32"]) < 1e-2


INDEFINITE_CASES = [(400, 4, 1.5, 8, 31), (500, 8, 1.0, 12, 32), (300, 3, 2.0, 6, 33)]   # N, k, spread, block width m, seed


@pytest.mark.parametrize("N,k,spread,m,seed", INDEFINITE_CASES)
def test_scaling_takes_the_largest_eigenvalues_not_the_largest_magnitudes(N, k, spread, m, seed):
    """MDS Steps 3-4 ask for the largest eigenvalues of G.  On these synthetic factors the squared-dissimilarity
    Gram matrix G = H P^ H - 1/2 H (P^ o P^) H has at least m negative eigenvalues that are larger in magnitude
    than its third-largest eigenvalue, so an unshifted block power iteration of width m cannot hold the wanted
    eigenvectors.  The dense reference must still return the algebraically largest three, and the implicit
    operator solved for the algebraically largest agrees with it."""
    Q, s = ri.random_int8_factor(N, k, spread, seed)
    G = oracle.mds_gram_dense(oracle.dequantise(Q, s), oracle.SQUARED)
    ev = np.linalg.eigvalsh(0.5 * (G + G.T))
    lam3 = ev[-3]
    assert lam3 > 0
    assert (ev < -lam3).sum() >= m                       # the dominant part of the spectrum is negative
    assert -ev[0] > 1.5 * ev[-1]
    coords, lam = oracle.mds3d_dense(Q, s, oracle.SQUARED)
    np.testing.assert_allclose(lam, ev[::-1][:3], rtol=1e-12)
    assert (lam > 0).all()
    np.testing.assert_allclose(coords.T @ coords, np.diag(lam), atol=1e-8 * lam[0])
    c2, lam2 = oracle.mds3d_implicit(Q, s, oracle.SQUARED)
    np.testing.assert_allclose(lam2, lam, rtol=1e-9)


def test_scaling_of_a_factor_of_rank_below_three():
    """LINEAR mode with k = 2: G = 1/2 H P^ H has rank 2, the third eigenvalue is zero and the third
    coordinate vanishes (a non-positive eigenvalue gives a zero column, MDS Step 4 with lambda_3 = 0)."""
    Q, s = ri.random_int8_factor(200, 2, 0.3, 34)
    coords, lam = oracle.mds3d_dense(Q, s, oracle.LINEAR)
    assert lam[1] > 1e-3 * lam[0] and abs(lam[2]) < 1e-10 * lam[0]
    assert np.abs(coords[:, 2]).max() < 1e-4 * np.abs(coords[:, 0]).max()


def test_implicit_eigensolver_equals_the_dense_eigendecomposition(cfg1, small2):
    """The ARPACK route on the implicit float64 operator (used where P cannot be materialised) against LAPACK on
    the materialised matrix: same leading eigenvalues, same invariant subspace."""
    for d, k in ((cfg1, 6), (small2, 8)):
        leaf = d["leaf"]
        B, N = leaf.shape
        P = oracle.counts_full(leaf).astype(np.float64) / B
        lam_d, U_d = oracle.dense_eig(P, k)
        lam_i, U_i = oracle.implicit_eig(leaf, k)
        np.testing.assert_allclose(lam_i, lam_d, rtol=1e-10)
        assert oracle.principal_angle(U_i, U_d) < 1e-6
        np.testing.assert_allclose(P @ U_i, U_i * lam_i[None, :], atol=1e-8 * lam_d[0])
