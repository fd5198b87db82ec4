// Small dense linear algebra for the block iterations (see dense_small.h).
#include "dense_small.h"

#include <algorithm>

namespace rfx {
namespace {

constexpr int kGramWaves = 4;   // waves per workgroup of the Gram kernel, each with its own row range
constexpr int kApplyRows = 32;  // rows per workgroup step of the tall-times-small product

typedef double double4_t __attribute__((ext_vector_type(4)));

// partial[workgroup][p][q] = sum over the workgroup's rows of A[i][p] * Bm[i][q] in float64 on the
// matrix cores: v_mfma_f64_16x16x4_f64 computes D(16x16) += Aop(16x4) Bop(4x16), 4 rows of the
// tall blocks per instruction.  Operand layout of a 64-lane wave: lane l supplies
// Aop[l % 16][l / 16] and Bop[l / 16][l % 16]; the result register v (0..3) of lane l is
// D[l / 16 + 4 v][l % 16].  With Aop[m][r] = A[i0 + r][16 u + m] and Bop[r][n] = Bm[i0 + r][16 w + n]
// both operands of lane l are the element (row i0 + l / 16, column 16 * tile + l % 16) of their block:
// 4 rows x 64 contiguous bytes per load.  A wave keeps PBC x NB output tiles (at most 16) in
// registers and passes over its own row range once per group of PBC tile rows, with the loads of the
// next 4 rows issued before the instructions of the current ones; the four waves of a workgroup add
// their tiles up in LDS in wave order.  kSame (A and Bm are the same block): the product is symmetric
// and only the tiles on and above the diagonal are computed and stored.
template <int NB, bool kSame>
__global__ __launch_bounds__(64 * kGramWaves) void gram_partial_kernel(const float* __restrict__ A,
                                                                      const float* __restrict__ Bm, int64_t N, int k,
                                                                      int64_t rows_per_wave,
                                                                      double* __restrict__ partial) {
    extern __shared__ double gram_sm[];  // [k][k]
    constexpr int PBC = NB <= 4 ? NB : (16 / NB > 0 ? 16 / NB : 1);
    constexpr bool kShare = kSame && PBC == NB;  // the left operands are the right ones
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int slot = blockIdx.x * kGramWaves + wave;
    const int64_t i_begin = min(N, (int64_t)slot * rows_per_wave);
    const int64_t i_end = min(N, i_begin + rows_per_wave);
    const int r = lane >> 4, c = lane & 15;
    for (int pg = 0; pg < NB; pg += PBC) {
        double4_t acc[PBC][NB];
#pragma unroll
        for (int u = 0; u < PBC; ++u)
#pragma unroll
            for (int w = 0; w < NB; ++w) acc[u][w] = double4_t{0.0, 0.0, 0.0, 0.0};
        float a_next[PBC], b_next[NB];
        auto load_rows = [&](int64_t i0) {
            const int64_t row = i0 + r;
            const bool live = row < i_end;
#pragma unroll
            for (int w = 0; w < NB; ++w) {
                const int col = 16 * w + c;
                b_next[w] = (live && col < k) ? Bm[row * k + col] : 0.0f;
            }
            if (!kShare) {
#pragma unroll
                for (int u = 0; u < PBC; ++u) {
                    const int col = 16 * (pg + u) + c;
                    a_next[u] = (live && pg + u < NB && col < k) ? A[row * k + col] : 0.0f;
                }
            }
        };
        load_rows(i_begin);
        for (int64_t i0 = i_begin; i0 < i_end; i0 += 4) {
            double a[PBC], b[NB];
#pragma unroll
            for (int w = 0; w < NB; ++w) b[w] = (double)b_next[w];
#pragma unroll
            for (int u = 0; u < PBC; ++u) a[u] = kShare ? b[u] : (double)a_next[u];
            load_rows(i0 + 4);
#pragma unroll
            for (int u = 0; u < PBC; ++u)
#pragma unroll
                for (int w = 0; w < NB; ++w)
                    if (!kSame || pg + u <= w)
                        acc[u][w] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[u], b[w], acc[u][w], 0, 0, 0);
        }
        for (int w4 = 0; w4 < kGramWaves; ++w4) {
            if (wave == w4) {
#pragma unroll
                for (int u = 0; u < PBC; ++u)
#pragma unroll
                    for (int w = 0; w < NB; ++w)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int p = 16 * (pg + u) + r + 4 * v, q = 16 * w + c;
                            if ((!kSame || pg + u <= w) && pg + u < NB && p < k && q < k)
                                gram_sm[p * k + q] = (w4 == 0 ? 0.0 : gram_sm[p * k + q]) + acc[u][w][v];
                        }
            }
            __syncthreads();
        }
    }
    double* out = partial + (int64_t)blockIdx.x * k * k;
    for (int e = threadIdx.x; e < k * k; e += 64 * kGramWaves) {
        const int p = e / k, q = e - p * k;
        if (!kSame || p / 16 <= q / 16) out[e] = gram_sm[e];
    }
}

// G[e] = sum over workgroups of partial[workgroup][e].  sym: symmetrised, (x[p][q] + x[q][p]) / 2.  upper_only: the
// 16 x 16 tiles below the diagonal were not stored (symmetric product); their entries are those of the mirrored tile,
// and the symmetrisation only concerns the diagonal tiles.  16 consecutive lanes share an entry: lane part p adds
// workgroups p, p+16, ..., then the 16 partial sums are added pairwise in a fixed order, so the result does not
// depend on scheduling.
__global__ __launch_bounds__(256) void gram_reduce_kernel(const double* __restrict__ partial, int blocks, int k, int sym,
                                                         int upper_only, double* __restrict__ G) {
    const int e = blockIdx.x * 16 + (threadIdx.x >> 4);
    const int part = threadIdx.x & 15;
    const bool live = e < k * k;
    int p = live ? e / k : 0, q = live ? e - p * k : 0;
    if (upper_only && p / 16 > q / 16) {
        const int t = p;
        p = q;
        q = t;
    }
    const bool both = sym && (!upper_only || p / 16 == q / 16);
    double s = 0.0;
    for (int b = part; b < blocks; b += 16) {
        s += partial[(int64_t)b * k * k + p * k + q];
        if (both) s += partial[(int64_t)b * k * k + q * k + p];
    }
    for (int off = 8; off > 0; off >>= 1) s += __shfl_xor(s, off, 16);
    if (live && part == 0) G[e] = both ? 0.5 * s : s;
}

// One workgroup.  R (upper, G = R^T R) is formed in LDS by the right-looking Cholesky algorithm,
// then thread c solves R x = e_c by back substitution and writes column c of T = R^-1.
__global__ __launch_bounds__(256) void chol_inverse_kernel(const double* __restrict__ G, int k, double* __restrict__ T,
                                                          int* __restrict__ flag) {
    extern __shared__ double chol_sm[];
    double* R = chol_sm;  // [k][k]
    for (int e = threadIdx.x; e < k * k; e += 256) R[e] = G[e];
    __syncthreads();
    double scale = 0.0;
    for (int j = 0; j < k; ++j) scale = fmax(scale, R[j * k + j]);
    for (int j = 0; j < k; ++j) {
        if (threadIdx.x == 0) {
            const double d = R[j * k + j];
            if (!(d > scale * 1e-28)) {
                // Column j lies in the span of the columns before it: the flag reports it, and an infinite pivot
                // drops the column (row j of the factor and column j of its inverse become zero, so column j of
                // the orthonormalised block is a zero vector and the remaining columns are unaffected).
                *flag = 1;
                R[j * k + j] = __builtin_inf();
            } else {
                R[j * k + j] = sqrt(d);
            }
        }
        __syncthreads();
        const double piv = R[j * k + j];
        for (int c = j + 1 + threadIdx.x; c < k; c += 256) R[j * k + c] /= piv;
        __syncthreads();
        // trailing block (j+1..k-1)^2, upper part: a 16 x 16 arrangement of the threads walks it in squares
        for (int r = j + 1 + (int)(threadIdx.x >> 4); r < k; r += 16) {
            const double rj = R[j * k + r];
            for (int c = j + 1 + (int)(threadIdx.x & 15); c < k; c += 16)
                if (c >= r) R[r * k + c] -= rj * R[j * k + c];
        }
        __syncthreads();
    }
    for (int c = threadIdx.x; c < k; c += 256) {
        for (int r = k - 1; r > c; --r) T[r * k + c] = 0.0;
        T[c * k + c] = 1.0 / R[c * k + c];  // 0 for a dropped column
        for (int r = c - 1; r >= 0; --r) {
            double s = 0.0;
            for (int p = r + 1; p <= c; ++p) s += R[r * k + p] * T[p * k + c];
            T[r * k + c] = -s / R[r * k + r];
        }
    }
}

// The same factorisation with one barrier per column and the Schur complement in registers, for k <= 16 NB16 small
// enough that two k x k arrays fit LDS.  Thread (ty, tx) of a 16 x 16 arrangement owns the entries (ty + 16 a,
// tx + 16 b) of the upper triangle for the whole factorisation.  Column step j: everybody reads the unscaled pivot
// row j (published in LDS by its owners), forms 1 / d and its square root itself, updates its entries
// (A[r][c] -= A[j][r] A[j][c] / d), and the owners of row j + 1 publish it into the other of two LDS slots; the
// scaled row goes to the factor R.  Then the inverse of R by back substitution: lane c of the first wave owns
// column c (columns are independent); the loops over r and p are the same for every lane, so R[r][p] is one
// broadcast read and Ti[p][c] a conflict-free one; entries below the diagonal are written as zeros before they
// are read.
template <int NB16>
__global__ __launch_bounds__(256) void chol_inverse_fast_kernel(const double* __restrict__ G, int k, double* __restrict__ T,
                                                               int* __restrict__ flag) {
    extern __shared__ double chol_sm[];
    double* Ti = chol_sm;       // [k][k] inverse of the factor
    double* R = Ti + k * k;     // [k][k] upper factor
    double* dinv = R + k * k;   // [k] diagonal of G, later reciprocals of the diagonal of R
    double* piv = dinv + k;     // [2][k] unscaled pivot rows of even and odd columns
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
    double a[NB16][NB16];
#pragma unroll
    for (int ia = 0; ia < NB16; ++ia)
#pragma unroll
        for (int ib = 0; ib < NB16; ++ib) {
            const int r = ty + 16 * ia, c = tx + 16 * ib;
            a[ia][ib] = (r < k && c < k && c >= r) ? G[r * k + c] : 0.0;
        }
    for (int c = threadIdx.x; c < k; c += 256) dinv[c] = G[c * k + c];
    if (ty == 0) {
#pragma unroll
        for (int ib = 0; ib < NB16; ++ib)
            if (tx + 16 * ib < k) piv[tx + 16 * ib] = a[0][ib];
    }
    __syncthreads();
    double scale = 0.0;
    for (int j = 0; j < k; ++j) scale = fmax(scale, dinv[j]);
    for (int j = 0; j < k; ++j) {
        const double* pr = piv + (j & 1) * k;
        const double d = pr[j];
        // A pivot that is not positive at the scale of the matrix: column j lies in the span of the columns
        // before it.  The flag reports it and the column is dropped: with 1 / d taken as 0 and the diagonal of the
        // factor as infinity, row j of the factor and column j of its inverse are zero, so column j of the
        // orthonormalised block is a zero vector and the remaining columns are unaffected.
        const bool dependent = !(d > scale * 1e-28);
        if (dependent && threadIdx.x == 0) *flag = 1;
        const double inv = dependent ? 0.0 : 1.0 / d, rs = sqrt(inv);
        if ((int)threadIdx.x >= j && (int)threadIdx.x < k)
            R[j * k + threadIdx.x] = ((int)threadIdx.x == j) ? (dependent ? __builtin_inf() : d * rs) : pr[threadIdx.x] * rs;
        double fr[NB16], pc[NB16];
#pragma unroll
        for (int ia = 0; ia < NB16; ++ia) {
            const int r = ty + 16 * ia;
            fr[ia] = (r > j && r < k) ? pr[r] * inv : 0.0;
        }
#pragma unroll
        for (int ib = 0; ib < NB16; ++ib) {
            const int c = tx + 16 * ib;
            pc[ib] = (c > j && c < k) ? pr[c] : 0.0;
        }
#pragma unroll
        for (int ia = 0; ia < NB16; ++ia)
#pragma unroll
            for (int ib = 0; ib < NB16; ++ib) a[ia][ib] -= fr[ia] * pc[ib];
        const int jr = j + 1;
        if (jr < k && ty == (jr & 15)) {
            double* pw = piv + (jr & 1) * k;
#pragma unroll
            for (int ib = 0; ib < NB16; ++ib) {
                double v = 0.0;
#pragma unroll
                for (int ia = 0; ia < NB16; ++ia)
                    if (ia == (jr >> 4)) v = a[ia][ib];
                const int c = tx + 16 * ib;
                if (c >= jr && c < k) pw[c] = v;
            }
        }
        __syncthreads();
    }
    for (int c = threadIdx.x; c < k; c += 256) dinv[c] = 1.0 / R[c * k + c];
    __syncthreads();
    if (threadIdx.x < 64) {
        for (int c0 = 0; c0 < k; c0 += 64) {
            const int c = c0 + (int)threadIdx.x;
            const bool on = c < k;
            const int cc = on ? c : k - 1;  // lanes without a column read a valid one and store nothing
            const int cmax = min(k - 1, c0 + 63);
            for (int r = k - 1; r > cmax; --r)
                if (on) Ti[r * k + c] = 0.0;
            for (int r = cmax; r >= 0; --r) {
                double s = 0.0;
#pragma unroll 4
                for (int p = r + 1; p <= cmax; ++p) s += R[r * k + p] * Ti[p * k + cc];
                const double t = r > c ? 0.0 : (r == c ? dinv[r] : -s * dinv[r]);
                if (on) Ti[r * k + c] = t;
            }
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < k * k; e += 256) T[e] = Ti[e];
}

// One workgroup: cyclic Jacobi on a symmetric k x k matrix held in LDS.  The rotations of one round-robin step
// act on disjoint index pairs; with pair a = (p_a, q_a) and pair b = (p_b, q_b), the update J^T A J changes the
// 2 x 2 block A[{p_a, q_a}][{p_b, q_b}] using nothing but that block and the two rotations, so every block is
// read, rotated by rows, then by columns, and written by one thread: two barriers per step (rotations known;
// blocks written).  The accumulated rotations are kept transposed (Wt[p][row], contiguous per rotated column),
// in LDS when both arrays fit (kLdsW) and in global memory otherwise.  theta is sorted descending and the
// columns of W follow.
template <bool kLdsW>
__global__ __launch_bounds__(256) void jacobi_kernel(const double* __restrict__ H, int k, int sweeps,
                                                    double* __restrict__ Wk, double* __restrict__ theta,
                                                    double* __restrict__ W) {
    extern __shared__ double jac_sm[];
    const int K = (k + 1) & ~1;  // even number of players; index k (if any) is a dummy
    const int half = K / 2;
    double* A = jac_sm;          // [k][k]
    double* cs = A + k * k;      // [K/2] cos, [K/2] sin
    double* sn = cs + half;
    int* pp = (int*)(sn + half);  // [K/2] p, [K/2] q
    int* qq = pp + half;
    double* Wt = kLdsW ? (double*)(qq + half) : Wk;  // [k][k], transposed
    for (int e = threadIdx.x; e < k * k; e += 256) {
        A[e] = H[e];
        Wt[e] = (e / k == e % k) ? 1.0 : 0.0;
    }
    __syncthreads();
    __shared__ double red_off[256], red_diag[256];
    const int ta = threadIdx.x >> 4, tb = threadIdx.x & 15;
    for (int sw = 0; sw < sweeps; ++sw) {
        // converged when the off-diagonal mass is negligible against the diagonal
        double off = 0.0, dg = 0.0;
        for (int e = threadIdx.x; e < k * k; e += 256) {
            const double v = A[e];
            if (e / k == e % k)
                dg += v * v;
            else
                off += v * v;
        }
        red_off[threadIdx.x] = off;
        red_diag[threadIdx.x] = dg;
        __syncthreads();
        for (int s2 = 128; s2 > 0; s2 >>= 1) {
            if (threadIdx.x < s2) {
                red_off[threadIdx.x] += red_off[threadIdx.x + s2];
                red_diag[threadIdx.x] += red_diag[threadIdx.x + s2];
            }
            __syncthreads();
        }
        const bool done = red_off[0] <= 1e-30 * red_diag[0];
        __syncthreads();
        if (done) break;
        for (int step = 0; step < K - 1; ++step) {
            for (int pr = threadIdx.x; pr < half; pr += 256) {
                int p = (step + pr) % (K - 1);
                int q = (pr == 0) ? K - 1 : (step + K - 1 - pr) % (K - 1);
                if (p > q) {
                    int t = p;
                    p = q;
                    q = t;
                }
                double c = 1.0, s = 0.0;
                if (q < k) {
                    const double apq = A[p * k + q];
                    if (apq != 0.0) {
                        const double tau = (A[q * k + q] - A[p * k + p]) / (2.0 * apq);
                        const double t = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
                        c = 1.0 / sqrt(1.0 + t * t);
                        s = t * c;
                    }
                } else {
                    q = -1;  // pair with the dummy: index p rests in this step (identity rotation, no second row)
                }
                cs[pr] = c;
                sn[pr] = s;
                pp[pr] = p;
                qq[pr] = q;
            }
            __syncthreads();
            for (int a = ta; a < half; a += 16) {
                const int pa = pp[a], qa = qq[a];
                const double ca = cs[a], sa = sn[a];
                for (int b = tb; b < half; b += 16) {
                    const int pb = pp[b], qb = qq[b];
                    const double cb = cs[b], sb = sn[b];
                    const double xpp = A[pa * k + pb];
                    const double xpq = qb >= 0 ? A[pa * k + qb] : 0.0;
                    const double xqp = qa >= 0 ? A[qa * k + pb] : 0.0;
                    const double xqq = (qa >= 0 && qb >= 0) ? A[qa * k + qb] : 0.0;
                    // rows p_a, q_a
                    const double rpp = ca * xpp - sa * xqp, rpq = ca * xpq - sa * xqq;
                    const double rqp = sa * xpp + ca * xqp, rqq = sa * xpq + ca * xqq;
                    // columns p_b, q_b
                    A[pa * k + pb] = cb * rpp - sb * rpq;
                    if (qb >= 0) A[pa * k + qb] = sb * rpp + cb * rpq;
                    if (qa >= 0) A[qa * k + pb] = cb * rqp - sb * rqq;
                    if (qa >= 0 && qb >= 0) A[qa * k + qb] = sb * rqp + cb * rqq;
                }
                // columns p_a, q_a of the accumulated rotations
                if (qa >= 0) {
                    for (int row = tb; row < k; row += 16) {
                        const double wp = Wt[pa * k + row], wq = Wt[qa * k + row];
                        Wt[pa * k + row] = ca * wp - sa * wq;
                        Wt[qa * k + row] = sa * wp + ca * wq;
                    }
                }
            }
            __syncthreads();
        }
    }
    // descending order; equal values keep their index order
    for (int i = threadIdx.x; i < k; i += 256) {
        const double ti = A[i * k + i];
        int rank = 0;
        for (int j = 0; j < k; ++j) {
            const double tj = A[j * k + j];
            rank += (tj > ti) || (tj == ti && j < i);
        }
        theta[rank] = ti;
        for (int r = 0; r < k; ++r) W[r * k + rank] = Wt[i * k + r];
    }
}

// Out[i][c] = sum_p A[i][p] T[p][c]; T (float64, [k][kout], row stride k) is staged in LDS.
__global__ __launch_bounds__(256) void apply_small_kernel(const float* __restrict__ A, int64_t N, int k,
                                                         const double* __restrict__ T, int kout,
                                                         float* __restrict__ Out) {
    extern __shared__ double app_sm[];
    double* Ts = app_sm;                     // [k][kout]
    float* As = (float*)(Ts + k * kout);     // [kApplyRows][k]
    for (int e = threadIdx.x; e < k * kout; e += 256) Ts[e] = T[(e / kout) * k + (e % kout)];
    for (int64_t i0 = (int64_t)blockIdx.x * kApplyRows; i0 < N; i0 += (int64_t)gridDim.x * kApplyRows) {
        const int rows = (int)min((int64_t)kApplyRows, N - i0);
        __syncthreads();
        for (int e = threadIdx.x; e < rows * k; e += 256) As[e] = A[i0 * k + e];
        __syncthreads();
        for (int e = threadIdx.x; e < rows * kout; e += 256) {
            const int r = e / kout, c = e - r * kout;
            double s = 0.0;
            for (int p = 0; p < k; ++p) s = fma((double)As[r * k + p], Ts[p * kout + c], s);
            Out[(i0 + r) * kout + c] = (float)s;
        }
    }
}

// The same product on the matrix cores for k a multiple of 16, k <= 64, kout <= 64, rows of A 16-byte aligned: a wave
// takes tiles of 16 rows; v_mfma_f64_16x16x4_f64 contracts 4 columns of A per instruction.  Lane l = (g = l / 16,
// r = l % 16) loads A[i0 + r][16 jj + 4 g .. + 3] as one 16-byte load per jj, which fixes the order in which the
// columns are contracted: instruction j = 4 jj + t handles columns 16 jj + 4 g' + t (g' = 0..3).  The matching
// entries of T (one per instruction and 16-column output tile) stay in registers for all tiles of the wave.
// Result register v of lane l is Out[i0 + g + 4 v][16 w + r].
template <int KB, int NBO>
__global__ __launch_bounds__(256) void apply_small_mfma_kernel(const float* __restrict__ A, int64_t N,
                                                              const double* __restrict__ T, int kout,
                                                              float* __restrict__ Out) {
    constexpr int k = 16 * KB, KO = 16 * NBO;
    extern __shared__ double app_sm[];  // [k][KO], columns beyond kout are zero
    for (int e = threadIdx.x; e < k * KO; e += 256) {
        const int p = e / KO, c = e - p * KO;
        app_sm[e] = c < kout ? T[p * k + c] : 0.0;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 4, r = lane & 15;
    double tb[4 * KB][NBO];
#pragma unroll
    for (int j = 0; j < 4 * KB; ++j)
#pragma unroll
        for (int w = 0; w < NBO; ++w) tb[j][w] = app_sm[(16 * (j / 4) + 4 * g + (j % 4)) * KO + 16 * w + r];
    const int64_t tiles = (N + 15) / 16;
    for (int64_t tile = (int64_t)blockIdx.x * 4 + wave; tile < tiles; tile += (int64_t)gridDim.x * 4) {
        const int64_t i0 = tile * 16;
        const bool live = i0 + r < N;
        float4 av[KB];
#pragma unroll
        for (int jj = 0; jj < KB; ++jj)
            av[jj] = live ? *reinterpret_cast<const float4*>(A + (i0 + r) * k + 16 * jj + 4 * g) : float4{0.f, 0.f, 0.f, 0.f};
        double4_t acc[NBO];
#pragma unroll
        for (int w = 0; w < NBO; ++w) acc[w] = double4_t{0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int jj = 0; jj < KB; ++jj) {
            const double a4[4] = {(double)av[jj].x, (double)av[jj].y, (double)av[jj].z, (double)av[jj].w};
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int w = 0; w < NBO; ++w)
                    acc[w] = __builtin_amdgcn_mfma_f64_16x16x4f64(a4[t], tb[4 * jj + t][w], acc[w], 0, 0, 0);
        }
#pragma unroll
        for (int w = 0; w < NBO; ++w)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t row = i0 + g + 4 * v;
                const int col = 16 * w + r;
                if (row < N && col < kout) Out[row * kout + col] = (float)acc[w][v];
            }
    }
}

// Sign convention, step 1: per workgroup (a range of rows) and column, the entry of largest magnitude (the first
// one on ties) with its row.  Thread t takes column t % kpad of rows g, g + 256 / kpad, ... (kpad = kc rounded
// up to a power of two), so a wave reads whole rows.
constexpr int kSignBlocks = 256;

__global__ __launch_bounds__(256) void sign_partial_kernel(const float* __restrict__ V, int64_t N, int kc, int kpad,
                                                          int64_t rows_per_block, float* __restrict__ best_val,
                                                          long long* __restrict__ best_row) {
    __shared__ float s_val[256];
    __shared__ long long s_idx[256];
    const int c = threadIdx.x & (kpad - 1), g = threadIdx.x / kpad, G = 256 / kpad;
    const int64_t i_begin = (int64_t)blockIdx.x * rows_per_block, i_end = min(N, i_begin + rows_per_block);
    float best = 0.0f, best_abs = -1.0f;
    long long bi = i_begin;
    if (c < kc)
        for (int64_t i = i_begin + g; i < i_end; i += G) {
            const float v = V[i * kc + c], a = fabsf(v);
            if (a > best_abs) {
                best_abs = a;
                best = v;
                bi = i;
            }
        }
    s_val[threadIdx.x] = best;
    s_idx[threadIdx.x] = best_abs < 0.0f ? -1 : bi;   // -1: nothing seen
    __syncthreads();
    for (int off = G >> 1; off > 0; off >>= 1) {
        if (g < off) {
            const int o = threadIdx.x + off * kpad;
            const float ov = s_val[o], mv = s_val[threadIdx.x];
            const long long oi = s_idx[o], mi = s_idx[threadIdx.x];
            if (oi >= 0 && (mi < 0 || fabsf(ov) > fabsf(mv) || (fabsf(ov) == fabsf(mv) && oi < mi))) {
                s_val[threadIdx.x] = ov;
                s_idx[threadIdx.x] = oi;
            }
        }
        __syncthreads();
    }
    if (g == 0 && c < kc) {
        best_val[(int64_t)blockIdx.x * kc + c] = s_val[threadIdx.x];
        best_row[(int64_t)blockIdx.x * kc + c] = s_idx[threadIdx.x];
    }
}

// Step 2: every workgroup picks each column's winner among the partial results (ranges are in ascending row
// order, so a strict comparison keeps the first on ties) and negates its rows of the columns whose winner is
// negative.  The decision uses the values recorded in step 1, never V itself, which other workgroups are changing.
__global__ __launch_bounds__(256) void sign_apply_kernel(float* __restrict__ V, int64_t N, int kc, int kpad,
                                                        int64_t rows_per_block, int blocks,
                                                        const float* __restrict__ best_val,
                                                        const long long* __restrict__ best_row) {
    __shared__ float s_sign[256];
    if ((int)threadIdx.x < kc) {
        float best = 0.0f, best_abs = -1.0f;
        for (int b = 0; b < blocks; ++b) {
            const float v = best_val[(int64_t)b * kc + threadIdx.x];
            if (best_row[(int64_t)b * kc + threadIdx.x] >= 0 && fabsf(v) > best_abs) {
                best_abs = fabsf(v);
                best = v;
            }
        }
        s_sign[threadIdx.x] = best < 0.0f ? -1.0f : 1.0f;
    }
    __syncthreads();
    const int c = threadIdx.x & (kpad - 1), g = threadIdx.x / kpad, G = 256 / kpad;
    if (c >= kc || s_sign[c] > 0.0f) return;
    const int64_t i_begin = (int64_t)blockIdx.x * rows_per_block, i_end = min(N, i_begin + rows_per_block);
    for (int64_t i = i_begin + g; i < i_end; i += G) V[i * kc + c] = -V[i * kc + c];
}

template <class K>
hipError_t allow_lds(K kern, size_t bytes) {
    if (bytes <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

}  // namespace

namespace {
__global__ void clear_flag_kernel(int* flag) { *flag = 0; }

struct SmallLayout {
    int gram_blocks;
    size_t doubles, sign_entries, total;
};
SmallLayout small_layout(int64_t N, int k) {
    SmallLayout l;
    l.gram_blocks = (int)std::min<int64_t>(512, ceil_div(N, 64 * kGramWaves));  // workgroups of the Gram kernel
    const size_t kk = (size_t)k * k;
    l.doubles = (size_t)l.gram_blocks * kk + 3 * kk + (size_t)k + kk /*jacobi work*/;
    l.sign_entries = (size_t)kSignBlocks * k;
    l.total = l.doubles * sizeof(double) + 64 + l.sign_entries * (sizeof(long long) + sizeof(float));
    return l;
}
}  // namespace

size_t SmallWs::bytes(int64_t N, int k) { return (small_layout(N, k).total + 255) & ~(size_t)255; }

int SmallWs::bind(void* mem, int64_t N, int k, hipStream_t st) {
    const SmallLayout l = small_layout(N, k);
    gram_blocks = l.gram_blocks;
    const size_t kk = (size_t)k * k;
    double* p = static_cast<double*>(mem);
    partial = p;
    p += (size_t)gram_blocks * kk;
    G = p;
    p += kk;
    T = p;
    p += kk;
    W = p;
    p += kk;
    theta = p;
    p += k;
    p += kk;  // jacobi work matrix sits at theta + k
    flag = (int*)p;
    p += 8;  // 64 bytes for the status word
    sign_row = (long long*)p;
    sign_val = (float*)(sign_row + l.sign_entries);
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, st, flag);
    RFX_LAUNCH_CHECK("clear_flag_kernel");
    return RFX_OK;
}

int SmallWs::alloc(int64_t N, int k, hipStream_t st) {
    RFX_HIP(buf.alloc(bytes(N, k)));
    return bind(buf.p, N, k, st);
}

int gram(const float* A, const float* Bm, int64_t N, int k, bool sym, SmallWs& ws, double* G, hipStream_t st) {
    // every wave takes a multiple of 4 rows (one matrix instruction covers 4)
    const int64_t rpw = ceil_div(ceil_div(N, (int64_t)ws.gram_blocks * kGramWaves), 4) * 4;
    const int blocks = (int)ceil_div(N, rpw * kGramWaves);  // workgroups with rows (<= gram_blocks)
    const int NB = (k + 15) / 16;
    const bool same = A == Bm;
    const size_t lds = sizeof(double) * (size_t)k * k;
#define RFX_GRAM(nb)                                                                                                 \
    case nb:                                                                                                         \
        if (same) {                                                                                                  \
            RFX_HIP(allow_lds(gram_partial_kernel<nb, true>, lds));                                                  \
            hipLaunchKernelGGL((gram_partial_kernel<nb, true>), dim3(blocks), dim3(64 * kGramWaves), lds, st, A, Bm, N, k, \
                               rpw, ws.partial);                                                                     \
        } else {                                                                                                     \
            RFX_HIP(allow_lds(gram_partial_kernel<nb, false>, lds));                                                 \
            hipLaunchKernelGGL((gram_partial_kernel<nb, false>), dim3(blocks), dim3(64 * kGramWaves), lds, st, A, Bm, N, k, \
                               rpw, ws.partial);                                                                     \
        }                                                                                                            \
        break;
    switch (NB) {
        RFX_GRAM(1) RFX_GRAM(2) RFX_GRAM(3) RFX_GRAM(4) RFX_GRAM(5) RFX_GRAM(6) RFX_GRAM(7) RFX_GRAM(8)
        default:
            return fail(RFX_ERR_INVALID_ARG, "gram: k=%d > %d", k, kMaxRank);
    }
#undef RFX_GRAM
    RFX_LAUNCH_CHECK("gram_partial_kernel");
    hipLaunchKernelGGL(gram_reduce_kernel, dim3((unsigned)ceil_div(k * k, 16)), dim3(256), 0, st, ws.partial, blocks, k,
                       sym ? 1 : 0, same ? 1 : 0, G);
    RFX_LAUNCH_CHECK("gram_reduce_kernel");
    return RFX_OK;
}

int chol_inverse(const double* G, int k, SmallWs& ws, double* T, hipStream_t st) {
    const size_t lds = sizeof(double) * (size_t)k * k;
    if (2 * lds <= 128 * 1024) {
        const size_t fast_lds = 2 * lds + sizeof(double) * 3 * (size_t)k;  // inverse, factor, diagonal, two pivot rows
#define RFX_CHOL(nb)                                                                                             \
    case nb:                                                                                                     \
        RFX_HIP(allow_lds(chol_inverse_fast_kernel<nb>, fast_lds));                                              \
        hipLaunchKernelGGL(chol_inverse_fast_kernel<nb>, dim3(1), dim3(256), fast_lds, st, G, k, T, ws.flag);    \
        break;
        switch ((k + 15) / 16) {
            RFX_CHOL(1) RFX_CHOL(2) RFX_CHOL(3) RFX_CHOL(4) RFX_CHOL(5)
            default:
                RFX_CHOL(6)
        }
#undef RFX_CHOL
    } else {
        RFX_HIP(allow_lds(chol_inverse_kernel, lds));
        hipLaunchKernelGGL(chol_inverse_kernel, dim3(1), dim3(256), lds, st, G, k, T, ws.flag);
    }
    RFX_LAUNCH_CHECK("chol_inverse_kernel");
    return RFX_OK;
}

int jacobi_eigh(const double* H, int k, SmallWs& ws, double* theta, double* W, hipStream_t st) {
    const int K = (k + 1) & ~1;
    const size_t lds = sizeof(double) * ((size_t)k * k + K) + sizeof(int) * K;
    const size_t lds_w = lds + sizeof(double) * (size_t)k * k;   // with the accumulated rotations in LDS as well
    double* work = ws.theta + k;  // [k][k] accumulated rotations when they do not fit LDS
    const int sweeps = 16;  // upper bound; the kernel stops when the off-diagonal mass is below 1e-30 of the diagonal
    if (lds_w <= 144 * 1024) {
        RFX_HIP(allow_lds(jacobi_kernel<true>, lds_w));
        hipLaunchKernelGGL(jacobi_kernel<true>, dim3(1), dim3(256), lds_w, st, H, k, sweeps, work, theta, W);
    } else {
        RFX_HIP(allow_lds(jacobi_kernel<false>, lds));
        hipLaunchKernelGGL(jacobi_kernel<false>, dim3(1), dim3(256), lds, st, H, k, sweeps, work, theta, W);
    }
    RFX_LAUNCH_CHECK("jacobi_kernel");
    return RFX_OK;
}

template <int KB, int NBO>
int launch_apply_mfma(const float* A, int64_t N, const double* T, int kout, float* Out, hipStream_t st) {
    const size_t lds = sizeof(double) * (size_t)(16 * KB) * (16 * NBO);
    const unsigned blocks = (unsigned)std::min<int64_t>(ceil_div(ceil_div(N, 16), 4), 512);
    hipLaunchKernelGGL((apply_small_mfma_kernel<KB, NBO>), dim3(blocks), dim3(256), lds, st, A, N, T, kout, Out);
    RFX_LAUNCH_CHECK("apply_small_mfma_kernel");
    return RFX_OK;
}

int apply_small(const float* A, int64_t N, int k, const double* T, int kout, float* Out, hipStream_t st) {
    if (k % 16 == 0 && k <= 64 && kout >= 1 && kout <= 64 && reinterpret_cast<uintptr_t>(A) % 16 == 0) {
        const int code = (k / 16) * 10 + (kout + 15) / 16;
        switch (code) {
#define RFX_APPLY(kb, nbo) \
    case kb * 10 + nbo:    \
        return launch_apply_mfma<kb, nbo>(A, N, T, kout, Out, st);
            // square factors (Cholesky-QR, Ritz rotation) and the three coordinate columns of a 16- or 32-wide block
            RFX_APPLY(1, 1) RFX_APPLY(2, 1) RFX_APPLY(2, 2) RFX_APPLY(3, 3) RFX_APPLY(4, 4)
#undef RFX_APPLY
            default:
                break;  // other shapes do not occur on the path; the general kernel takes them
        }
    }
    const size_t lds = sizeof(double) * (size_t)k * kout + sizeof(float) * kApplyRows * (size_t)k;
    RFX_HIP(allow_lds(apply_small_kernel, lds));
    const unsigned blocks = (unsigned)std::min<int64_t>(ceil_div(N, kApplyRows), 2048);
    hipLaunchKernelGGL(apply_small_kernel, dim3(blocks), dim3(256), lds, st, A, N, k, T, kout, Out);
    RFX_LAUNCH_CHECK("apply_small_kernel");
    return RFX_OK;
}

int orthonormalise(const float* Y, int64_t N, int k, SmallWs& ws, float* Z, float* V, hipStream_t st, int passes) {
    int rc;
    if (passes <= 1) {
        if ((rc = gram(Y, Y, N, k, true, ws, ws.G, st)) != RFX_OK) return rc;
        if ((rc = chol_inverse(ws.G, k, ws, ws.T, st)) != RFX_OK) return rc;
        return apply_small(Y, N, k, ws.T, k, V, st);
    }
    if ((rc = gram(Y, Y, N, k, true, ws, ws.G, st)) != RFX_OK) return rc;
    if ((rc = chol_inverse(ws.G, k, ws, ws.T, st)) != RFX_OK) return rc;
    if ((rc = apply_small(Y, N, k, ws.T, k, Z, st)) != RFX_OK) return rc;
    if ((rc = gram(Z, Z, N, k, true, ws, ws.G, st)) != RFX_OK) return rc;
    if ((rc = chol_inverse(ws.G, k, ws, ws.T, st)) != RFX_OK) return rc;
    return apply_small(Z, N, k, ws.T, k, V, st);
}

int fix_signs(float* V, int64_t N, int kc, SmallWs& ws, hipStream_t st) {
    if (kc < 1 || kc > kMaxRank || !ws.sign_val) return fail(RFX_ERR_INVALID_ARG, "fix_signs: kc=%d", kc);
    int kpad = 1;
    while (kpad < kc) kpad <<= 1;
    const int64_t rows_per_block = ceil_div(N, kSignBlocks);
    const int blocks = (int)ceil_div(N, rows_per_block);
    hipLaunchKernelGGL(sign_partial_kernel, dim3(blocks), dim3(256), 0, st, V, N, kc, kpad, rows_per_block, ws.sign_val,
                       ws.sign_row);
    hipLaunchKernelGGL(sign_apply_kernel, dim3(blocks), dim3(256), 0, st, V, N, kc, kpad, rows_per_block, blocks,
                       ws.sign_val, ws.sign_row);
    RFX_LAUNCH_CHECK("fix_signs kernels");
    return RFX_OK;
}

}  // namespace rfx
