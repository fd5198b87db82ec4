// 3-D scaling coordinates from the INT8 proximity factors (paper, "GPU-Accelerated 3D MDS from
// Low-Rank Proximity Matrices", Steps 1-4).
//
// With A^ = Q diag(scales) (N x k), P^ = A^ A^^T and D = 1 - P^, the Gram matrix of the scaling is
// G = -1/2 H D2 H, H = I - 11^T/N, D2 = D o D (SQUARED) or D (LINEAR).  G is never formed.  For a
// vector v: u = H v (so sum u = 0), z = D2 u, w = H z, G v = -w/2 (Step 3), and with
// p_ij = a_i . a_j
//     SQUARED: (1 - p)^2 = 1 - 2p + p^2  =>  z_i = -2 a_i . t + a_i^T M a_i
//     LINEAR :                               z_i = -a_i . t
// where t = A^^T u (k) and M = A^^T diag(u) A^ (k x k); the constant term vanishes because sum u = 0.
// A block of m vectors is iterated at once with a Rayleigh-Ritz step per iteration.
#include <cmath>
#include <vector>

#include "common.h"
#include "dense_small.h"

namespace {

constexpr int kRowsStage = 32;

// The factor is read either as float32 (A itself) or as INT8 codes with one float32 scale per column; the codes are
// decoded where they are used (code * scale, rounded to float32: the value a separate decoding pass would store),
// so an INT8 factor is streamed at one byte per entry and no float32 copy of it exists.
__device__ __forceinline__ float factor_at(const float* A, const float*, int64_t at, int) { return A[at]; }
__device__ __forceinline__ float factor_at(const int8_t* A, const float* scales, int64_t at, int col) {
    return (float)A[at] * scales[col];
}
// four consecutive entries of a row starting at column `col` (a multiple of 4; the row start is aligned for the load)
__device__ __forceinline__ float4 factor_at4(const float* A, const float*, int64_t at, int) {
    return *reinterpret_cast<const float4*>(A + at);
}
__device__ __forceinline__ float4 factor_at4(const int8_t* A, const float* scales, int64_t at, int col) {
    const char4 q = *reinterpret_cast<const char4*>(A + at);
    return float4{(float)q.x * scales[col], (float)q.y * scales[col + 1], (float)q.z * scales[col + 2],
                  (float)q.w * scales[col + 3]};
}

// partial[block][c] = sum of column c over the block's rows (float64)
__global__ __launch_bounds__(256) void col_sums_partial_kernel(const float* __restrict__ X, int64_t N, int m,
                                                              int64_t rows_per_block, double* __restrict__ partial) {
    __shared__ double red[256];
    const int64_t i_begin = (int64_t)blockIdx.x * rows_per_block;
    const int64_t i_end = min(N, i_begin + rows_per_block);
    // thread t handles column t % m of rows t / m, t / m + 256 / m, ...
    const int per = 256 / m;  // rows in flight (m <= 32)
    const int c = threadIdx.x % m, r0 = threadIdx.x / m;
    double s = 0.0;
    if (r0 < per)
        for (int64_t i = i_begin + r0; i < i_end; i += per) s += (double)X[i * m + c];
    red[threadIdx.x] = (r0 < per) ? s : 0.0;
    __syncthreads();
    if (threadIdx.x < m) {
        double tot = 0.0;
        for (int r = 0; r < per; ++r) tot += red[r * m + threadIdx.x];
        partial[(int64_t)blockIdx.x * m + threadIdx.x] = tot;
    }
}

// sums[c] = sum over blocks of partial[block][c].  Eight lanes share a column (m <= 32): lane part p adds blocks
// p, p + 8, ..., then the eight sums are added pairwise in a fixed order.
__global__ __launch_bounds__(256) void col_sums_reduce_kernel(const double* __restrict__ partial, int blocks, int m,
                                                             double* __restrict__ sums) {
    const int c = threadIdx.x >> 3, part = threadIdx.x & 7;
    double s = 0.0;
    if (c < m) {
#pragma unroll 4
        for (int b = part; b < blocks; b += 8) s += partial[(int64_t)b * m + c];
    }
    for (int off = 4; off > 0; off >>= 1) s += __shfl_xor(s, off, 8);
    if (c < m && part == 0) sums[c] = s;
}

// For column c = blockIdx.y, over the block's rows, with u_i = X[i][c] - mean_c:
//   partialT[block][c][q]    = sum_i u_i a_iq
//   partialM[block][c][p][q] = sum_i u_i a_ip a_iq        (SQUARED only)
template <int NB, class TA>
__global__ __launch_bounds__(256) void mds_moments_kernel(const TA* __restrict__ A, const float* __restrict__ scales,
                                                         const float* __restrict__ X, const double* __restrict__ colsum,
                                                         int64_t N, int k, int m, int64_t rows_per_block, int squared,
                                                         double* __restrict__ partialM, double* __restrict__ partialT) {
    extern __shared__ float mom_sm[];
    float* As = mom_sm;                                   // [kRowsStage][k]
    double* us = (double*)(mom_sm + kRowsStage * k);      // [kRowsStage]
    const int c = blockIdx.y;
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
    const double mean = colsum[c] / (double)N;
    double acc[NB][NB], tacc[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        tacc[u] = 0.0;
#pragma unroll
        for (int v = 0; v < NB; ++v) acc[u][v] = 0.0;
    }
    const int64_t i_begin = (int64_t)blockIdx.x * rows_per_block;
    const int64_t i_end = min(N, i_begin + rows_per_block);
    for (int64_t i0 = i_begin; i0 < i_end; i0 += kRowsStage) {
        const int rows = (int)min((int64_t)kRowsStage, i_end - i0);
        for (int e = threadIdx.x; e < rows * k; e += 256) As[e] = factor_at(A, scales, i0 * k + e, e % k);
        if (threadIdx.x < rows) us[threadIdx.x] = (double)X[(i0 + threadIdx.x) * m + c] - mean;
        __syncthreads();
        for (int r = 0; r < rows; ++r) {
            const double ur = us[r];
            double a[NB], b[NB];
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int p = ty + 16 * u, q = tx + 16 * u;
                a[u] = p < k ? (double)As[r * k + p] : 0.0;
                b[u] = q < k ? ur * (double)As[r * k + q] : 0.0;
            }
            if (ty == 0) {
#pragma unroll
                for (int v = 0; v < NB; ++v) tacc[v] += b[v];
            }
            if (squared) {
#pragma unroll
                for (int u = 0; u < NB; ++u)
#pragma unroll
                    for (int v = 0; v < NB; ++v) acc[u][v] = fma(a[u], b[v], acc[u][v]);
            }
        }
        __syncthreads();
    }
    const int64_t slot = (int64_t)blockIdx.x * m + c;
    if (ty == 0) {
#pragma unroll
        for (int v = 0; v < NB; ++v) {
            const int q = tx + 16 * v;
            if (q < k) partialT[slot * k + q] = tacc[v];
        }
    }
    if (squared) {
        double* out = partialM + slot * k * k;
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
            for (int v = 0; v < NB; ++v) {
                const int p = ty + 16 * u, q = tx + 16 * v;
                if (p < k && q < k) out[p * k + q] = acc[u][v];
            }
    }
}

// The same moments on the matrix cores (SQUARED, k <= 64): M_c = sum_i a_i (u_i a_i)^T is a Gram product with
// the sample index as the contraction, 4 samples per v_mfma_f64_16x16x4_f64.  Lane l of a wave supplies element
// (row i0 + l / 16, column 16 tile + l % 16) of A for the left operand and of diag(u) A for the right one; result
// register v of lane l is entry (16 tile_p + l / 16 + 4 v, 16 tile_q + l % 16).  The four waves of a workgroup take
// a quarter of its rows each and add their tiles up in LDS in wave order, so the sums do not depend on timing.
// Tiles below the diagonal are copies of their mirror images.
typedef double mds_double4_t __attribute__((ext_vector_type(4)));

template <int NB, class TA>
__global__ __launch_bounds__(256) void mds_moments_mfma_kernel(const TA* __restrict__ A, const float* __restrict__ scales,
                                                              const float* __restrict__ X,
                                                              const double* __restrict__ colsum, int64_t N, int k, int m,
                                                              int64_t rows_per_block, double* __restrict__ partialM,
                                                              double* __restrict__ partialT) {
    extern __shared__ double mfma_sm[];  // [k][k] tiles of M, then [k] of T
    const int c = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane >> 4, c16 = lane & 15;
    const double mean = colsum[c] / (double)N;
    const int64_t b_begin = (int64_t)blockIdx.x * rows_per_block;
    const int64_t b_end = min(N, b_begin + rows_per_block);
    const int64_t per_wave = ((b_end - b_begin + 3) / 4 + 3) / 4 * 4;  // whole groups of 4 rows
    const int64_t i_begin = min(b_end, b_begin + wave * per_wave), i_end = min(b_end, i_begin + per_wave);
    mds_double4_t acc[NB][NB];
    double tacc[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        tacc[u] = 0.0;
#pragma unroll
        for (int w = 0; w < NB; ++w) acc[u][w] = mds_double4_t{0.0, 0.0, 0.0, 0.0};
    }
    for (int64_t i0 = i_begin; i0 < i_end; i0 += 4) {
        const int64_t row = i0 + r;
        const bool live = row < i_end;
        const double u_i = live ? (double)X[row * m + c] - mean : 0.0;
        double a[NB], b[NB];
#pragma unroll
        for (int w = 0; w < NB; ++w) {
            const int col = 16 * w + c16;
            a[w] = (live && col < k) ? (double)factor_at(A, scales, row * k + col, col) : 0.0;
            b[w] = u_i * a[w];
            tacc[w] += b[w];
        }
        // M_c is symmetric: only the tiles on and above the diagonal are accumulated
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
            for (int w = u; w < NB; ++w) acc[u][w] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[u], b[w], acc[u][w], 0, 0, 0);
    }
    // T: the four row groups of a wave (lanes c16, c16 + 16, ...) hold partial sums of the same columns
#pragma unroll
    for (int w = 0; w < NB; ++w) {
        tacc[w] += __shfl_xor(tacc[w], 16);
        tacc[w] += __shfl_xor(tacc[w], 32);
    }
    double* Ms = mfma_sm;
    double* Ts = mfma_sm + k * k;
    for (int w4 = 0; w4 < 4; ++w4) {
        if (wave == w4) {
#pragma unroll
            for (int u = 0; u < NB; ++u)
#pragma unroll
                for (int w = u; w < NB; ++w)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int p = 16 * u + r + 4 * v, q = 16 * w + c16;
                        if (p < k && q < k) {
                            const double sum = (w4 == 0 ? 0.0 : Ms[p * k + q]) + acc[u][w][v];
                            Ms[p * k + q] = sum;
                            if (w > u) Ms[q * k + p] = sum;  // the mirrored tile below the diagonal
                        }
                    }
            if (r == 0) {
#pragma unroll
                for (int w = 0; w < NB; ++w) {
                    const int q = 16 * w + c16;
                    if (q < k) Ts[q] = (w4 == 0 ? 0.0 : Ts[q]) + tacc[w];
                }
            }
        }
        __syncthreads();
    }
    const int64_t slot = (int64_t)blockIdx.x * m + c;
    for (int e = threadIdx.x; e < k * k; e += 256) partialM[slot * k * k + e] = Ms[e];
    for (int e = threadIdx.x; e < k; e += 256) partialT[slot * k + e] = Ts[e];
}

// M[c][e] = sum_block partialM[block][c][e];  T[c][q] likewise.  len = k*k or k.
__global__ __launch_bounds__(256) void moments_reduce_kernel(const double* __restrict__ partial, int blocks, int m,
                                                            int len, double* __restrict__ out) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    const int c = blockIdx.y;
    if (e >= len) return;
    double s = 0.0;
    for (int b = 0; b < blocks; ++b) s += partial[((int64_t)b * m + c) * len + e];
    out[(int64_t)c * len + e] = s;
}

// Z[i][c] for a tile of RT rows and column c = blockIdx.y:
//   SQUARED: a_i^T (M_c a_i) - 2 t_c . a_i      LINEAR: -t_c . a_i
// (RT/16) x NB register tile per thread of the product A^ M_c, then a row reduction over the
// 16 threads that share a row.
template <int NB, int RT, class TA>
__global__ __launch_bounds__(256) void mds_quad_kernel(const TA* __restrict__ A, const float* __restrict__ scales,
                                                      const double* __restrict__ M, const double* __restrict__ T,
                                                      int64_t N, int k, int m, int squared, float* __restrict__ Z) {
    extern __shared__ double quad_sm[];
    double* Ms = quad_sm;                     // [k][k]   (SQUARED only)
    double* ts = Ms + (squared ? k * k : 0);  // [k]
    float* As = (float*)(ts + k);             // [RT][k]
    const int c = blockIdx.y;
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
    const int64_t i0 = (int64_t)blockIdx.x * RT;
    const int rows = (int)min((int64_t)RT, N - i0);
    if (squared)
        for (int e = threadIdx.x; e < k * k; e += 256) Ms[e] = M[(int64_t)c * k * k + e];
    for (int e = threadIdx.x; e < k; e += 256) ts[e] = T[(int64_t)c * k + e];
    for (int e = threadIdx.x; e < RT * k; e += 256)
        As[e] = e < rows * k ? factor_at(A, scales, i0 * k + e, e % k) : 0.0f;
    __syncthreads();
    constexpr int RU = RT / 16;
    double acc[RU][NB];
#pragma unroll
    for (int u = 0; u < RU; ++u)
#pragma unroll
        for (int v = 0; v < NB; ++v) acc[u][v] = 0.0;
    if (squared) {
        for (int q = 0; q < k; ++q) {
            double a[RU], mq[NB];
#pragma unroll
            for (int u = 0; u < RU; ++u) a[u] = (double)As[(ty + 16 * u) * k + q];
#pragma unroll
            for (int v = 0; v < NB; ++v) {
                const int p = tx + 16 * v;
                mq[v] = p < k ? Ms[q * k + p] : 0.0;
            }
#pragma unroll
            for (int u = 0; u < RU; ++u)
#pragma unroll
                for (int v = 0; v < NB; ++v) acc[u][v] = fma(a[u], mq[v], acc[u][v]);
        }
    }
#pragma unroll
    for (int u = 0; u < RU; ++u) {
        const int r = ty + 16 * u;
        double z = 0.0;
#pragma unroll
        for (int v = 0; v < NB; ++v) {
            const int p = tx + 16 * v;
            if (p < k) {
                const double ap = (double)As[r * k + p];
                z += squared ? (acc[u][v] - 2.0 * ts[p]) * ap : -ts[p] * ap;
            }
        }
        // sum over the 16 consecutive lanes that hold this row
        for (int off = 8; off > 0; off >>= 1) z += __shfl_xor(z, off, 16);
        if (tx == 0 && r < rows) Z[(i0 + r) * m + c] = (float)z;
    }
}

// The SQUARED quadratic form on the matrix cores for k a multiple of 16, k <= 64, rows of A aligned for a 4-entry load:
// B = A M_c by v_mfma_f64_16x16x4_f64 on tiles of 16 rows, then Z[i][c] = sum_q (B[i][q] - 2 t_c[q]) A[i][q].
// Lane l = (g = l / 16, r = l % 16) loads A[i0 + r][16 jj + 4 g .. + 3] with one load per jj (16 bytes of float32, 4 of INT8 codes); instruction
// j = 4 jj + t contracts columns 16 jj + 4 g' + t (g' = 0..3) and the matching entries of M_c stay in registers for
// all tiles of the wave.  Result register v of lane l is B[i0 + g + 4 v][16 w + r]; the entries of A at those
// positions are read again (they are in the first-level cache) and the 16 lanes of a row group are summed.
template <int KB, class TA>
__global__ __launch_bounds__(256) void mds_quad_mfma_kernel(const TA* __restrict__ A, const float* __restrict__ scales,
                                                           const double* __restrict__ M,
                                                           const double* __restrict__ T, int64_t N, int m,
                                                           float* __restrict__ Z) {
    constexpr int k = 16 * KB;
    extern __shared__ double quad_sm[];  // [k][k] M_c, then [k] t_c
    const int c = blockIdx.y;
    for (int e = threadIdx.x; e < k * k; e += 256) quad_sm[e] = M[(int64_t)c * k * k + e];
    for (int e = threadIdx.x; e < k; e += 256) quad_sm[k * k + e] = T[(int64_t)c * k + e];
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 4, r = lane & 15;
    double mb[4 * KB][KB], t2[KB];
#pragma unroll
    for (int j = 0; j < 4 * KB; ++j)
#pragma unroll
        for (int w = 0; w < KB; ++w) mb[j][w] = quad_sm[(16 * (j / 4) + 4 * g + (j % 4)) * k + 16 * w + r];
#pragma unroll
    for (int w = 0; w < KB; ++w) t2[w] = 2.0 * quad_sm[k * k + 16 * w + r];
    const int64_t tiles = (N + 15) / 16;
    for (int64_t tile = (int64_t)blockIdx.x * 4 + wave; tile < tiles; tile += (int64_t)gridDim.x * 4) {
        const int64_t i0 = tile * 16;
        const bool live = i0 + r < N;
        float4 av[KB];
#pragma unroll
        for (int jj = 0; jj < KB; ++jj)
            av[jj] = live ? factor_at4(A, scales, (i0 + r) * k + 16 * jj + 4 * g, 16 * jj + 4 * g) : float4{0.f, 0.f, 0.f, 0.f};
        float ad[4][KB];  // A at the positions of the result registers
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int w = 0; w < KB; ++w) ad[v][w] = i0 + g + 4 * v < N ? factor_at(A, scales, (i0 + g + 4 * v) * k + 16 * w + r, 16 * w + r) : 0.0f;
        mds_double4_t acc[KB];
#pragma unroll
        for (int w = 0; w < KB; ++w) acc[w] = mds_double4_t{0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int jj = 0; jj < KB; ++jj) {
            const double a4[4] = {(double)av[jj].x, (double)av[jj].y, (double)av[jj].z, (double)av[jj].w};
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int w = 0; w < KB; ++w)
                    acc[w] = __builtin_amdgcn_mfma_f64_16x16x4f64(a4[t], mb[4 * jj + t][w], acc[w], 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            double z = 0.0;
#pragma unroll
            for (int w = 0; w < KB; ++w) z += (acc[w][v] - t2[w]) * (double)ad[v][w];
            for (int off = 8; off > 0; off >>= 1) z += __shfl_xor(z, off, 16);
            const int64_t row = i0 + g + 4 * v;
            if (r == 0 && row < N) Z[row * m + c] = (float)z;
        }
    }
}

// Y[i][c] = -1/2 (Z[i][c] - mean_c(Z))
__global__ __launch_bounds__(256) void mds_center_kernel(const float* __restrict__ Z, const double* __restrict__ colsum,
                                                        int64_t N, int m, float* __restrict__ Y) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= N * m) return;
    const int c = (int)(e % m);
    Y[e] = (float)(-0.5 * ((double)Z[e] - colsum[c] / (double)N));
}

// coords[i][d] = sqrt(max(theta_d, 0)) * V[i][d] for d < 3 (V has row stride 3); eigvals[d] = theta_d
__global__ __launch_bounds__(256) void mds_coords_kernel(float* __restrict__ V, const double* __restrict__ theta, int64_t N,
                                                        float* __restrict__ eigvals) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < 3) eigvals[e] = (float)theta[e];
    if (e >= N * 3) return;
    const double th = theta[e % 3];
    V[e] = (float)((double)V[e] * sqrt(th > 0.0 ? th : 0.0));
}

// What the iteration carries from one application of G to the next, on the device.
struct MdsState {
    double prev[3];  // the three leading Ritz values of the previous application
    double sigma;    // spectral shift: the largest -theta_min seen so far (0 while no Ritz value was negative)
    double rel;      // largest relative change of the three leading Ritz values in the last application
    int32_t lost_rank;
    int32_t pad;
};

__global__ void mds_state_init_kernel(MdsState* s) {
    s->prev[0] = s->prev[1] = s->prev[2] = 0.0;
    s->sigma = 0.0;
    s->rel = __builtin_inf();
    s->lost_rank = 0;
    s->pad = 0;
}

// After a Rayleigh-Ritz step (theta descending, m values).  Records the relative change of the three leading Ritz
// values, and raises the shift to -theta_min when the smallest Ritz value of the block is negative.  Ritz values lie
// inside the spectrum of G, so the shift never exceeds |lambda_min(G)|; it only grows, and once the block contains the
// most negative eigenvector the shift reaches |lambda_min|, G + sigma I is positive semi-definite and the iteration
// converges to the algebraically largest eigenvalues (MDS Steps 3-4 ask for the largest eigenvalues, not the
// largest magnitudes).
__global__ void mds_track_kernel(const double* __restrict__ theta, int m, int first, MdsState* s, float* rel_out) {
    double rel = first ? __builtin_inf() : 0.0;
    for (int d = 0; d < 3; ++d) {
        const double diff = fabs(theta[d] - s->prev[d]), mag = fabs(theta[d]);
        if (!first) rel = fmax(rel, diff > 0.0 ? (mag > 0.0 ? diff / mag : __builtin_inf()) : 0.0);
        s->prev[d] = theta[d];
    }
    s->rel = rel;
    if (rel_out) *rel_out = (float)rel;
    const double lo = theta[m - 1];
    if (lo < 0.0 && -lo > s->sigma) s->sigma = -lo;
}

// Y += sigma X (the block that is orthonormalised next spans (G + sigma I) X)
__global__ __launch_bounds__(256) void mds_shift_kernel(float* __restrict__ Y, const float* __restrict__ X, int64_t total,
                                                       const MdsState* __restrict__ s) {
    const double sigma = s->sigma;
    if (sigma == 0.0) return;
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < total) Y[e] = (float)((double)Y[e] + sigma * (double)X[e]);
}

// Scratch of one run, carved from one buffer: the small dense workspace, the float64 partial moments, three blocks
// of N x m floats and the iteration state.
struct MdsWs {
    int blocks = 0;
    int64_t rows_per_block = 0;
    double* colsum_partial = nullptr;  // [blocks][m]
    double* colsum = nullptr;          // [m]
    double* partialM = nullptr;        // [blocks][m][k][k]
    double* partialT = nullptr;        // [blocks][m][k]
    double* M = nullptr;               // [m][k][k]
    double* T = nullptr;               // [m][k]
    float *X = nullptr, *Y = nullptr, *Z = nullptr;  // [N][m] each
    MdsState* state = nullptr;
    rfx::SmallWs small;
};

struct MdsLayout {
    int blocks;
    int64_t rows_per_block;
    size_t small_bytes, doubles, block_floats, total;
};

MdsLayout mds_layout(int64_t N, int k, int m, int squared) {
    MdsLayout l;
    l.blocks = (int)std::min<int64_t>(256, rfx::ceil_div(N, kRowsStage));
    l.rows_per_block = rfx::ceil_div(rfx::ceil_div(N, l.blocks), kRowsStage) * kRowsStage;
    l.blocks = (int)rfx::ceil_div(N, l.rows_per_block);
    const size_t kk = (size_t)k * k;
    l.small_bytes = rfx::SmallWs::bytes(N, m);
    l.doubles = (size_t)l.blocks * m + m + (size_t)l.blocks * m * (squared ? kk : 0) + (size_t)l.blocks * m * k +
                (size_t)m * kk + (size_t)m * k;
    l.block_floats = ((size_t)N * m + 63) & ~(size_t)63;
    l.total = l.small_bytes + ((l.doubles * sizeof(double) + 255) & ~(size_t)255) + 3 * l.block_floats * sizeof(float) + 256;
    return l;
}

int mds_bind(MdsWs& w, void* mem, int64_t N, int k, int m, int squared, hipStream_t st) {
    const MdsLayout l = mds_layout(N, k, m, squared);
    w.blocks = l.blocks;
    w.rows_per_block = l.rows_per_block;
    char* base = static_cast<char*>(mem);
    int rc = w.small.bind(base, N, m, st);
    if (rc != RFX_OK) return rc;
    base += l.small_bytes;
    const size_t kk = (size_t)k * k;
    double* p = reinterpret_cast<double*>(base);
    w.colsum_partial = p;
    p += (size_t)w.blocks * m;
    w.colsum = p;
    p += m;
    w.partialM = p;
    p += (size_t)w.blocks * m * (squared ? kk : 0);
    w.partialT = p;
    p += (size_t)w.blocks * m * k;
    w.M = p;
    p += (size_t)m * kk;
    w.T = p;
    base += (l.doubles * sizeof(double) + 255) & ~(size_t)255;
    w.X = reinterpret_cast<float*>(base);
    w.Y = w.X + l.block_floats;
    w.Z = w.Y + l.block_floats;
    w.state = reinterpret_cast<MdsState*>(w.Z + l.block_floats);
    hipLaunchKernelGGL(mds_state_init_kernel, dim3(1), dim3(1), 0, st, w.state);
    RFX_LAUNCH_CHECK("mds_state_init_kernel");
    return RFX_OK;
}

int col_sums(const float* X, int64_t N, int m, MdsWs& w, hipStream_t st) {
    hipLaunchKernelGGL(col_sums_partial_kernel, dim3(w.blocks), dim3(256), 0, st, X, N, m, w.rows_per_block,
                       w.colsum_partial);
    hipLaunchKernelGGL(col_sums_reduce_kernel, dim3(1), dim3(256), 0, st, w.colsum_partial, w.blocks, m, w.colsum);
    RFX_LAUNCH_CHECK("col_sums");
    return RFX_OK;
}

template <int NB, class TA>
int apply_gram_nb(const TA* A, const float* scales, int64_t N, int k, int m, int squared, const float* X, float* Z,
                  float* Y, MdsWs& w, hipStream_t st) {
    int rc;
    if ((rc = col_sums(X, N, m, w, st)) != RFX_OK) return rc;
    {
        int mom_blocks = w.blocks;
        if (squared && NB <= 4) {
            // few, long row ranges: the tiles are added up and written once per workgroup
            mom_blocks = std::min(w.blocks, 64);
            const int64_t rows_per = rfx::ceil_div(rfx::ceil_div(N, mom_blocks), 16) * 16;
            mom_blocks = (int)rfx::ceil_div(N, rows_per);
            const size_t lds = sizeof(double) * ((size_t)k * k + k);
            hipLaunchKernelGGL((mds_moments_mfma_kernel<(NB <= 4 ? NB : 1), TA>), dim3(mom_blocks, m), dim3(256), lds, st, A,
                               scales, X, w.colsum, N, k, m, rows_per, w.partialM, w.partialT);
        } else {
            const size_t lds = sizeof(float) * kRowsStage * (size_t)k + sizeof(double) * kRowsStage;
            hipLaunchKernelGGL((mds_moments_kernel<NB, TA>), dim3(w.blocks, m), dim3(256), lds, st, A, scales, X, w.colsum, N,
                               k, m, w.rows_per_block, squared, w.partialM, w.partialT);
        }
        RFX_LAUNCH_CHECK("mds_moments_kernel");
        if (squared)
            hipLaunchKernelGGL(moments_reduce_kernel, dim3((unsigned)rfx::ceil_div(k * k, 256), m), dim3(256), 0, st,
                               w.partialM, mom_blocks, m, k * k, w.M);
        hipLaunchKernelGGL(moments_reduce_kernel, dim3((unsigned)rfx::ceil_div(k, 256), m), dim3(256), 0, st, w.partialT,
                           mom_blocks, m, k, w.T);
        RFX_LAUNCH_CHECK("moments_reduce_kernel");
    }
    if (squared && k % 16 == 0 && k <= 64 && reinterpret_cast<uintptr_t>(A) % (4 * sizeof(TA)) == 0) {
        const size_t lds = sizeof(double) * ((size_t)k * k + k);
        dim3 grid((unsigned)std::min<int64_t>(rfx::ceil_div(rfx::ceil_div(N, 16), 4), 64), m);
        switch (k / 16) {
            case 1: hipLaunchKernelGGL((mds_quad_mfma_kernel<1, TA>), grid, dim3(256), lds, st, A, scales, w.M, w.T, N, m, Z); break;
            case 2: hipLaunchKernelGGL((mds_quad_mfma_kernel<2, TA>), grid, dim3(256), lds, st, A, scales, w.M, w.T, N, m, Z); break;
            case 3: hipLaunchKernelGGL((mds_quad_mfma_kernel<3, TA>), grid, dim3(256), lds, st, A, scales, w.M, w.T, N, m, Z); break;
            default: hipLaunchKernelGGL((mds_quad_mfma_kernel<4, TA>), grid, dim3(256), lds, st, A, scales, w.M, w.T, N, m, Z); break;
        }
        RFX_LAUNCH_CHECK("mds_quad_mfma_kernel");
    } else {
        const bool small_tile = k > 96;
        const int RT = small_tile ? 32 : 64;
        const size_t lds = sizeof(double) * ((squared ? (size_t)k * k : 0) + k) + sizeof(float) * (size_t)RT * k;
        dim3 grid((unsigned)rfx::ceil_div(N, RT), m);
        if (small_tile) {
            auto kern = mds_quad_kernel<NB, 32, TA>;
            if (lds > 64 * 1024)
                RFX_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, A, scales, w.M, w.T, N, k, m, squared, Z);
        } else {
            auto kern = mds_quad_kernel<NB, 64, TA>;
            if (lds > 64 * 1024)
                RFX_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, A, scales, w.M, w.T, N, k, m, squared, Z);
        }
        RFX_LAUNCH_CHECK("mds_quad_kernel");
    }
    if ((rc = col_sums(Z, N, m, w, st)) != RFX_OK) return rc;
    hipLaunchKernelGGL(mds_center_kernel, dim3((unsigned)rfx::ceil_div(N * m, 256)), dim3(256), 0, st, Z, w.colsum, N, m, Y);
    RFX_LAUNCH_CHECK("mds_center_kernel");
    return RFX_OK;
}

// Y = G X for a block X [N][m]; Z is an [N][m] temporary.
template <class TA>
int apply_gram(const TA* A, const float* scales, int64_t N, int k, int m, int squared, const float* X, float* Z, float* Y,
               MdsWs& w, hipStream_t st) {
    switch ((k + 15) / 16) {
#define RFX_CASE(nb) \
    case nb:         \
        return apply_gram_nb<nb, TA>(A, scales, N, k, m, squared, X, Z, Y, w, st);
        RFX_CASE(1) RFX_CASE(2) RFX_CASE(3) RFX_CASE(4) RFX_CASE(5) RFX_CASE(6) RFX_CASE(7) RFX_CASE(8)
#undef RFX_CASE
    }
    return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_mds3d: k=%d", k);
}

int check_args(const void* A, int64_t N, int32_t k, int dissim_mode, int32_t m, int32_t iters, const float* x0,
               const float* coords, const float* eigvals) {
    (void)x0;  // null: the block starts from the leading columns of the factor
    if (!A || !coords || !eigvals) return rfx::fail(RFX_ERR_NULL, "rfx_mds3d: null argument");
    if (N < 3 || N * 32 / 256 > 0x7fffffffLL) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_mds3d: N=%lld", (long long)N);
    if (k < 1 || k > rfx::kMaxRank) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_mds3d: k=%d outside 1..%d", k, rfx::kMaxRank);
    if (m < 3 || m > 32 || m > N) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_mds3d: m=%d outside 3..min(32, N)", m);
    if (dissim_mode != RFX_MDS_SQUARED && dissim_mode != RFX_MDS_LINEAR)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_mds3d: dissim_mode=%d", dissim_mode);
    if (iters < 1) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_mds3d: iterations=%d", iters);
    return RFX_OK;
}

// The host looks at the convergence state every kCheckEvery applications (one 8-byte copy and one wait), not after
// each of them (the relative change needs two applications anyway).
constexpr int kCheckEvery = 2;

// Start block when the caller gives none: the m leading columns of the factor.  G is H A A^T H plus (squared mode) a term of the
// same column space squared, so the columns of A that belong to the largest eigenvalues of P nearly span the subspace wanted
// and the iteration has little left to do.  Where m > k the block is filled up with fixed pseudo-random columns (a mixing
// function of row and column: the same block on every call).
template <class TA>
__global__ __launch_bounds__(256) void mds_start_kernel(const TA* __restrict__ A, const float* __restrict__ scales, int64_t N,
                                                       int32_t k, int32_t m, float* __restrict__ X0) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= N * m) return;
    const int64_t i = e / m;
    const int c = (int)(e % m);
    if (c < k) {
        X0[e] = factor_at(A, scales, i * k + c, c);
    } else {
        unsigned long long z = (unsigned long long)e * 0x9e3779b97f4a7c15ull + 0xbf58476d1ce4e5b9ull;
        z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
        z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
        z ^= z >> 31;
        X0[e] = (float)(z >> 40) * (1.0f / 8388608.0f) - 1.0f;   // 24 bits -> [-1, 1)
    }
}

// Simultaneous iteration on the block.  tol < 0: exactly max_iters applications and no host read-back (nothing in
// this function waits for the device); otherwise the run stops at the first check that finds the last application's
// relative change of the three leading Ritz values at or below tol.
template <class TA>
int mds_iterate(const TA* A, const float* scales, int64_t N, int32_t k, int squared, int32_t m, int32_t max_iters, float tol,
                const float* x0, float* coords, float* eigvals, float* rel_change, int32_t* iters_done, MdsWs& w,
                hipStream_t st) {
    rfx::SmallWs& ws = w.small;
    float *X = w.X, *Y = w.Y, *Z = w.Z;
    int rc;
    if (!x0) {
        hipLaunchKernelGGL(mds_start_kernel<TA>, dim3((unsigned)rfx::ceil_div(N * m, 256)), dim3(256), 0, st, A, scales, N, k, m, Y);
        RFX_LAUNCH_CHECK("mds_start_kernel");
        x0 = Y;
    }
    if ((rc = rfx::orthonormalise(x0, N, m, ws, Z, X, st, 2)) != RFX_OK) return rc;
    int it = 0;
    while (true) {
        // Y = G X, H = sym(X^T Y) = W diag(theta) W^T (theta descending by algebraic value)
        if ((rc = apply_gram(A, scales, N, k, m, squared, X, Z, Y, w, st)) != RFX_OK) return rc;
        ++it;
        if ((rc = rfx::gram(X, Y, N, m, true, ws, ws.G, st)) != RFX_OK) return rc;
        if ((rc = rfx::jacobi_eigh(ws.G, m, ws, ws.theta, ws.W, st)) != RFX_OK) return rc;
        hipLaunchKernelGGL(mds_track_kernel, dim3(1), dim3(1), 0, st, ws.theta, m, it == 1 ? 1 : 0, w.state, rel_change);
        RFX_LAUNCH_CHECK("mds_track_kernel");
        if (it >= max_iters) break;
        if (tol >= 0.0f && it > 1 && it % kCheckEvery == 0) {
            double rel = 0.0;
            RFX_HIP(hipMemcpyAsync(&rel, &w.state->rel, sizeof(double), hipMemcpyDeviceToHost, st));
            RFX_HIP(hipStreamSynchronize(st));
            if (rel <= (double)tol) break;
        }
        // next block: orth((G + sigma I) X)
        hipLaunchKernelGGL(mds_shift_kernel, dim3((unsigned)rfx::ceil_div(N * m, 256)), dim3(256), 0, st, Y, X, N * m, w.state);
        RFX_LAUNCH_CHECK("mds_shift_kernel");
        if ((rc = rfx::orthonormalise(Y, N, m, ws, Z, X, st, 2)) != RFX_OK) return rc;
    }
    // Ritz vectors of the three largest values: coords = X W[:, 0:3] scaled by sqrt(theta)
    if ((rc = rfx::apply_small(X, N, m, ws.W, 3, coords, st)) != RFX_OK) return rc;
    if ((rc = rfx::fix_signs(coords, N, 3, ws, st)) != RFX_OK) return rc;
    hipLaunchKernelGGL(mds_coords_kernel, dim3((unsigned)rfx::ceil_div(N * 3, 256)), dim3(256), 0, st, coords, ws.theta, N,
                       eigvals);
    RFX_LAUNCH_CHECK("mds_coords_kernel");
    if (iters_done) *iters_done = it;
    return RFX_OK;
}

// The synchronous entry points: scratch allocated for the call and freed after a final wait.
template <class TA>
int mds_sync(const TA* A, const float* scales, int64_t N, int32_t k, int dissim_mode, int32_t m, int32_t max_iters, float tol,
             const float* x0, float* coords, float* eigvals, int32_t* iters_done, hipStream_t st) {
    int rc = check_args(A, N, k, dissim_mode, m, max_iters, x0, coords, eigvals);
    if (rc != RFX_OK) return rc;
    if (!(tol >= 0.0f)) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_mds3d: tol=%g", tol);
    const int squared = dissim_mode == RFX_MDS_SQUARED;
    rfx::DevBuf buf;
    RFX_HIP(buf.alloc(mds_layout(N, k, m, squared).total));
    MdsWs w;
    if ((rc = mds_bind(w, buf.p, N, k, m, squared, st)) != RFX_OK) return rc;
    rc = mds_iterate(A, scales, N, k, squared, m, max_iters, tol, x0, coords, eigvals, nullptr, iters_done, w, st);
    hipError_t e = hipStreamSynchronize(st);  // the scratch is freed on return
    if (rc != RFX_OK) return rc;
    if (e != hipSuccess) return rfx::fail(RFX_ERR_HIP, "rfx_mds3d: kernels failed: %s", hipGetErrorString(e));
    return RFX_OK;
}

}  // namespace

extern "C" {

int rfx_mds3d_workspace_bytes(int64_t N, int32_t k, int32_t m, int dissim_mode, int64_t* bytes) {
    if (!bytes) return rfx::fail(RFX_ERR_NULL, "rfx_mds3d_workspace_bytes: bytes is null");
    float dummy = 0.0f;
    int rc = check_args(&dummy, N, k, dissim_mode, m, 1, &dummy, &dummy, &dummy);
    if (rc != RFX_OK) return rc;
    *bytes = (int64_t)mds_layout(N, k, m, dissim_mode == RFX_MDS_SQUARED).total;
    return RFX_OK;
}

int rfx_mds3d_ws(const int8_t* Q, const float* scales, int64_t N, int32_t k, int dissim_mode, int32_t m, int32_t iters,
                 const float* x0, float* coords, float* eigvals, float* rel_change, void* workspace, int64_t workspace_bytes,
                 void* stream) {
    if (!scales) return rfx::fail(RFX_ERR_NULL, "rfx_mds3d_ws: null argument");
    int rc = check_args(Q, N, k, dissim_mode, m, iters, x0, coords, eigvals);
    if (rc != RFX_OK) return rc;
    const int squared = dissim_mode == RFX_MDS_SQUARED;
    if (!workspace) return rfx::fail(RFX_ERR_NULL, "rfx_mds3d_ws: workspace is null");
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_mds3d_ws: workspace is not 256-byte aligned");
    const size_t need = mds_layout(N, k, m, squared).total;
    if (workspace_bytes < 0 || (size_t)workspace_bytes < need)
        return rfx::fail(RFX_ERR_CAPACITY, "rfx_mds3d_ws: workspace of %lld bytes, %zu needed", (long long)workspace_bytes, need);
    hipStream_t st = rfx::as_stream(stream);
    MdsWs w;
    if ((rc = mds_bind(w, workspace, N, k, m, squared, st)) != RFX_OK) return rc;
    return mds_iterate(Q, scales, N, k, squared, m, iters, -1.0f, x0, coords, eigvals, rel_change, nullptr, w, st);
}

int rfx_mds3d(const int8_t* Q, const float* scales, int64_t N, int32_t k, int dissim_mode, int32_t m, int32_t max_iters,
              float tol, const float* x0, float* coords, float* eigvals, int32_t* iters_done, void* stream) {
    if (!scales) return rfx::fail(RFX_ERR_NULL, "rfx_mds3d: null argument");
    return mds_sync(Q, scales, N, k, dissim_mode, m, max_iters, tol, x0, coords, eigvals, iters_done, rfx::as_stream(stream));
}

int rfx_mds3d_factor(const float* A, int64_t N, int32_t k, int dissim_mode, int32_t m, int32_t max_iters, float tol,
                     const float* x0, float* coords, float* eigvals, int32_t* iters_done, void* stream) {
    return mds_sync(A, static_cast<const float*>(nullptr), N, k, dissim_mode, m, max_iters, tol, x0, coords, eigvals,
                    iters_done, rfx::as_stream(stream));
}

}  // extern "C"
