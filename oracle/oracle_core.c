/* CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, literal implementations of the integer and float64 steps of
 * the random-forest proximity path, written from the paper's definitions.
 * Nothing here is shared with the HIP library; only tests, the smoke check
 * and the benchmark's CPU-baseline leg may call it.
 *
 * Steps (paper passages):
 *   orc_leaf_assign   terminal node of every sample in every tree; rows with
 *                     x <= tau go left, rows with x > tau go right
 *                     (Methodology, "Threshold-based Splits"; every sample,
 *                     in-bag or not, is dropped down every tree: CPU
 *                     Proximity Computation).
 *   orc_counts_rows   cnt(i,j) = #{b : node_b(i) = node_b(j)}, the numerator
 *                     of the proximity equation p(i,j) = (1/B) sum_b I(...)
 *                     (Methodology, "Proximity Matrices").
 *   orc_oob_rows      the same restricted to trees where both samples are
 *                     out-of-bag (OOB_i = {b : i not in bootstrap sample b},
 *                     "Case-wise Bootstrap Tracking"), and the number of such
 *                     trees.
 *   orc_pv_implicit   Y = P V with P = (1/B) sum_b Z_b Z_b^T, Z_b the one-hot
 *                     leaf-membership matrix of tree b, in float64.
 *   orc_pv_rows       Y[i,:] = (1/B) sum_j cnt(i,j) V[j,:] straight from the
 *                     proximity equation (the dense product), in float64.
 *
 * Threads split the outermost independent loop only (trees or rows); there is
 * no blocking or fusion.
 *
 * Build: gcc -O2 -std=c99 -fopenmp -shared -fPIC oracle_core.c -o liboracle_core.so
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Forest arrays are concatenated over trees; tree b owns nodes
 * [node_offset[b], node_offset[b+1]) and its root is local node 0.  Writes
 * leaf[b*N + i] and, if path_len is not null, the summed number of internal
 * nodes visited over all (tree, sample) pairs.  Returns 0, or -1 when a walk
 * leaves the tree's node range (malformed forest). */
int orc_leaf_assign(int32_t B, const int64_t* node_offset, const int32_t* feature, const float* threshold,
                    const int32_t* left, const int32_t* right, const int32_t* leaf_id, const float* X, int64_t N,
                    int32_t M, uint32_t* leaf, int64_t* path_len) {
    int bad = 0;
    int64_t total = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : total) reduction(| : bad)
    for (int32_t b = 0; b < B; ++b) {
        int64_t off = node_offset[b];
        int64_t n_nodes = node_offset[b + 1] - off;
        for (int64_t i = 0; i < N; ++i) {
            int64_t node = 0;
            int64_t steps = 0;
            while (feature[off + node] >= 0) {
                float x = X[i * M + feature[off + node]];
                node = (x <= threshold[off + node]) ? left[off + node] : right[off + node];
                ++steps;
                if (node < 0 || node >= n_nodes || steps > n_nodes) {
                    bad = 1;
                    node = -1;
                    break;
                }
            }
            leaf[(int64_t)b * N + i] = node < 0 ? 0xffffffffu : (uint32_t)leaf_id[off + node];
            total += steps;
        }
    }
    if (path_len) *path_len = total;
    return bad ? -1 : 0;
}

/* Rows i0..i1-1 of the full co-occurrence count matrix: cnt[(i-i0)*N + j]. */
void orc_counts_rows(const uint32_t* leaf, int64_t N, int32_t B, int64_t i0, int64_t i1, uint32_t* cnt) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = i0; i < i1; ++i) {
        uint32_t* row = cnt + (i - i0) * N;
        memset(row, 0, sizeof(uint32_t) * (size_t)N);
        for (int32_t b = 0; b < B; ++b) {
            const uint32_t* lb = leaf + (int64_t)b * N;
            uint32_t li = lb[i];
            for (int64_t j = 0; j < N; ++j) row[j] += (lb[j] == li);
        }
    }
}

/* Rows i0..i1-1 of the out-of-bag-only numerator and denominator:
 *   num(i,j) = #{b : c_b(i) = 0, c_b(j) = 0, node_b(i) = node_b(j)}
 *   den(i,j) = #{b : c_b(i) = 0, c_b(j) = 0}
 * with c_b the in-bag counts inbag[b*N + .]. */
void orc_oob_rows(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int64_t i0, int64_t i1,
                  uint32_t* num, uint32_t* den) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = i0; i < i1; ++i) {
        uint32_t* nr = num + (i - i0) * N;
        uint32_t* dr = den + (i - i0) * N;
        memset(nr, 0, sizeof(uint32_t) * (size_t)N);
        memset(dr, 0, sizeof(uint32_t) * (size_t)N);
        for (int32_t b = 0; b < B; ++b) {
            const uint32_t* lb = leaf + (int64_t)b * N;
            const uint16_t* cb = inbag + (int64_t)b * N;
            if (cb[i] != 0) continue;
            uint32_t li = lb[i];
            for (int64_t j = 0; j < N; ++j) {
                if (cb[j] == 0) {
                    dr[j] += 1;
                    nr[j] += (lb[j] == li);
                }
            }
        }
    }
}

/* Y = (1/B) sum_b Z_b (Z_b^T V), V and Y row-major [N][k] float64.
 * Per tree: S[l,:] = sum of V rows in leaf l, then Y[i,:] += S[leaf_b(i),:].
 * Each column of V is handled by one thread, trees in order, so the summation
 * order is fixed.  Returns 0, -1 if a leaf id is >= max_leaves, -2 on
 * allocation failure. */
int orc_pv_implicit(const uint32_t* leaf, int64_t N, int32_t B, int64_t max_leaves, const double* V, int32_t k,
                    double* Y) {
    int status = 0;
#pragma omp parallel for schedule(static, 1)
    for (int32_t c = 0; c < k; ++c) {
        /* column c of V and of Y, copied out so the loops below run over contiguous memory */
        double* S = (double*)malloc(sizeof(double) * (size_t)max_leaves);
        double* v = (double*)malloc(sizeof(double) * (size_t)N);
        double* y = (double*)malloc(sizeof(double) * (size_t)N);
        if (!S || !v || !y) {
#pragma omp atomic write
            status = -2;
            free(S);
            free(v);
            free(y);
            continue;
        }
        for (int64_t j = 0; j < N; ++j) {
            v[j] = V[j * k + c];
            y[j] = 0.0;
        }
        for (int32_t b = 0; b < B; ++b) {
            const uint32_t* lb = leaf + (int64_t)b * N;
            for (int64_t l = 0; l < max_leaves; ++l) S[l] = 0.0;
            int bad = 0;
            for (int64_t j = 0; j < N; ++j) {
                if (lb[j] >= (uint64_t)max_leaves) {
                    bad = 1;
                    break;
                }
                S[lb[j]] += v[j];
            }
            if (bad) {
#pragma omp atomic write
                status = -1;
                break;
            }
            for (int64_t i = 0; i < N; ++i) y[i] += S[lb[i]];
        }
        for (int64_t i = 0; i < N; ++i) Y[i * k + c] = y[i] / (double)B;
        free(S);
        free(v);
        free(y);
    }
    return status;
}

/* Rows i0..i1-1 of the dense product: Y[(i-i0)*k + c] = (1/B) sum_j cnt(i,j) V[j*k + c]. */
void orc_pv_rows(const uint32_t* leaf, int64_t N, int32_t B, int64_t i0, int64_t i1, const double* V, int32_t k,
                 double* Y) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = i0; i < i1; ++i) {
        double* y = Y + (i - i0) * k;
        for (int32_t c = 0; c < k; ++c) y[c] = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            uint32_t cnt = 0;
            for (int32_t b = 0; b < B; ++b) cnt += (leaf[(int64_t)b * N + i] == leaf[(int64_t)b * N + j]);
            if (cnt) {
                double p = (double)cnt / (double)B;
                for (int32_t c = 0; c < k; ++c) y[c] += p * V[j * k + c];
            }
        }
    }
}
