// Small dense linear algebra on device used by the block iterations: k x k Gram matrices of
// tall N x k blocks, Cholesky factor and its inverse, symmetric eigen-decomposition (cyclic
// Jacobi), and tall-times-small products.  All reductions and k x k work are float64; tall
// blocks are float32 in memory.  Host-side launch wrappers; every call is asynchronous on `st`.
#pragma once

#include "common.h"

namespace rfx {

constexpr int kMaxRank = 128;  // largest block width the small-matrix kernels are built for

// Scratch shared by the wrappers below, sized for N rows and width k.
struct SmallWs {
    double* partial = nullptr;  // [gram_blocks][k][k], one per workgroup of the Gram kernel
    double* G = nullptr;        // [k][k]
    double* T = nullptr;        // [k][k]
    double* theta = nullptr;    // [k]
    double* W = nullptr;        // [k][k]
    int* flag = nullptr;        // device status word (non-positive Cholesky pivot)
    long long* sign_row = nullptr;  // [256][k] per row range and column: row of the largest-magnitude entry
    float* sign_val = nullptr;      // [256][k] and its value
    int gram_blocks = 0;
    DevBuf buf;
    // Either the scratch is carved from caller memory (`bytes` of it, 256-byte aligned; bind clears the status word
    // with a kernel on `st`), or alloc takes it from hipMalloc and binds it.
    static size_t bytes(int64_t N, int k);
    int bind(void* mem, int64_t N, int k, hipStream_t st);
    int alloc(int64_t N, int k, hipStream_t st);
};

// G = A^T Bm (k x k, float64), A and Bm float32 [N][k]; symmetrised (G + G^T)/2 if sym.
int gram(const float* A, const float* Bm, int64_t N, int k, bool sym, SmallWs& ws, double* G, hipStream_t st);
// T = inverse of the upper Cholesky factor R of G (G = R^T R).  A column of G whose pivot is not positive (the
// column of the block lies in the span of the columns before it) sets *ws.flag and is dropped: row and column of T
// are zero, so the orthonormalised block gets a zero column there.
int chol_inverse(const double* G, int k, SmallWs& ws, double* T, hipStream_t st);
// Eigen-decomposition of the symmetric k x k matrix H: theta descending, W columns = vectors.
int jacobi_eigh(const double* H, int k, SmallWs& ws, double* theta, double* W, hipStream_t st);
// Out = A T with A float32 [N][k], T float64 [k][kout] (row stride k), Out float32 [N][kout].
int apply_small(const float* A, int64_t N, int k, const double* T, int kout, float* Out, hipStream_t st);
// Cholesky QR: V = orthonormal basis of span(Y); Z is an [N][k] temporary (used by the second pass).
// The Gram matrix and its factor are float64, so one pass already leaves V orthonormal to float32
// rounding when cond(Y)^2 is well below 1e16 (a block that has just been multiplied by P from an
// orthonormal block); passes = 2 repeats the step for blocks of unknown conditioning (start blocks).
int orthonormalise(const float* Y, int64_t N, int k, SmallWs& ws, float* Z, float* V, hipStream_t st, int passes);
// Flips every column of V [N][kc] so that its largest-magnitude entry (first one on ties) is positive.
int fix_signs(float* V, int64_t N, int kc, SmallWs& ws, hipStream_t st);  // kc <= the width ws was sized for

}  // namespace rfx
