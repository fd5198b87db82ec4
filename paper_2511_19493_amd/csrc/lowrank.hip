// Rank-k factorisation of the proximity matrix by block power iteration on the implicit product,
// and INT8 quantisation of the factor (paper: "QLORA" low-rank proximity P ~ Q U^T, quantisation
// levels in "Low-Rank Factorization and Quantization Trade-offs").  P is symmetric positive
// semi-definite, so the factorisation is taken in its symmetric form P ~ A A^T,
// A = V diag(sqrt(lambda)), with (lambda, V) the leading eigenpairs of P.
#include "common.h"
#include "dense_small.h"

namespace {

// scales[c] = max_i |V[i][c] * sqrt(max(lambda_c, 0))| / 127, or 1 for an all-zero column.
__global__ __launch_bounds__(256) void column_scale_kernel(const float* __restrict__ V, const float* __restrict__ lam,
                                                          int64_t N, int k, float* __restrict__ scales) {
    __shared__ float red[256];
    const int c = blockIdx.x;
    const float root = sqrtf(fmaxf(lam[c], 0.0f));
    float best = 0.0f;
    for (int64_t i = threadIdx.x; i < N; i += 256) best = fmaxf(best, fabsf(V[i * k + c] * root));
    red[threadIdx.x] = best;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + off]);
        __syncthreads();
    }
    if (threadIdx.x == 0) scales[c] = red[0] > 0.0f ? red[0] / 127.0f : 1.0f;
}

// Q[i][c] = clamp(round-half-even(V[i][c] * sqrt(lambda_c) / scales[c]), -127, 127)
__global__ __launch_bounds__(256) void quantise_kernel(const float* __restrict__ V, const float* __restrict__ lam,
                                                      const float* __restrict__ scales, int64_t total, int k,
                                                      int8_t* __restrict__ Q) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    const int c = (int)(e % k);
    const float a = V[e] * sqrtf(fmaxf(lam[c], 0.0f));
    const float q = rintf(a / scales[c]);
    Q[e] = (int8_t)fminf(127.0f, fmaxf(-127.0f, q));
}

__global__ void theta_to_float_kernel(const double* __restrict__ theta, int k, float* __restrict__ out) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < k) out[c] = (float)theta[c];
}

int quantise(const float* V, const float* eigvals, int64_t N, int32_t k, int8_t* Q, float* scales, hipStream_t st) {
    hipLaunchKernelGGL(column_scale_kernel, dim3(k), dim3(256), 0, st, V, eigvals, N, k, scales);
    RFX_LAUNCH_CHECK("column_scale_kernel");
    const int64_t total = N * k;
    hipLaunchKernelGGL(quantise_kernel, dim3((unsigned)rfx::ceil_div(total, 256)), dim3(256), 0, st, V, eigvals, scales,
                       total, k, Q);
    RFX_LAUNCH_CHECK("quantise_kernel");
    return RFX_OK;
}

}  // namespace

extern "C" {

int rfx_quantise_int8(const float* V, const float* eigvals, int64_t N, int32_t k, int8_t* Q, float* scales,
                      void* stream) {
    if (!V || !eigvals || !Q || !scales) return rfx::fail(RFX_ERR_NULL, "rfx_quantise_int8: null argument");
    if (N < 1 || k < 1 || N * (int64_t)k / 256 > 0x7fffffffLL)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_quantise_int8: N=%lld k=%d", (long long)N, k);
    return quantise(V, eigvals, N, k, Q, scales, rfx::as_stream(stream));
}

int rfx_prox_lowrank(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int32_t k, int32_t iters,
                     const float* V0, float* eigvals, float* V, int8_t* Q, float* scales, void* stream) {
    if (!leaf || !V0 || !eigvals || !V) return rfx::fail(RFX_ERR_NULL, "rfx_prox_lowrank: null argument");
    if ((Q == nullptr) != (scales == nullptr))
        return rfx::fail(RFX_ERR_NULL, "rfx_prox_lowrank: Q and scales must be given together");
    if (k < 1 || k > rfx::kMaxRank || k > N)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_lowrank: k=%d outside 1..min(%d, N)", k, rfx::kMaxRank);
    if (iters < 1) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_lowrank: iters=%d", iters);
    hipStream_t st = rfx::as_stream(stream);

    rfx_pv_plan* plan = nullptr;
    int rc = rfx_pv_plan_create(leaf, N, B, leaf_bound, &plan, stream);
    if (rc != RFX_OK) return rc;
    struct PlanGuard {
        rfx_pv_plan* p;
        ~PlanGuard() { rfx_pv_plan_destroy(p); }
    } guard{plan};

    rfx::SmallWs ws;
    rfx::DevBuf blocks;
    RFX_HIP(ws.alloc(N, k));
    RFX_HIP(blocks.alloc(sizeof(float) * 2 * (size_t)N * (size_t)k));
    float* Y = blocks.as<float>();
    float* Z = Y + (size_t)N * k;

    // V <- orth(V0); (iters - 1) x V <- orth(P V)
    if ((rc = rfx::orthonormalise(V0, N, k, ws, Z, V, st, 2)) != RFX_OK) return rc;
    for (int it = 1; it < iters; ++it) {
        if ((rc = rfx_pv_apply(plan, V, k, Y, stream)) != RFX_OK) return rc;
        if ((rc = rfx::orthonormalise(Y, N, k, ws, Z, V, st, 1)) != RFX_OK) return rc;
    }
    // Rayleigh-Ritz: Y = P V, H = sym(V^T Y) = W diag(theta) W^T, V <- V W
    if ((rc = rfx_pv_apply(plan, V, k, Y, stream)) != RFX_OK) return rc;
    if ((rc = rfx::gram(V, Y, N, k, true, ws, ws.G, st)) != RFX_OK) return rc;
    if ((rc = rfx::jacobi_eigh(ws.G, k, ws, ws.theta, ws.W, st)) != RFX_OK) return rc;
    if ((rc = rfx::apply_small(V, N, k, ws.W, k, Z, st)) != RFX_OK) return rc;
    RFX_HIP(hipMemcpyAsync(V, Z, sizeof(float) * (size_t)N * k, hipMemcpyDeviceToDevice, st));
    hipLaunchKernelGGL(theta_to_float_kernel, dim3((k + 63) / 64), dim3(64), 0, st, ws.theta, k, eigvals);
    RFX_LAUNCH_CHECK("theta_to_float_kernel");
    if ((rc = rfx::fix_signs(V, N, k, ws, st)) != RFX_OK) return rc;
    if (Q && (rc = quantise(V, eigvals, N, k, Q, scales, st)) != RFX_OK) return rc;

    int h_flag = 0;
    RFX_HIP(hipMemcpyAsync(&h_flag, ws.flag, sizeof(int), hipMemcpyDeviceToHost, st));
    RFX_HIP(hipStreamSynchronize(st));
    if (h_flag)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_lowrank: block lost rank (start block or P has rank < k=%d)", k);
    return RFX_OK;
}

}  // extern "C"
