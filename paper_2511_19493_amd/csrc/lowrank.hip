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

// eigvals = theta in float32; the status word of the orthonormalisations (a block that lost rank) goes to the caller
__global__ void theta_to_float_kernel(const double* __restrict__ theta, int k, float* __restrict__ out,
                                      const int* __restrict__ flag, int32_t* __restrict__ status) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < k) out[c] = (float)theta[c];
    if (c == 0 && status) *status = *flag;
}

// Scratch of one factorisation: the small dense workspace, then two N x k float32 blocks.
struct LowrankLayout {
    size_t small_bytes, block_floats, total;
};
LowrankLayout lowrank_layout(int64_t N, int k) {
    LowrankLayout l;
    l.small_bytes = rfx::SmallWs::bytes(N, k);
    l.block_floats = ((size_t)N * k + 63) & ~(size_t)63;
    l.total = l.small_bytes + 2 * l.block_floats * sizeof(float);
    return l;
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

int rfx_lowrank_workspace_bytes(int64_t N, int32_t k, int64_t* bytes) {
    if (!bytes) return rfx::fail(RFX_ERR_NULL, "rfx_lowrank_workspace_bytes: bytes is null");
    if (N < 1 || k < 1 || k > rfx::kMaxRank || k > N)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_lowrank_workspace_bytes: N=%lld k=%d", (long long)N, k);
    *bytes = (int64_t)lowrank_layout(N, k).total;
    return RFX_OK;
}

int rfx_prox_lowrank_plan(rfx_pv_plan* plan, int32_t k, int32_t iters, const float* V0, float* eigvals, float* V, int8_t* Q,
                          float* scales, int32_t* status, void* workspace, int64_t workspace_bytes, void* stream) {
    if (!plan || !V0 || !eigvals || !V) return rfx::fail(RFX_ERR_NULL, "rfx_prox_lowrank_plan: null argument");
    if ((Q == nullptr) != (scales == nullptr))
        return rfx::fail(RFX_ERR_NULL, "rfx_prox_lowrank_plan: Q and scales must be given together");
    int64_t N = 0;
    int32_t B = 0, k_ready = 0;
    int rc = rfx_pv_plan_info(plan, &N, &B, &k_ready);
    if (rc != RFX_OK) return rc;
    if (k < 1 || k > rfx::kMaxRank || k > N)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_lowrank_plan: k=%d outside 1..min(%d, N)", k, rfx::kMaxRank);
    if (iters < 1) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_lowrank_plan: iters=%d", iters);
    if (k_ready < k)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_lowrank_plan: the plan is sized for rank %d, call rfx_pv_plan_reserve(plan, %d) first",
                         k_ready, k);
    if (!workspace) return rfx::fail(RFX_ERR_NULL, "rfx_prox_lowrank_plan: workspace is null");
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_lowrank_plan: workspace is not 256-byte aligned");
    const LowrankLayout l = lowrank_layout(N, k);
    if (workspace_bytes < 0 || (size_t)workspace_bytes < l.total)
        return rfx::fail(RFX_ERR_CAPACITY, "rfx_prox_lowrank_plan: workspace of %lld bytes, %zu needed", (long long)workspace_bytes, l.total);
    hipStream_t st = rfx::as_stream(stream);

    rfx::SmallWs ws;
    if ((rc = ws.bind(workspace, N, k, st)) != RFX_OK) return rc;
    float* Y = reinterpret_cast<float*>(static_cast<char*>(workspace) + l.small_bytes);
    float* Z = Y + l.block_floats;

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
    hipLaunchKernelGGL(theta_to_float_kernel, dim3((k + 63) / 64), dim3(64), 0, st, ws.theta, k, eigvals, ws.flag, status);
    RFX_LAUNCH_CHECK("theta_to_float_kernel");
    if ((rc = rfx::fix_signs(V, N, k, ws, st)) != RFX_OK) return rc;
    if (Q && (rc = quantise(V, eigvals, N, k, Q, scales, st)) != RFX_OK) return rc;
    return RFX_OK;
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
    if ((rc = rfx_pv_plan_reserve(plan, k)) != RFX_OK) return rc;

    const LowrankLayout l = lowrank_layout(N, k);
    rfx::DevBuf buf;
    RFX_HIP(buf.alloc(l.total + 256));
    int32_t* d_status = reinterpret_cast<int32_t*>(static_cast<char*>(buf.p) + l.total);
    rc = rfx_prox_lowrank_plan(plan, k, iters, V0, eigvals, V, Q, scales, d_status, buf.p, (int64_t)l.total, stream);
    int32_t h_status = 0;
    hipError_t e = hipSuccess;
    if (rc == RFX_OK) e = hipMemcpyAsync(&h_status, d_status, sizeof(int32_t), hipMemcpyDeviceToHost, st);
    hipError_t e2 = hipStreamSynchronize(st);  // plan and scratch are released on return
    if (rc != RFX_OK) return rc;
    if (e != hipSuccess || e2 != hipSuccess)
        return rfx::fail(RFX_ERR_HIP, "rfx_prox_lowrank: %s", hipGetErrorString(e != hipSuccess ? e : e2));
    if (h_status)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_lowrank: block lost rank (start block or P has rank < k=%d)", k);
    return RFX_OK;
}

}  // extern "C"
