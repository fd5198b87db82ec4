// Encodings of the low-rank factor A = V diag(sqrt(lambda)) (paper, "Low-Rank Factorization and
// Quantization Trade-offs": NF4 (4-bit), INT8, FP16 and FP32 levels).  INT8 lives in lowrank.hip;
// this file has the other three and the decoders.
//   FP32 / FP16: A rounded to nearest-even, no scales.
//   NF4: the 4-bit NormalFloat type of the QLoRA paper: 16 fixed levels in [-1, 1] applied to values
//        normalised by the absolute maximum of their block.  Blocks are 64 consecutive rows of one
//        column; codes are packed two per byte (even row in the low nibble, a missing last row is
//        the zero level); the nearest level is decided in float32 by counting the midpoints between
//        adjacent levels that lie below the normalised value.
#include <hip/hip_fp16.h>

#include "common.h"

namespace {

constexpr int kNf4Block = 64;

__constant__ float kNf4Levels[16] = {-1.0f,
                                     -0.6961928009986877f,
                                     -0.5250730514526367f,
                                     -0.39491748809814453f,
                                     -0.28444138169288635f,
                                     -0.18477343022823334f,
                                     -0.09105003625154495f,
                                     0.0f,
                                     0.07958029955625534f,
                                     0.16093020141124725f,
                                     0.24611230194568634f,
                                     0.33791524171829224f,
                                     0.44070982933044434f,
                                     0.5626170039176941f,
                                     0.7229568362236023f,
                                     1.0f};

__device__ __forceinline__ float factor_value(const float* V, const float* lam, int64_t e, int k) {
    return V[e] * sqrtf(fmaxf(lam[e % k], 0.0f));
}

__global__ __launch_bounds__(256) void encode_fp32_kernel(const float* __restrict__ V, const float* __restrict__ lam,
                                                         int64_t total, int k, float* __restrict__ out) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < total) out[e] = factor_value(V, lam, e, k);
}

__global__ __launch_bounds__(256) void encode_fp16_kernel(const float* __restrict__ V, const float* __restrict__ lam,
                                                         int64_t total, int k, __half* __restrict__ out) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < total) {
        // The product is rounded to float32 first and to half precision second.  The empty asm keeps the
        // compiler from merging both into one mixed-precision multiply that rounds the exact product once.
        float a = factor_value(V, lam, e, k);
        asm volatile("" : "+v"(a));
        out[e] = __float2half_rn(a);
    }
}

// One workgroup per block of 64 rows; each of its 4 waves takes every 4th column, lane = row.
__global__ __launch_bounds__(256) void encode_nf4_kernel(const float* __restrict__ V, const float* __restrict__ lam,
                                                        int64_t N, int k, uint8_t* __restrict__ codes,
                                                        float* __restrict__ scales) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t blk = blockIdx.x;
    const int64_t row = blk * kNf4Block + lane;
    for (int c = w; c < k; c += 4) {
        const float a = row < N ? V[row * k + c] * sqrtf(fmaxf(lam[c], 0.0f)) : 0.0f;
        float amax = fabsf(a);
        for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
        const float s = amax > 0.0f ? amax : 1.0f;
        const float x = a / s;
        uint32_t code = 0;
#pragma unroll
        for (int t = 0; t < 15; ++t) code += x > (kNf4Levels[t] + kNf4Levels[t + 1]) * 0.5f ? 1u : 0u;
        const uint32_t hi = __shfl_down(code, 1);
        if ((lane & 1) == 0 && row < N) codes[(row >> 1) * k + c] = (uint8_t)(code | (hi << 4));
        if (lane == 0) scales[blk * k + c] = s;
    }
}

__global__ __launch_bounds__(256) void decode_fp16_kernel(const __half* __restrict__ codes, int64_t total,
                                                         float* __restrict__ A) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < total) A[e] = __half2float(codes[e]);
}

__global__ __launch_bounds__(256) void decode_int8_kernel(const int8_t* __restrict__ codes, const float* __restrict__ scales,
                                                         int64_t total, int k, float* __restrict__ A) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < total) A[e] = (float)codes[e] * scales[e % k];
}

__global__ __launch_bounds__(256) void decode_nf4_kernel(const uint8_t* __restrict__ codes, const float* __restrict__ scales,
                                                        int64_t N, int k, float* __restrict__ A) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= N * k) return;
    const int64_t row = e / k;
    const int c = (int)(e - row * k);
    const uint8_t byte = codes[(row >> 1) * k + c];
    const uint32_t code = (row & 1) ? (byte >> 4) : (byte & 15u);
    A[e] = kNf4Levels[code] * scales[(row / kNf4Block) * k + c];
}

int check(const char* who, int64_t N, int32_t k, int encoding) {
    if (N < 1 || k < 1 || N * (int64_t)k / 256 > 0x7fffffffLL)
        return rfx::fail(RFX_ERR_INVALID_ARG, "%s: N=%lld k=%d", who, (long long)N, k);
    if (encoding < RFX_ENC_INT8 || encoding > RFX_ENC_FP32) return rfx::fail(RFX_ERR_INVALID_ARG, "%s: encoding=%d", who, encoding);
    return RFX_OK;
}

}  // namespace

extern "C" {

int rfx_factor_sizes(int encoding, int64_t N, int32_t k, int64_t* code_bytes, int64_t* n_scales) {
    if (!code_bytes || !n_scales) return rfx::fail(RFX_ERR_NULL, "rfx_factor_sizes: null argument");
    int rc = check("rfx_factor_sizes", N, k, encoding);
    if (rc != RFX_OK) return rc;
    switch (encoding) {
        case RFX_ENC_INT8: *code_bytes = N * k; *n_scales = k; break;
        case RFX_ENC_FP16: *code_bytes = 2 * N * k; *n_scales = 0; break;
        case RFX_ENC_NF4: *code_bytes = ((N + 1) / 2) * k; *n_scales = ((N + kNf4Block - 1) / kNf4Block) * k; break;
        default: *code_bytes = 4 * N * k; *n_scales = 0; break;
    }
    return RFX_OK;
}

int rfx_quantise_factor(const float* V, const float* eigvals, int64_t N, int32_t k, int encoding, void* codes,
                        float* scales, void* stream) {
    if (!V || !eigvals || !codes) return rfx::fail(RFX_ERR_NULL, "rfx_quantise_factor: null argument");
    int rc = check("rfx_quantise_factor", N, k, encoding);
    if (rc != RFX_OK) return rc;
    hipStream_t st = rfx::as_stream(stream);
    const int64_t total = N * k;
    const dim3 grid((unsigned)rfx::ceil_div(total, 256));
    switch (encoding) {
        case RFX_ENC_INT8:
            return rfx_quantise_int8(V, eigvals, N, k, static_cast<int8_t*>(codes), scales, stream);
        case RFX_ENC_FP32:
            hipLaunchKernelGGL(encode_fp32_kernel, grid, dim3(256), 0, st, V, eigvals, total, k, static_cast<float*>(codes));
            break;
        case RFX_ENC_FP16:
            hipLaunchKernelGGL(encode_fp16_kernel, grid, dim3(256), 0, st, V, eigvals, total, k, static_cast<__half*>(codes));
            break;
        default:
            if (!scales) return rfx::fail(RFX_ERR_NULL, "rfx_quantise_factor: NF4 needs scales");
            hipLaunchKernelGGL(encode_nf4_kernel, dim3((unsigned)rfx::ceil_div(N, kNf4Block)), dim3(256), 0, st, V, eigvals, N, k,
                               static_cast<uint8_t*>(codes), scales);
            break;
    }
    RFX_LAUNCH_CHECK("factor encoding kernel");
    return RFX_OK;
}

int rfx_dequantise_factor(const void* codes, const float* scales, int64_t N, int32_t k, int encoding, float* A,
                          void* stream) {
    if (!codes || !A) return rfx::fail(RFX_ERR_NULL, "rfx_dequantise_factor: null argument");
    int rc = check("rfx_dequantise_factor", N, k, encoding);
    if (rc != RFX_OK) return rc;
    if ((encoding == RFX_ENC_INT8 || encoding == RFX_ENC_NF4) && !scales)
        return rfx::fail(RFX_ERR_NULL, "rfx_dequantise_factor: scales required");
    hipStream_t st = rfx::as_stream(stream);
    const int64_t total = N * k;
    const dim3 grid((unsigned)rfx::ceil_div(total, 256));
    switch (encoding) {
        case RFX_ENC_INT8:
            hipLaunchKernelGGL(decode_int8_kernel, grid, dim3(256), 0, st, static_cast<const int8_t*>(codes), scales, total, k, A);
            break;
        case RFX_ENC_FP16:
            hipLaunchKernelGGL(decode_fp16_kernel, grid, dim3(256), 0, st, static_cast<const __half*>(codes), total, A);
            break;
        case RFX_ENC_NF4:
            hipLaunchKernelGGL(decode_nf4_kernel, grid, dim3(256), 0, st, static_cast<const uint8_t*>(codes), scales, N, k, A);
            break;
        default:
            RFX_HIP(hipMemcpyAsync(A, codes, sizeof(float) * (size_t)total, hipMemcpyDeviceToDevice, st));
            return RFX_OK;
    }
    RFX_LAUNCH_CHECK("factor decoding kernel");
    return RFX_OK;
}

}  // extern "C"
