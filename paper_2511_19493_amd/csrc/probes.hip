// Measurement aids: the rates this GPU reaches on a dependency-free integer vector loop and on a
// plain device-to-device copy, as practical ceilings next to the published peaks (256 CU x 64
// lanes x 2.4 GHz lane-ops/s; 8 TB/s).  Not part of the proximity path.
#include "common.h"

namespace {

constexpr int kChains = 8;       // independent dependency chains per lane
constexpr int kOpsPerRound = 16; // vector ops per chain and loop round

// Each lane runs kChains independent chains of the two operations the compare-and-count loop is
// made of: t = t | (a ^ b) as one 3-input boolean op, and a population count with accumulate.
__global__ __launch_bounds__(256) void valu_probe_kernel(const uint32_t* __restrict__ seed, int32_t rounds,
                                                        uint32_t* __restrict__ out) {
    const uint32_t s = seed[threadIdx.x & 63];
    uint32_t t[kChains], a[kChains], c[kChains];
#pragma unroll
    for (int q = 0; q < kChains; ++q) {
        t[q] = s * (2u * q + 1u);
        a[q] = s ^ (0x9e3779b9u * (q + 1));
        c[q] = 0;
    }
    for (int r = 0; r < rounds; ++r) {
#pragma unroll
        for (int o = 0; o < kOpsPerRound / 2; ++o)
#pragma unroll
            for (int q = 0; q < kChains; ++q) {
                t[q] = __builtin_amdgcn_bitop3_b32(t[q], a[q], c[q], 0xf6);
                c[q] += __builtin_popcount(t[q]);
            }
    }
    uint32_t acc = 0;
#pragma unroll
    for (int q = 0; q < kChains; ++q) acc += c[q] ^ t[q];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

int elapsed_ms(hipEvent_t e0, hipEvent_t e1, float* ms) {
    RFX_HIP(hipEventSynchronize(e1));
    RFX_HIP(hipEventElapsedTime(ms, e0, e1));
    return RFX_OK;
}

}  // namespace

extern "C" {

int rfx_probe_valu(int32_t rounds, double* lane_ops_per_s, void* stream) {
    if (!lane_ops_per_s) return rfx::fail(RFX_ERR_NULL, "rfx_probe_valu: null argument");
    if (rounds < 1 || rounds > (1 << 20)) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_probe_valu: rounds=%d", rounds);
    hipStream_t st = rfx::as_stream(stream);
    const int blocks = 256 * 8;  // 8 workgroups of 4 waves per CU: 8 waves per SIMD
    rfx::DevBuf seed, out;
    RFX_HIP(seed.alloc(64 * sizeof(uint32_t)));
    RFX_HIP(out.alloc((size_t)blocks * 256 * sizeof(uint32_t)));
    uint32_t h[64];
    for (int i = 0; i < 64; ++i) h[i] = 0x85ebca6bu * (uint32_t)(i + 1);
    RFX_HIP(hipMemcpyAsync(seed.p, h, sizeof(h), hipMemcpyHostToDevice, st));
    hipEvent_t e0, e1;
    RFX_HIP(hipEventCreate(&e0));
    RFX_HIP(hipEventCreate(&e1));
    float ms = 0.0f;
    int rc = RFX_OK;
    for (int rep = 0; rep < 2 && rc == RFX_OK; ++rep) {  // the first launch warms up
        (void)hipEventRecord(e0, st);
        hipLaunchKernelGGL(valu_probe_kernel, dim3(blocks), dim3(256), 0, st, seed.as<uint32_t>(), rounds, out.as<uint32_t>());
        (void)hipEventRecord(e1, st);
        rc = elapsed_ms(e0, e1, &ms);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != RFX_OK) return rc;
    const double ops = (double)blocks * 256.0 * (double)rounds * kOpsPerRound * kChains;
    *lane_ops_per_s = ops / (ms * 1e-3);
    return RFX_OK;
}

int rfx_probe_copy(int64_t bytes, double* bytes_per_s, void* stream) {
    if (!bytes_per_s) return rfx::fail(RFX_ERR_NULL, "rfx_probe_copy: null argument");
    if (bytes < (1 << 20) || bytes > (1ll << 36)) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_probe_copy: bytes=%lld", (long long)bytes);
    hipStream_t st = rfx::as_stream(stream);
    const size_t n = (size_t)bytes / sizeof(uint4);
    rfx::DevBuf src, dst;
    RFX_HIP(src.alloc(n * sizeof(uint4)));
    RFX_HIP(dst.alloc(n * sizeof(uint4)));
    RFX_HIP(hipMemsetAsync(src.p, 1, n * sizeof(uint4), st));
    hipEvent_t e0, e1;
    RFX_HIP(hipEventCreate(&e0));
    RFX_HIP(hipEventCreate(&e1));
    float ms = 0.0f, best = 0.0f;
    int rc = RFX_OK;
    for (int rep = 0; rep < 4 && rc == RFX_OK; ++rep) {
        (void)hipEventRecord(e0, st);
        hipLaunchKernelGGL(copy_probe_kernel, dim3(256 * 16), dim3(256), 0, st, src.as<uint4>(), dst.as<uint4>(), n);
        (void)hipEventRecord(e1, st);
        rc = elapsed_ms(e0, e1, &ms);
        if (rep > 0 && (best == 0.0f || ms < best)) best = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != RFX_OK) return rc;
    *bytes_per_s = 2.0 * (double)(n * sizeof(uint4)) / (best * 1e-3);  // bytes read + bytes written
    return RFX_OK;
}

}  // extern "C"
