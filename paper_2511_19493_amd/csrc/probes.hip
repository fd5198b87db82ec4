// Measurement aids: the rates this GPU reaches on a dependency-free integer vector loop, on a plain
// device-to-device copy, on row gathers from a table of a given size (the access pattern of the
// implicit product, whose tables live in the caches) and on chains of dependent loads (the access
// pattern of tree traversal), as practical ceilings next to the published peaks (256 CU x 64
// lanes x 2.4 GHz lane-ops/s; 8 TB/s).  Not part of the proximity path.
#include <algorithm>

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

__device__ __forceinline__ uint32_t probe_hash(uint64_t x) {
    x ^= x >> 33;
    x *= 0xff51afd7ed558ccdull;
    x ^= x >> 33;
    x *= 0xc4ceb9fe1a85ec53ull;
    x ^= x >> 33;
    return (uint32_t)x;
}

// Row indices of the gather probe: workgroup w draws its per_wg rows uniformly from the whole table, or (xcd_local)
// from the eighth of the table that belongs to the XCD running it (workgroup id mod 8).
__global__ __launch_bounds__(256) void gather_index_kernel(uint32_t* __restrict__ idx, int64_t total, int32_t per_wg,
                                                          uint32_t table_rows, int32_t xcd_local) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const uint32_t wg = (uint32_t)(t / per_wg);
    uint32_t lo = 0, span = table_rows;
    if (xcd_local) {
        span = table_rows / 8;
        lo = (wg & 7u) * span;
    }
    idx[t] = lo + probe_hash((uint64_t)t * 0x9e3779b97f4a7c15ull + 12345u) % span;
}

// The access pattern of the implicit product's two kernels with everything else taken away: a wave reads rows of
// k floats at listed indices, eight row loads in flight, and adds them up.  16 waves per workgroup, each with its
// own contiguous share of the workgroup's index list; one row of sums is written per workgroup.
template <int KCH, int RPW>
__global__ __launch_bounds__(1024) void gather_probe_kernel(const float* __restrict__ V, const uint32_t* __restrict__ idx,
                                                           int32_t per_wg, int32_t k, float* __restrict__ out) {
    __shared__ float red[16][KCH * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per_wave = per_wg / 16;
    const uint32_t* my = idx + (size_t)blockIdx.x * per_wg + (size_t)wave * per_wave;
    const int sub = lane / (64 / RPW), col = lane & (64 / RPW - 1);
    float acc[KCH];
#pragma unroll
    for (int c = 0; c < KCH; ++c) acc[c] = 0.0f;
    for (int t = 0; t < per_wave; t += 8 * RPW) {
        float v[8][KCH];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t j = my[t + u * RPW + sub];
#pragma unroll
            for (int c = 0; c < KCH; ++c) v[u][c] = V[(size_t)j * k + col + 64 * c];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int c = 0; c < KCH; ++c) acc[c] += v[u][c];
    }
#pragma unroll
    for (int c = 0; c < KCH; ++c) red[wave][lane + 64 * c] = acc[c];
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
            float s = 0.0f;
            for (int w = 0; w < 16; ++w) s += red[w][lane + 64 * c];
            out[(size_t)blockIdx.x * (KCH * 64) + lane + 64 * c] = s;
        }
    }
}

// Table of the chase probe: record i points to a pseudo-random record (its .y) and carries a pseudo-random
// 32-bit payload (.x), like an 8-byte tree node (threshold bits, child index).
__global__ __launch_bounds__(256) void chase_table_kernel(uint2* __restrict__ table, uint32_t n) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) table[i] = make_uint2(probe_hash(i * 2ull + 1), probe_hash(i * 2ull) % n);
}

// Dependent loads, as in tree traversal: every thread advances kWalks independent walks; one step of a walk is an
// 8-byte load at an address that depends on the previous step's record and (kLds) a 4-byte LDS read whose address
// depends on the record just loaded and whose value decides which of two neighbouring records comes next, the way a
// feature value picked by the node's feature index decides between two children.
template <int kWalks, bool kLds>
__global__ __launch_bounds__(1024, 2) void chase_probe_kernel(const uint2* __restrict__ table, uint32_t n, int32_t steps,
                                                            uint32_t* __restrict__ out) {
    __shared__ uint32_t feat[8192];
    if (kLds) {
        for (int i = threadIdx.x; i < 8192; i += 1024) feat[i] = probe_hash(i + 77u);
        __syncthreads();
    }
    uint32_t at[kWalks];
#pragma unroll
    for (int q = 0; q < kWalks; ++q) at[q] = probe_hash(((uint64_t)blockIdx.x * 1024 + threadIdx.x) * kWalks + q) % n;
    for (int s = 0; s < steps; ++s) {
        uint2 rec[kWalks];
#pragma unroll
        for (int q = 0; q < kWalks; ++q) rec[q] = table[at[q]];
#pragma unroll
        for (int q = 0; q < kWalks; ++q) {
            uint32_t next = rec[q].y;
            if (kLds) next = min(next + ((feat[rec[q].x & 8191u] <= rec[q].x) ? 0u : 1u), n - 1);
            at[q] = next;
        }
    }
    uint32_t acc = 0;
#pragma unroll
    for (int q = 0; q < kWalks; ++q) acc ^= at[q];
    out[(size_t)blockIdx.x * 1024 + threadIdx.x] = acc;
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

int rfx_probe_gather(int64_t table_rows, int32_t k, int64_t gathers, int32_t xcd_local, double* bytes_per_s, void* stream) {
    if (!bytes_per_s) return rfx::fail(RFX_ERR_NULL, "rfx_probe_gather: null argument");
    const bool k_ok = k == 16 || k == 32 || k == 64 || k == 128 || k == 192 || k == 256;
    if (!k_ok || table_rows < 64 || table_rows > (1ll << 26) || gathers < 1 || gathers > (1ll << 32))
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_probe_gather: table_rows=%lld k=%d gathers=%lld", (long long)table_rows, k,
                         (long long)gathers);
    hipStream_t st = rfx::as_stream(stream);
    const int per_wg = 8192;  // rows per workgroup: 512 per wave, 64 batches of 8
    const int64_t wgs = std::max<int64_t>(1, gathers / per_wg);
    const int64_t total = wgs * per_wg;
    rfx::DevBuf V, idx, out;
    RFX_HIP(V.alloc(sizeof(float) * (size_t)table_rows * k));
    RFX_HIP(idx.alloc(sizeof(uint32_t) * (size_t)total));
    RFX_HIP(out.alloc(sizeof(float) * (size_t)wgs * 256));
    RFX_HIP(hipMemsetAsync(V.p, 0, sizeof(float) * (size_t)table_rows * k, st));
    hipLaunchKernelGGL(gather_index_kernel, dim3((unsigned)rfx::ceil_div(total, 256)), dim3(256), 0, st, idx.as<uint32_t>(),
                       total, per_wg, (uint32_t)table_rows, xcd_local);
    RFX_LAUNCH_CHECK("gather_index_kernel");
    hipEvent_t e0, e1;
    RFX_HIP(hipEventCreate(&e0));
    RFX_HIP(hipEventCreate(&e1));
    float ms = 0.0f, best = 0.0f;
    int rc = RFX_OK;
    for (int rep = 0; rep < 4 && rc == RFX_OK; ++rep) {
        (void)hipEventRecord(e0, st);
#define RFX_GATHER(kch, rpw)                                                                                             \
    hipLaunchKernelGGL((gather_probe_kernel<kch, rpw>), dim3((unsigned)wgs), dim3(1024), 0, st, V.as<float>(), idx.as<uint32_t>(), \
                       per_wg, k, out.as<float>())
        if (k == 16) RFX_GATHER(1, 4);
        else if (k == 32) RFX_GATHER(1, 2);
        else if (k == 64) RFX_GATHER(1, 1);
        else if (k == 128) RFX_GATHER(2, 1);
        else if (k == 192) RFX_GATHER(3, 1);
        else RFX_GATHER(4, 1);
#undef RFX_GATHER
        (void)hipEventRecord(e1, st);
        rc = elapsed_ms(e0, e1, &ms);
        if (rep > 0 && (best == 0.0f || ms < best)) best = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != RFX_OK) return rc;
    *bytes_per_s = (double)total * 4.0 * k / (best * 1e-3);
    return RFX_OK;
}

int rfx_probe_chase(int64_t table_bytes, int32_t walks_per_thread, int32_t steps, int32_t with_lds, double* steps_per_s,
                    void* stream) {
    if (!steps_per_s) return rfx::fail(RFX_ERR_NULL, "rfx_probe_chase: null argument");
    if (table_bytes < 4096 || table_bytes > (1ll << 34) || steps < 1 || steps > (1 << 20) ||
        (walks_per_thread != 1 && walks_per_thread != 2 && walks_per_thread != 4))
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_probe_chase: table_bytes=%lld walks_per_thread=%d steps=%d",
                         (long long)table_bytes, walks_per_thread, steps);
    hipStream_t st = rfx::as_stream(stream);
    const uint32_t n = (uint32_t)(table_bytes / sizeof(uint2));
    const int blocks = 256 * 2;  // two workgroups of 16 waves per CU, as the traversal kernel runs
    rfx::DevBuf table, out;
    RFX_HIP(table.alloc(sizeof(uint2) * (size_t)n));
    RFX_HIP(out.alloc(sizeof(uint32_t) * (size_t)blocks * 1024));
    hipLaunchKernelGGL(chase_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, table.as<uint2>(), n);
    RFX_LAUNCH_CHECK("chase_table_kernel");
    hipEvent_t e0, e1;
    RFX_HIP(hipEventCreate(&e0));
    RFX_HIP(hipEventCreate(&e1));
    float ms = 0.0f, best = 0.0f;
    int rc = RFX_OK;
    for (int rep = 0; rep < 3 && rc == RFX_OK; ++rep) {
        (void)hipEventRecord(e0, st);
#define RFX_CHASE(w)                                                                                                      \
    if (with_lds)                                                                                                         \
        hipLaunchKernelGGL((chase_probe_kernel<w, true>), dim3(blocks), dim3(1024), 0, st, table.as<uint2>(), n, steps,   \
                           out.as<uint32_t>());                                                                           \
    else                                                                                                                  \
        hipLaunchKernelGGL((chase_probe_kernel<w, false>), dim3(blocks), dim3(1024), 0, st, table.as<uint2>(), n, steps,  \
                           out.as<uint32_t>())
        if (walks_per_thread == 1) { RFX_CHASE(1); }
        else if (walks_per_thread == 2) { RFX_CHASE(2); }
        else { RFX_CHASE(4); }
#undef RFX_CHASE
        (void)hipEventRecord(e1, st);
        rc = elapsed_ms(e0, e1, &ms);
        if (rep > 0 && (best == 0.0f || ms < best)) best = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != RFX_OK) return rc;
    *steps_per_s = (double)blocks * 1024.0 * walks_per_thread * (double)steps / (best * 1e-3);
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
