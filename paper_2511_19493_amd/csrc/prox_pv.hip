// Implicit product Y = P V = (1/B) sum_b Z_b (Z_b^T V) without forming P
// (P from the paper's proximity equation; Z_b = one-hot leaf membership of tree b).
//
// Plan (once per forest): for every tree the samples are grouped by leaf with a stable counting
// sort, giving perm[B][N] (sample indices, leaf by leaf, ascending inside a leaf) and
// seg_start[B*Lb + 1] (Lb = leaf_bound; slot = b*Lb + leaf).  Ascending order inside a leaf
// fixes the float summation order, so results are reproducible run to run.
//
// Apply, two kernels, both pure row traffic of k floats:
//   leaf sums : S[slot,:] = sum over the slot's samples of V[sample,:]   (one wave per chunk
//               of a slot; long slots are split and their partial sums added in order)
//   gather    : Y[i,:] = (1/B) sum_b S[slot_b(i),:]   (a wave keeps a tile of Y rows in
//               registers and sweeps the trees in order, so all waves touch the same trees'
//               sums at about the same time and those rows stay cache-resident)
#include <vector>

#include "common.h"

struct rfx_pv_plan {
    int64_t N = 0;
    int32_t B = 0, Lb = 0;
    uint32_t* d_slot = nullptr;       // [B][N]  b*Lb + leaf_b(i)
    uint32_t* d_perm = nullptr;       // [B*N]
    uint32_t* d_seg_start = nullptr;  // [B*Lb + 1]
    float* d_S = nullptr;             // [B*Lb][k_cap]
    int32_t k_cap = 0;
};

namespace {

constexpr int kGatherTile = 32;  // Y rows per wave in the gather

__global__ __launch_bounds__(256) void pv_hist_kernel(const uint32_t* __restrict__ leaf, int64_t N, int32_t B, int32_t Lb,
                                                     uint32_t* __restrict__ slot, uint32_t* __restrict__ count,
                                                     int* __restrict__ bad) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int b = blockIdx.y;
    if (i >= N) return;
    uint32_t id = leaf[(int64_t)b * N + i];
    if (id >= (uint32_t)Lb) {
        *bad = 1;
        id = (uint32_t)Lb - 1;
    }
    const uint32_t s = (uint32_t)b * (uint32_t)Lb + id;
    slot[(int64_t)b * N + i] = s;
    atomicAdd(&count[s], 1u);
}

// One workgroup per tree: seg_start[b*Lb + l] = b*N + (number of samples of tree b in leaves < l);
// cursor = seg_start.
__global__ __launch_bounds__(256) void pv_scan_kernel(const uint32_t* __restrict__ count, int64_t N, int32_t B, int32_t Lb,
                                                     uint32_t* __restrict__ seg_start, uint32_t* __restrict__ cursor) {
    __shared__ uint32_t part[256];
    const int b = blockIdx.x;
    const int t = threadIdx.x;
    const int per = (Lb + 255) / 256;
    const int lo = min(Lb, t * per), hi = min(Lb, lo + per);
    const uint32_t* c = count + (int64_t)b * Lb;
    uint32_t sum = 0;
    for (int l = lo; l < hi; ++l) sum += c[l];
    part[t] = sum;
    __syncthreads();
    if (t == 0) {
        uint32_t run = (uint32_t)((int64_t)b * N);
        for (int q = 0; q < 256; ++q) {
            uint32_t v = part[q];
            part[q] = run;
            run += v;
        }
    }
    __syncthreads();
    uint32_t run = part[t];
    for (int l = lo; l < hi; ++l) {
        const int64_t at = (int64_t)b * Lb + l;
        const uint32_t v = c[l];
        seg_start[at] = run;
        cursor[at] = run;
        run += v;
    }
    if (b == B - 1 && t == 255) seg_start[(int64_t)B * Lb] = (uint32_t)((int64_t)B * N);
}

// Stable scatter: one wave per tree walks the samples 64 at a time in ascending order.  Lanes with
// the same slot are ranked by lane index; the group's first lane reserves the group's range with
// one atomic add, so the order inside every leaf is ascending sample index.
__global__ __launch_bounds__(64) void pv_scatter_kernel(const uint32_t* __restrict__ slot, int64_t N,
                                                       uint32_t* __restrict__ cursor, uint32_t* __restrict__ perm) {
    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    const uint32_t* s = slot + (int64_t)b * N;
    for (int64_t i0 = 0; i0 < N; i0 += 64) {
        const int64_t i = i0 + lane;
        const bool valid = i < N;
        const uint32_t key = valid ? s[i] : 0xffffffffu;
        uint64_t remaining = __ballot(valid);
        int my_leader = lane;
        uint32_t rank = 0, gcount = 0;
        while (remaining) {
            const int leader = __ffsll((unsigned long long)remaining) - 1;
            const uint32_t lk = __builtin_amdgcn_readlane(key, leader);
            const uint64_t m = __ballot(valid && key == lk);
            if (valid && key == lk) {
                my_leader = leader;
                rank = (uint32_t)__popcll(m & lt_mask);
                gcount = (uint32_t)__popcll(m);
            }
            remaining &= ~m;
        }
        uint32_t base = 0;
        if (valid && my_leader == lane) base = atomicAdd(&cursor[key], gcount);
        base = __shfl(base, my_leader);
        if (valid) perm[base + rank] = (uint32_t)i;
    }
}

// ---------------------------------------------------------------------------------------------
// Column handled by a lane.  RPW = rows (samples) a wave touches with one load instruction:
// 1 for k > 32 (lanes are columns lane, lane+64, ...), 2 for 16 < k <= 32, 4 for k <= 16 (each
// group of 64/RPW lanes is one row).  Lanes beyond k read a clamped column and are never stored,
// which keeps every load unconditional so that the loads of a batch are all in flight together.
template <int RPW>
__device__ __forceinline__ int lane_col(int lane) {
    return lane & (64 / RPW - 1);
}

// Leaf sums.  One wave per slot; the RPW lane groups take members t, t+RPW, ... of the slot in
// batches of kSumBatch loads, and their partial sums are added in group order at the end.
constexpr int kSumBatch = 8;

template <int KCH, int RPW>
__global__ __launch_bounds__(256) void pv_leaf_sum_kernel(const uint32_t* __restrict__ seg_start,
                                                         const uint32_t* __restrict__ perm, int64_t n_slots,
                                                         const float* __restrict__ V, int32_t k, float* __restrict__ S) {
    const int lane = threadIdx.x & 63;
    const int64_t slot = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (slot >= n_slots) return;
    const uint32_t lo = seg_start[slot], hi = seg_start[slot + 1];
    if (lo == hi) return;  // empty leaf: its row of S is never read
    const int grp = lane / (64 / RPW);
    int col[KCH];
#pragma unroll
    for (int c = 0; c < KCH; ++c) col[c] = min(lane_col<RPW>(lane) + 64 * c, k - 1);
    float acc[KCH];
#pragma unroll
    for (int c = 0; c < KCH; ++c) acc[c] = 0.0f;
    for (uint32_t t0 = lo; t0 < hi; t0 += kSumBatch * RPW) {
        float v[kSumBatch][KCH];
#pragma unroll
        for (int u = 0; u < kSumBatch; ++u) {
            const uint32_t t = t0 + u * RPW + grp;
            const uint32_t j = perm[min(t, hi - 1)];   // clamped: always a valid member
#pragma unroll
            for (int c = 0; c < KCH; ++c) v[u][c] = V[(int64_t)j * k + col[c]];
        }
#pragma unroll
        for (int u = 0; u < kSumBatch; ++u) {
            const bool live = t0 + u * RPW + grp < hi;
#pragma unroll
            for (int c = 0; c < KCH; ++c) acc[c] += live ? v[u][c] : 0.0f;
        }
    }
    if (RPW > 1) {
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
            float tot = acc[c];
#pragma unroll
            for (int g = 1; g < RPW; ++g) tot += __shfl(acc[c], lane_col<RPW>(lane) + g * (64 / RPW));
            acc[c] = tot;
        }
    }
    if (grp == 0) {
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
            const int cc = lane_col<RPW>(lane) + 64 * c;
            if (cc < k) S[slot * k + cc] = acc[c];
        }
    }
}

// Gather.  A wave owns kGatherTile consecutive samples and sweeps all trees in order, two trees
// per step; all row loads of a step are issued before any is consumed.
constexpr int kGatherTrees = 2;

template <int KCH, int RPW>
__global__ __launch_bounds__(256) void pv_gather_kernel(const uint32_t* __restrict__ slot, int64_t N, int32_t B,
                                                       const float* __restrict__ S, int32_t k, float* __restrict__ Y) {
    constexpr int kSteps = kGatherTile / RPW;  // load instructions per tree
    const int lane = threadIdx.x & 63;
    const int64_t tile = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t i0 = tile * kGatherTile;
    if (i0 >= N) return;
    const int rows = (int)min((int64_t)kGatherTile, N - i0);
    const int grp = lane / (64 / RPW);
    int col[KCH];
#pragma unroll
    for (int c = 0; c < KCH; ++c) col[c] = min(lane_col<RPW>(lane) + 64 * c, k - 1);
    float acc[kSteps][KCH];
#pragma unroll
    for (int s = 0; s < kSteps; ++s)
#pragma unroll
        for (int c = 0; c < KCH; ++c) acc[s][c] = 0.0f;
    // lane l < 32 carries the slot of sample i0 + l (clamped to the tile's last valid row)
    const int64_t my_row = i0 + min(lane & (kGatherTile - 1), rows - 1);
    for (int b = 0; b < B; b += kGatherTrees) {
        uint32_t mine[kGatherTrees];
#pragma unroll
        for (int t = 0; t < kGatherTrees; ++t) mine[t] = slot[(int64_t)min(b + t, B - 1) * N + my_row];
        float v[kGatherTrees][kSteps][KCH];
#pragma unroll
        for (int t = 0; t < kGatherTrees; ++t)
#pragma unroll
            for (int s = 0; s < kSteps; ++s) {
                uint32_t row;
                if (RPW == 1)
                    row = __builtin_amdgcn_readlane(mine[t], s);
                else
                    row = __shfl(mine[t], s * RPW + grp);
#pragma unroll
                for (int c = 0; c < KCH; ++c) v[t][s][c] = S[(int64_t)row * k + col[c]];
            }
#pragma unroll
        for (int t = 0; t < kGatherTrees; ++t) {
            const bool live = b + t < B;
#pragma unroll
            for (int s = 0; s < kSteps; ++s)
#pragma unroll
                for (int c = 0; c < KCH; ++c) acc[s][c] += live ? v[t][s][c] : 0.0f;
        }
    }
    const float Bf = (float)B;
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
        const int r = s * RPW + grp;
        if (r < rows) {
#pragma unroll
            for (int c = 0; c < KCH; ++c) {
                const int cc = lane_col<RPW>(lane) + 64 * c;
                if (cc < k) Y[(i0 + r) * k + cc] = acc[s][c] / Bf;
            }
        }
    }
}

template <int KCH, int RPW>
int launch_apply(const rfx_pv_plan* p, const float* V, int32_t k, float* Y, hipStream_t st) {
    const int64_t n_slots = (int64_t)p->B * p->Lb;
    {
        rfx::TimedLaunch timed("pv_leaf_sum_kernel", st);
        hipLaunchKernelGGL((pv_leaf_sum_kernel<KCH, RPW>), dim3((unsigned)rfx::ceil_div(n_slots, 4)), dim3(256), 0, st,
                           p->d_seg_start, p->d_perm, n_slots, V, k, p->d_S);
    }
    RFX_LAUNCH_CHECK("pv_leaf_sum_kernel");
    const int64_t tiles = rfx::ceil_div(p->N, kGatherTile);
    rfx::TimedLaunch timed("pv_gather_kernel", st);
    hipLaunchKernelGGL((pv_gather_kernel<KCH, RPW>), dim3((unsigned)rfx::ceil_div(tiles, 4)), dim3(256), 0, st, p->d_slot,
                       p->N, p->B, p->d_S, k, Y);
    RFX_LAUNCH_CHECK("pv_gather_kernel");
    return RFX_OK;
}

}  // namespace

extern "C" {

int rfx_pv_plan_destroy(rfx_pv_plan* p) {
    if (!p) return RFX_OK;
    if (p->d_slot) (void)hipFree(p->d_slot);
    if (p->d_perm) (void)hipFree(p->d_perm);
    if (p->d_seg_start) (void)hipFree(p->d_seg_start);
    if (p->d_S) (void)hipFree(p->d_S);
    delete p;
    return RFX_OK;
}

int rfx_pv_plan_create(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, rfx_pv_plan** out, void* stream) {
    if (!leaf || !out) return rfx::fail(RFX_ERR_NULL, "rfx_pv_plan_create: null argument");
    *out = nullptr;
    if (N < 1 || B < 1 || leaf_bound < 1)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_pv_plan_create: N=%lld B=%d leaf_bound=%d", (long long)N, B, leaf_bound);
    if ((int64_t)B * N >= (1ll << 32) || (int64_t)B * leaf_bound >= (1ll << 32) || B > 65535)
        return rfx::fail(RFX_ERR_UNSUPPORTED, "rfx_pv_plan_create: B*N or B*leaf_bound does not fit 32 bits");
    hipStream_t st = rfx::as_stream(stream);
    rfx_pv_plan* p = new (std::nothrow) rfx_pv_plan;
    if (!p) return rfx::fail(RFX_ERR_OOM, "rfx_pv_plan_create: host allocation failed");
    p->N = N;
    p->B = B;
    p->Lb = leaf_bound;
    const int64_t n_slots = (int64_t)B * leaf_bound;
    rfx::DevBuf count, bad;
    hipError_t e = hipMalloc((void**)&p->d_slot, sizeof(uint32_t) * (size_t)B * (size_t)N);
    if (e == hipSuccess) e = hipMalloc((void**)&p->d_perm, sizeof(uint32_t) * (size_t)B * (size_t)N);
    if (e == hipSuccess) e = hipMalloc((void**)&p->d_seg_start, sizeof(uint32_t) * (size_t)(n_slots + 1));
    if (e == hipSuccess) e = count.alloc(sizeof(uint32_t) * (size_t)n_slots * 2);
    if (e == hipSuccess) e = bad.alloc(sizeof(int));
    if (e == hipSuccess) e = hipMemsetAsync(count.p, 0, sizeof(uint32_t) * (size_t)n_slots, st);
    if (e == hipSuccess) e = hipMemsetAsync(bad.p, 0, sizeof(int), st);
    if (e != hipSuccess) {
        rfx_pv_plan_destroy(p);
        return rfx::fail(e == hipErrorOutOfMemory ? RFX_ERR_OOM : RFX_ERR_HIP, "rfx_pv_plan_create: %s", hipGetErrorString(e));
    }
    uint32_t* cnt = count.as<uint32_t>();
    uint32_t* cursor = cnt + n_slots;
    hipLaunchKernelGGL(pv_hist_kernel, dim3((unsigned)rfx::ceil_div(N, 256), (unsigned)B), dim3(256), 0, st, leaf, N, B,
                       leaf_bound, p->d_slot, cnt, bad.as<int>());
    hipLaunchKernelGGL(pv_scan_kernel, dim3((unsigned)B), dim3(256), 0, st, cnt, N, B, leaf_bound, p->d_seg_start, cursor);
    hipLaunchKernelGGL(pv_scatter_kernel, dim3((unsigned)B), dim3(64), 0, st, p->d_slot, N, cursor, p->d_perm);
    int h_bad = 0;
    e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(&h_bad, bad.p, sizeof(int), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess || h_bad) {
        rfx_pv_plan_destroy(p);
        if (e != hipSuccess) return rfx::fail(RFX_ERR_HIP, "rfx_pv_plan_create: %s", hipGetErrorString(e));
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_pv_plan_create: a leaf id is >= leaf_bound=%d", leaf_bound);
    }
    *out = p;
    return RFX_OK;
}

int rfx_pv_apply(rfx_pv_plan* p, const float* V, int32_t k, float* Y, void* stream) {
    if (!p || !V || !Y) return rfx::fail(RFX_ERR_NULL, "rfx_pv_apply: null argument");
    if (k < 1 || k > 256) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_pv_apply: k=%d outside 1..256", k);
    if (V == Y) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_pv_apply: V and Y must not overlap");
    hipStream_t st = rfx::as_stream(stream);
    if (k > p->k_cap) {
        // earlier applies on any stream may still read the old buffer
        RFX_HIP(hipDeviceSynchronize());
        if (p->d_S) (void)hipFree(p->d_S);
        p->d_S = nullptr;
        p->k_cap = 0;
        RFX_HIP(hipMalloc((void**)&p->d_S, sizeof(float) * (size_t)p->B * (size_t)p->Lb * (size_t)k));
        p->k_cap = k;
    }
    if (k <= 16) return launch_apply<1, 4>(p, V, k, Y, st);
    if (k <= 32) return launch_apply<1, 2>(p, V, k, Y, st);
    switch ((k + 63) / 64) {
        case 1: return launch_apply<1, 1>(p, V, k, Y, st);
        case 2: return launch_apply<2, 1>(p, V, k, Y, st);
        case 3: return launch_apply<3, 1>(p, V, k, Y, st);
        default: return launch_apply<4, 1>(p, V, k, Y, st);
    }
}

int rfx_prox_matvec(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, const float* V, int32_t k,
                    float* Y, void* stream) {
    if (!V || !Y) return rfx::fail(RFX_ERR_NULL, "rfx_prox_matvec: null argument");
    if (k < 1 || k > 256) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_matvec: k=%d outside 1..256", k);
    rfx_pv_plan* p = nullptr;
    int rc = rfx_pv_plan_create(leaf, N, B, leaf_bound, &p, stream);
    if (rc != RFX_OK) return rc;
    rc = rfx_pv_apply(p, V, k, Y, stream);
    hipError_t e = hipStreamSynchronize(rfx::as_stream(stream));
    rfx_pv_plan_destroy(p);
    if (rc != RFX_OK) return rc;
    if (e != hipSuccess) return rfx::fail(RFX_ERR_HIP, "rfx_prox_matvec: %s", hipGetErrorString(e));
    return RFX_OK;
}

}  // extern "C"
