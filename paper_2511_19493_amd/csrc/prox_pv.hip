// Implicit product Y = P V = (1/B) sum_b Z_b (Z_b^T V) without forming P
// (P from the paper's proximity equation; Z_b = one-hot leaf membership of tree b).
//
// Plan (once per forest): for every tree the samples are grouped by leaf with a stable counting
// sort, giving perm[B][N] (sample indices, leaf by leaf, ascending inside a leaf) and
// seg_start[B*Lb + 1] (Lb = leaf_bound; slot = b*Lb + leaf).  Ascending order inside a leaf
// fixes the float summation order, so results are reproducible run to run.  The sort splits
// each tree's samples into Q parts: per-part leaf histograms (in LDS when Lb allows), a per-tree
// scan that turns them into segment starts and per-part cursors, and a stable per-part scatter.
//
// Apply, both kernels pure row traffic of k floats:
//   leaf sums : S[slot,:] = sum over the slot's samples of V[sample,:].  Purity-grown trees have
//               thousands of tiny leaves and a few huge ones (most samples sit in leaves of more
//               than a thousand members), so slots up to kBigLeaf members take one wave each and
//               the rest, listed at plan time, take a 16-wave workgroup each whose waves sum
//               contiguous ranges and combine their partial sums in wave order.
//   gather    : Y[i,:] = (1/B) sum_b S[slot_b(i),:]   (a wave keeps a tile of Y rows in
//               registers and sweeps the trees in order, so all waves touch the same trees'
//               sums at about the same time and those rows stay cache-resident)
// The leaf sums are bound by row reads that come from the last-level cache, the gather by reads that
// hit L2, so one application runs in groups of trees: the sums of a group on the caller's stream, its
// gather on a second stream of the plan as soon as they are done (Y carries the partial sums from group
// to group, the same additions in the same order as one sweep), the caller's stream joining at the end.
#include <algorithm>
#include <mutex>
#include <optional>
#include <type_traits>
#include <vector>

#include "common.h"
#include "prox_pv.h"


namespace {

constexpr int kGatherTile = 32;   // Y rows per wave in the gather
#ifndef RFX_PV_GATHER_WAVES
#define RFX_PV_GATHER_WAVES 4096
#endif
constexpr int kGatherWaves = RFX_PV_GATHER_WAVES;  // waves the gather of a group should at least have (one per wave slot of the chip)
// Groups of trees per application.  Measured at N = 100,000, B = 1,000, k = 64: 5.66 ms in one group, 5.17 in two,
// 5.07 in four, 5.30 in eight.  Small problems stay in one group: their kernels are too short to pay for the extra
// launches and the cross-stream events (N = 10,000, B = 500: 0.57 ms in one group, 0.67 ms in four).
constexpr int kApplyChunks = rfx_pv_plan::kMaxChunks;
constexpr int64_t kApplyChunkMinPairs = 10000000;   // B * N from which the groups pay
#ifndef RFX_PV_BIG_LEAF
#define RFX_PV_BIG_LEAF 256
#endif
constexpr int kBigLeaf = RFX_PV_BIG_LEAF;     // slots with more members are summed by a whole workgroup
#ifndef RFX_PV_SPLIT
#define RFX_PV_SPLIT 1
#endif
constexpr bool kSplitBigLeaves = RFX_PV_SPLIT != 0;
constexpr int64_t kSplitMaxRangeBytes = 3584 * 1024;  // an eighth of V must fit a 4 MB second-level cache with room to spare
constexpr int kBigWaves = 16;
constexpr int kHistLdsLeaves = 16384;  // largest Lb whose histogram fits LDS (64 KB)

// Histogram of one part (blockIdx.x) of one tree (blockIdx.y) and the slot ids of its samples.
// kLds 1: the part's histogram is built in LDS, one 32-bit counter per leaf, and stored whole; kLds 2: the same
// with two 16-bit counters per LDS word (parts shorter than 65,536 samples, so no counter can carry into its
// neighbour); kLds 0: `count` was zeroed and takes global atomics.
template <int kLds>
__global__ __launch_bounds__(1024) void pv_hist_kernel(const uint32_t* __restrict__ leaf, int64_t N, int32_t Lb,
                                                      int64_t part_len, uint32_t* __restrict__ slot,
                                                      uint32_t* __restrict__ count, int* __restrict__ bad) {
    extern __shared__ uint32_t hist[];
    const int q = blockIdx.x, Q = gridDim.x, b = blockIdx.y;
    uint32_t* mine = count + ((int64_t)b * Q + q) * Lb;
    const int words = kLds == 2 ? (Lb + 1) / 2 : Lb;
    if (kLds) {
        for (int l = threadIdx.x; l < words; l += blockDim.x) hist[l] = 0;
        __syncthreads();
    }
    const int64_t lo = (int64_t)q * part_len, hi = min(N, lo + part_len);
    for (int64_t i = lo + threadIdx.x; i < hi; i += blockDim.x) {
        uint32_t id = leaf[(int64_t)b * N + i];
        if (id >= (uint32_t)Lb) {
            *bad = 1;
            id = (uint32_t)Lb - 1;
        }
        slot[(int64_t)b * N + i] = (uint32_t)b * (uint32_t)Lb + id;
        if (kLds == 1)
            atomicAdd(&hist[id], 1u);
        else if (kLds == 2)
            atomicAdd(&hist[id >> 1], 1u << (16 * (id & 1)));
        else
            atomicAdd(&mine[id], 1u);
    }
    if (kLds) {
        __syncthreads();
        for (int l = threadIdx.x; l < Lb; l += blockDim.x)
            mine[l] = kLds == 2 ? (hist[l >> 1] >> (16 * (l & 1))) & 0xffffu : hist[l];
    }
}

__global__ __launch_bounds__(256) void pv_zero_kernel(uint32_t* __restrict__ p, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// Groups of trees (consecutive ranges) and where each group's list of big slots starts.
struct BigGroups {
    int n;
    int tree_end[rfx_pv_plan::kMaxChunks];
    int64_t base[rfx_pv_plan::kMaxChunks];
};

// One workgroup per tree.  With c[q][l] the part histograms: seg_start[b*Lb + l] = b*N + (samples of
// the tree in leaves < l); c[q][l] is replaced by the cursor seg_start + sum_{q' < q} c[q'][l]; slots
// with more than kBigLeaf members are appended to the big list of the tree's group.  Leaves are taken 256 at a time,
// one per thread, so that every access to c is coalesced; the running offset is carried across tiles.
__global__ __launch_bounds__(256) void pv_scan_kernel(uint32_t* __restrict__ count, int64_t N, int32_t B, int32_t Lb, int32_t Q,
                                                     uint32_t* __restrict__ seg_start, uint32_t* __restrict__ big,
                                                     int* __restrict__ n_big, BigGroups groups) {
    __shared__ uint32_t wave_tot[4];
    __shared__ uint32_t carry;
    const int b = blockIdx.x;
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    int grp = 0;
    while (grp + 1 < groups.n && b >= groups.tree_end[grp]) ++grp;
    uint32_t* c = count + (int64_t)b * Q * Lb;
    if (t == 0) carry = (uint32_t)((int64_t)b * N);
    __syncthreads();
    for (int l0 = 0; l0 < Lb; l0 += 256) {
        const int l = l0 + t;
        uint32_t tot = 0;
        if (l < Lb)
            for (int q = 0; q < Q; ++q) tot += c[(int64_t)q * Lb + l];
        // inclusive scan inside the wave, then across the 4 waves
        uint32_t inc = tot;
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(inc, off);
            if (lane >= off) inc += up;
        }
        if (lane == 63) wave_tot[w] = inc;
        __syncthreads();
        uint32_t before = carry;
        for (int u = 0; u < w; ++u) before += wave_tot[u];
        uint32_t run = before + inc - tot;  // exclusive
        if (l < Lb) {
            seg_start[(int64_t)b * Lb + l] = run;
            for (int q = 0; q < Q; ++q) {
                const uint32_t v = c[(int64_t)q * Lb + l];
                c[(int64_t)q * Lb + l] = run;
                run += v;
            }
            if (tot > (uint32_t)kBigLeaf)
                big[groups.base[grp] + atomicAdd(&n_big[grp], 1)] = (uint32_t)b * (uint32_t)Lb + (uint32_t)l;
        }
        __syncthreads();
        if (t == 255) carry = before + inc;
        __syncthreads();
    }
    if (b == B - 1 && t == 0) seg_start[(int64_t)B * Lb] = (uint32_t)((int64_t)B * N);
}

// Groups the lanes of a wave by key: my_leader = lowest lane with this lane's key, rank = lanes with the same key below this
// one, gcount = size of the group.  In a deep forest nearly all 64 keys of a step differ, so the lanes first find out which
// of them may share a key at all: every lane writes its number into a 1,024-entry LDS table at a hash of its key and reads
// the entry back; a lane that reads its own number has a key no other lane holds, unless that other lane lost the entry to
// it and is therefore among the rest.  Only the keys of the rest are then compared across the wave, one ballot per key.
constexpr int kRankTable = 1024;

__device__ __forceinline__ void rank_equal_keys(uint32_t key, bool valid, int lane, uint32_t* tab, int& my_leader, uint32_t& rank,
                                                uint32_t& gcount) {
    const uint32_t h = (key * 2654435761u) >> 22;
    if (valid) tab[h] = (uint32_t)lane;
    __builtin_amdgcn_wave_barrier();   // one wave: its LDS accesses complete in order
    const bool lost = valid && tab[h] != (uint32_t)lane;
    __builtin_amdgcn_wave_barrier();   // the next step's writes stay behind these reads
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    uint64_t remaining = __ballot(lost);
    my_leader = lane;
    rank = 0;
    gcount = 1;
    while (remaining) {
        const int leader = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)remaining) - 1);
        const uint32_t lk = __builtin_amdgcn_readlane(key, leader);
        const uint64_t m = __ballot(valid && key == lk);
        if (valid && key == lk) {
            my_leader = __ffsll((unsigned long long)m) - 1;
            rank = (uint32_t)__popcll(m & lt_mask);
            gcount = (uint32_t)__popcll(m);
        }
        remaining &= ~m;
    }
}

// Stable scatter: one wave per (part, tree) walks its samples 64 at a time in ascending order.  Lanes
// with the same slot are ranked by lane index; the group's first lane reserves the group's range
// with one atomic add on the part's cursor, so the order inside every leaf is ascending sample index.
__global__ __launch_bounds__(64) void pv_scatter_kernel(const uint32_t* __restrict__ slot, int64_t N, int32_t Lb,
                                                       int64_t part_len, uint32_t* __restrict__ cursor,
                                                       uint32_t* __restrict__ perm, int32_t b_first) {
    __shared__ uint32_t tab[kRankTable];
    const int q = blockIdx.x, Q = gridDim.x, b = b_first + blockIdx.y;
    const int lane = threadIdx.x;
    const uint32_t* s = slot + (int64_t)b * N;
    uint32_t* cur = cursor + ((int64_t)b * Q + q) * Lb - (int64_t)b * Lb;  // indexed by slot = b*Lb + leaf
    const int64_t lo = (int64_t)q * part_len, hi = min(N, lo + part_len);
    for (int64_t i0 = lo; i0 < hi; i0 += 64) {
        const int64_t i = i0 + lane;
        const bool valid = i < hi;
        const uint32_t key = valid ? s[i] : 0xffffffffu;
        int my_leader;
        uint32_t rank, gcount;
        rank_equal_keys(key, valid, lane, tab, my_leader, rank, gcount);
        uint32_t base = 0;
        if (valid && my_leader == lane) base = atomicAdd(&cur[key], gcount);
        base = __shfl(base, my_leader);
        if (valid) perm[base + rank] = (uint32_t)i;
    }
}

// The same scatter with the part's cursors in LDS (leaf bounds up to kScatterLdsLeaves): they are loaded once,
// coalesced, and the first lane of every group of equal slots advances its cursor with a plain read and write
// (the groups of a step have distinct slots), so no global atomic and no round trip per step is left.
constexpr int kScatterLdsLeaves = 8192;  // 32 KB of cursors per wave, five waves per CU

__global__ __launch_bounds__(64) void pv_scatter_lds_kernel(const uint32_t* __restrict__ slot, int64_t N, int32_t Lb,
                                                           int64_t part_len, const uint32_t* __restrict__ cursor,
                                                           uint32_t* __restrict__ perm) {
    extern __shared__ uint32_t cur[];  // [Lb]
    __shared__ uint32_t tab[kRankTable];
    const int q = blockIdx.x, Q = gridDim.x, b = blockIdx.y;
    const int lane = threadIdx.x;
    const uint32_t* s = slot + (int64_t)b * N;
    const uint32_t* mine = cursor + ((int64_t)b * Q + q) * Lb;
    for (int l = lane; l < Lb; l += 64) cur[l] = mine[l];
    __builtin_amdgcn_wave_barrier();
    const uint32_t slot0 = (uint32_t)b * (uint32_t)Lb;
    const int64_t lo = (int64_t)q * part_len, hi = min(N, lo + part_len);
    for (int64_t i0 = lo; i0 < hi; i0 += 64) {
        const int64_t i = i0 + lane;
        const bool valid = i < hi;
        const uint32_t key = valid ? s[i] - slot0 : 0xffffffffu;
        int my_leader;
        uint32_t rank, gcount;
        rank_equal_keys(key, valid, lane, tab, my_leader, rank, gcount);
        uint32_t base = 0;
        if (valid && my_leader == lane) {
            base = cur[key];
            cur[key] = base + gcount;
        }
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

constexpr int kSumBatch = 8;

// Sum of the V rows of members perm[lo .. hi) for this lane's columns.  The RPW lane groups take
// members t, t+RPW, ... in batches of kSumBatch loads; their partial sums are added in group order,
// so every lane of a column ends with the same total.
template <int KCH, int RPW>
__device__ __forceinline__ void sum_members(const uint32_t* __restrict__ perm, uint32_t lo, uint32_t hi,
                                            const float* __restrict__ V, int32_t k, int lane, float (&acc)[KCH]) {
    const int grp = lane / (64 / RPW);
    int col[KCH];
#pragma unroll
    for (int c = 0; c < KCH; ++c) {
        col[c] = min(lane_col<RPW>(lane) + 64 * c, k - 1);
        acc[c] = 0.0f;
    }
    if (lo >= hi) return;
    // one batch of NBATCH row loads per lane group, all issued before any is added
    auto batch = [&](uint32_t t0, auto nbatch) {
        constexpr int NBATCH = decltype(nbatch)::value;
        float v[NBATCH][KCH];
#pragma unroll
        for (int u = 0; u < NBATCH; ++u) {
            const uint32_t t = t0 + u * RPW + grp;
            const uint32_t j = perm[min(t, hi - 1)];  // clamped: always a valid member
#pragma unroll
            for (int c = 0; c < KCH; ++c) v[u][c] = V[(int64_t)j * k + col[c]];
        }
#pragma unroll
        for (int u = 0; u < NBATCH; ++u) {
            const bool live = t0 + u * RPW + grp < hi;
#pragma unroll
            for (int c = 0; c < KCH; ++c) acc[c] += live ? v[u][c] : 0.0f;
        }
    };
    // most leaves of a purity-grown tree hold one to four samples: do not pay for a full batch there
    const uint32_t n = hi - lo;
    if (n <= 2u * RPW) {
        batch(lo, std::integral_constant<int, 2>{});
    } else if (n <= 4u * RPW) {
        batch(lo, std::integral_constant<int, 4>{});
    } else {
        for (uint32_t t0 = lo; t0 < hi; t0 += kSumBatch * RPW) batch(t0, std::integral_constant<int, kSumBatch>{});
    }
    if (RPW > 1) {
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
            float tot = __shfl(acc[c], lane_col<RPW>(lane));
#pragma unroll
            for (int g = 1; g < RPW; ++g) tot += __shfl(acc[c], lane_col<RPW>(lane) + g * (64 / RPW));
            acc[c] = tot;
        }
    }
}

// Leaf sums of the slots with at most kBigLeaf members.  Most of them hold one to four samples, so
// a wave's time is three dependent memory round trips (segment bounds, member indices, rows) and
// almost no traffic; a wave therefore takes kSlotsPerWave consecutive slots at once and has the
// first four rows of each in flight together before it finishes the longer ones.
constexpr int kSlotsPerWave = 4;

template <int KCH, int RPW>
__global__ __launch_bounds__(256) void pv_leaf_sum_kernel(const uint32_t* __restrict__ seg_start,
                                                         const uint32_t* __restrict__ perm, int64_t slot_begin,
                                                         int64_t n_slots, uint32_t n_perm, const float* __restrict__ V,
                                                         int32_t k, float* __restrict__ S) {
    // slots slot_begin .. n_slots - 1
    constexpr int G = kSlotsPerWave, NF = 4;  // NF = rows per lane group in the first batch
    const int lane = threadIdx.x & 63;
    const int grp = lane / (64 / RPW);
    const int64_t slot0 = slot_begin + ((int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6)) * G;
    if (slot0 >= n_slots) return;
    int col[KCH];
#pragma unroll
    for (int c = 0; c < KCH; ++c) col[c] = min(lane_col<RPW>(lane) + 64 * c, k - 1);
    uint32_t lo[G], hi[G];
    bool mine[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int64_t s = min(slot0 + g, n_slots - 1);
        lo[g] = seg_start[s];
        hi[g] = seg_start[s + 1];
        // empty slots are never read by the gather; big ones belong to the workgroup kernel
        mine[g] = slot0 + g < n_slots && hi[g] > lo[g] && hi[g] - lo[g] <= (uint32_t)kBigLeaf;
    }
    float v[G][NF][KCH];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int u = 0; u < NF; ++u) {
            const uint32_t t = lo[g] + u * RPW + grp;
            const uint32_t j = perm[min(min(t, hi[g] - 1), n_perm - 1)];  // clamped: always a valid index
#pragma unroll
            for (int c = 0; c < KCH; ++c) v[g][u][c] = V[(int64_t)j * k + col[c]];
        }
    float acc[G][KCH];
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int c = 0; c < KCH; ++c) acc[g][c] = 0.0f;
#pragma unroll
        for (int u = 0; u < NF; ++u) {
            const bool live = mine[g] && lo[g] + u * RPW + grp < hi[g];
#pragma unroll
            for (int c = 0; c < KCH; ++c) acc[g][c] += live ? v[g][u][c] : 0.0f;
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (!mine[g]) continue;
        for (uint32_t t0 = lo[g] + NF * RPW; t0 < hi[g]; t0 += kSumBatch * RPW) {
            float w[kSumBatch][KCH];
#pragma unroll
            for (int u = 0; u < kSumBatch; ++u) {
                const uint32_t t = t0 + u * RPW + grp;
                const uint32_t j = perm[min(t, hi[g] - 1)];
#pragma unroll
                for (int c = 0; c < KCH; ++c) w[u][c] = V[(int64_t)j * k + col[c]];
            }
#pragma unroll
            for (int u = 0; u < kSumBatch; ++u) {
                const bool live = t0 + u * RPW + grp < hi[g];
#pragma unroll
                for (int c = 0; c < KCH; ++c) acc[g][c] += live ? w[u][c] : 0.0f;
            }
        }
        if (RPW > 1) {
#pragma unroll
            for (int c = 0; c < KCH; ++c) {
                float tot = __shfl(acc[g][c], lane_col<RPW>(lane));
#pragma unroll
                for (int q = 1; q < RPW; ++q) tot += __shfl(acc[g][c], lane_col<RPW>(lane) + q * (64 / RPW));
                acc[g][c] = tot;
            }
        }
        if (lane < 64 / RPW) {
#pragma unroll
            for (int c = 0; c < KCH; ++c) {
                const int cc = lane + 64 * c;
                if (cc < k) S[(slot0 + g) * k + cc] = acc[g][c];
            }
        }
    }
}

// Leaf sums of the listed big slots: one 16-wave workgroup per slot.  Wave w sums the w-th contiguous
// share of the members; the 16 partial rows are then added in wave order.
template <int KCH, int RPW>
__global__ __launch_bounds__(64 * kBigWaves) void pv_leaf_sum_big_kernel(const uint32_t* __restrict__ big,
                                                                        const uint32_t* __restrict__ seg_start,
                                                                        const uint32_t* __restrict__ perm,
                                                                        const float* __restrict__ V, int32_t k,
                                                                        float* __restrict__ S) {
    __shared__ float part[kBigWaves][KCH * 64];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t slot = big[blockIdx.x];
    const uint32_t lo = seg_start[slot], hi = seg_start[slot + 1];
    const uint32_t share = ((hi - lo + kBigWaves - 1) / kBigWaves + kSumBatch * RPW - 1) / (kSumBatch * RPW) * (kSumBatch * RPW);
    const uint32_t wlo = min(hi, lo + w * share), whi = min(hi, wlo + share);
    float acc[KCH];
    sum_members<KCH, RPW>(perm, wlo, whi, V, k, lane, acc);
    if (lane < 64 / RPW) {
#pragma unroll
        for (int c = 0; c < KCH; ++c) part[w][lane + 64 * c] = acc[c];
    }
    __syncthreads();
    for (int cc = threadIdx.x; cc < k; cc += 64 * kBigWaves) {
        float tot = part[0][cc];
#pragma unroll
        for (int u = 1; u < kBigWaves; ++u) tot += part[u][cc];
        S[slot * k + cc] = tot;
    }
}

// The same sums in pieces.  The members of a slot are ascending sample indices, so the samples of range x (the x-th of
// kRanges equal parts of 0..N-1) are one contiguous piece of the segment; bounds[idx][x] is where it begins.  Workgroup
// 8 idx + x sums piece x of big slot idx: consecutive workgroup ids go to the 8 XCDs in turn, so the XCD that runs
// pieces x only ever gathers rows from the x-th eighth of V, which stays in its second-level cache when that eighth
// is smaller than the cache (the rows of a whole segment are spread over all of V and come from the last-level cache).
// The pieces' sums go to `part` and are added in range order by pv_combine_kernel, so the result does not depend on timing.
#ifndef RFX_PV_SPLIT_WAVES
#define RFX_PV_SPLIT_WAVES 4
#endif
constexpr int kSplitWaves = RFX_PV_SPLIT_WAVES;

__global__ __launch_bounds__(256) void pv_big_bounds_kernel(const uint32_t* __restrict__ big, int32_t n_big,
                                                           const uint32_t* __restrict__ seg_start,
                                                           const uint32_t* __restrict__ perm, int64_t N,
                                                           uint32_t* __restrict__ bounds) {
    constexpr int R = rfx_pv_plan::kRanges;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_big * (R + 1)) return;
    const int idx = t / (R + 1), x = t % (R + 1);
    const uint32_t slot = big[idx];
    uint32_t lo = seg_start[slot], hi = seg_start[slot + 1];
    const uint32_t first = (uint32_t)(((int64_t)x * N + R - 1) / R);  // first sample of range x (x = R: N)
    while (lo < hi) {  // first position whose sample is >= first
        const uint32_t mid = lo + (hi - lo) / 2;
        if (perm[mid] < first)
            lo = mid + 1;
        else
            hi = mid;
    }
    bounds[(int64_t)idx * (R + 1) + x] = lo;
}

template <int KCH, int RPW>
__global__ __launch_bounds__(64 * kSplitWaves) void pv_leaf_sum_split_kernel(const uint32_t* __restrict__ bounds,
                                                                            const uint32_t* __restrict__ perm,
                                                                            const float* __restrict__ V, int32_t k,
                                                                            float* __restrict__ part) {
    constexpr int R = rfx_pv_plan::kRanges;
    __shared__ float sm[kSplitWaves][KCH * 64];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t idx = blockIdx.x / R;
    const int x = blockIdx.x % R;
    const uint32_t lo = bounds[idx * (R + 1) + x], hi = bounds[idx * (R + 1) + x + 1];
    const uint32_t share = ((hi - lo + kSplitWaves - 1) / kSplitWaves + kSumBatch * RPW - 1) / (kSumBatch * RPW) * (kSumBatch * RPW);
    const uint32_t wlo = min(hi, lo + w * share), whi = min(hi, wlo + share);
    float acc[KCH];
    sum_members<KCH, RPW>(perm, wlo, whi, V, k, lane, acc);
    if (lane < 64 / RPW) {
#pragma unroll
        for (int c = 0; c < KCH; ++c) sm[w][lane + 64 * c] = acc[c];
    }
    __syncthreads();
    for (int cc = threadIdx.x; cc < k; cc += 64 * kSplitWaves) {
        float tot = sm[0][cc];
#pragma unroll
        for (int u = 1; u < kSplitWaves; ++u) tot += sm[u][cc];
        part[((int64_t)blockIdx.x) * k + cc] = tot;
    }
}

// S[big[idx]] = sum over the ranges, in range order, of the pieces' sums
__global__ __launch_bounds__(256) void pv_combine_kernel(const uint32_t* __restrict__ big, int32_t n_big,
                                                        const float* __restrict__ part, int32_t k, float* __restrict__ S) {
    constexpr int R = rfx_pv_plan::kRanges;
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (int64_t)n_big * k) return;
    const int64_t idx = e / k;
    const int cc = (int)(e % k);
    float tot = part[(idx * R) * k + cc];
#pragma unroll
    for (int x = 1; x < R; ++x) tot += part[(idx * R + x) * k + cc];
    S[(int64_t)big[idx] * k + cc] = tot;
}

// Gather.  A wave owns kGatherTile consecutive samples and sweeps the trees b_begin .. b_end - 1 in order, two
// trees per step; all row loads of a step are issued before any is consumed.  The sums start from zero for the
// first group of trees (kFirst) and from the values the previous group left in Y otherwise (the same additions in the same
// order as one sweep over all trees); the last group divides by B.
constexpr int kGatherTrees = 2;
// For k in 33..64 the kernel needs 131 registers as written; held to 128 (four waves per SIMD instead of three, one
// register spilled) an application takes 4.89 instead of 5.07 ms; at 102 (five waves) the spills cost more (5.26 ms).

template <int KCH, int RPW, bool kFirst>
__global__ __launch_bounds__(256, (KCH == 1 && RPW == 1) ? 4 : 1) void pv_gather_kernel(const uint32_t* __restrict__ slot, int64_t N, int32_t B,
                                                       int32_t b_begin, int32_t b_end,
                                                       const float* __restrict__ S, int32_t k, float* __restrict__ Y,
                                                       int32_t trees_per_piece) {
    constexpr int kSteps = kGatherTile / RPW;  // load instructions per tree
    // A small N gives too few tiles to fill the chip and each of them a long chain of dependent steps, so the trees are
    // then cut into pieces (blockIdx.y) whose sums go to Y = part[piece][N][k] unscaled and are added in piece order afterwards.
    const bool pieces = trees_per_piece > 0;
    if (pieces) {
        b_begin += (int32_t)blockIdx.y * trees_per_piece;
        b_end = min(b_end, b_begin + trees_per_piece);
        Y += (int64_t)blockIdx.y * N * k;
    }
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
        for (int c = 0; c < KCH; ++c) {
            const int r = s * RPW + grp, cc = lane_col<RPW>(lane) + 64 * c;
            acc[s][c] = (!kFirst && r < rows && cc < k) ? Y[(i0 + r) * k + cc] : 0.0f;
        }
    // lane l < 32 carries the slot of sample i0 + l (clamped to the tile's last valid row)
    const int64_t my_row = i0 + min(lane & (kGatherTile - 1), rows - 1);
    for (int b = b_begin; b < b_end; b += kGatherTrees) {
        uint32_t mine[kGatherTrees];
#pragma unroll
        for (int t = 0; t < kGatherTrees; ++t) mine[t] = slot[(int64_t)min(b + t, b_end - 1) * N + my_row];
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
            const bool live = b + t < b_end;
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
                if (cc < k) Y[(i0 + r) * k + cc] = (b_end == B && !pieces) ? acc[s][c] / Bf : acc[s][c];
            }
        }
    }
}

// Y = (Y of the groups of trees before, unless this is the first group) + the pieces' sums in piece order, divided by the
// number of trees after the last group
__global__ __launch_bounds__(256) void pv_gather_combine_kernel(const float* __restrict__ part, int32_t n_pieces, int64_t n,
                                                               int first, int last, float n_trees, float* __restrict__ Y) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    float acc = first ? 0.0f : Y[e];
    for (int32_t c = 0; c < n_pieces; ++c) acc += part[(int64_t)c * n + e];
    Y[e] = last ? acc / n_trees : acc;
}

// The second stream of the overlapped application: one per device for the life of the process, created on first use
// (default priority, not synchronised with the null stream).
hipError_t side_stream(hipStream_t* out) {
    static std::mutex mu;
    static hipStream_t streams[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(mu);
    if (!streams[dev]) e = hipStreamCreateWithFlags(&streams[dev], hipStreamNonBlocking);
    *out = streams[dev];
    return e;
}

template <int KCH, int RPW>
int launch_apply(const rfx_pv_plan* p, const float* V, int32_t k, float* Y, hipStream_t st) {
    const int64_t tiles = rfx::ceil_div(p->N, kGatherTile);
    // with one group the two kernel brackets below add up to the application; no third pair of events then
    std::optional<rfx::TimedLaunch> whole;
    if (p->n_chunks > 1) whole.emplace("pv_apply", st);
    // Big slots in pieces by sample range when an eighth of V fits the second-level cache of an XCD with room to spare and
    // the pieces' buffer holds them all (every group of trees has its own part of that buffer)
    int64_t n_big_all = 0, part_off = 0;
    for (int c = 0; c < p->n_chunks; ++c) n_big_all += p->big_cnt[c];
    const bool split = kSplitBigLeaves && p->d_part && n_big_all <= p->part_cap &&
                       (int64_t)p->N * k * 4 / rfx_pv_plan::kRanges <= kSplitMaxRangeBytes;
    for (int c = 0; c < p->n_chunks; ++c) {
        const int b0 = p->tree_off[c], b1 = p->tree_off[c + 1];
        const int64_t slot_begin = (int64_t)b0 * p->Lb, slot_end = (int64_t)b1 * p->Lb;
        const int n_big = p->big_cnt[c];
        {
            rfx::TimedLaunch timed("pv_leaf_sum_kernel", st);
            hipLaunchKernelGGL((pv_leaf_sum_kernel<KCH, RPW>),
                               dim3((unsigned)rfx::ceil_div(slot_end - slot_begin, 4 * kSlotsPerWave)), dim3(256), 0, st,
                               p->d_seg_start, p->d_perm, slot_begin, slot_end, (uint32_t)((int64_t)p->B * p->N), V, k, p->d_S);
            if (n_big > 0 && split) {
                float* part = p->d_part + part_off * rfx_pv_plan::kRanges * k;
                hipLaunchKernelGGL((pv_leaf_sum_split_kernel<KCH, RPW>), dim3((unsigned)n_big * rfx_pv_plan::kRanges),
                                   dim3(64 * kSplitWaves), 0, st, p->d_big_bounds + p->big_base[c] * (rfx_pv_plan::kRanges + 1),
                                   p->d_perm, V, k, part);
                hipLaunchKernelGGL(pv_combine_kernel, dim3((unsigned)rfx::ceil_div((int64_t)n_big * k, 256)), dim3(256), 0, st,
                                   p->d_big + p->big_base[c], n_big, part, k, p->d_S);
                part_off += n_big;
            } else if (n_big > 0) {
                hipLaunchKernelGGL((pv_leaf_sum_big_kernel<KCH, RPW>), dim3((unsigned)n_big), dim3(64 * kBigWaves), 0, st,
                                   p->d_big + p->big_base[c], p->d_seg_start, p->d_perm, V, k, p->d_S);
            }
        }
        RFX_LAUNCH_CHECK("pv_leaf_sum_kernel");
        // one group of trees: everything stays on the caller's stream
        hipStream_t gs = p->n_chunks > 1 ? p->side : st;
        if (p->n_chunks > 1) {
            RFX_HIP(hipEventRecord(p->ev_sum[c], st));
            RFX_HIP(hipStreamWaitEvent(gs, p->ev_sum[c], 0));
        }
        {
            rfx::TimedLaunch timed("pv_gather_kernel", gs);
            if (p->gather_pieces > 1) {
                const int32_t per = (b1 - b0 + p->gather_pieces - 1) / p->gather_pieces;
                const int32_t n_pieces = (b1 - b0 + per - 1) / per;   // no empty piece
                hipLaunchKernelGGL((pv_gather_kernel<KCH, RPW, true>), dim3((unsigned)rfx::ceil_div(tiles, 4), (unsigned)n_pieces),
                                   dim3(256), 0, gs, p->d_slot, p->N, p->B, b0, b1, p->d_S, k, p->d_gather_part, per);
                hipLaunchKernelGGL(pv_gather_combine_kernel, dim3((unsigned)rfx::ceil_div(p->N * k, 256)), dim3(256), 0, gs,
                                   p->d_gather_part, n_pieces, p->N * k, c == 0 ? 1 : 0, c == p->n_chunks - 1 ? 1 : 0, (float)p->B, Y);
            } else if (c == 0)
                hipLaunchKernelGGL((pv_gather_kernel<KCH, RPW, true>), dim3((unsigned)rfx::ceil_div(tiles, 4)), dim3(256), 0,
                                   gs, p->d_slot, p->N, p->B, b0, b1, p->d_S, k, Y, 0);
            else
                hipLaunchKernelGGL((pv_gather_kernel<KCH, RPW, false>), dim3((unsigned)rfx::ceil_div(tiles, 4)), dim3(256), 0,
                                   gs, p->d_slot, p->N, p->B, b0, b1, p->d_S, k, Y, 0);
        }
        RFX_LAUNCH_CHECK("pv_gather_kernel");
    }
    if (p->n_chunks > 1) {
        RFX_HIP(hipEventRecord(p->ev_done, p->side));
        RFX_HIP(hipStreamWaitEvent(st, p->ev_done, 0));
    }
    return RFX_OK;
}

}  // namespace

extern "C" {

int rfx_pv_plan_destroy(rfx_pv_plan* p) {
    if (!p) return RFX_OK;
    if (p->d_slot) (void)hipFree(p->d_slot);
    if (p->d_perm) (void)hipFree(p->d_perm);
    if (p->d_seg_start) (void)hipFree(p->d_seg_start);
    if (p->d_big) (void)hipFree(p->d_big);
    if (p->d_big_bounds) (void)hipFree(p->d_big_bounds);
    if (p->d_part) (void)hipFree(p->d_part);
    if (p->d_gather_part) (void)hipFree(p->d_gather_part);
    if (p->d_S) (void)hipFree(p->d_S);
    if (p->d_count) (void)hipFree(p->d_count);
    if (p->d_flags) (void)hipFree(p->d_flags);
    for (hipEvent_t e : p->ev_sum)
        if (e) (void)hipEventDestroy(e);
    if (p->ev_done) (void)hipEventDestroy(p->ev_done);
    delete p;
    return RFX_OK;
}

namespace {
constexpr int kPlanFlags = 1 + rfx_pv_plan::kMaxChunks;  // bad id seen; big slots per group

// Groups the samples of every tree by leaf into the plan's arrays (histograms, scan, stable scatter) and reads the
// counts of big slots back.  Allocates nothing; waits for the stream.
int build_plan(rfx_pv_plan* p, const uint32_t* leaf, hipStream_t st) {
    const int64_t N = p->N;
    const int32_t B = p->B, Lb = p->Lb, Q = p->Q;
    const int64_t n_slots = (int64_t)B * Lb;
    BigGroups groups;
    groups.n = p->n_chunks;
    for (int c = 0; c < rfx_pv_plan::kMaxChunks; ++c) {
        groups.tree_end[c] = c < p->n_chunks ? p->tree_off[c + 1] : B;
        groups.base[c] = p->big_base[c];
    }
    uint32_t* cnt = p->d_count;
    int* bad = p->d_flags;
    int* n_big = bad + 1;
    const size_t hist16_lds = sizeof(uint32_t) * (size_t)((Lb + 1) / 2);
    // the two clears are kernels, not memsets, so that a caller may capture the build into a graph
    if (!p->lds_hist) {
        hipLaunchKernelGGL(pv_zero_kernel, dim3((unsigned)std::min<int64_t>(rfx::ceil_div(n_slots * Q, 256), 65535)), dim3(256), 0,
                           st, cnt, n_slots * Q);
    }
    hipLaunchKernelGGL(pv_zero_kernel, dim3(1), dim3(256), 0, st, reinterpret_cast<uint32_t*>(p->d_flags), (int64_t)kPlanFlags);
    if (p->lds_hist == 1)
        hipLaunchKernelGGL(pv_hist_kernel<1>, dim3(Q, B), dim3(1024), sizeof(uint32_t) * Lb, st, leaf, N, Lb, p->part_len,
                           p->d_slot, cnt, bad);
    else if (p->lds_hist == 2)
        hipLaunchKernelGGL(pv_hist_kernel<2>, dim3(Q, B), dim3(1024), hist16_lds, st, leaf, N, Lb, p->part_len, p->d_slot, cnt,
                           bad);
    else
        hipLaunchKernelGGL(pv_hist_kernel<0>, dim3(Q, B), dim3(1024), 0, st, leaf, N, Lb, p->part_len, p->d_slot, cnt, bad);
    hipLaunchKernelGGL(pv_scan_kernel, dim3((unsigned)B), dim3(256), 0, st, cnt, N, B, Lb, Q, p->d_seg_start, p->d_big, n_big,
                       groups);
    if (Lb <= kScatterLdsLeaves)
        hipLaunchKernelGGL(pv_scatter_lds_kernel, dim3(Q, B), dim3(64), sizeof(uint32_t) * Lb, st, p->d_slot, N, Lb, p->part_len,
                           cnt, p->d_perm);
    else {
        // Trees are taken in batches whose cursors (4 Q Lb bytes per tree) fit the last-level cache together: the scatter is
        // one read-modify-write of a cursor per sample, and with all trees in flight those go to HBM (workload 5, 3 MB of
        // cursors per tree: 51 ms in one launch, 32 ms in batches of 64 trees, 37 / 40 ms in batches of 32 / 128).
        const int64_t per_tree = 4ll * Q * Lb;
        const int32_t batch = (int32_t)std::max<int64_t>(1, std::min<int64_t>(B, (192ll << 20) / per_tree));
        for (int32_t b0 = 0; b0 < B; b0 += batch)
            hipLaunchKernelGGL(pv_scatter_kernel, dim3(Q, std::min<int32_t>(batch, B - b0)), dim3(64), 0, st, p->d_slot, N, Lb,
                               p->part_len, cnt, p->d_perm, b0);
    }
    int h_flags[kPlanFlags] = {};
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(h_flags, p->d_flags, kPlanFlags * sizeof(int), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return rfx::fail(RFX_ERR_HIP, "rfx_pv_plan: %s", hipGetErrorString(e));
    if (h_flags[0]) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_pv_plan: a leaf id is >= leaf_bound=%d", Lb);
    for (int c = 0; c < p->n_chunks; ++c) p->big_cnt[c] = h_flags[1 + c];
    for (int c = 0; c < p->n_chunks; ++c) {
        if (p->big_cnt[c] == 0) continue;
        const int threads = p->big_cnt[c] * (rfx_pv_plan::kRanges + 1);
        hipLaunchKernelGGL(pv_big_bounds_kernel, dim3((unsigned)rfx::ceil_div(threads, 256)), dim3(256), 0, st,
                           p->d_big + p->big_base[c], p->big_cnt[c], p->d_seg_start, p->d_perm, N,
                           p->d_big_bounds + p->big_base[c] * (rfx_pv_plan::kRanges + 1));
    }
    RFX_LAUNCH_CHECK("pv_big_bounds_kernel");
    p->built = true;
    return RFX_OK;
}
}  // namespace

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
    const int Lb = leaf_bound;
    const int64_t n_slots = (int64_t)B * Lb;
    // parts per tree: enough (part, tree) pairs to fill the chip, parts of at least 4096 samples
    const int Q = p->Q = (int)std::max<int64_t>(1, std::min<int64_t>(16, N / 4096));
    const int64_t part_len = p->part_len = rfx::ceil_div(rfx::ceil_div(N, Q), 64) * 64;
    // groups of trees for the overlapped application, each with its own list of big slots
    p->n_chunks = (B >= 16 * kApplyChunks && (int64_t)B * N >= kApplyChunkMinPairs) ? kApplyChunks : 1;
    int64_t max_big = 0;
    for (int c = 0; c <= p->n_chunks; ++c) p->tree_off[c] = (int32_t)((int64_t)c * B / p->n_chunks);
    for (int c = 0; c < rfx_pv_plan::kMaxChunks; ++c) {
        const int trees = c < p->n_chunks ? p->tree_off[c + 1] - p->tree_off[c] : 0;
        p->big_base[c] = max_big;
        max_big += (int64_t)trees * N / kBigLeaf + 1;
    }
    // pieces of a group's tree range in the gather when the sample tiles are few: enough (tile, piece) pairs for about 4096
    // waves, at least 4 trees per piece, at most 16 pieces
    {
        const int64_t tiles = rfx::ceil_div(N, kGatherTile), group_trees = B / p->n_chunks;
        p->gather_pieces = (int32_t)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(16, group_trees / 4), kGatherWaves / tiles));
    }
    // 1: 32-bit LDS counters; 2: 16-bit pairs (up to 65,536 leaves, parts below 65,536 samples); 0: global atomics
    p->lds_hist = Lb <= kHistLdsLeaves ? 1 : ((Lb <= 65536 && part_len < 65536) ? 2 : 0);
    hipError_t e = hipMalloc((void**)&p->d_slot, sizeof(uint32_t) * (size_t)B * (size_t)N);
    if (e == hipSuccess) e = hipMalloc((void**)&p->d_perm, sizeof(uint32_t) * (size_t)B * (size_t)N);
    if (e == hipSuccess) e = hipMalloc((void**)&p->d_seg_start, sizeof(uint32_t) * (size_t)(n_slots + 1));
    if (e == hipSuccess) e = hipMalloc((void**)&p->d_big, sizeof(uint32_t) * (size_t)max_big);
    if (e == hipSuccess) e = hipMalloc((void**)&p->d_big_bounds, sizeof(uint32_t) * (size_t)max_big * (rfx_pv_plan::kRanges + 1));
    if (e == hipSuccess) e = hipMalloc((void**)&p->d_count, sizeof(uint32_t) * (size_t)n_slots * Q);
    if (e == hipSuccess) e = hipMalloc((void**)&p->d_flags, kPlanFlags * sizeof(int));
    const size_t hist16_lds = sizeof(uint32_t) * (size_t)((Lb + 1) / 2);
    if (e == hipSuccess && p->lds_hist == 2 && hist16_lds > 64 * 1024)
        e = hipFuncSetAttribute((const void*)pv_hist_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)hist16_lds);
    if (e == hipSuccess && p->n_chunks > 1) {
        e = side_stream(&p->side);
        for (int c = 0; c < p->n_chunks && e == hipSuccess; ++c)
            e = hipEventCreateWithFlags(&p->ev_sum[c], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&p->ev_done, hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        rfx_pv_plan_destroy(p);
        return rfx::fail(e == hipErrorOutOfMemory ? RFX_ERR_OOM : RFX_ERR_HIP, "rfx_pv_plan_create: %s", hipGetErrorString(e));
    }
    int rc = build_plan(p, leaf, st);
    if (rc != RFX_OK) {
        rfx_pv_plan_destroy(p);
        return rc;
    }
    *out = p;
    return RFX_OK;
}

int rfx_pv_plan_rebuild(rfx_pv_plan* p, const uint32_t* leaf, void* stream) {
    if (!p || !leaf) return rfx::fail(RFX_ERR_NULL, "rfx_pv_plan_rebuild: null argument");
    // applications of the old grouping on other streams must have finished; the caller orders that
    p->built = false;
    return build_plan(p, leaf, rfx::as_stream(stream));
}

int rfx_pv_plan_reserve(rfx_pv_plan* p, int32_t k) {
    if (!p) return rfx::fail(RFX_ERR_NULL, "rfx_pv_plan_reserve: plan is null");
    if (k < 1 || k > 256) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_pv_plan_reserve: k=%d outside 1..256", k);
    if (k <= p->k_cap) return RFX_OK;
    // earlier applications on any stream may still read the old buffer
    RFX_HIP(hipDeviceSynchronize());
    if (p->d_S) (void)hipFree(p->d_S);
    p->d_S = nullptr;
    p->k_cap = 0;
    RFX_HIP(hipMalloc((void**)&p->d_S, sizeof(float) * (size_t)p->B * (size_t)p->Lb * (size_t)k));
    // room for the pieces of a quarter more big slots than the current grouping has (a regrouped plan with more than that
    // sums its big slots whole)
    if (p->d_part) (void)hipFree(p->d_part);
    p->d_part = nullptr;
    int64_t n_big_all = 0;
    for (int c = 0; c < p->n_chunks; ++c) n_big_all += p->big_cnt[c];
    p->part_cap = n_big_all + n_big_all / 4 + 64;
    RFX_HIP(hipMalloc((void**)&p->d_part, sizeof(float) * (size_t)p->part_cap * rfx_pv_plan::kRanges * (size_t)k));
    if (p->d_gather_part) (void)hipFree(p->d_gather_part);
    p->d_gather_part = nullptr;
    if (p->gather_pieces > 1)
        RFX_HIP(hipMalloc((void**)&p->d_gather_part, sizeof(float) * (size_t)p->gather_pieces * (size_t)p->N * (size_t)k));
    p->k_cap = k;
    return RFX_OK;
}

int rfx_pv_plan_info(const rfx_pv_plan* p, int64_t* N, int32_t* B, int32_t* k_reserved) {
    if (!p) return rfx::fail(RFX_ERR_NULL, "rfx_pv_plan_info: plan is null");
    if (N) *N = p->N;
    if (B) *B = p->B;
    if (k_reserved) *k_reserved = p->k_cap;
    return RFX_OK;
}

int rfx_pv_apply(rfx_pv_plan* p, const float* V, int32_t k, float* Y, void* stream) {
    if (!p || !V || !Y) return rfx::fail(RFX_ERR_NULL, "rfx_pv_apply: null argument");
    if (k < 1 || k > 256) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_pv_apply: k=%d outside 1..256", k);
    if (V == Y) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_pv_apply: V and Y must not overlap");
    if (!p->built) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_pv_apply: the plan's last rebuild failed");
    hipStream_t st = rfx::as_stream(stream);
    if (k > p->k_cap) {
        int rc = rfx_pv_plan_reserve(p, k);
        if (rc != RFX_OK) return rc;
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
