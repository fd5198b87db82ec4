// Exact sparse proximity, row by row, from the samples grouped by leaf (paper, "CPU TriBlock Proximity": forests grown to
// purity put most pairs of samples in no common leaf, so only the pairs that do share one need work).
//
// cnt(i, j) = #{b : leaf_b(i) = leaf_b(j)}: for a sample i and a tree b the samples j that add 1 to cnt(i, j) are exactly
// the other members of i's leaf in b.  With the samples of every tree grouped by leaf and ascending inside a leaf (the
// grouping of the implicit product), the members j > i of i's leaf are the entries of `perm` that follow i's own entry up to
// the end of the segment.  Row i of the strict upper triangle is therefore sum over b of one short run of perm: in all
// sum_b sum_leaf s (s - 1) / 2 counter increments instead of N^2 B / 2 equality tests, a saving of two to three orders of
// magnitude on deep forests (N = 500,000, B = 1,000: 8e10 increments against 1.25e14 tests).
//
// One workgroup owns a row.  It walks the row's columns in chunks of kChunk: 16-bit counters of the chunk (two per 32-bit LDS
// word, B < 65,536) are cleared, every wave takes four of its trees at a time, reads the next members of the row's leaf in
// each (they are ascending, so the members inside the chunk are a prefix of what is left; a cursor per tree in LDS carries
// over to the next chunk, and a wave drops a tree from its list once the segment is used up), and counts them with LDS
// atomics; then the chunk's counters are compacted into (i, j, count) triplets behind a 64-bit cursor, one reservation per
// chunk.
#include <algorithm>

#include "common.h"
#include "prox_pv.h"

namespace {

#ifndef RFX_ROWS_CHUNK
#define RFX_ROWS_CHUNK 32768
#endif
constexpr int kChunk = RFX_ROWS_CHUNK;   // columns per pass: 16-bit LDS counters, two per word
constexpr int kRowThreads = 1024;        // 16 waves
constexpr int kRowWaves = kRowThreads / 64;
constexpr int kTreesPerWave = 4;         // member loads a wave keeps in flight
constexpr int kGroupTrees = 8;           // quarter-wave load instructions (four trees each) a wave keeps in flight
constexpr int kGroupLoads = 2;           // 16-member loads of a tree and chunk by a quarter wave before the wave-wide loads
constexpr int kNarrowLoads = 2;          // 64-member loads of a tree and chunk before the segment counts as long
constexpr uint32_t kDone = 0xffffffffu;  // cursor of a tree whose segment is used up
constexpr uint32_t kEndFlag = 0x80000000u;

// For every entry t of perm: marks the last entry of its segment (bit 31) and records, for the sample i = perm[t], where the
// members that follow it start: start[i][b] = t + 1, or kDone if i is the last of its leaf.
__global__ __launch_bounds__(256) void row_starts_kernel(uint32_t* __restrict__ perm, const uint32_t* __restrict__ slot,
                                                        const uint32_t* __restrict__ seg_start, int64_t N, int32_t B,
                                                        uint32_t* __restrict__ start) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)B * N) return;
    const int64_t b = t / N;
    const uint32_t i = perm[t];
    const uint32_t s = slot[b * N + i];
    const bool last = (uint32_t)(t + 1) == seg_start[s + 1];
    start[(int64_t)i * B + b] = last ? kDone : (uint32_t)(t + 1);
    if (last) perm[t] = i | kEndFlag;
}

// Takes the marks of row_starts_kernel out of perm again: the last entry of every segment that holds anything.
__global__ __launch_bounds__(256) void row_ends_clear_kernel(uint32_t* __restrict__ perm, const uint32_t* __restrict__ seg_start,
                                                            int64_t n_slots) {
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n_slots) return;
    const uint32_t lo = seg_start[s], hi = seg_start[s + 1];
    if (hi > lo) perm[hi - 1] &= ~kEndFlag;
}

// sum over all segments of len * (len - 1) / 2: the number of counter increments of the row pass
__global__ __launch_bounds__(256) void pair_work_kernel(const uint32_t* __restrict__ seg_start, int64_t n_slots,
                                                       unsigned long long* __restrict__ out) {
    unsigned long long acc = 0;
    for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s < n_slots; s += (int64_t)gridDim.x * blockDim.x) {
        const unsigned long long len = seg_start[s + 1] - seg_start[s];
        acc += len * (len - 1) / 2;  // len = 0: 0 * huge / 2 = 0
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0 && acc) atomicAdd(out, acc);
}

// Entries p + 4 * lane .. + 3 of the flagged member list as one 16-byte load (the address is 4-byte aligned only).  Lanes
// that would reach past the array read its last entry instead: that entry ends the last segment, so whatever follows it
// in a wave's 256 entries is never counted.
struct __attribute__((packed, aligned(4))) Members4 {
    uint32_t a, b, c, d;
};
__device__ __forceinline__ uint4 load_members(const uint32_t* __restrict__ permx, uint32_t p, int lane, uint32_t last_pos) {
    const uint64_t at = (uint64_t)p + 4u * (uint32_t)lane;
    if (at + 3 <= last_pos) {
        const Members4 m = *reinterpret_cast<const Members4*>(permx + at);
        return make_uint4(m.a, m.b, m.c, m.d);
    }
    const uint32_t tail = permx[last_pos];
    return make_uint4(at <= last_pos ? permx[at] : tail, at + 1 <= last_pos ? permx[at + 1] : tail,
                      at + 2 <= last_pos ? permx[at + 2] : tail, tail);
}

// Leaf sizes of a sample of trees (tree_step apart): hist[s][leaf] by global atomics (hist cleared beforehand).
__global__ __launch_bounds__(256) void sample_hist_kernel(const uint32_t* __restrict__ leaf, int64_t N, int32_t Lb, int32_t tree_step,
                                                         uint32_t* __restrict__ hist) {
    const int s = blockIdx.y;
    const uint32_t* row = leaf + (int64_t)s * tree_step * N;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t id = row[i];
        if (id < (uint32_t)Lb) atomicAdd(&hist[(int64_t)s * Lb + id], 1u);
    }
}
__global__ __launch_bounds__(256) void zero_u32_kernel(uint32_t* p, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}
// sum over the sampled leaves of len * (len - 1) / 2; hist has one more readable word after its n entries
__global__ __launch_bounds__(256) void hist_work_kernel(const uint32_t* __restrict__ hist, int64_t n, unsigned long long* __restrict__ out) {
    unsigned long long acc = 0;
    for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s < n; s += (int64_t)gridDim.x * blockDim.x) {
        const unsigned long long len = hist[s];
        acc += len * (len - 1) / 2;
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0 && acc) atomicAdd(out, acc);
}

struct RowOut {
    uint32_t* rows;
    uint32_t* cols;
    void* counts;
    float* prox;
    unsigned long long* cursor;
    unsigned long long capacity;
    uint32_t min_count;
    int32_t u16;
};

__global__ __launch_bounds__(kRowThreads, kChunk > 32768 ? 4 : 8) void sparse_rows_kernel(const uint32_t* __restrict__ permx,
                                                                    const uint32_t* __restrict__ start, int64_t N, int32_t B,
                                                                    RowOut out) {
    extern __shared__ uint32_t lds[];
    uint32_t* cnt = lds;                       // [kChunk / 2] two 16-bit counters per word
    uint32_t* cur = lds + kChunk / 2;          // [B] position in permx of the next member of the row's leaf, per tree
    uint32_t* act = cur + B;                   // [2][16][ceil(B / 16)] per wave: its trees that are not finished, and the long ones
    __shared__ uint32_t wave_tot[kRowWaves];
    __shared__ unsigned long long base_sh;
    // Rows are taken in the order of tree 0's grouping (the first N entries of the member list): samples that share a leaf
    // there share leaves in many other trees, so workgroups that run at the same time read the same segments and find them
    // in the caches.
    const int64_t i = permx[blockIdx.x] & ~kEndFlag;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t last_pos = (uint32_t)((int64_t)B * N - 1);
    const float Bf = (float)B;

    for (int b = threadIdx.x; b < B; b += kRowThreads) cur[b] = start[i * B + b];
    __syncthreads();
    // Wave w owns the trees w, w + 16, w + 32, ... for the whole row and keeps the list of those whose segment still has
    // members ahead; most trees put the row's sample in a small leaf and drop out after the first chunk.
    const int cap = (B + kRowWaves - 1) / kRowWaves;
    uint32_t* mine_act = act + wave * cap;
    uint32_t* mine_long = act + (kRowWaves + wave) * cap;  // its trees with many members left in the current chunk
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    int n_act = 0;
    auto compact_list = [&](bool first) {
        const int n_old = first ? (B - wave + kRowWaves - 1) / kRowWaves : n_act;
        int n_new = 0;
        for (int t0 = 0; t0 < n_old; t0 += 64) {
            const int t = t0 + lane;
            const uint32_t tree = t < n_old ? (first ? (uint32_t)(wave + kRowWaves * t) : mine_act[t]) : 0u;
            const bool alive = t < n_old && cur[tree] != kDone;
            const uint64_t m = __ballot(alive);
            if (alive) mine_act[n_new + __popcll(m & lt_mask)] = tree;  // at or before the slot it was read from
            n_new += __popcll(m);
        }
        n_act = n_new;
    };
    compact_list(true);
    const int64_t c0 = (i + 1) / kChunk, n_chunks = (N + kChunk - 1) / kChunk;
    for (int64_t c = c0; c < n_chunks; ++c) {
        for (int w = threadIdx.x; w < kChunk / 2; w += kRowThreads) cnt[w] = 0;
        if (!__syncthreads_or(n_act > 0)) break;  // no tree has members in the columns that are left
        const uint32_t col0 = (uint32_t)(c * kChunk);
        const uint32_t limit = (uint32_t)min((c + 1) * (int64_t)kChunk, N);
        // ---- count: kTreesPerWave trees of the wave's list per round, their first loads in flight together.  The first
        // loads of a tree bring 64 members each (most segments have fewer inside a chunk, and wider loads would mostly
        // fetch members of later chunks); a segment that fills kNarrowLoads of them is long, and from then on one load
        // brings 256 consecutive members (four per lane) and the next 256 are requested before the current ones are counted.
        //
        // Before that, every tree gets kGroupLoads loads of 16 members by a quarter of the wave (four trees per load
        // instruction, sixteen per round): in a deep forest a tree has some twenty members of a row's leaf inside a chunk,
        // and a 64-member load would fetch three times what it counts.  Only trees that fill those loads go on to the
        // wave-wide loads below.
        int n_long = 0;
        {
            const int g = lane >> 4, l = lane & 15;
            for (int t0 = 0; t0 < n_act; t0 += 4 * kGroupTrees) {
                // kGroupTrees load instructions (four trees each) in flight; tree and cursor are read again from LDS
                // when a load is consumed, which is cheaper than holding them in registers
                uint32_t v[kGroupTrees];
#pragma unroll
                for (int q = 0; q < kGroupTrees; ++q) {
                    const int t = t0 + 4 * q + g;
                    const uint32_t p0 = t < n_act ? cur[mine_act[t]] : kDone;
                    v[q] = permx[p0 == kDone ? 0u : min(p0 + (uint32_t)l, last_pos)];
                }
#pragma unroll
                for (int q = 0; q < kGroupTrees; ++q) {
                    const int t = t0 + 4 * q + g;
                    const uint32_t tree = t < n_act ? mine_act[t] : 0u;
                    const uint32_t p0 = t < n_act ? cur[tree] : kDone;
                    bool active = p0 != kDone, is_long = false;
                    uint32_t p = p0, val = v[q];
                    for (int step = 0; step < kGroupLoads; ++step) {
                        if (!__ballot(active)) break;  // wave-uniform
                        const uint32_t j = val & ~kEndFlag;
                        const uint64_t ends = __ballot(active && (val & kEndFlag));
                        const uint32_t e16 = (uint32_t)(ends >> (16 * g)) & 0xffffu;
                        const int end_l = e16 ? __ffs((int)e16) - 1 : 16;
                        const bool take = active && l <= end_l && j < limit;
                        if (take) atomicAdd(&cnt[(j - col0) >> 1], 1u << (16 * (j & 1u)));
                        const int n_take = __popc((uint32_t)(__ballot(take) >> (16 * g)) & 0xffffu);
                        if (active) {
                            if (n_take == end_l + 1) {  // the whole rest of the segment lay in this chunk
                                p = kDone;
                                active = false;
                            } else {
                                p += (uint32_t)n_take;
                                if (n_take < 16) active = false;  // stopped at the chunk's limit
                            }
                        }
                        if (step + 1 < kGroupLoads) {
                            if (active) val = permx[min(p + (uint32_t)l, last_pos)];
                        } else if (active) {
                            is_long = true;
                        }
                    }
                    if (p0 != kDone && l == 0) cur[tree] = p;
                    const uint64_t lm = __ballot(is_long && l == 0);
                    if (is_long && l == 0) mine_long[n_long + __popcll(lm & lt_mask)] = tree;
                    n_long += __popcll(lm);
                }
            }
        }
        for (int t0 = 0; t0 < n_long; t0 += kTreesPerWave) {
            uint32_t tree[kTreesPerWave], pos[kTreesPerWave], v[kTreesPerWave];
#pragma unroll
            for (int q = 0; q < kTreesPerWave; ++q) {
                // the same for all lanes; entries past the list's end repeat its last tree and are skipped below
                tree[q] = (uint32_t)__builtin_amdgcn_readfirstlane((int)mine_long[min(t0 + q, n_long - 1)]);
                pos[q] = t0 + q < n_long ? (uint32_t)__builtin_amdgcn_readfirstlane((int)cur[tree[q]]) : kDone;
            }
#pragma unroll
            for (int q = 0; q < kTreesPerWave; ++q) {
                // a finished tree reads a valid address and ignores the value
                const uint32_t at = pos[q] == kDone ? 0u : min(pos[q] + (uint32_t)lane, last_pos);
                v[q] = permx[at];
            }
#pragma unroll
            for (int q = 0; q < kTreesPerWave; ++q) {
                if (pos[q] == kDone) continue;  // wave-uniform
                uint32_t p = pos[q];
                // members are ascending and the segment ends at the first flagged entry: the entries to count are a prefix
                bool finished = false;
                uint32_t narrow = v[q];
                for (int step = 0; step < kNarrowLoads; ++step) {
                    const uint32_t j = narrow & ~kEndFlag;
                    const uint64_t ends = __ballot(narrow & kEndFlag);
                    const int end_lane = ends ? __ffsll((unsigned long long)ends) - 1 : 64;  // wave-uniform
                    const bool take = lane <= end_lane && j < limit;
                    if (take) atomicAdd(&cnt[(j - col0) >> 1], 1u << (16 * (j & 1u)));
                    const int n_take = __popcll(__ballot(take));
                    if (n_take == end_lane + 1) {  // the whole rest of the segment lay in this chunk
                        p = kDone;
                        finished = true;
                        break;
                    }
                    p += (uint32_t)n_take;
                    if (n_take < 64) {             // stopped at the chunk's limit
                        finished = true;
                        break;
                    }
                    if (step + 1 < kNarrowLoads) narrow = permx[min(p + (uint32_t)lane, last_pos)];
                }
                if (finished) {
                    if (lane == 0) cur[tree[q]] = p;
                    continue;
                }
                uint4 val = load_members(permx, p, lane, last_pos);
                uint4 nxt = load_members(permx, p + 256u, lane, last_pos);
                while (true) {
                    // entry 4 * lane + r of the 256 sits in component r of lane `lane`
                    const uint32_t e[4] = {val.x, val.y, val.z, val.w};
                    const uint32_t my_end = (e[0] & kEndFlag) ? 0u : (e[1] & kEndFlag) ? 1u : (e[2] & kEndFlag) ? 2u : (e[3] & kEndFlag) ? 3u : 4u;
                    const uint64_t ends = __ballot(my_end < 4u);
                    const int end_lane = ends ? __ffsll((unsigned long long)ends) - 1 : 64;           // wave-uniform
                    const uint32_t end_r = (uint32_t)__builtin_amdgcn_readlane((int)my_end, end_lane & 63);
                    const int end_pos = ends ? 4 * end_lane + (int)end_r : 256;                       // index of the last member
                    int n_take = 0;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const uint32_t j = e[r] & ~kEndFlag;
                        const bool take = 4 * lane + r <= end_pos && j < limit;
                        if (take) atomicAdd(&cnt[(j - col0) >> 1], 1u << (16 * (j & 1u)));
                        n_take += __popcll(__ballot(take));
                    }
                    if (n_take == end_pos + 1) {
                        p = kDone;
                        break;
                    }
                    p += (uint32_t)n_take;
                    if (n_take < 256) break;
                    val = nxt;
                    nxt = load_members(permx, p + 256u, lane, last_pos);
                }
                if (lane == 0) cur[tree[q]] = p;
            }
        }
        compact_list(false);
        __syncthreads();
        // ---- compact the chunk's counters into triplets
        constexpr int kWordsPerThread = kChunk / 2 / kRowThreads;
        uint32_t w[kWordsPerThread];
        uint32_t mine = 0;
#pragma unroll
        for (int u = 0; u < kWordsPerThread; ++u) {
            w[u] = cnt[u * kRowThreads + threadIdx.x];
            mine += ((w[u] & 0xffffu) >= out.min_count ? 1u : 0u) + ((w[u] >> 16) >= out.min_count ? 1u : 0u);
        }
        uint32_t incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int u = 0; u < kRowWaves; ++u) {
            before += u < wave ? wave_tot[u] : 0u;
            total += wave_tot[u];
        }
        if (total) {  // uniform over the workgroup
            if (threadIdx.x == 0) base_sh = atomicAdd(out.cursor, (unsigned long long)total);
            // The kept pairs are first packed into the counter array itself (every thread holds its words in registers
            // by now, and entry e of the chunk goes to word e: column offset in the upper, count in the lower half), so
            // that the list leaves as contiguous runs, one entry per thread and store, instead of every thread writing
            // a short run of its own.
            __syncthreads();
            const unsigned long long base = base_sh;
            if (base + total > out.capacity) {
                // counted, not stored
            } else if (total > (uint32_t)(kChunk / 2)) {
                // more kept pairs than the counter array has words (a row that shares leaves with most of the chunk):
                // every thread writes its own run
                unsigned long long at = base + before + incl - mine;
#pragma unroll
                for (int u = 0; u < kWordsPerThread; ++u) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const uint32_t c16 = h ? w[u] >> 16 : w[u] & 0xffffu;
                        if (c16 >= out.min_count) {
                            out.rows[at] = (uint32_t)i;
                            out.cols[at] = col0 + 2u * (uint32_t)(u * kRowThreads + threadIdx.x) + (uint32_t)h;
                            if (out.counts) {
                                if (out.u16)
                                    static_cast<uint16_t*>(out.counts)[at] = (uint16_t)c16;
                                else
                                    static_cast<uint32_t*>(out.counts)[at] = c16;
                            }
                            if (out.prox) out.prox[at] = (float)c16 / Bf;
                            ++at;
                        }
                    }
                }
            } else {
                uint32_t e = before + incl - mine;
#pragma unroll
                for (int u = 0; u < kWordsPerThread; ++u) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const uint32_t c16 = h ? w[u] >> 16 : w[u] & 0xffffu;
                        if (c16 >= out.min_count) cnt[e++] = ((2u * (uint32_t)(u * kRowThreads + threadIdx.x) + (uint32_t)h) << 16) | c16;
                    }
                }
                __syncthreads();
                for (uint32_t t = threadIdx.x; t < total; t += kRowThreads) {
                    const uint32_t x = cnt[t], c16 = x & 0xffffu;
                    const unsigned long long at = base + t;
                    out.rows[at] = (uint32_t)i;
                    out.cols[at] = col0 + (x >> 16);
                    if (out.counts) {
                        if (out.u16)
                            static_cast<uint16_t*>(out.counts)[at] = (uint16_t)c16;
                        else
                            static_cast<uint32_t*>(out.counts)[at] = c16;
                    }
                    if (out.prox) out.prox[at] = (float)c16 / Bf;
                }
            }
        }
        __syncthreads();  // the counters and base_sh are reused by the next chunk
    }
}

__global__ void zero_u64_kernel(unsigned long long* p) { *p = 0; }

}  // namespace

namespace rfx {

// Number of counter increments the row pass needs for this grouping (host value; waits for the stream).
int sparse_rows_work(const rfx_pv_plan* plan, unsigned long long* d_scratch, unsigned long long* increments, hipStream_t st) {
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, st, d_scratch);
    const int64_t n_slots = (int64_t)plan->B * plan->Lb;
    hipLaunchKernelGGL(pair_work_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(n_slots, 256), 4096)), dim3(256), 0, st,
                       plan->d_seg_start, n_slots, d_scratch);
    RFX_LAUNCH_CHECK("pair_work_kernel");
    RFX_HIP(hipMemcpyAsync(increments, d_scratch, sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
    RFX_HIP(hipStreamSynchronize(st));
    return RFX_OK;
}

// Which of the two ways of listing the non-zero pairs is expected to be faster for these leaf ids: the row pass (true)
// or the pair tests on bit planes (false).  Leaf sizes of 16 evenly spaced trees give the number of counter increments;
// the constants are the measured rates of the two kernels on an MI355X (row pass: 0.71 ps per increment and 68 ps per
// (row, column chunk, tree) visit, 80 ps per (tree, sample) for the grouping; tile pass: 78 % of 39.3 T lane-ops/s with
// (bits + 1) / 32 lane-ops per pair and tree).  The row pass must win by a fifth to be chosen.  Synchronous.
int sparse_rows_cheaper(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, hipStream_t st, bool* rows_cheaper) {
    *rows_cheaper = false;
    if (B > kSparseRowsMaxTrees || N < 4096 || (int64_t)B * N >= (1ll << 32) || (int64_t)B * leaf_bound >= (1ll << 32))
        return RFX_OK;
    const int S = std::min(B, 16), tree_step = B / S;
    DevBuf hist, total;
    RFX_HIP(hist.alloc(sizeof(uint32_t) * (size_t)S * leaf_bound));
    RFX_HIP(total.alloc(sizeof(unsigned long long)));
    const int64_t n = (int64_t)S * leaf_bound;
    hipLaunchKernelGGL(zero_u32_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(n, 256), 4096)), dim3(256), 0, st, hist.as<uint32_t>(), n);
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, st, total.as<unsigned long long>());
    hipLaunchKernelGGL(sample_hist_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(N, 256), 1024), S), dim3(256), 0, st, leaf, N,
                       leaf_bound, tree_step, hist.as<uint32_t>());
    hipLaunchKernelGGL(hist_work_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(n, 256), 4096)), dim3(256), 0, st,
                       hist.as<uint32_t>(), n, total.as<unsigned long long>());
    RFX_LAUNCH_CHECK("sample_hist_kernel");
    unsigned long long sampled = 0;
    RFX_HIP(hipMemcpyAsync(&sampled, total.p, sizeof(sampled), hipMemcpyDeviceToHost, st));
    RFX_HIP(hipStreamSynchronize(st));
    const double increments = (double)sampled * (double)B / (double)S;
    const double chunks = (double)ceil_div(N, kChunk);
    const double visits = (double)N * (chunks + 1.0) / 2.0 * (double)B;
    const double t_rows = 0.71e-12 * increments + 68e-12 * visits + 80e-12 * (double)B * (double)N;
    int bits = 1;
    while ((1 << bits) < leaf_bound) ++bits;
    bits = std::max(bits, 8);
    const double t_tiles = 0.5 * (double)N * (double)N * (double)B * (bits + 1) / 32.0 / (0.78 * 256 * 64 * 2.4e9);
    *rows_cheaper = t_rows < 0.8 * t_tiles;
    return RFX_OK;
}

// Enqueues the row pass on a grouping.  `start` is scratch of 4 B N bytes; the grouping's perm is flagged in place, so the
// plan cannot serve the implicit product afterwards.  *cursor must have been cleared.
int sparse_rows_enqueue(rfx_pv_plan* plan, uint32_t* start, int32_t min_count, int u16, int64_t capacity, uint32_t* rows,
                        uint32_t* cols, void* counts, float* prox, unsigned long long* cursor, hipStream_t st) {
    const int64_t N = plan->N;
    const int32_t B = plan->B;
    const int64_t total = (int64_t)B * N;
    plan->built = false;
    hipLaunchKernelGGL(row_starts_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, st, plan->d_perm, plan->d_slot,
                       plan->d_seg_start, N, B, start);
    RFX_LAUNCH_CHECK("row_starts_kernel");
    RowOut out{rows, cols, counts, prox, cursor, (unsigned long long)capacity, (uint32_t)min_count, u16};
    const size_t lds = sizeof(uint32_t) * ((size_t)kChunk / 2 + (size_t)B + 2 * (size_t)kRowWaves * ((B + kRowWaves - 1) / kRowWaves));
    RFX_HIP(hipFuncSetAttribute((const void*)sparse_rows_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    TimedLaunch timed("sparse_rows_kernel", st);
    hipLaunchKernelGGL(sparse_rows_kernel, dim3((unsigned)N), dim3(kRowThreads), lds, st, plan->d_perm, start, N, B, out);
    RFX_LAUNCH_CHECK("sparse_rows_kernel");
    return RFX_OK;
}

}  // namespace rfx

extern "C" int rfx_prox_sparse_plan_workspace_bytes(const rfx_pv_plan* plan, int64_t* bytes) {
    if (!plan || !bytes) return rfx::fail(RFX_ERR_NULL, "rfx_prox_sparse_plan_workspace_bytes: null argument");
    *bytes = (int64_t)((sizeof(uint32_t) * (size_t)plan->B * (size_t)plan->N + 255) / 256 * 256);
    return RFX_OK;
}

extern "C" int rfx_prox_sparse_plan(rfx_pv_plan* plan, int32_t min_count, int count_dtype, int64_t capacity, uint32_t* rows,
                                    uint32_t* cols, void* counts, float* prox, uint64_t* nnz, void* workspace,
                                    int64_t workspace_bytes, void* stream) {
    if (!plan || !nnz || !workspace) return rfx::fail(RFX_ERR_NULL, "rfx_prox_sparse_plan: null argument");
    if (!plan->built) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse_plan: the plan's last rebuild failed");
    if (count_dtype != RFX_U16 && count_dtype != RFX_U32)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse_plan: count_dtype=%d", count_dtype);
    if (min_count < 1) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse_plan: min_count=%d below 1", min_count);
    if (capacity < 0) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse_plan: capacity=%lld", (long long)capacity);
    if (capacity > 0 && (!rows || !cols)) return rfx::fail(RFX_ERR_NULL, "rfx_prox_sparse_plan: rows / cols are null");
    if (plan->B > rfx::kSparseRowsMaxTrees)
        return rfx::fail(RFX_ERR_UNSUPPORTED, "rfx_prox_sparse_plan: more than %d trees (use rfx_prox_sparse_ws)", rfx::kSparseRowsMaxTrees);
    if (plan->N >= (1ll << 31)) return rfx::fail(RFX_ERR_UNSUPPORTED, "rfx_prox_sparse_plan: N=%lld", (long long)plan->N);
    int64_t need = 0;
    (void)rfx_prox_sparse_plan_workspace_bytes(plan, &need);
    if (workspace_bytes < need)
        return rfx::fail(RFX_ERR_CAPACITY, "rfx_prox_sparse_plan: workspace of %lld bytes, %lld needed", (long long)workspace_bytes,
                         (long long)need);
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0 || reinterpret_cast<uintptr_t>(nnz) % 8 != 0)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse_plan: workspace must be 256-byte aligned, nnz 8-byte aligned");
    hipStream_t st = rfx::as_stream(stream);
    static_assert(sizeof(unsigned long long) == sizeof(uint64_t), "the pair counter is a 64-bit atomic");
    unsigned long long* cursor = reinterpret_cast<unsigned long long*>(nnz);
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, st, cursor);
    int rc = rfx::sparse_rows_enqueue(plan, static_cast<uint32_t*>(workspace), min_count, count_dtype == RFX_U16, capacity, rows, cols,
                                      counts, prox, cursor, st);
    // whatever happened, the marks come out of the member lists again, so the plan serves the implicit product as before
    const int64_t n_slots = (int64_t)plan->B * plan->Lb;
    hipLaunchKernelGGL(row_ends_clear_kernel, dim3((unsigned)rfx::ceil_div(n_slots, 256)), dim3(256), 0, st, plan->d_perm,
                       plan->d_seg_start, n_slots);
    if (rc != RFX_OK) return rc;
    RFX_LAUNCH_CHECK("row_ends_clear_kernel");
    plan->built = true;
    return RFX_OK;
}

extern "C" int rfx_prox_sparse_rows(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int32_t min_count,
                                    int count_dtype, int64_t capacity, uint32_t* rows, uint32_t* cols, void* counts,
                                    float* prox, int64_t* nnz, void* stream) {
    if (!leaf || !nnz) return rfx::fail(RFX_ERR_NULL, "rfx_prox_sparse_rows: null argument");
    if (N < 1 || N >= (1ll << 31) || B < 1 || leaf_bound < 1)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse_rows: N=%lld B=%d leaf_bound=%d", (long long)N, B, leaf_bound);
    if (count_dtype != RFX_U16 && count_dtype != RFX_U32)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse_rows: count_dtype=%d", count_dtype);
    if (min_count < 1) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse_rows: min_count=%d below 1", min_count);
    if (capacity < 0) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse_rows: capacity=%lld", (long long)capacity);
    if (capacity > 0 && (!rows || !cols)) return rfx::fail(RFX_ERR_NULL, "rfx_prox_sparse_rows: rows / cols are null");
    if (B > rfx::kSparseRowsMaxTrees)
        return rfx::fail(RFX_ERR_UNSUPPORTED, "rfx_prox_sparse_rows: more than %d trees (use rfx_prox_sparse)", rfx::kSparseRowsMaxTrees);
    hipStream_t st = rfx::as_stream(stream);
    rfx_pv_plan* plan = nullptr;
    int rc = rfx_pv_plan_create(leaf, N, B, leaf_bound, &plan, stream);
    if (rc != RFX_OK) return rc;
    struct PlanGuard {
        rfx_pv_plan* p;
        ~PlanGuard() { rfx_pv_plan_destroy(p); }
    } guard{plan};
    rfx::DevBuf start, cursor;
    RFX_HIP(start.alloc(sizeof(uint32_t) * (size_t)B * (size_t)N));
    RFX_HIP(cursor.alloc(sizeof(unsigned long long)));
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, st, cursor.as<unsigned long long>());
    rc = rfx::sparse_rows_enqueue(plan, start.as<uint32_t>(), min_count, count_dtype == RFX_U16, capacity, rows, cols, counts,
                                  prox, cursor.as<unsigned long long>(), st);
    unsigned long long total = 0;
    hipError_t e = hipSuccess;
    if (rc == RFX_OK) e = hipMemcpyAsync(&total, cursor.p, sizeof(total), hipMemcpyDeviceToHost, st);
    hipError_t e2 = hipStreamSynchronize(st);  // plan and scratch are released on return
    if (rc != RFX_OK) return rc;
    if (e != hipSuccess || e2 != hipSuccess)
        return rfx::fail(RFX_ERR_HIP, "rfx_prox_sparse_rows: %s", hipGetErrorString(e != hipSuccess ? e : e2));
    *nnz = (int64_t)total;
    if (total > (unsigned long long)capacity && capacity > 0)
        return rfx::fail(RFX_ERR_CAPACITY, "rfx_prox_sparse_rows: %llu pairs reach the threshold, capacity is %lld", total,
                         (long long)capacity);
    return RFX_OK;
}
