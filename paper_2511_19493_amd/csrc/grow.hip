// Forest growth on the GPU (paper, "GPU Tree Growth Strategies" / "Batched Multi-Tree Processing":
// trees of a batch are grown together; Methodology: bootstrap sample per tree, mtry random features
// per node, the split with the largest Gini decrease over the values present in the node, x <= tau
// goes left, growth until the nodes are pure).
//
// The trees of a batch advance level by level.  Per level, for all impure nodes of all trees at once:
//   1. every node draws its mtry features (counter-based generator keyed by tree and node number,
//      so the draws do not depend on the processing order);
//   2. for every (node, feature) pair the node's rows are copied as (order-preserving key of the
//      float value, row) pairs and every segment is sorted: bitonic networks for up to 4096 pairs,
//      rocPRIM's segmented radix sort (the one library primitive left in this file) for the longer
//      ones of the first levels;
//   3. one wave per segment sweeps its sorted rows 64 at a time, keeping the left-side class weights
//      as prefix sums, and scores every boundary between two different values;
//   4. the best boundary of a node is taken over its features; rows are split, children that hold
//      one class become leaves, the others form the next level.
// Split scores are compared exactly: maximising the Gini decrease is maximising
//   sum_c wL_c^2 / nL + sum_c wR_c^2 / nR = (A nR + C nL) / (nL nR)
// and two such fractions of integers are compared by cross-multiplication in 128 bits, so the trees
// do not depend on floating-point rounding or on the order of the rows inside a node.
// Nodes are numbered breadth first in creation order (children of the split nodes of a level, in
// node order), leaves 0..L-1 in node order.
#include <cstring>  // rocPRIM's host code calls memset

#include <rocprim/rocprim.hpp>

#include <algorithm>
#include <new>
#include <vector>

#include "common.h"

namespace {

typedef unsigned long long u64;

constexpr int kMaxClasses = 64;  // a lane holds the running weight of one class
constexpr int kMaxMtry = 64;

__host__ __device__ inline u64 mix(u64 z) {
    z += 0x9e3779b97f4a7c15ull;
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}
// counter-based draw: the output function of splitmix64 applied three times
__host__ __device__ inline u64 draw(u64 seed, u64 tree, u64 a, u64 b) {
    u64 h = mix(seed ^ ((tree + 1) * 0x9e3779b97f4a7c15ull));
    h = mix(h ^ a);
    return mix(h ^ b);
}
__host__ __device__ inline uint32_t bounded(u64 r, uint32_t n) { return (uint32_t)(((r >> 32) * (u64)n) >> 32); }

// unsigned key with the order of the float values; -0 and +0 get the same key
__device__ __forceinline__ uint32_t order_key(float x) {
    const uint32_t u = __float_as_uint(x + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// a * b > c * d, exactly
__device__ __forceinline__ bool prod_gt(u64 a, u64 b, u64 c, u64 d) {
    const u64 h1 = __umul64hi(a, b), l1 = a * b, h2 = __umul64hi(c, d), l2 = c * d;
    return h1 > h2 || (h1 == h2 && l1 > l2);
}
__device__ __forceinline__ bool prod_eq(u64 a, u64 b, u64 c, u64 d) {
    return __umul64hi(a, b) == __umul64hi(c, d) && a * b == c * d;
}

struct SegBest {
    u64 num;  // score = num / den
    u64 den;
    uint32_t pos;  // last row of the left side, as an index into the sorted segment
    uint32_t valid;
};

// impure nodes of the current level, ordered by (tree, node number)
struct Level {
    int32_t* tree;    // tree index inside the batch
    int32_t* node;    // node number inside the tree
    uint32_t* start;  // first row of the node in rows[]
    uint32_t* count;
    uint32_t* tot;    // [A][C] class weights
};

// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bootstrap_kernel(u64 seed, int32_t first_tree, int32_t Tb, int64_t N,
                                                       uint32_t* __restrict__ cnt) {
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= (int64_t)Tb * N) return;
    const int64_t tb = g / N, t = g - tb * N;
    atomicAdd(&cnt[tb * N + bounded(draw(seed, (u64)(first_tree + tb), 0, (u64)t), (uint32_t)N)], 1u);
}

// In-bag counts as uint16, a 0/1 flag per (tree, row) whose prefix sum places the in-bag rows, and the
// class weights of every root.  blockIdx.y is the tree, so a workgroup first adds its rows' weights
// up in LDS and then issues one global atomic per class.
__global__ __launch_bounds__(256) void inbag_kernel(const uint32_t* __restrict__ cnt, const int32_t* __restrict__ y, int64_t N,
                                                   int32_t C, uint16_t* __restrict__ inbag, uint32_t* __restrict__ flag,
                                                   uint32_t* __restrict__ root_tot) {
    __shared__ uint32_t hist[kMaxClasses];
    const int64_t tb = blockIdx.y;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (threadIdx.x < kMaxClasses) hist[threadIdx.x] = 0;
    __syncthreads();
    if (i < N) {
        const uint32_t c = cnt[tb * N + i];
        inbag[tb * N + i] = (uint16_t)c;
        flag[tb * N + i] = c ? 1u : 0u;
        if (c) atomicAdd(&hist[y[i]], c);
    }
    __syncthreads();
    if ((int)threadIdx.x < C && hist[threadIdx.x]) atomicAdd(&root_tot[tb * C + threadIdx.x], hist[threadIdx.x]);
}

__device__ __forceinline__ int32_t heaviest_class(const uint32_t* tot, int32_t C, int32_t* present) {
    int32_t top = 0, np = 0;
    for (int32_t c = 0; c < C; ++c) {
        np += tot[c] > 0;
        if (tot[c] > tot[top]) top = c;  // strict: the lowest class wins a tie
    }
    *present = np;
    return top;
}

// Level 0: a root that holds one class is a leaf, the others are the first level.  One thread.
__global__ void roots_kernel(int32_t Tb, int32_t C, int64_t N, int64_t cap, const uint32_t* __restrict__ pos,
                             const uint32_t* __restrict__ root_tot, Level lv, int32_t* __restrict__ root_active,
                             int32_t* __restrict__ nd_feature, int32_t* __restrict__ nd_class, int32_t* __restrict__ nd_depth,
                             int32_t* __restrict__ next_id, uint32_t* __restrict__ n_active) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    uint32_t A = 0;
    for (int32_t tb = 0; tb < Tb; ++tb) {
        int32_t present;
        const int32_t top = heaviest_class(root_tot + (int64_t)tb * C, C, &present);
        nd_depth[tb * cap] = 0;
        next_id[tb] = 1;
        if (present > 1) {
            lv.tree[A] = tb;
            lv.node[A] = 0;
            lv.start[A] = pos[(int64_t)tb * N];  // in-bag rows are placed in (tree, row) order
            lv.count[A] = pos[(int64_t)(tb + 1) * N] - pos[(int64_t)tb * N];
            for (int32_t c = 0; c < C; ++c) lv.tot[(int64_t)A * C + c] = root_tot[(int64_t)tb * C + c];
            root_active[tb] = (int32_t)A;
            ++A;
        } else {
            nd_feature[tb * cap] = -1;
            nd_class[tb * cap] = top;
            root_active[tb] = -1;
        }
    }
    *n_active = A;
}

__global__ __launch_bounds__(256) void fill_rows_kernel(const uint32_t* __restrict__ flag, const uint32_t* __restrict__ pos,
                                                       int32_t Tb, int64_t N, const int32_t* __restrict__ root_active,
                                                       uint32_t* __restrict__ rows, int32_t* __restrict__ row_node) {
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= (int64_t)Tb * N) return;
    const int64_t tb = g / N, i = g - tb * N;
    if (!flag[g]) return;
    const uint32_t e = pos[g];
    rows[e] = (uint32_t)i;
    row_node[e] = root_active[tb];
}

// The first mtry entries of a Fisher-Yates shuffle of 0..M-1, kept as the short list of entries that
// differ from the identity.  One thread per node.
__global__ __launch_bounds__(256) void draw_features_kernel(u64 seed, int32_t first_tree, uint32_t A, int32_t M, int32_t mtry,
                                                           Level lv, int32_t* __restrict__ seg_node,
                                                           int32_t* __restrict__ seg_feat, uint32_t* __restrict__ seg_begin,
                                                           uint32_t* __restrict__ seg_end, int32_t* __restrict__ node_first_seg,
                                                           int32_t* __restrict__ node_nseg) {
    const uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= A) return;
    int32_t idx[2 * kMaxMtry], val[2 * kMaxMtry];
    int n_sw = 0;
    auto get = [&](int32_t i) {
        for (int s = 0; s < n_sw; ++s)
            if (idx[s] == i) return val[s];
        return i;
    };
    auto set = [&](int32_t i, int32_t v) {
        for (int s = 0; s < n_sw; ++s)
            if (idx[s] == i) {
                val[s] = v;
                return;
            }
        idx[n_sw] = i;
        val[n_sw] = v;
        ++n_sw;
    };
    const u64 tree = (u64)(first_tree + lv.tree[a]);
    const u64 node = (u64)lv.node[a];
    const uint32_t st = lv.start[a], n = lv.count[a];
    for (int32_t q = 0; q < mtry; ++q) {
        const int32_t j = q + (int32_t)bounded(draw(seed, tree, 1 + node, (u64)q), (uint32_t)(M - q));
        const int32_t vq = get(q), vj = get(j);
        set(q, vj);
        set(j, vq);
        const int64_t s = (int64_t)a * mtry + q;
        seg_node[s] = (int32_t)a;
        seg_feat[s] = vj;
        seg_begin[s] = (uint32_t)mtry * st + (uint32_t)q * n;
        seg_end[s] = (uint32_t)mtry * st + (uint32_t)q * n + n;
    }
    node_first_seg[a] = (int32_t)(a * mtry);
    node_nseg[a] = mtry;
}

// (key, row) pairs of every segment of every node: thread (e, q) copies row e into the q-th segment
// of its node, if the node has one.
__global__ __launch_bounds__(256) void build_keys_kernel(const float* __restrict__ X, int32_t M, uint32_t S, int32_t max_nseg,
                                                        const uint32_t* __restrict__ rows, const int32_t* __restrict__ row_node,
                                                        Level lv, const int32_t* __restrict__ node_first_seg,
                                                        const int32_t* __restrict__ node_nseg,
                                                        const int32_t* __restrict__ seg_feat,
                                                        const uint32_t* __restrict__ seg_begin, uint32_t* __restrict__ keys,
                                                        uint32_t* __restrict__ vals) {
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= (int64_t)S * max_nseg) return;
    const uint32_t e = (uint32_t)(g % S);
    const int32_t q = (int32_t)(g / S);
    const int32_t a = row_node[e];
    if (a < 0 || q >= node_nseg[a]) return;
    const int32_t s = node_first_seg[a] + q;
    const uint32_t r = rows[e];
    const uint32_t dst = seg_begin[s] + (e - lv.start[a]);
    keys[dst] = order_key(X[(int64_t)r * M + seg_feat[s]]);
    vals[dst] = r;
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(v, off);
        if (lane >= off) v += t;
    }
    return v;
}
__device__ __forceinline__ u64 wave_incl_scan(u64 v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const u64 t = __shfl_up(v, off);
        if (lane >= off) v += t;
    }
    return v;
}

// One wave per sorted segment.  Lane c keeps the weight of class c on the left side so far (wl) and
// the node's total of class c (tot); a row finds the left weight of its own class as wl[own class]
// plus the weights of the same class on lower lanes of its tile.  With A = sum_c wl_c^2 and
// T = sum_c tot_c wl_c, moving a row of weight w and class c to the left adds 2 w wl_c + w^2 to A and
// w tot_c to T, and the right side's sum_c (tot_c - wl_c)^2 is S2 - 2 T + A.
constexpr int kEvalWaves = 4;
__global__ __launch_bounds__(64 * kEvalWaves) void eval_segments_kernel(
    uint32_t n_seg, int32_t C, int64_t N, const int32_t* __restrict__ seg_node, const uint32_t* __restrict__ seg_begin,
    Level lv, const uint32_t* __restrict__ keys, const uint32_t* __restrict__ vals, const int32_t* __restrict__ y,
    const uint16_t* __restrict__ inbag, SegBest* __restrict__ best_out) {
    const int lane = threadIdx.x & 63;
    const uint32_t seg = blockIdx.x * kEvalWaves + (threadIdx.x >> 6);
    if (seg >= n_seg) return;
    const int32_t a = seg_node[seg];
    const uint32_t n = lv.count[a];
    const uint32_t base = seg_begin[seg];
    const uint16_t* w_of = inbag + (int64_t)lv.tree[a] * N;
    const uint32_t tot = lane < C ? lv.tot[(int64_t)a * C + lane] : 0u;
    u64 s2 = (u64)tot * tot, n_tot64 = tot;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        s2 += __shfl_xor(s2, off);
        n_tot64 += __shfl_xor(n_tot64, off);
    }
    const uint32_t n_tot = (uint32_t)n_tot64;
    uint32_t wl = 0;             // lane c: left weight of class c before the current tile
    uint32_t nl_run = 0;         // uniform carries
    u64 a_run = 0, t_run = 0;
    u64 b_num = 0, b_den = 1;
    uint32_t b_pos = 0;
    bool have = false;
    for (uint32_t t0 = 0; t0 < n; t0 += 64) {
        const uint32_t p = t0 + lane;
        const bool in = p < n;
        const uint32_t key = in ? keys[base + p] : 0u;
        const uint32_t nxt = (p + 1 < n) ? keys[base + p + 1] : key;
        const uint32_t row = in ? vals[base + p] : 0u;
        const int32_t cls = in ? y[row] : 0;
        const uint32_t w = in ? (uint32_t)w_of[row] : 0u;
        // one prefix sum per class that occurs in the tile (deep nodes hold two or three classes, not all C)
        uint32_t own_prefix = 0, add = 0;
        u64 todo = __ballot(in);
        while (todo) {
            const int c = __shfl(cls, __ffsll((unsigned long long)todo) - 1);  // wave-uniform
            const bool mine = in && cls == c;
            const uint32_t v = mine ? w : 0u;
            const uint32_t incl = wave_incl_scan(v, lane);
            if (mine) own_prefix = incl - v;
            const uint32_t tile_tot = __shfl(incl, 63);
            if (lane == c) add = tile_tot;
            todo &= ~__ballot(mine);
        }
        const uint32_t wl_own = (uint32_t)__shfl((int)wl, cls) + own_prefix;
        const uint32_t tot_own = (uint32_t)__shfl((int)tot, cls);
        const u64 da = 2ull * w * wl_own + (u64)w * w;
        const u64 dt = (u64)w * tot_own;
        const uint32_t nl = nl_run + wave_incl_scan(w, lane);
        const u64 ai = a_run + wave_incl_scan(da, lane);
        const u64 ti = t_run + wave_incl_scan(dt, lane);
        if (in && p + 1 < n && nxt != key) {
            const u64 nr = n_tot - nl;
            const u64 right = s2 - 2ull * ti + ai;
            const u64 num = ai * nr + right * (u64)nl;
            const u64 den = (u64)nl * nr;
            if (!have || prod_gt(num, b_den, b_num, den)) {
                have = true;
                b_num = num;
                b_den = den;
                b_pos = p;
            }
        }
        wl += add;
        nl_run = __shfl(nl, 63);
        a_run = __shfl(ai, 63);
        t_run = __shfl(ti, 63);
    }
    // best over the lanes: larger score, then the smaller position
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const u64 o_num = __shfl_xor(b_num, off), o_den = __shfl_xor(b_den, off);
        const uint32_t o_pos = __shfl_xor(b_pos, off);
        const bool o_have = __shfl_xor((int)have, off) != 0;
        bool take = false;
        if (o_have) {
            if (!have)
                take = true;
            else if (prod_gt(o_num, b_den, b_num, o_den))
                take = true;
            else if (prod_eq(o_num, b_den, b_num, o_den) && o_pos < b_pos)
                take = true;
        }
        if (take) {
            have = true;
            b_num = o_num;
            b_den = o_den;
            b_pos = o_pos;
        }
    }
    if (lane == 0) best_out[seg] = SegBest{b_num, b_den, b_pos, have ? 1u : 0u};
}

// Best segment of every node, features in draw order, a later one only if strictly better.
__global__ __launch_bounds__(256) void choose_split_kernel(uint32_t A, int32_t mtry, int32_t M, const float* __restrict__ X,
                                                          const int32_t* __restrict__ seg_feat,
                                                          const uint32_t* __restrict__ seg_begin,
                                                          const SegBest* __restrict__ best, const uint32_t* __restrict__ keys,
                                                          const uint32_t* __restrict__ vals, int32_t* __restrict__ has_split,
                                                          int32_t* __restrict__ split_feat, uint32_t* __restrict__ split_key,
                                                          float* __restrict__ split_thr, uint32_t* __restrict__ n_unresolved) {
    const uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= A) return;
    int32_t bq = -1;
    u64 b_num = 0, b_den = 1;
    for (int32_t q = 0; q < mtry; ++q) {
        const SegBest b = best[(int64_t)a * mtry + q];
        if (b.valid && (bq < 0 || prod_gt(b.num, b_den, b_num, b.den))) {
            bq = q;
            b_num = b.num;
            b_den = b.den;
        }
    }
    if (bq < 0) {
        has_split[a] = 0;
        atomicAdd(n_unresolved, 1u);
        return;
    }
    const int64_t s = (int64_t)a * mtry + bq;
    const uint32_t at = seg_begin[s] + best[s].pos;
    has_split[a] = 1;
    split_feat[a] = seg_feat[s];
    split_key[a] = keys[at];
    split_thr[a] = X[(int64_t)vals[at] * M + seg_feat[s]] + 0.0f;
}

// Nodes whose drawn features are all constant try the features that were not drawn, in index
// order, one per round: this kernel gives every such node its next candidate and a segment.
__global__ __launch_bounds__(256) void fallback_pick_kernel(uint32_t A, int32_t M, int32_t mtry, Level lv,
                                                           const int32_t* __restrict__ has_split,
                                                           const int32_t* __restrict__ drawn_feat, int32_t* __restrict__ fb_next,
                                                           int32_t* __restrict__ seg_node, int32_t* __restrict__ seg_feat,
                                                           uint32_t* __restrict__ seg_begin, uint32_t* __restrict__ seg_end,
                                                           int32_t* __restrict__ node_first_seg, int32_t* __restrict__ node_nseg,
                                                           uint32_t* __restrict__ counters /* [0] segments, [1] elements */) {
    const uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= A) return;
    node_nseg[a] = 0;
    node_first_seg[a] = -1;
    if (has_split[a]) return;
    int32_t f = fb_next[a];
    for (; f < M; ++f) {
        bool drawn = false;
        for (int32_t q = 0; q < mtry; ++q) drawn |= drawn_feat[(int64_t)a * mtry + q] == f;
        if (!drawn) break;
    }
    fb_next[a] = f + 1;
    if (f >= M) return;  // every feature is constant in this node: it stays without a split
    const uint32_t slot = atomicAdd(&counters[0], 1u);
    const uint32_t at = atomicAdd(&counters[1], lv.count[a]);
    seg_node[slot] = (int32_t)a;
    seg_feat[slot] = f;
    seg_begin[slot] = at;
    seg_end[slot] = at + lv.count[a];
    node_first_seg[a] = (int32_t)slot;
    node_nseg[a] = 1;
}

__global__ __launch_bounds__(256) void fallback_choose_kernel(uint32_t n_seg, int32_t M, const float* __restrict__ X,
                                                             const int32_t* __restrict__ seg_node,
                                                             const int32_t* __restrict__ seg_feat,
                                                             const uint32_t* __restrict__ seg_begin,
                                                             const SegBest* __restrict__ best, const uint32_t* __restrict__ keys,
                                                             const uint32_t* __restrict__ vals, int32_t* __restrict__ has_split,
                                                             int32_t* __restrict__ split_feat, uint32_t* __restrict__ split_key,
                                                             float* __restrict__ split_thr, uint32_t* __restrict__ n_resolved) {
    const uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n_seg || !best[s].valid) return;
    const int32_t a = seg_node[s];
    const uint32_t at = seg_begin[s] + best[s].pos;
    has_split[a] = 1;
    split_feat[a] = seg_feat[s];
    split_key[a] = keys[at];
    split_thr[a] = X[(int64_t)vals[at] * M + seg_feat[s]] + 0.0f;
    atomicAdd(n_resolved, 1u);
}

// The rows of a split node are reordered inside the node's own range, left child first: a 0/1 flag
// per row (1 = goes left), its prefix sum over all rows, and a scatter.  Nothing here needs atomics,
// and the order of the rows stays ascending inside each child.
__global__ __launch_bounds__(256) void sides_kernel(const float* __restrict__ X, int32_t M, uint32_t S,
                                                   const uint32_t* __restrict__ rows, const int32_t* __restrict__ row_node,
                                                   const int32_t* __restrict__ has_split,
                                                   const int32_t* __restrict__ split_feat, const uint32_t* __restrict__ split_key,
                                                   uint32_t* __restrict__ goes_left) {
    const uint32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= S) return;
    const int32_t a = row_node[e];
    uint32_t l = 0;
    if (a >= 0 && has_split[a]) l = order_key(X[(int64_t)rows[e] * M + split_feat[a]]) <= split_key[a] ? 1u : 0u;
    goes_left[e] = l;
}

__global__ __launch_bounds__(256) void partition_kernel(uint32_t S, const uint32_t* __restrict__ rows,
                                                       const int32_t* __restrict__ row_node, Level lv,
                                                       const int32_t* __restrict__ has_split,
                                                       const uint32_t* __restrict__ goes_left,
                                                       const uint32_t* __restrict__ left_before, uint32_t* __restrict__ rows_tmp) {
    const uint32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= S) return;
    const int32_t a = row_node[e];
    if (a < 0 || !has_split[a]) return;
    const uint32_t st = lv.start[a];
    const uint32_t lb = left_before[e] - left_before[st];                  // left rows of the node before this one
    const uint32_t nl = left_before[st + lv.count[a]] - left_before[st];   // left rows of the node
    rows_tmp[goes_left[e] ? st + lb : st + nl + (e - st - lb)] = rows[e];
}

// class weights and row count of both children of every split node: one wave per child, lane c sums class c
__global__ __launch_bounds__(256) void child_stats_kernel(uint32_t A, int32_t C, int64_t N, Level lv,
                                                         const int32_t* __restrict__ has_split,
                                                         const uint32_t* __restrict__ left_before,
                                                         const uint32_t* __restrict__ rows_tmp, const int32_t* __restrict__ y,
                                                         const uint16_t* __restrict__ inbag, uint32_t* __restrict__ child_tot,
                                                         uint32_t* __restrict__ child_cnt) {
    const int lane = threadIdx.x & 63;
    const uint32_t ch = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (ch >= 2 * A) return;
    const uint32_t a = ch >> 1;
    if (!has_split[a]) return;
    const uint32_t st = lv.start[a], n = lv.count[a];
    const uint32_t nl = left_before[st + n] - left_before[st];
    const uint32_t lo = (ch & 1) ? st + nl : st, hi = (ch & 1) ? st + n : st + nl;
    const uint16_t* w_of = inbag + (int64_t)lv.tree[a] * N;
    uint32_t mine = 0;  // lane c: weight of class c
    for (uint32_t t0 = lo; t0 < hi; t0 += 64) {
        const uint32_t p = t0 + lane;
        const uint32_t r = p < hi ? rows_tmp[p] : 0u;
        const int32_t cls = p < hi ? y[r] : -1;
        const uint32_t w = p < hi ? (uint32_t)w_of[r] : 0u;
        u64 todo = __ballot(p < hi);
        while (todo) {  // the classes that occur in this tile
            const int c = __shfl(cls, __ffsll((unsigned long long)todo) - 1);
            uint32_t v = cls == c ? w : 0u;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
            if (lane == c) mine += v;
            todo &= ~__ballot(cls == c);
        }
    }
    if (lane < C) child_tot[(int64_t)ch * C + lane] = mine;
    if (lane == 0) child_cnt[ch] = hi - lo;
}

// per node: is it split, how many of its children go on to the next level, with how many rows
__global__ __launch_bounds__(256) void children_kernel(uint32_t A, int32_t C, const int32_t* __restrict__ has_split,
                                                      const uint32_t* __restrict__ child_tot,
                                                      const uint32_t* __restrict__ child_cnt, uint32_t* __restrict__ f_split,
                                                      uint32_t* __restrict__ f_active, uint32_t* __restrict__ f_rows) {
    const uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= A) return;
    uint32_t act = 0, nrows = 0;
    if (has_split[a]) {
        for (int s = 0; s < 2; ++s) {
            int32_t present;
            heaviest_class(child_tot + (2 * (int64_t)a + s) * C, C, &present);
            if (present > 1) {
                ++act;
                nrows += child_cnt[2 * (int64_t)a + s];
            }
        }
    }
    f_split[a] = has_split[a] ? 1u : 0u;
    f_active[a] = act;
    f_rows[a] = nrows;
}

__global__ __launch_bounds__(256) void tree_first_kernel(uint32_t A, const int32_t* __restrict__ an_tree,
                                                        uint32_t* __restrict__ tree_first) {
    const uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= A) return;
    if (a == 0 || an_tree[a - 1] != an_tree[a]) tree_first[an_tree[a]] = a;
}

// Writes the records of the level's nodes and of the children that are leaves, and the next level.
__global__ __launch_bounds__(256) void emit_kernel(uint32_t A, int32_t C, int64_t cap, int32_t level, Level lv, Level nx,
                                                  const int32_t* __restrict__ has_split, const int32_t* __restrict__ split_feat,
                                                  const float* __restrict__ split_thr, const uint32_t* __restrict__ child_tot,
                                                  const uint32_t* __restrict__ child_cnt, const uint32_t* __restrict__ x_split,
                                                  const uint32_t* __restrict__ x_active, const uint32_t* __restrict__ x_rows,
                                                  const uint32_t* __restrict__ tree_first, const int32_t* __restrict__ next_id,
                                                  int32_t* __restrict__ nd_feature, float* __restrict__ nd_thr,
                                                  int32_t* __restrict__ nd_left, int32_t* __restrict__ nd_right,
                                                  int32_t* __restrict__ nd_class, int32_t* __restrict__ nd_depth,
                                                  int32_t* __restrict__ child_dest, int32_t* __restrict__ child_next) {
    const uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= A) return;
    const int32_t tb = lv.tree[a];
    const int64_t at = (int64_t)tb * cap + lv.node[a];
    if (!has_split[a]) {
        // no feature takes two values here: an impure leaf
        int32_t present;
        nd_feature[at] = -1;
        nd_class[at] = heaviest_class(lv.tot + (int64_t)a * C, C, &present);
        child_dest[2 * (int64_t)a] = child_dest[2 * (int64_t)a + 1] = -1;
        return;
    }
    const int32_t left = next_id[tb] + 2 * (int32_t)(x_split[a] - x_split[tree_first[tb]]);
    nd_feature[at] = split_feat[a];
    nd_thr[at] = split_thr[a];
    nd_left[at] = left;
    nd_right[at] = left + 1;
    uint32_t na = x_active[a], ns = x_rows[a];
    for (int s = 0; s < 2; ++s) {
        const int64_t ch = 2 * (int64_t)a + s;
        const int64_t cat = (int64_t)tb * cap + left + s;
        nd_depth[cat] = level + 1;
        int32_t present;
        const int32_t top = heaviest_class(child_tot + ch * C, C, &present);
        if (present > 1) {
            nx.tree[na] = tb;
            nx.node[na] = left + s;
            nx.start[na] = ns;
            nx.count[na] = child_cnt[ch];
            for (int32_t c = 0; c < C; ++c) nx.tot[(int64_t)na * C + c] = child_tot[ch * C + c];
            child_dest[ch] = (int32_t)ns;
            child_next[ch] = (int32_t)na;
            ++na;
            ns += child_cnt[ch];
        } else {
            nd_feature[cat] = -1;
            nd_class[cat] = top;
            child_dest[ch] = -1;
        }
    }
}

__global__ __launch_bounds__(256) void advance_ids_kernel(uint32_t A, const int32_t* __restrict__ an_tree,
                                                         const uint32_t* __restrict__ x_split, const uint32_t* __restrict__ f_split,
                                                         const uint32_t* __restrict__ tree_first, int32_t* __restrict__ next_id) {
    const uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= A) return;
    if (a + 1 == A || an_tree[a + 1] != an_tree[a]) {
        const int32_t tb = an_tree[a];
        next_id[tb] += 2 * (int32_t)(x_split[a] + f_split[a] - x_split[tree_first[tb]]);
    }
}

// rows of the children that go on, moved to the next level's (dense) row array
__global__ __launch_bounds__(256) void compact_rows_kernel(uint32_t S, const uint32_t* __restrict__ rows_tmp,
                                                          const int32_t* __restrict__ row_node, Level lv,
                                                          const int32_t* __restrict__ has_split,
                                                          const uint32_t* __restrict__ left_before,
                                                          const int32_t* __restrict__ child_dest,
                                                          const int32_t* __restrict__ child_next, uint32_t* __restrict__ rows_next,
                                                          int32_t* __restrict__ row_node_next) {
    const uint32_t p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= S) return;
    const int32_t a = row_node[p];  // a node keeps its range of positions while its rows are reordered
    if (a < 0 || !has_split[a]) return;
    const uint32_t st = lv.start[a];
    const uint32_t nl = left_before[st + lv.count[a]] - left_before[st];
    const uint32_t s = (p - st < nl) ? 0u : 1u;
    const int64_t ch = 2 * (int64_t)a + s;
    const int32_t d = child_dest[ch];
    if (d < 0) return;
    const uint32_t q = (uint32_t)d + (s ? p - st - nl : p - st);
    rows_next[q] = rows_tmp[p];
    row_node_next[q] = child_next[ch];
}

// leaves numbered in node order: one wave per tree
__global__ __launch_bounds__(64) void leaf_ids_kernel(int64_t cap, const int32_t* __restrict__ n_nodes,
                                                     const int32_t* __restrict__ nd_feature, int32_t* __restrict__ nd_leaf_id,
                                                     int32_t* __restrict__ n_leaves) {
    const int tb = blockIdx.x, lane = threadIdx.x;
    const int32_t n = n_nodes[tb];
    int32_t run = 0;
    for (int32_t t0 = 0; t0 < n; t0 += 64) {
        const int32_t v = t0 + lane;
        const bool leaf = v < n && nd_feature[(int64_t)tb * cap + v] < 0;
        const u64 m = __ballot(leaf);
        if (v < n) nd_leaf_id[(int64_t)tb * cap + v] = leaf ? run + (int32_t)__builtin_popcountll(m & ((1ull << lane) - 1ull)) : -1;
        run += (int32_t)__builtin_popcountll(m);
    }
    if (lane == 0) n_leaves[tb] = run;
}

// the seven 4-byte fields of a node record (the threshold travels as its bit pattern)
struct NodeFields {
    const int32_t* f[7];
};

// [Tb][cap] per field -> the trees' first n_nodes records, tree after tree, field after field
__global__ __launch_bounds__(256) void pack_nodes_kernel(int64_t cap, const int64_t* __restrict__ off, int64_t n_batch,
                                                        NodeFields src, int32_t* __restrict__ packed) {
    const int64_t tb = blockIdx.y;
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= off[tb + 1] - off[tb]) return;
#pragma unroll
    for (int f = 0; f < 7; ++f) packed[(int64_t)f * n_batch + off[tb] + v] = src.f[f][tb * cap + v];
}

// scratch of the library primitives; it only grows, and before it is replaced the stream is drained
// because earlier work may still be using the old block
struct Scratch {
    rfx::DevBuf buf;
    size_t bytes = 0;
    hipError_t reserve(size_t need, hipStream_t st) {
        if (need <= bytes) return hipSuccess;
        hipError_t e = hipStreamSynchronize(st);
        if (e != hipSuccess) return e;
        e = buf.alloc(need + need / 4);
        bytes = e == hipSuccess ? need + need / 4 : 0;
        return e;
    }
};


// Exclusive prefix sum of n 32-bit values in three launches: totals of tiles of kScanTile values, the prefix of those
// totals by one workgroup, and the tiles again with their offsets.  A thread owns 16 consecutive values.
constexpr int kScanTile = 4096;

// exclusive prefix of v over the 256 threads of the workgroup (sm: 4 words); *total = sum over the workgroup
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* sm, uint32_t* total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = __shfl_up(inc, off);
        if (lane >= off) inc += up;
    }
    __syncthreads();  // sm may still be read by the previous call
    if (lane == 63) sm[w] = inc;
    __syncthreads();
    uint32_t before = 0;
    for (int u = 0; u < w; ++u) before += sm[u];
    *total = sm[0] + sm[1] + sm[2] + sm[3];
    return before + inc - v;
}

__global__ __launch_bounds__(256) void scan_tile_sums_kernel(const uint32_t* __restrict__ in, uint32_t n,
                                                            uint32_t* __restrict__ tile_sum) {
    __shared__ uint32_t sm[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + threadIdx.x * 16;
    uint32_t v = 0;
#pragma unroll
    for (int u = 0; u < 16; ++u)
        if (base + u < (int64_t)n) v += in[base + u];
    uint32_t total;
    (void)block_excl_scan(v, sm, &total);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void scan_tile_offsets_kernel(uint32_t* __restrict__ tile_sum, uint32_t n_tiles) {
    __shared__ uint32_t sm[4];
    uint32_t carry = 0;
    for (uint32_t t0 = 0; t0 < n_tiles; t0 += 256 * 16) {
        const uint32_t base = t0 + threadIdx.x * 16;
        uint32_t x[16];
        uint32_t v = 0;
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            x[u] = base + u < n_tiles ? tile_sum[base + u] : 0u;
            v += x[u];
        }
        uint32_t total;
        uint32_t run = carry + block_excl_scan(v, sm, &total);
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            if (base + u < n_tiles) tile_sum[base + u] = run;
            run += x[u];
        }
        carry += total;
    }
}

__global__ __launch_bounds__(256) void scan_tiles_kernel(const uint32_t* __restrict__ in, uint32_t n,
                                                        const uint32_t* __restrict__ tile_off, uint32_t* __restrict__ out) {
    __shared__ uint32_t sm[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + threadIdx.x * 16;
    uint32_t x[16];
    uint32_t v = 0;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        x[u] = base + u < (int64_t)n ? in[base + u] : 0u;
        v += x[u];
    }
    uint32_t total;
    uint32_t run = tile_off[blockIdx.x] + block_excl_scan(v, sm, &total);
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        if (base + u < (int64_t)n) out[base + u] = run;
        run += x[u];
    }
}

int scan_u32(Scratch& tmp, const uint32_t* in, uint32_t* out, uint32_t n, hipStream_t st) {
    if (n == 0) return RFX_OK;
    const uint32_t n_tiles = (uint32_t)(((uint64_t)n + kScanTile - 1) / kScanTile);
    RFX_HIP(tmp.reserve(sizeof(uint32_t) * (size_t)n_tiles, st));
    uint32_t* tile_sum = static_cast<uint32_t*>(tmp.buf.p);
    hipLaunchKernelGGL(scan_tile_sums_kernel, dim3(n_tiles), dim3(256), 0, st, in, n, tile_sum);
    hipLaunchKernelGGL(scan_tile_offsets_kernel, dim3(1), dim3(256), 0, st, tile_sum, n_tiles);
    hipLaunchKernelGGL(scan_tiles_kernel, dim3(n_tiles), dim3(256), 0, st, in, n, tile_sum, out);
    RFX_LAUNCH_CHECK("scan_tiles_kernel");
    return RFX_OK;
}

// ---------------------------------------------------------------------------------------------
// Segmented sort of the (key, row) pairs.  After the first few levels almost every segment is short (the nodes of a
// level are many and small).  All sizes up to kSortBlockMax go through bitonic networks on the 64-bit value
// key << 32 | row (the rows of a segment are distinct and arrive ascending, so this is the order a stable sort by key
// gives): up to 16 pairs in a quarter wave, up to 64 in a wave, up to kSortBlockMax in a workgroup that keeps up to 16
// pairs per thread in registers and exchanges through LDS only at distances of a wave or more.  Only the few long
// segments of the top levels are left to the library's radix sort.
constexpr int kSortBlockMax = 4096;
constexpr int kSortWaveMax = 256;   // up to here a single wave sorts the segment, four pairs per lane

__device__ __forceinline__ u64 shfl_xor_u64(u64 x, int m) {
    const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)x, m), hi = (uint32_t)__shfl_xor((int)(uint32_t)(x >> 32), m);
    return ((u64)hi << 32) | lo;
}

// compare-exchange with the lane at distance j; this lane keeps the smaller value if keep_min
__device__ __forceinline__ u64 exchange_step(u64 x, int j, bool keep_min) {
    const u64 other = shfl_xor_u64(x, j);
    return (x < other) == keep_min ? x : other;
}

// Four segments per wave, one per quarter.  A quarter sorts a segment of up to 16 pairs by itself; segments of 17 .. 64
// pairs are then taken one after the other by the whole wave; longer ones are appended to the list of medium segments
// (those a wave can take from the front of the list, those for a workgroup from its back) or to the begin / end arrays of the
// long ones.  counts[0] = medium for a wave, counts[3] = medium for a workgroup, counts[1] = long segments.
__global__ __launch_bounds__(256) void sort_short_segments_kernel(uint32_t n_seg, const uint32_t* __restrict__ seg_begin,
                                                                 const uint32_t* __restrict__ seg_end,
                                                                 const uint32_t* keys_in, const uint32_t* vals_in, uint32_t* keys_out, uint32_t* vals_out,
                                                                 uint32_t* __restrict__ medium, uint32_t medium_cap,
                                                                 uint32_t* __restrict__ long_begin,
                                                                 uint32_t* __restrict__ long_end, uint32_t* __restrict__ counts) {
    const int lane = threadIdx.x & 63, gl = lane & 15;
    const uint32_t seg = ((blockIdx.x * 4 + (threadIdx.x >> 6)) << 2) + (lane >> 4);
    const bool valid = seg < n_seg;
    const uint32_t b = valid ? seg_begin[seg] : 0u, len = valid ? seg_end[seg] - b : 0u;
    {
        const bool mine = (uint32_t)gl < len && len <= 16;
        u64 x = ~0ull;
        if (mine) x = ((u64)keys_in[b + gl] << 32) | vals_in[b + gl];
#pragma unroll
        for (int k = 2; k <= 16; k <<= 1) {
#pragma unroll
            for (int j = k >> 1; j > 0; j >>= 1) x = exchange_step(x, j, ((gl & j) == 0) == ((gl & k) == 0));
        }
        if (mine) {
            keys_out[b + gl] = (uint32_t)(x >> 32);
            vals_out[b + gl] = (uint32_t)x;
        }
    }
    if (gl == 0 && len > 64) {
        if (len <= (uint32_t)kSortWaveMax) {
            medium[atomicAdd(&counts[0], 1u)] = seg;                       // from the front: one wave each
        } else if (len <= (uint32_t)kSortBlockMax) {
            medium[medium_cap - 1u - atomicAdd(&counts[3], 1u)] = seg;     // from the back: one workgroup each
        } else {
            const uint32_t at = atomicAdd(&counts[1], 1u);
            long_begin[at] = b;
            long_end[at] = b + len;
        }
    }
    u64 todo = __ballot(gl == 0 && len > 16 && len <= 64);
    while (todo) {
        const int src = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        const uint32_t wb = (uint32_t)__shfl((int)b, src), wl = (uint32_t)__shfl((int)len, src);
        u64 x = ~0ull;
        if ((uint32_t)lane < wl) x = ((u64)keys_in[wb + lane] << 32) | vals_in[wb + lane];
#pragma unroll
        for (int k = 2; k <= 64; k <<= 1) {
#pragma unroll
            for (int j = k >> 1; j > 0; j >>= 1) x = exchange_step(x, j, ((lane & j) == 0) == ((lane & k) == 0));
        }
        if ((uint32_t)lane < wl) {
            keys_out[wb + lane] = (uint32_t)(x >> 32);
            vals_out[wb + lane] = (uint32_t)x;
        }
    }
}

// Bitonic sort of T E values over T threads (a wave, or a workgroup of 256): thread t holds the values at positions
// t E .. t E + E - 1.  Steps at distances below E stay in the thread's registers, distances below 64 E are lane exchanges,
// the rest (workgroup only) goes through LDS, laid out [r][t] so that consecutive lanes touch consecutive words.
template <int E, int T>
__device__ __forceinline__ void sort_block(u64 (&x)[E], u64* sm, int t) {
#pragma unroll
    for (int k = 2; k < E; k <<= 1) {  // direction fixed by the position inside the thread
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
#pragma unroll
            for (int r = 0; r < E; ++r) {
                if ((r & j) == 0) {
                    const u64 a = x[r], c = x[r | j];
                    const bool sw = (a > c) == ((r & k) == 0);
                    x[r] = sw ? c : a;
                    x[r | j] = sw ? a : c;
                }
            }
        }
    }
    for (int k = (E > 1 ? E : 2); k <= T * E; k <<= 1) {
        const bool asc = ((t * E) & k) == 0;
        for (int j = k >> 1; j >= E; j >>= 1) {
            const int d = j / E;
            const bool keep_min = ((t & d) == 0) == asc;
            if (T <= 64 || d < 64) {
#pragma unroll
                for (int r = 0; r < E; ++r) x[r] = exchange_step(x[r], d, keep_min);
            } else {
#pragma unroll
                for (int r = 0; r < E; ++r) sm[r * T + t] = x[r];
                __syncthreads();
#pragma unroll
                for (int r = 0; r < E; ++r) {
                    const u64 other = sm[r * T + (t ^ d)];
                    x[r] = (x[r] < other) == keep_min ? x[r] : other;
                }
                __syncthreads();
            }
        }
#pragma unroll
        for (int j = E >> 1; j > 0; j >>= 1) {
#pragma unroll
            for (int r = 0; r < E; ++r) {
                if ((r & j) == 0) {
                    const u64 a = x[r], c = x[r | j];
                    const bool sw = (a > c) == asc;
                    x[r] = sw ? c : a;
                    x[r | j] = sw ? a : c;
                }
            }
        }
    }
}

// One wave per listed segment of 65 .. kSortWaveMax pairs, four segments per workgroup.
__global__ __launch_bounds__(256) void sort_wave_segments_kernel(const uint32_t* __restrict__ medium, uint32_t n_listed,
                                                                const uint32_t* __restrict__ seg_begin,
                                                                const uint32_t* __restrict__ seg_end, const uint32_t* keys_in,
                                                                const uint32_t* vals_in, uint32_t* keys_out, uint32_t* vals_out) {
    constexpr int E = kSortWaveMax / 64;
    const int lane = threadIdx.x & 63;
    const uint32_t at = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (at >= n_listed) return;
    const uint32_t seg = medium[at];
    const uint32_t b = seg_begin[seg], len = seg_end[seg] - b;
    u64 x[E];
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const uint32_t i = (uint32_t)(r * 64 + lane);
        x[r] = i < len ? ((u64)keys_in[b + i] << 32) | vals_in[b + i] : ~0ull;
    }
    sort_block<E, 64>(x, nullptr, lane);
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const uint32_t i = (uint32_t)(lane * E + r);
        if (i < len) {
            keys_out[b + i] = (uint32_t)(x[r] >> 32);
            vals_out[b + i] = (uint32_t)x[r];
        }
    }
}

template <int E>
__device__ __forceinline__ void sort_medium_segment(uint32_t b, uint32_t len, const uint32_t* keys_in, const uint32_t* vals_in,
                                                    uint32_t* keys_out, uint32_t* vals_out, u64* sm) {
    const int t = threadIdx.x;
    u64 x[E];
#pragma unroll
    for (int r = 0; r < E; ++r) {  // where a value starts does not matter: read coalesced
        const uint32_t i = (uint32_t)(r * 256 + t);
        x[r] = i < len ? ((u64)keys_in[b + i] << 32) | vals_in[b + i] : ~0ull;
    }
    sort_block<E, 256>(x, sm, t);
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const uint32_t i = (uint32_t)(t * E + r);
        if (i < len) {
            keys_out[b + i] = (uint32_t)(x[r] >> 32);
            vals_out[b + i] = (uint32_t)x[r];
        }
    }
}

// One workgroup per listed segment of 65 .. kSortBlockMax pairs.
__global__ __launch_bounds__(256) void sort_medium_segments_kernel(const uint32_t* __restrict__ medium,
                                                                  const uint32_t* __restrict__ seg_begin,
                                                                  const uint32_t* __restrict__ seg_end,
                                                                  const uint32_t* keys_in, const uint32_t* vals_in, uint32_t* keys_out,
                                                                  uint32_t* vals_out) {
    __shared__ u64 sm[kSortBlockMax];
    const uint32_t seg = medium[blockIdx.x];  // (the caller passes the end of the list that holds the workgroup-sized ones)
    const uint32_t b = seg_begin[seg], len = seg_end[seg] - b;
    if (len <= 512) sort_medium_segment<2>(b, len, keys_in, vals_in, keys_out, vals_out, sm);
    else if (len <= 1024) sort_medium_segment<4>(b, len, keys_in, vals_in, keys_out, vals_out, sm);
    else if (len <= 2048) sort_medium_segment<8>(b, len, keys_in, vals_in, keys_out, vals_out, sm);
    else sort_medium_segment<16>(b, len, keys_in, vals_in, keys_out, vals_out, sm);
}

__global__ __launch_bounds__(256) void zero_u32_kernel(uint32_t* __restrict__ p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0;
}

// Lists of the segmented sort: ids of the medium segments (those for a wave from the front, those for a workgroup from the
// back), begin / end of the long ones, and the counters ([0] medium for a wave, [1] long, [3] medium for a workgroup).
struct SortLists {
    rfx::DevBuf buf;
    size_t cap = 0;
    uint32_t *medium = nullptr, *long_begin = nullptr, *long_end = nullptr, *counts = nullptr;
    hipError_t reserve(size_t n, hipStream_t st) {
        if (n > cap) {
            hipError_t e = hipStreamSynchronize(st);
            if (e != hipSuccess) return e;
            cap = 0;
            const size_t c = n + n / 4 + 64;
            e = buf.alloc(sizeof(uint32_t) * (3 * c + 64));
            if (e != hipSuccess) return e;
            cap = c;
        }
        medium = buf.as<uint32_t>();
        long_begin = medium + cap;
        long_end = long_begin + cap;
        counts = long_end + cap;
        return hipSuccess;
    }
};

// Every segment up to kSortBlockMax pairs by the networks; the long ones, listed by the first kernel, by the library's
// segmented radix sort (stable, and the rows arrive ascending, so equal keys keep ascending rows there too).
int sort_segments(Scratch& tmp, const uint32_t* keys_in, uint32_t* keys_out, const uint32_t* vals_in, uint32_t* vals_out,
                  uint32_t size, uint32_t n_seg, const uint32_t* seg_begin, const uint32_t* seg_end, SortLists& r,
                  hipStream_t st) {
    if (n_seg == 0) return RFX_OK;
    RFX_HIP(r.reserve(n_seg, st));
    hipLaunchKernelGGL(zero_u32_kernel, dim3(1), dim3(64), 0, st, r.counts, (size_t)4);
    hipLaunchKernelGGL(sort_short_segments_kernel, dim3((n_seg + 15) / 16), dim3(256), 0, st, n_seg, seg_begin, seg_end, keys_in,
                       vals_in, keys_out, vals_out, r.medium, (uint32_t)r.cap, r.long_begin, r.long_end, r.counts);
    RFX_LAUNCH_CHECK("sort_short_segments_kernel");
    uint32_t h[4];
    RFX_HIP(hipMemcpyAsync(h, r.counts, sizeof(h), hipMemcpyDeviceToHost, st));
    RFX_HIP(hipStreamSynchronize(st));
    if (h[0] > 0) {
        hipLaunchKernelGGL(sort_wave_segments_kernel, dim3((h[0] + 3) / 4), dim3(256), 0, st, r.medium, h[0], seg_begin, seg_end,
                           keys_in, vals_in, keys_out, vals_out);
        RFX_LAUNCH_CHECK("sort_wave_segments_kernel");
    }
    if (h[3] > 0) {
        hipLaunchKernelGGL(sort_medium_segments_kernel, dim3(h[3]), dim3(256), 0, st, r.medium + (r.cap - h[3]), seg_begin, seg_end,
                           keys_in, vals_in, keys_out, vals_out);
        RFX_LAUNCH_CHECK("sort_medium_segments_kernel");
    }
    if (h[1] > 0) {
        size_t need = 0;
        RFX_HIP(rocprim::segmented_radix_sort_pairs(nullptr, need, keys_in, keys_out, vals_in, vals_out, size, h[1], r.long_begin,
                                                    r.long_end, 0, 32, st));
        RFX_HIP(tmp.reserve(need, st));
        RFX_HIP(rocprim::segmented_radix_sort_pairs(tmp.buf.p, need, keys_in, keys_out, vals_in, vals_out, size, h[1], r.long_begin,
                                                    r.long_end, 0, 32, st));
    }
    return RFX_OK;
}

inline dim3 blocks_for(int64_t n, int per = 256) { return dim3((unsigned)std::max<int64_t>(1, rfx::ceil_div(n, per))); }

}  // namespace

// the grown forest, on the host, in the layout rfx_forest_desc takes
struct rfx_grown {
    int32_t n_trees = 0, n_features = 0, n_classes = 0;
    int64_t N = 0;
    std::vector<int64_t> node_offset;
    std::vector<int32_t> feature, left, right, leaf_id, depth, node_class, n_leaves;
    std::vector<float> threshold;
    std::vector<uint16_t> inbag;
    int32_t levels = 0;        // level passes of the deepest batch
    int64_t sorted_pairs = 0;  // (row, feature) pairs sorted and scored over all levels and batches
};

namespace {

template <class T>
hipError_t alloc_n(rfx::DevBuf& b, size_t n) {
    return b.alloc(sizeof(T) * std::max<size_t>(n, 1));
}

// Grows trees [first, first + Tb) and appends them to g.
int grow_batch(rfx_grown& g, const float* X, const int32_t* y, int64_t N, int32_t M, int32_t C, int32_t first, int32_t Tb,
               int32_t mtry, u64 seed, hipStream_t st) {
    const int64_t cap = 2 * N;  // node numbers of a tree stay below twice its number of in-bag rows
    const int64_t TN = (int64_t)Tb * N;
    rfx::DevBuf cnt32, inbag, ib_flag, ib_pos, root_tot, root_active, next_id, counters;
    Scratch tmp;
    SortLists sort_lists;
    RFX_HIP(alloc_n<uint32_t>(cnt32, TN));
    RFX_HIP(alloc_n<uint16_t>(inbag, TN));
    RFX_HIP(alloc_n<uint32_t>(ib_flag, TN + 1));
    RFX_HIP(alloc_n<uint32_t>(ib_pos, TN + 1));
    RFX_HIP(alloc_n<uint32_t>(root_tot, (size_t)Tb * C));
    RFX_HIP(alloc_n<int32_t>(root_active, Tb));
    RFX_HIP(alloc_n<int32_t>(next_id, Tb));
    RFX_HIP(alloc_n<uint32_t>(counters, 8));
    RFX_HIP(hipMemsetAsync(cnt32.p, 0, sizeof(uint32_t) * TN, st));
    RFX_HIP(hipMemsetAsync(root_tot.p, 0, sizeof(uint32_t) * Tb * C, st));
    hipLaunchKernelGGL(bootstrap_kernel, blocks_for(TN), dim3(256), 0, st, seed, first, Tb, N, cnt32.as<uint32_t>());
    hipLaunchKernelGGL(inbag_kernel, dim3((unsigned)rfx::ceil_div(N, 256), (unsigned)Tb), dim3(256), 0, st, cnt32.as<uint32_t>(), y, N,
                       C, inbag.as<uint16_t>(), ib_flag.as<uint32_t>(), root_tot.as<uint32_t>());
    RFX_LAUNCH_CHECK("bootstrap kernels");
    // position of every in-bag (tree, row) pair among all of them: the rows of the roots, tree after tree
    int rc0 = scan_u32(tmp, ib_flag.as<uint32_t>(), ib_pos.as<uint32_t>(), (uint32_t)(TN + 1), st);
    if (rc0 != RFX_OK) return rc0;
    uint32_t s0 = 0;
    RFX_HIP(hipMemcpyAsync(&s0, ib_pos.as<uint32_t>() + TN, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    RFX_HIP(hipStreamSynchronize(st));
    const uint64_t S0 = s0;
    if (S0 * (uint64_t)std::max(mtry, 1) >= (1ull << 31)) return rfx::fail(RFX_ERR_INVALID_ARG, "forest growth: batch too large");

    // node records of the batch: [Tb][cap]
    rfx::DevBuf nd_feature, nd_thr, nd_left, nd_right, nd_class, nd_depth, nd_leaf;
    const size_t n_rec = (size_t)Tb * (size_t)cap;
    RFX_HIP(alloc_n<int32_t>(nd_feature, n_rec));
    RFX_HIP(alloc_n<float>(nd_thr, n_rec));
    RFX_HIP(alloc_n<int32_t>(nd_left, n_rec));
    RFX_HIP(alloc_n<int32_t>(nd_right, n_rec));
    RFX_HIP(alloc_n<int32_t>(nd_class, n_rec));
    RFX_HIP(alloc_n<int32_t>(nd_depth, n_rec));
    RFX_HIP(alloc_n<int32_t>(nd_leaf, n_rec));
    RFX_HIP(hipMemsetAsync(nd_thr.p, 0, sizeof(float) * n_rec, st));
    RFX_HIP(hipMemsetAsync(nd_left.p, 0xff, sizeof(int32_t) * n_rec, st));   // -1
    RFX_HIP(hipMemsetAsync(nd_right.p, 0xff, sizeof(int32_t) * n_rec, st));  // -1
    RFX_HIP(hipMemsetAsync(nd_class.p, 0xff, sizeof(int32_t) * n_rec, st));  // -1

    // rows of the impure nodes (two buffers), per-level node tables (two sets), per-level scratch
    const size_t S_max = (size_t)S0, A_max = (size_t)S0 / 2 + 1;  // an impure node holds at least two rows
    rfx::DevBuf rows[2], row_node[2], lv_tree[2], lv_node[2], lv_start[2], lv_count[2], lv_tot[2];
    for (int i = 0; i < 2; ++i) {
        RFX_HIP(alloc_n<uint32_t>(rows[i], S_max));
        RFX_HIP(alloc_n<int32_t>(row_node[i], S_max));
        RFX_HIP(alloc_n<int32_t>(lv_tree[i], A_max));
        RFX_HIP(alloc_n<int32_t>(lv_node[i], A_max));
        RFX_HIP(alloc_n<uint32_t>(lv_start[i], A_max));
        RFX_HIP(alloc_n<uint32_t>(lv_count[i], A_max));
        RFX_HIP(alloc_n<uint32_t>(lv_tot[i], A_max * C));
    }
    auto level_of = [&](int i) {
        return Level{lv_tree[i].as<int32_t>(), lv_node[i].as<int32_t>(), lv_start[i].as<uint32_t>(), lv_count[i].as<uint32_t>(),
                     lv_tot[i].as<uint32_t>()};
    };
    const size_t K_max = S_max * (size_t)mtry, G_max = A_max * (size_t)mtry;
    rfx::DevBuf keys[2], vals[2], seg_node, seg_feat, seg_begin, seg_end, node_first_seg, node_nseg, best, has_split, split_feat,
        split_key, split_thr, fb_next, fb_seg_node, fb_seg_feat, fb_seg_begin, fb_seg_end, fb_best, rows_tmp, goes_left,
        left_before, child_tot, child_cnt, child_dest, child_next, f_split, f_active, f_rows, x_split, x_active, x_rows, tree_first;
    for (int i = 0; i < 2; ++i) {
        RFX_HIP(alloc_n<uint32_t>(keys[i], K_max));
        RFX_HIP(alloc_n<uint32_t>(vals[i], K_max));
    }
    RFX_HIP(alloc_n<int32_t>(seg_node, G_max));
    RFX_HIP(alloc_n<int32_t>(seg_feat, G_max));
    RFX_HIP(alloc_n<uint32_t>(seg_begin, G_max));
    RFX_HIP(alloc_n<uint32_t>(seg_end, G_max));
    RFX_HIP(alloc_n<SegBest>(best, G_max));
    RFX_HIP(alloc_n<int32_t>(node_first_seg, A_max));
    RFX_HIP(alloc_n<int32_t>(node_nseg, A_max));
    RFX_HIP(alloc_n<int32_t>(has_split, A_max));
    RFX_HIP(alloc_n<int32_t>(split_feat, A_max));
    RFX_HIP(alloc_n<uint32_t>(split_key, A_max));
    RFX_HIP(alloc_n<float>(split_thr, A_max));
    RFX_HIP(alloc_n<int32_t>(fb_next, A_max));
    RFX_HIP(alloc_n<int32_t>(fb_seg_node, A_max));
    RFX_HIP(alloc_n<int32_t>(fb_seg_feat, A_max));
    RFX_HIP(alloc_n<uint32_t>(fb_seg_begin, A_max));
    RFX_HIP(alloc_n<uint32_t>(fb_seg_end, A_max));
    RFX_HIP(alloc_n<SegBest>(fb_best, A_max));
    RFX_HIP(alloc_n<uint32_t>(rows_tmp, S_max));
    RFX_HIP(alloc_n<uint32_t>(goes_left, S_max + 1));
    RFX_HIP(alloc_n<uint32_t>(left_before, S_max + 1));
    RFX_HIP(alloc_n<uint32_t>(child_tot, 2 * A_max * C));
    RFX_HIP(alloc_n<uint32_t>(child_cnt, 2 * A_max));
    RFX_HIP(alloc_n<int32_t>(child_dest, 2 * A_max));
    RFX_HIP(alloc_n<int32_t>(child_next, 2 * A_max));
    RFX_HIP(alloc_n<uint32_t>(f_split, A_max + 1));
    RFX_HIP(alloc_n<uint32_t>(f_active, A_max + 1));
    RFX_HIP(alloc_n<uint32_t>(f_rows, A_max + 1));
    RFX_HIP(alloc_n<uint32_t>(x_split, A_max + 1));
    RFX_HIP(alloc_n<uint32_t>(x_active, A_max + 1));
    RFX_HIP(alloc_n<uint32_t>(x_rows, A_max + 1));
    RFX_HIP(alloc_n<uint32_t>(tree_first, Tb));

    int cur = 0;
    hipLaunchKernelGGL(roots_kernel, dim3(1), dim3(64), 0, st, Tb, C, N, cap, ib_pos.as<uint32_t>(), root_tot.as<uint32_t>(),
                       level_of(cur), root_active.as<int32_t>(), nd_feature.as<int32_t>(), nd_class.as<int32_t>(),
                       nd_depth.as<int32_t>(), next_id.as<int32_t>(), counters.as<uint32_t>());
    hipLaunchKernelGGL(fill_rows_kernel, blocks_for(TN), dim3(256), 0, st, ib_flag.as<uint32_t>(), ib_pos.as<uint32_t>(), Tb, N,
                       root_active.as<int32_t>(), rows[cur].as<uint32_t>(), row_node[cur].as<int32_t>());
    RFX_LAUNCH_CHECK("root kernels");
    uint32_t A = 0, S = (uint32_t)S0;
    RFX_HIP(hipMemcpyAsync(&A, counters.p, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    RFX_HIP(hipStreamSynchronize(st));

    int32_t level = 0;
    while (A > 0) {
        if ((size_t)A > A_max || (size_t)S > S_max) return rfx::fail(RFX_ERR_HIP, "forest growth: level tables overflow");
        Level lv = level_of(cur), nx = level_of(cur ^ 1);
        const uint32_t n_seg = A * (uint32_t)mtry;
        g.sorted_pairs += (int64_t)S * mtry;
        RFX_HIP(hipMemsetAsync(counters.p, 0, sizeof(uint32_t) * 8, st));
        hipLaunchKernelGGL(draw_features_kernel, blocks_for(A), dim3(256), 0, st, seed, first, A, M, mtry, lv, seg_node.as<int32_t>(),
                           seg_feat.as<int32_t>(), seg_begin.as<uint32_t>(), seg_end.as<uint32_t>(),
                           node_first_seg.as<int32_t>(), node_nseg.as<int32_t>());
        hipLaunchKernelGGL(build_keys_kernel, blocks_for((int64_t)S * mtry), dim3(256), 0, st, X, M, S, mtry, rows[cur].as<uint32_t>(),
                           row_node[cur].as<int32_t>(), lv, node_first_seg.as<int32_t>(), node_nseg.as<int32_t>(),
                           seg_feat.as<int32_t>(), seg_begin.as<uint32_t>(), keys[0].as<uint32_t>(), vals[0].as<uint32_t>());
        RFX_LAUNCH_CHECK("segment kernels");
        int rc = sort_segments(tmp, keys[0].as<uint32_t>(), keys[1].as<uint32_t>(), vals[0].as<uint32_t>(), vals[1].as<uint32_t>(),
                               S * (uint32_t)mtry, n_seg, seg_begin.as<uint32_t>(), seg_end.as<uint32_t>(), sort_lists, st);
        if (rc != RFX_OK) return rc;
        {
            rfx::TimedLaunch timed("grow_eval_segments_kernel", st);
            hipLaunchKernelGGL(eval_segments_kernel, blocks_for(n_seg, kEvalWaves), dim3(64 * kEvalWaves), 0, st, n_seg, C, N,
                               seg_node.as<int32_t>(), seg_begin.as<uint32_t>(), lv, keys[1].as<uint32_t>(), vals[1].as<uint32_t>(),
                               y, inbag.as<uint16_t>(), best.as<SegBest>());
        }
        hipLaunchKernelGGL(choose_split_kernel, blocks_for(A), dim3(256), 0, st, A, mtry, M, X, seg_feat.as<int32_t>(),
                           seg_begin.as<uint32_t>(), best.as<SegBest>(), keys[1].as<uint32_t>(), vals[1].as<uint32_t>(),
                           has_split.as<int32_t>(), split_feat.as<int32_t>(), split_key.as<uint32_t>(), split_thr.as<float>(),
                           counters.as<uint32_t>() + 2);
        RFX_LAUNCH_CHECK("split kernels");
        uint32_t unresolved = 0;
        RFX_HIP(hipMemcpyAsync(&unresolved, counters.as<uint32_t>() + 2, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        RFX_HIP(hipStreamSynchronize(st));
        if (unresolved > 0 && M > mtry) {
            // rare: features outside the drawn set, in index order, one per round
            RFX_HIP(hipMemsetAsync(fb_next.p, 0, sizeof(int32_t) * A, st));
            for (int32_t round = 0; round < M - mtry && unresolved > 0; ++round) {
                RFX_HIP(hipMemsetAsync(counters.p, 0, sizeof(uint32_t) * 2, st));
                RFX_HIP(hipMemsetAsync(counters.as<uint32_t>() + 3, 0, sizeof(uint32_t), st));
                hipLaunchKernelGGL(fallback_pick_kernel, blocks_for(A), dim3(256), 0, st, A, M, mtry, lv, has_split.as<int32_t>(),
                                   seg_feat.as<int32_t>(), fb_next.as<int32_t>(), fb_seg_node.as<int32_t>(),
                                   fb_seg_feat.as<int32_t>(), fb_seg_begin.as<uint32_t>(), fb_seg_end.as<uint32_t>(),
                                   node_first_seg.as<int32_t>(), node_nseg.as<int32_t>(), counters.as<uint32_t>());
                RFX_LAUNCH_CHECK("fallback_pick_kernel");
                uint32_t h[2] = {0, 0};
                RFX_HIP(hipMemcpyAsync(h, counters.p, sizeof(h), hipMemcpyDeviceToHost, st));
                RFX_HIP(hipStreamSynchronize(st));
                if (h[0] == 0) break;  // the unresolved nodes have tried every feature
                hipLaunchKernelGGL(build_keys_kernel, blocks_for((int64_t)S), dim3(256), 0, st, X, M, S, 1, rows[cur].as<uint32_t>(),
                                   row_node[cur].as<int32_t>(), lv, node_first_seg.as<int32_t>(), node_nseg.as<int32_t>(),
                                   fb_seg_feat.as<int32_t>(), fb_seg_begin.as<uint32_t>(), keys[0].as<uint32_t>(),
                                   vals[0].as<uint32_t>());
                RFX_LAUNCH_CHECK("build_keys_kernel");
                rc = sort_segments(tmp, keys[0].as<uint32_t>(), keys[1].as<uint32_t>(), vals[0].as<uint32_t>(), vals[1].as<uint32_t>(),
                                   h[1], h[0], fb_seg_begin.as<uint32_t>(), fb_seg_end.as<uint32_t>(), sort_lists, st);
                if (rc != RFX_OK) return rc;
                hipLaunchKernelGGL(eval_segments_kernel, blocks_for(h[0], kEvalWaves), dim3(64 * kEvalWaves), 0, st, h[0], C, N,
                                   fb_seg_node.as<int32_t>(), fb_seg_begin.as<uint32_t>(), lv, keys[1].as<uint32_t>(),
                                   vals[1].as<uint32_t>(), y, inbag.as<uint16_t>(), fb_best.as<SegBest>());
                hipLaunchKernelGGL(fallback_choose_kernel, blocks_for(h[0]), dim3(256), 0, st, h[0], M, X, fb_seg_node.as<int32_t>(),
                                   fb_seg_feat.as<int32_t>(), fb_seg_begin.as<uint32_t>(), fb_best.as<SegBest>(),
                                   keys[1].as<uint32_t>(), vals[1].as<uint32_t>(), has_split.as<int32_t>(),
                                   split_feat.as<int32_t>(), split_key.as<uint32_t>(), split_thr.as<float>(),
                                   counters.as<uint32_t>() + 3);
                RFX_LAUNCH_CHECK("fallback kernels");
                uint32_t resolved = 0;
                RFX_HIP(hipMemcpyAsync(&resolved, counters.as<uint32_t>() + 3, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
                RFX_HIP(hipStreamSynchronize(st));
                unresolved -= std::min(resolved, unresolved);
            }
        }
        // split the rows, classify the children, number them, build the next level
        hipLaunchKernelGGL(sides_kernel, blocks_for(S), dim3(256), 0, st, X, M, S, rows[cur].as<uint32_t>(), row_node[cur].as<int32_t>(),
                           has_split.as<int32_t>(), split_feat.as<int32_t>(), split_key.as<uint32_t>(), goes_left.as<uint32_t>());
        RFX_LAUNCH_CHECK("sides_kernel");
        if ((rc = scan_u32(tmp, goes_left.as<uint32_t>(), left_before.as<uint32_t>(), S + 1, st)) != RFX_OK) return rc;
        hipLaunchKernelGGL(partition_kernel, blocks_for(S), dim3(256), 0, st, S, rows[cur].as<uint32_t>(), row_node[cur].as<int32_t>(),
                           lv, has_split.as<int32_t>(), goes_left.as<uint32_t>(), left_before.as<uint32_t>(),
                           rows_tmp.as<uint32_t>());
        hipLaunchKernelGGL(child_stats_kernel, blocks_for(2 * (int64_t)A, 4), dim3(256), 0, st, A, C, N, lv, has_split.as<int32_t>(),
                           left_before.as<uint32_t>(), rows_tmp.as<uint32_t>(), y, inbag.as<uint16_t>(), child_tot.as<uint32_t>(),
                           child_cnt.as<uint32_t>());
        hipLaunchKernelGGL(children_kernel, blocks_for(A), dim3(256), 0, st, A, C, has_split.as<int32_t>(), child_tot.as<uint32_t>(),
                           child_cnt.as<uint32_t>(), f_split.as<uint32_t>(), f_active.as<uint32_t>(), f_rows.as<uint32_t>());
        hipLaunchKernelGGL(tree_first_kernel, blocks_for(A), dim3(256), 0, st, A, lv.tree, tree_first.as<uint32_t>());
        RFX_LAUNCH_CHECK("children kernels");
        if ((rc = scan_u32(tmp, f_split.as<uint32_t>(), x_split.as<uint32_t>(), A + 1, st)) != RFX_OK) return rc;
        if ((rc = scan_u32(tmp, f_active.as<uint32_t>(), x_active.as<uint32_t>(), A + 1, st)) != RFX_OK) return rc;
        if ((rc = scan_u32(tmp, f_rows.as<uint32_t>(), x_rows.as<uint32_t>(), A + 1, st)) != RFX_OK) return rc;
        hipLaunchKernelGGL(emit_kernel, blocks_for(A), dim3(256), 0, st, A, C, cap, level, lv, nx, has_split.as<int32_t>(),
                           split_feat.as<int32_t>(), split_thr.as<float>(), child_tot.as<uint32_t>(), child_cnt.as<uint32_t>(),
                           x_split.as<uint32_t>(), x_active.as<uint32_t>(), x_rows.as<uint32_t>(), tree_first.as<uint32_t>(),
                           next_id.as<int32_t>(), nd_feature.as<int32_t>(), nd_thr.as<float>(), nd_left.as<int32_t>(),
                           nd_right.as<int32_t>(), nd_class.as<int32_t>(), nd_depth.as<int32_t>(), child_dest.as<int32_t>(),
                           child_next.as<int32_t>());
        hipLaunchKernelGGL(advance_ids_kernel, blocks_for(A), dim3(256), 0, st, A, lv.tree, x_split.as<uint32_t>(),
                           f_split.as<uint32_t>(), tree_first.as<uint32_t>(), next_id.as<int32_t>());
        hipLaunchKernelGGL(compact_rows_kernel, blocks_for(S), dim3(256), 0, st, S, rows_tmp.as<uint32_t>(), row_node[cur].as<int32_t>(),
                           lv, has_split.as<int32_t>(), left_before.as<uint32_t>(), child_dest.as<int32_t>(),
                           child_next.as<int32_t>(), rows[cur ^ 1].as<uint32_t>(), row_node[cur ^ 1].as<int32_t>());
        RFX_LAUNCH_CHECK("emit kernels");
        uint32_t nextA = 0, nextS = 0;
        RFX_HIP(hipMemcpyAsync(&nextA, x_active.as<uint32_t>() + A, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        RFX_HIP(hipMemcpyAsync(&nextS, x_rows.as<uint32_t>() + A, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        RFX_HIP(hipStreamSynchronize(st));
        A = nextA;
        S = nextS;
        cur ^= 1;
        ++level;
    }
    g.levels = std::max(g.levels, level);

    // leaf numbers, then the batch's trees to the host
    rfx::DevBuf n_leaves;
    RFX_HIP(alloc_n<int32_t>(n_leaves, Tb));
    hipLaunchKernelGGL(leaf_ids_kernel, dim3(Tb), dim3(64), 0, st, cap, next_id.as<int32_t>(), nd_feature.as<int32_t>(),
                       nd_leaf.as<int32_t>(), n_leaves.as<int32_t>());
    RFX_LAUNCH_CHECK("leaf_ids_kernel");
    std::vector<int32_t> h_nodes(Tb), h_leaves(Tb);
    RFX_HIP(hipMemcpyAsync(h_nodes.data(), next_id.p, sizeof(int32_t) * Tb, hipMemcpyDeviceToHost, st));
    RFX_HIP(hipMemcpyAsync(h_leaves.data(), n_leaves.p, sizeof(int32_t) * Tb, hipMemcpyDeviceToHost, st));
    RFX_HIP(hipStreamSynchronize(st));
    // the batch's records, packed tree after tree on the device and copied with one transfer per field
    std::vector<int64_t> h_off(Tb + 1, 0);
    for (int32_t t = 0; t < Tb; ++t) h_off[t + 1] = h_off[t] + h_nodes[t];
    const size_t n_batch = (size_t)h_off[Tb], base = g.feature.size();
    rfx::DevBuf d_off, packed;
    RFX_HIP(alloc_n<int64_t>(d_off, Tb + 1));
    RFX_HIP(alloc_n<int32_t>(packed, 7 * n_batch));
    RFX_HIP(hipMemcpyAsync(d_off.p, h_off.data(), sizeof(int64_t) * (Tb + 1), hipMemcpyHostToDevice, st));
    NodeFields src{nd_feature.as<int32_t>(), reinterpret_cast<const int32_t*>(nd_thr.p), nd_left.as<int32_t>(), nd_right.as<int32_t>(),
                   nd_leaf.as<int32_t>(), nd_depth.as<int32_t>(), nd_class.as<int32_t>()};
    hipLaunchKernelGGL(pack_nodes_kernel, dim3((unsigned)rfx::ceil_div(cap, 256), (unsigned)Tb), dim3(256), 0, st, cap,
                       d_off.as<int64_t>(), (int64_t)n_batch, src, packed.as<int32_t>());
    RFX_LAUNCH_CHECK("pack_nodes_kernel");
    g.feature.resize(base + n_batch);
    g.threshold.resize(base + n_batch);
    g.left.resize(base + n_batch);
    g.right.resize(base + n_batch);
    g.leaf_id.resize(base + n_batch);
    g.depth.resize(base + n_batch);
    g.node_class.resize(base + n_batch);
    void* dst[7] = {g.feature.data() + base, g.threshold.data() + base, g.left.data() + base, g.right.data() + base,
                    g.leaf_id.data() + base, g.depth.data() + base, g.node_class.data() + base};
    for (int f = 0; f < 7; ++f)
        RFX_HIP(hipMemcpyAsync(dst[f], packed.as<int32_t>() + (size_t)f * n_batch, sizeof(int32_t) * n_batch,
                               hipMemcpyDeviceToHost, st));
    for (int32_t t = 0; t < Tb; ++t) {
        g.node_offset.push_back((int64_t)base + h_off[t + 1]);
        g.n_leaves.push_back(h_leaves[t]);
    }
    const size_t ib = g.inbag.size();
    g.inbag.resize(ib + (size_t)TN);
    RFX_HIP(hipMemcpyAsync(g.inbag.data() + ib, inbag.p, sizeof(uint16_t) * TN, hipMemcpyDeviceToHost, st));
    RFX_HIP(hipStreamSynchronize(st));
    return RFX_OK;
}

}  // namespace

extern "C" {

int rfx_forest_grow(const float* X, const int32_t* y, int64_t N, int32_t M, int32_t n_classes, int32_t first_tree,
                    int32_t n_trees, int32_t mtry, uint64_t seed, rfx_grown** out, void* stream) {
    if (!X || !y || !out) return rfx::fail(RFX_ERR_NULL, "rfx_forest_grow: null argument");
    if (N < 1 || N >= (1 << 20)) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_forest_grow: N=%lld outside 1..2^20-1", (long long)N);
    if (M < 1 || mtry < 1 || mtry > M || mtry > kMaxMtry)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_forest_grow: M=%d mtry=%d (1 <= mtry <= min(M, %d))", M, mtry, kMaxMtry);
    if (n_classes < 1 || n_classes > kMaxClasses)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_forest_grow: n_classes=%d outside 1..%d", n_classes, kMaxClasses);
    if (n_trees < 1 || first_tree < 0) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_forest_grow: trees %d + %d", first_tree, n_trees);
    hipStream_t st = rfx::as_stream(stream);
    rfx_grown* g = new (std::nothrow) rfx_grown();
    if (!g) return rfx::fail(RFX_ERR_OOM, "rfx_forest_grow: host allocation failed");
    g->n_trees = n_trees;
    g->n_features = M;
    g->n_classes = n_classes;
    g->N = N;
    g->node_offset.push_back(0);
    // trees per batch: about 5e8 (key, row) pairs per level at most (some 20 GB of level buffers), 256 trees at most;
    // few trees per batch leave the first levels, whose segments are whole trees, with too few waves
    const double per_tree = 0.64 * (double)N * mtry;
    const int32_t batch = (int32_t)std::max(1.0, std::min(256.0, 5.0e8 / per_tree));
    int rc = RFX_OK;
    try {
        for (int32_t t0 = 0; t0 < n_trees && rc == RFX_OK; t0 += batch)
            rc = grow_batch(*g, X, y, N, M, n_classes, first_tree + t0, std::min(batch, n_trees - t0), mtry, seed, st);
    } catch (const std::bad_alloc&) {
        rc = rfx::fail(RFX_ERR_OOM, "rfx_forest_grow: host allocation failed");
    }
    if (rc != RFX_OK) {
        delete g;
        return rc;
    }
    *out = g;
    return RFX_OK;
}

int rfx_grown_sizes(const rfx_grown* g, int64_t* total_nodes, int32_t* max_leaves, int32_t* levels, int64_t* sorted_pairs) {
    if (!g) return rfx::fail(RFX_ERR_NULL, "rfx_grown_sizes: null handle");
    if (total_nodes) *total_nodes = (int64_t)g->feature.size();
    if (max_leaves) *max_leaves = g->n_leaves.empty() ? 0 : *std::max_element(g->n_leaves.begin(), g->n_leaves.end());
    if (levels) *levels = g->levels;
    if (sorted_pairs) *sorted_pairs = g->sorted_pairs;
    return RFX_OK;
}

int rfx_grown_export(const rfx_grown* g, int64_t* node_offset, int32_t* feature, float* threshold, int32_t* left,
                     int32_t* right, int32_t* leaf_id, int32_t* depth, int32_t* n_leaves, uint16_t* inbag,
                     int32_t* leaf_class) {
    if (!g || !node_offset || !feature || !threshold || !left || !right || !leaf_id || !n_leaves)
        return rfx::fail(RFX_ERR_NULL, "rfx_grown_export: null argument");
    const size_t nn = g->feature.size();
    std::copy(g->node_offset.begin(), g->node_offset.end(), node_offset);
    std::copy(g->feature.begin(), g->feature.end(), feature);
    std::copy(g->threshold.begin(), g->threshold.end(), threshold);
    std::copy(g->left.begin(), g->left.end(), left);
    std::copy(g->right.begin(), g->right.end(), right);
    std::copy(g->leaf_id.begin(), g->leaf_id.end(), leaf_id);
    if (depth) std::copy(g->depth.begin(), g->depth.end(), depth);
    std::copy(g->n_leaves.begin(), g->n_leaves.end(), n_leaves);
    if (inbag) std::copy(g->inbag.begin(), g->inbag.end(), inbag);
    if (leaf_class) {
        const int32_t ml = *std::max_element(g->n_leaves.begin(), g->n_leaves.end());
        std::fill(leaf_class, leaf_class + (size_t)g->n_trees * ml, -1);
        for (int32_t t = 0; t < g->n_trees; ++t)
            for (int64_t v = g->node_offset[t]; v < g->node_offset[t + 1]; ++v)
                if (g->leaf_id[v] >= 0) leaf_class[(size_t)t * ml + g->leaf_id[v]] = g->node_class[v];
    }
    (void)nn;
    return RFX_OK;
}

uint64_t rfx_growth_draw(uint64_t seed, uint64_t tree, uint64_t a, uint64_t b) { return draw(seed, tree, a, b); }

int rfx_grown_destroy(rfx_grown* g) {
    delete g;
    return RFX_OK;
}

}  // extern "C"
