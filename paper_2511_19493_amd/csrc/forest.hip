// Forest handle (validation, breadth-first re-layout, upload) and the leaf-assignment kernel.
//
// Traversal rule (paper, "Threshold-based Splits"): at an internal node a sample goes left iff
// x[feature] <= threshold, right otherwise; every sample is dropped down every tree (paper, CPU
// Proximity Computation).
//
// Device layout.  Each tree is stored breadth-first with the two children of a node adjacent, so
// one child index suffices (right = left + 1) and the upper levels of a tree, which every sample
// visits, sit in a few contiguous cache lines.  A node is one 8-byte record
//     .x = threshold bits (float32)
//     .y = payload << fbits | feature     internal node: payload = index of the left child
//          payload << fbits | fmask       leaf:          payload = dense leaf id
// with fmask = 2^fbits - 1 >= n_features, so a single 8-byte load per visited node brings
// everything the step needs.
#include <algorithm>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "common.h"

namespace rfx {

static thread_local std::string g_last_error;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

namespace {
struct TimingState {
    std::mutex mu;
    bool enabled = false;
    struct Pending {
        std::string name;
        hipEvent_t a, b;
    };
    std::vector<Pending> pending;
    std::map<std::string, std::pair<double, int64_t>> totals;  // name -> (ms, launches)
};
TimingState& timing() {
    static TimingState s;
    return s;
}
}  // namespace

TimedLaunch::TimedLaunch(const char* name, hipStream_t st) : name_(name), st_(st) {
    TimingState& t = timing();
    std::lock_guard<std::mutex> lk(t.mu);
    if (!t.enabled) return;
    if (hipEventCreate(&start_) != hipSuccess) {
        start_ = nullptr;
        return;
    }
    (void)hipEventRecord(start_, st_);
}

TimedLaunch::~TimedLaunch() {
    if (!start_) return;
    hipEvent_t stop = nullptr;
    if (hipEventCreate(&stop) != hipSuccess) {
        (void)hipEventDestroy(start_);
        return;
    }
    (void)hipEventRecord(stop, st_);
    TimingState& t = timing();
    std::lock_guard<std::mutex> lk(t.mu);
    t.pending.push_back({name_, start_, stop});
}

}  // namespace rfx

struct rfx_forest {
    int32_t B = 0, M = 0, fbits = 0, leaf_bound = 0;
    int64_t total_nodes = 0;
    uint2* d_nodes = nullptr;      // [total_nodes]
    int64_t* d_tree_off = nullptr; // [B+1]
};

namespace {

constexpr int kTileSamples = 128;  // samples per workgroup
constexpr int kTreeSlots = 8;      // thread groups (of kTileSamples threads) walking different trees
constexpr int kWalks = 2;          // trees a thread walks at once
constexpr int kBlock = kTileSamples * kTreeSlots;
constexpr int kRound = kTreeSlots * kWalks;  // trees per round of a workgroup

// A workgroup owns a tile of 128 samples and keeps their feature rows in LDS (row stride odd, so a
// wave reading one feature of 64 different rows hits 64 different banks).  It walks them down a
// contiguous range of trees, 16 trees per round: each of the 8 thread groups takes 2 trees and each
// thread advances its 2 walks together.  A walk is a dependent chain (node record -> feature value ->
// child index), so throughput comes from walks in flight: 1024 threads x 2 walks per workgroup and,
// with the 128-row tile, two workgroups per compute unit.  (Measured at N = 100k, M = 100: 256-row
// tiles with one walk per thread 4.4 ms per 1000 trees, this shape 2.3 ms; staging the upper tree
// levels in LDS did not pay.)  A wave is 64 consecutive samples of one tree pair, so leaf ids are
// written coalesced along the sample axis of leaf[B][N].
template <bool kRowsInLds>
__global__ __launch_bounds__(kBlock) void leaf_assign_kernel(const uint2* __restrict__ nodes,
                                                            const int64_t* __restrict__ tree_off, int32_t B,
                                                            const float* __restrict__ X, int64_t N, int32_t M,
                                                            int32_t fbits, int32_t lds_stride,
                                                            int32_t trees_per_block, uint32_t* __restrict__ leaf) {
    extern __shared__ float xs[];
    const int s = threadIdx.x % kTileSamples;
    const int slot = threadIdx.x / kTileSamples;
    const int64_t i0 = (int64_t)blockIdx.x * kTileSamples;
    const int64_t i = i0 + s;
    if (kRowsInLds) {
        const int rows = (int)min((int64_t)kTileSamples, N - i0);
        const float* src = X + i0 * M;
        for (int idx = threadIdx.x; idx < rows * M; idx += kBlock) {
            int r = idx / M;
            xs[r * lds_stride + (idx - r * M)] = src[idx];
        }
        __syncthreads();
    }
    if (i >= N) return;
    const uint32_t fmask = (1u << fbits) - 1u;
    const int b0 = blockIdx.y * trees_per_block;
    const int b1 = min(B, b0 + trees_per_block);
    const float* xrow = kRowsInLds ? xs + s * lds_stride : X + i * M;
    for (int bb = b0; bb < b1; bb += kRound) {
        const uint2* t[kWalks];
        uint2 rec[kWalks];
#pragma unroll
        for (int u = 0; u < kWalks; ++u) {
            const int b = min(bb + slot * kWalks + u, b1 - 1);
            t[u] = nodes + tree_off[b];
            rec[u] = t[u][0];
        }
        bool any = true;
        while (any) {
            any = false;
#pragma unroll
            for (int u = 0; u < kWalks; ++u) {
                if ((rec[u].y & fmask) != fmask) {
                    const float x = xrow[rec[u].y & fmask];
                    const uint32_t child = (rec[u].y >> fbits) + ((x <= __uint_as_float(rec[u].x)) ? 0u : 1u);
                    rec[u] = t[u][child];
                    any = true;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kWalks; ++u) {
            const int b = bb + slot * kWalks + u;
            if (b < b1) leaf[(int64_t)b * N + i] = rec[u].y >> fbits;
        }
    }
}

int bit_width(uint64_t v) {
    int w = 0;
    while (v) {
        ++w;
        v >>= 1;
    }
    return w;
}

}  // namespace

extern "C" {

const char* rfx_last_error(void) { return rfx::g_last_error.c_str(); }

int rfx_timing_enable(int on) {
    rfx::TimingState& t = rfx::timing();
    std::lock_guard<std::mutex> lk(t.mu);
    t.enabled = on != 0;
    for (auto& p : t.pending) {
        (void)hipEventSynchronize(p.b);
        (void)hipEventDestroy(p.a);
        (void)hipEventDestroy(p.b);
    }
    t.pending.clear();
    t.totals.clear();
    return RFX_OK;
}

int rfx_timing_get(const char* kernel, double* total_ms, int64_t* launches) {
    if (!kernel || !total_ms || !launches) return rfx::fail(RFX_ERR_NULL, "rfx_timing_get: null argument");
    rfx::TimingState& t = rfx::timing();
    std::lock_guard<std::mutex> lk(t.mu);
    for (auto& p : t.pending) {
        float ms = 0.0f;
        if (hipEventSynchronize(p.b) == hipSuccess && hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
            auto& tot = t.totals[p.name];
            tot.first += ms;
            tot.second += 1;
        }
        (void)hipEventDestroy(p.a);
        (void)hipEventDestroy(p.b);
    }
    t.pending.clear();
    auto it = t.totals.find(kernel);
    *total_ms = it == t.totals.end() ? 0.0 : it->second.first;
    *launches = it == t.totals.end() ? 0 : it->second.second;
    return RFX_OK;
}

int rfx_forest_create(const rfx_forest_desc* d, rfx_forest** out) {
    if (!d || !out) return rfx::fail(RFX_ERR_NULL, "rfx_forest_create: null argument");
    *out = nullptr;
    if (!d->node_offset || !d->feature || !d->threshold || !d->left || !d->right || !d->leaf_id || !d->n_leaves)
        return rfx::fail(RFX_ERR_NULL, "rfx_forest_create: null array in description");
    const int32_t B = d->n_trees, M = d->n_features;
    if (B < 1 || M < 1) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_forest_create: n_trees=%d n_features=%d", B, M);
    if (d->node_offset[0] != 0) return rfx::fail(RFX_ERR_FOREST, "node_offset[0] must be 0");

    const int fbits = bit_width((uint64_t)M);  // 2^fbits - 1 >= M
    const uint32_t fmask = (1u << fbits) - 1u;
    const uint64_t payload_cap = 1ull << (32 - fbits);
    const int64_t total = d->node_offset[B];
    if (total < B) return rfx::fail(RFX_ERR_FOREST, "node_offset[B]=%lld", (long long)total);

    std::vector<uint2> nodes((size_t)total);
    std::vector<int32_t> order, newidx;
    std::vector<char> leaf_seen;
    int32_t leaf_bound = 0;
    for (int32_t b = 0; b < B; ++b) {
        const int64_t off = d->node_offset[b];
        const int64_t n = d->node_offset[b + 1] - off;
        const int32_t L = d->n_leaves[b];
        if (n < 1 || off < 0 || off + n > total)
            return rfx::fail(RFX_ERR_FOREST, "tree %d: bad node range", b);
        if (L < 1 || n != 2 * (int64_t)L - 1)
            return rfx::fail(RFX_ERR_FOREST, "tree %d: %lld nodes do not form a binary tree with %d leaves", b,
                             (long long)n, L);
        if ((uint64_t)n > payload_cap || (uint64_t)L > payload_cap)
            return rfx::fail(RFX_ERR_UNSUPPORTED, "tree %d: %lld nodes and %d features do not fit a 32-bit node word", b,
                             (long long)n, M);
        leaf_bound = std::max(leaf_bound, L);
        // breadth-first order from the root; a node's children take the next two slots
        order.clear();
        order.reserve((size_t)n);
        newidx.assign((size_t)n, -1);
        leaf_seen.assign((size_t)L, 0);
        order.push_back(0);
        newidx[0] = 0;
        for (size_t head = 0; head < order.size(); ++head) {
            const int32_t v = order[head];
            if (d->feature[off + v] < 0) continue;
            const int32_t kids[2] = {d->left[off + v], d->right[off + v]};
            for (int32_t c : kids) {
                if (c < 0 || c >= n || newidx[c] >= 0)
                    return rfx::fail(RFX_ERR_FOREST, "tree %d node %d: child %d out of range or visited twice", b, v, c);
                newidx[c] = (int32_t)order.size();
                order.push_back(c);
            }
        }
        if ((int64_t)order.size() != n)
            return rfx::fail(RFX_ERR_FOREST, "tree %d: %zu of %lld nodes reachable from the root", b, order.size(),
                             (long long)n);
        for (int64_t p = 0; p < n; ++p) {
            const int32_t v = order[(size_t)p];
            const int32_t f = d->feature[off + v];
            uint2 rec;
            if (f >= 0) {
                if (f >= M) return rfx::fail(RFX_ERR_FOREST, "tree %d node %d: feature %d >= %d", b, v, f, M);
                float thr = d->threshold[off + v];
                std::memcpy(&rec.x, &thr, 4);
                const int32_t l = newidx[d->left[off + v]];
                if (newidx[d->right[off + v]] != l + 1)
                    return rfx::fail(RFX_ERR_FOREST, "tree %d node %d: internal layout error", b, v);
                rec.y = ((uint32_t)l << fbits) | (uint32_t)f;
            } else {
                const int32_t id = d->leaf_id[off + v];
                if (id < 0 || id >= L || leaf_seen[id])
                    return rfx::fail(RFX_ERR_FOREST, "tree %d node %d: leaf id %d out of range or repeated", b, v, id);
                leaf_seen[id] = 1;
                rec.x = 0;
                rec.y = ((uint32_t)id << fbits) | fmask;
            }
            nodes[(size_t)(off + p)] = rec;
        }
    }

    rfx_forest* F = new (std::nothrow) rfx_forest;
    if (!F) return rfx::fail(RFX_ERR_OOM, "rfx_forest_create: host allocation failed");
    F->B = B;
    F->M = M;
    F->fbits = fbits;
    F->leaf_bound = leaf_bound;
    F->total_nodes = total;
    hipError_t e = hipMalloc((void**)&F->d_nodes, sizeof(uint2) * (size_t)total);
    if (e == hipSuccess) e = hipMalloc((void**)&F->d_tree_off, sizeof(int64_t) * (size_t)(B + 1));
    if (e == hipSuccess) e = hipMemcpy(F->d_nodes, nodes.data(), sizeof(uint2) * (size_t)total, hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(F->d_tree_off, d->node_offset, sizeof(int64_t) * (size_t)(B + 1), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        rfx_forest_destroy(F);
        return rfx::fail(e == hipErrorOutOfMemory ? RFX_ERR_OOM : RFX_ERR_HIP, "rfx_forest_create: %s",
                         hipGetErrorString(e));
    }
    *out = F;
    return RFX_OK;
}

int rfx_forest_destroy(rfx_forest* F) {
    if (!F) return RFX_OK;
    if (F->d_nodes) (void)hipFree(F->d_nodes);
    if (F->d_tree_off) (void)hipFree(F->d_tree_off);
    delete F;
    return RFX_OK;
}

int32_t rfx_forest_leaf_bound(const rfx_forest* F) { return F ? F->leaf_bound : 0; }

int rfx_leaf_assign(const rfx_forest* F, const float* X, int64_t N, int32_t M, uint32_t* leaf, void* stream) {
    if (!F || !X || !leaf) return rfx::fail(RFX_ERR_NULL, "rfx_leaf_assign: null argument");
    if (N < 1 || N > (int64_t)1 << 31) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_leaf_assign: N=%lld", (long long)N);
    if (M != F->M) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_leaf_assign: M=%d but the forest has %d features", M, F->M);

    const int64_t tiles = rfx::ceil_div(N, kTileSamples);
    // enough workgroups to fill 256 compute units several times over.  A forest much larger than the L2 caches
    // (32 MB in all) is walked tree-major instead (one round of trees per workgroup, sample tiles fastest in the
    // grid): all samples pass through a round's trees while their nodes are cached, instead of every group of
    // resident workgroups pulling the whole forest in again, one first touch per deep node.  (500,000 rows, trees
    // of 90,000 nodes: 142 -> 48 us per tree; at 54 MB of nodes the extra staging of the sample tiles costs 10 %.)
    const bool forest_fits_cache = F->total_nodes * (int64_t)sizeof(uint2) <= (64ll << 20);
    int64_t chunks = std::min<int64_t>(rfx::ceil_div(F->B, kRound), std::max<int64_t>(1, rfx::ceil_div(4096, tiles)));
    if (!forest_fits_cache) chunks = rfx::ceil_div(F->B, kRound);
    int32_t tpb = (int32_t)(rfx::ceil_div(rfx::ceil_div(F->B, chunks), kRound) * kRound);
    chunks = rfx::ceil_div(F->B, tpb);
    if (chunks > 65535) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_leaf_assign: too many tree chunks");
    dim3 grid((unsigned)tiles, (unsigned)chunks);

    const int32_t stride = (M & 1) ? M : M + 1;
    const size_t lds = sizeof(float) * (size_t)kTileSamples * (size_t)stride;
    hipStream_t st = rfx::as_stream(stream);
    rfx::TimedLaunch timed("leaf_assign_kernel", st);
    if (lds <= 156 * 1024) {  // up to about 300 features; beyond that the rows are read from global memory
        auto kern = leaf_assign_kernel<true>;
        RFX_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(kern, grid, dim3(kBlock), lds, st, F->d_nodes, F->d_tree_off, F->B, X, N, M, F->fbits, stride,
                           tpb, leaf);
    } else {
        hipLaunchKernelGGL(leaf_assign_kernel<false>, grid, dim3(kBlock), 0, st, F->d_nodes, F->d_tree_off, F->B, X, N, M,
                           F->fbits, stride, tpb, leaf);
    }
    RFX_LAUNCH_CHECK("leaf_assign_kernel");
    return RFX_OK;
}

}  // extern "C"
