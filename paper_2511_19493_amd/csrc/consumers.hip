// Out-of-bag vote (paper, "OOB Error Estimation"): for sample i only the trees whose bootstrap
// sample missed i vote, each with the class label of the leaf that i falls in; the prediction is
// the class with most votes.  Reads the leaf ids and in-bag counts once (coalesced over samples,
// one tree after another) and gathers the leaf labels, which stay cache-resident.
#include "common.h"

namespace {

constexpr int kVoteThreads = 256;
constexpr int kVoteUnroll = 4;

// One sample per thread; its C vote counters live in LDS at [class][thread] (conflict-free).
__global__ __launch_bounds__(kVoteThreads) void oob_vote_kernel(const uint32_t* __restrict__ leaf,
                                                               const uint16_t* __restrict__ inbag,
                                                               const int32_t* __restrict__ leaf_class, int64_t N,
                                                               int32_t B, int32_t leaf_stride, int32_t C,
                                                               const int32_t* __restrict__ y, uint32_t* __restrict__ votes,
                                                               int32_t* __restrict__ pred,
                                                               unsigned long long* __restrict__ tallies) {
    extern __shared__ uint32_t v[];
    const int tid = threadIdx.x;
    const int64_t i = (int64_t)blockIdx.x * kVoteThreads + tid;
    for (int c = 0; c < C; ++c) v[c * kVoteThreads + tid] = 0;
    const int64_t ic = i < N ? i : N - 1;  // clamped: loads are unconditional, the votes of padding threads are dropped
    for (int b0 = 0; b0 < B; b0 += kVoteUnroll) {
        uint32_t id[kVoteUnroll];
        uint32_t in[kVoteUnroll];
        int32_t cls[kVoteUnroll];
#pragma unroll
        for (int u = 0; u < kVoteUnroll; ++u) {
            const int b = min(b0 + u, B - 1);
            id[u] = leaf[(int64_t)b * N + ic];
            in[u] = inbag[(int64_t)b * N + ic];
        }
#pragma unroll
        for (int u = 0; u < kVoteUnroll; ++u) {
            const int b = min(b0 + u, B - 1);
            cls[u] = leaf_class[(int64_t)b * leaf_stride + min(id[u], (uint32_t)(leaf_stride - 1))];
        }
#pragma unroll
        for (int u = 0; u < kVoteUnroll; ++u) {
            // a leaf id or a label out of range casts no vote
            const bool ok = b0 + u < B && in[u] == 0 && id[u] < (uint32_t)leaf_stride && (uint32_t)cls[u] < (uint32_t)C;
            if (ok) v[cls[u] * kVoteThreads + tid] += 1;
        }
    }
    int32_t best = -1;
    uint32_t best_votes = 0;
    for (int c = 0; c < C; ++c) {
        const uint32_t n = v[c * kVoteThreads + tid];
        if (n > best_votes) {  // strict: the lowest class wins a tie
            best_votes = n;
            best = c;
        }
        if (votes && i < N) votes[i * C + c] = n;
    }
    const bool voted = i < N && best >= 0;
    const bool wrong = voted && y && y[ic] != best;
    if (i < N) pred[i] = best;
    const unsigned long long nv = __builtin_popcountll(__ballot(voted));
    const unsigned long long nw = __builtin_popcountll(__ballot(wrong));
    if ((tid & 63) == 0) {
        if (nw) atomicAdd(tallies + 0, nw);
        if (nv) atomicAdd(tallies + 1, nv);
    }
}

}  // namespace

extern "C" {

int rfx_oob_vote(const uint32_t* leaf, const uint16_t* inbag, const int32_t* leaf_class, int64_t N, int32_t B,
                 int32_t leaf_stride, int32_t n_classes, const int32_t* y, uint32_t* votes, int32_t* pred,
                 int64_t* wrong, int64_t* voted, void* stream) {
    if (!leaf || !inbag || !leaf_class || !pred) return rfx::fail(RFX_ERR_NULL, "rfx_oob_vote: null argument");
    if (wrong && !y) return rfx::fail(RFX_ERR_NULL, "rfx_oob_vote: the error count needs the labels y");
    if (N < 1 || B < 1 || leaf_stride < 1)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_oob_vote: N=%lld B=%d leaf_stride=%d", (long long)N, B, leaf_stride);
    if (n_classes < 1 || n_classes > 128)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_oob_vote: n_classes=%d outside 1..128", n_classes);
    if (rfx::ceil_div(N, kVoteThreads) > 0x7fffffffLL) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_oob_vote: N too large");
    hipStream_t st = rfx::as_stream(stream);
    rfx::DevBuf tallies;
    RFX_HIP(tallies.alloc(2 * sizeof(unsigned long long)));
    RFX_HIP(hipMemsetAsync(tallies.p, 0, 2 * sizeof(unsigned long long), st));
    const size_t lds = sizeof(uint32_t) * (size_t)n_classes * kVoteThreads;
    if (lds > 64 * 1024)
        RFX_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(oob_vote_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    {
        rfx::TimedLaunch timed("oob_vote_kernel", st);
        hipLaunchKernelGGL(oob_vote_kernel, dim3((unsigned)rfx::ceil_div(N, kVoteThreads)), dim3(kVoteThreads), lds, st, leaf,
                           inbag, leaf_class, N, B, leaf_stride, n_classes, y, votes, pred,
                           tallies.as<unsigned long long>());
    }
    RFX_LAUNCH_CHECK("oob_vote_kernel");
    unsigned long long h[2] = {0, 0};
    RFX_HIP(hipMemcpyAsync(h, tallies.p, sizeof(h), hipMemcpyDeviceToHost, st));
    RFX_HIP(hipStreamSynchronize(st));
    if (wrong) *wrong = (int64_t)h[0];
    if (voted) *voted = (int64_t)h[1];
    return RFX_OK;
}

}  // extern "C"
