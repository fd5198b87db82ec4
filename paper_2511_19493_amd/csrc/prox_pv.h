// The grouping of samples by (tree, leaf) that the implicit product and the row-wise sparse proximity share.
#pragma once

#include "common.h"

struct rfx_pv_plan {
    int64_t N = 0;
    int32_t B = 0, Lb = 0;
    uint32_t* d_slot = nullptr;       // [B][N]  b*Lb + leaf_b(i)
    uint32_t* d_perm = nullptr;       // [B*N]
    uint32_t* d_seg_start = nullptr;  // [B*Lb + 1]
    uint32_t* d_big = nullptr;        // slots with more than kBigLeaf members, one list per group of trees
    float* d_S = nullptr;             // [B*Lb][k_cap]
    int32_t k_cap = 0;
    // big slots summed in kRanges pieces by sample range (each XCD then gathers from its own eighth of V)
    uint32_t* d_big_bounds = nullptr; // [as d_big][kRanges + 1] positions in perm where the sample ranges begin
    float* d_part = nullptr;          // [part_cap][kRanges][k_cap] partial sums of the pieces
    int64_t part_cap = 0;             // big slots d_part has room for
    static constexpr int kRanges = 8;
    // few sample tiles: the gather cuts the trees of a group into pieces and adds their sums in order
    int32_t gather_pieces = 1;
    float* d_gather_part = nullptr;   // [gather_pieces][N][k_cap]
    // scratch of the grouping, kept so that the plan can be rebuilt for new leaf ids without allocating
    uint32_t* d_count = nullptr;      // [B][Q][Lb] part histograms, then cursors
    int* d_flags = nullptr;           // bad id seen; big slots per group
    int32_t Q = 1;                    // parts per tree
    int64_t part_len = 0;
    int32_t lds_hist = 0;
    bool built = false;               // false after a rebuild that failed: applications are refused
    // An application runs in n_chunks groups of trees: the leaf sums of a group on the caller's stream, its gather on
    // `side` as soon as they are done, so the gather of one group overlaps the sums of the next.
    static constexpr int kMaxChunks = 4;
    int32_t n_chunks = 1;
    int32_t tree_off[kMaxChunks + 1] = {};   // trees of group c: [tree_off[c], tree_off[c + 1])
    int64_t big_base[kMaxChunks] = {};       // its big slots: d_big[big_base[c] .. big_base[c] + big_cnt[c])
    int32_t big_cnt[kMaxChunks] = {};
    hipStream_t side = nullptr;              // shared by all plans of the device, never destroyed
    hipEvent_t ev_sum[kMaxChunks] = {};
    hipEvent_t ev_done = nullptr;
};

namespace rfx {
constexpr int kSparseRowsMaxTrees = 4096;  // per-tree cursors of a row live in LDS next to 64 KB of counters
int sparse_rows_work(const rfx_pv_plan* plan, unsigned long long* d_scratch, unsigned long long* increments, hipStream_t st);
int sparse_rows_enqueue(rfx_pv_plan* plan, uint32_t* start, int32_t min_count, int u16, int64_t capacity, uint32_t* rows,
                        uint32_t* cols, void* counts, float* prox, unsigned long long* cursor, hipStream_t st);
}  // namespace rfx
