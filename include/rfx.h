/* rfx.h -- C ABI of librfx: the random-forest proximity path on one MI355X (gfx950).
 *
 * The library computes, for a grown Breiman-Cutler classification forest,
 *   1. the terminal node of every sample in every tree,
 *   2. the dense proximity matrix p(i,j) = (1/B) #{b : node_b(i) = node_b(j)} and its
 *      out-of-bag-only variant,
 *   3. a rank-k factorisation of P obtained without forming P, quantised to INT8, and
 *      3-D scaling coordinates computed from those factors.
 * Citations name sections / equations of the RFX paper (arXiv 2511.19493).
 *
 * Conventions
 *   - Every function returns an int status: RFX_OK (0) or a negative RFX_ERR_* code.  No
 *     exception or abort crosses this boundary.  rfx_last_error() returns a thread-local
 *     message for the last failing call on the calling thread.
 *   - Pointers marked [device] are device (HBM) addresses owned by the caller; the library
 *     neither frees nor keeps them after the call returns.  Pointers marked [host] are host
 *     addresses.  All arrays are dense, row-major, with the index order written in brackets.
 *   - `stream` is a hipStream_t passed as void* (null = the default stream).  Work is
 *     enqueued on that stream in order.  Calls documented as "asynchronous" return before
 *     the work has finished, never wait for the device, allocate nothing, and their outputs are
 *     valid once the caller has synchronised the stream; the others synchronise the stream
 *     before returning.
 *   - Scratch memory.  Every step has an asynchronous form that takes its scratch from the
 *     caller: rfx_*_workspace_bytes reports the size for a problem, and the *_ws / *_plan call
 *     takes `workspace` [device], 256-byte aligned, of at least that many bytes (else
 *     RFX_ERR_CAPACITY).  The workspace holds nothing between calls and may be reused by the
 *     next call on the same stream; two calls that use one workspace on different streams race.
 *     The calls without a workspace argument are conveniences for one-off use: they allocate
 *     their scratch (hipMalloc / hipFree inside the call), run the asynchronous form and wait.
 *     Plans and forests own their memory until destroyed.
 *   - Arguments are validated on the host before anything is launched: a call that returns an
 *     argument error (RFX_ERR_NULL, _INVALID_ARG, _OVERFLOW, _UNSUPPORTED, _FOREST, and
 *     _CAPACITY of a workspace) has launched nothing that writes caller memory.  Conditions that
 *     only the device can see are reported after the outputs were written: a leaf id at or above
 *     leaf_bound (rfx_pv_plan_create), a block that lost rank (rfx_prox_lowrank), more
 *     qualifying pairs than the capacity (rfx_prox_sparse), and failures of the HIP runtime.
 */
#ifndef RFX_H
#define RFX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RFX_OK 0
#define RFX_ERR_INVALID_ARG (-1) /* a size, enum or combination of arguments is out of range */
#define RFX_ERR_NULL (-2)        /* a required pointer is null */
#define RFX_ERR_OVERFLOW (-3)    /* a count does not fit the requested output type */
#define RFX_ERR_OOM (-4)         /* device or host allocation failed */
#define RFX_ERR_HIP (-5)         /* a HIP runtime call failed (message has the HIP error) */
#define RFX_ERR_UNSUPPORTED (-6) /* valid request outside what this build implements */
#define RFX_ERR_FOREST (-7)      /* the forest description is malformed */
#define RFX_ERR_CAPACITY (-8)    /* an output of caller-chosen capacity is too small (the needed size is reported) */

/* count_dtype */
#define RFX_U16 0
#define RFX_U32 1
/* layout of an N x N symmetric output */
#define RFX_FULL 0         /* [N][N]: both triangles and the diagonal */
#define RFX_UPPER_PACKED 1 /* strict upper triangle, row-major, N(N-1)/2 entries:
                              idx(i,j) = i*N - i(i+1)/2 + (j-i-1) for i < j
                              ("Packed Upper Triangle Storage") */
/* dissim_mode of rfx_mds3d */
#define RFX_MDS_SQUARED 0 /* D = 1 - P squared element-wise before double-centring (MDS Steps 1-2) */
#define RFX_MDS_LINEAR 1  /* 1 - P itself taken as the squared distance */

const char* rfx_last_error(void);

/* Measurement aid.  While enabled, the library brackets each launch of its main kernels
 * ("leaf_assign_kernel", "prox_tile_kernel", "prox_tile_kernel_oob", "pv_leaf_sum_kernel",
 * "pv_gather_kernel") with HIP events on the launch stream.  rfx_timing_enable(on) switches it
 * and clears the totals; rfx_timing_get waits for the recorded events and returns the summed
 * kernel time in milliseconds and the number of launches of one kernel since the last enable.
 *   total_ms, launches [host] out. */
int rfx_timing_enable(int on);
int rfx_timing_get(const char* kernel, double* total_ms, int64_t* launches);

/* ------------------------------------------------------------------------------------------
 * Forest: flattened trees ("Flattened arrays": per-node split variable, split value, child
 * pointers and node status, concatenated over trees).  All pointers [host].
 * Tree b owns nodes [node_offset[b], node_offset[b+1]); its root is local node 0; child
 * indices are tree-local.  A node is a leaf iff feature < 0; then leaf_id is its dense index
 * in 0..n_leaves[b]-1.  Internal nodes send a sample left iff x[feature] <= threshold, right
 * otherwise ("Threshold-based Splits"); a NaN feature value therefore goes right.
 */
typedef struct {
    int32_t n_trees;            /* B >= 1 */
    int32_t n_features;         /* M >= 1 */
    const int64_t* node_offset; /* [B+1] */
    const int32_t* feature;     /* [nodes] */
    const float* threshold;     /* [nodes] */
    const int32_t* left;        /* [nodes] */
    const int32_t* right;       /* [nodes] */
    const int32_t* leaf_id;     /* [nodes] */
    const int32_t* n_leaves;    /* [B] */
} rfx_forest_desc;

typedef struct rfx_forest rfx_forest;

/* Validates the description (every tree is a proper binary tree reachable from its root,
 * indices in range, leaf ids dense), re-lays each tree breadth-first with sibling pairs
 * adjacent, and uploads it to the current device.  Synchronous.  The handle owns its device
 * copy; the description's arrays may be freed after the call.
 * Errors: RFX_ERR_NULL, RFX_ERR_INVALID_ARG, RFX_ERR_FOREST, RFX_ERR_UNSUPPORTED (feature
 * index and child index of some tree do not fit one 32-bit word together), RFX_ERR_OOM. */
int rfx_forest_create(const rfx_forest_desc* desc, rfx_forest** out);
int rfx_forest_destroy(rfx_forest* forest);
/* Largest n_leaves over the trees: an exclusive upper bound on every leaf id the forest can
 * emit, to be passed as `leaf_bound` below. */
int32_t rfx_forest_leaf_bound(const rfx_forest* forest);

/* Forest growth on the GPU ("GPU Tree Growth Strategies", "Batched Multi-Tree Processing";
 * Methodology: every tree on a bootstrap sample, mtry random features per node, the split with
 * the largest Gini decrease over the values present in the node, x <= tau goes left, growth until
 * the nodes are pure).  Trees first_tree .. first_tree + n_trees - 1 are grown in batches, level
 * by level.  What the paper leaves open is fixed as follows:
 *   - random numbers: draw(seed, tree, a, b) = mix(mix(mix(seed ^ (tree+1) K) ^ a) ^ b), mix = the
 *     output function of splitmix64, K = 0x9e3779b97f4a7c15; an integer below n is
 *     ((draw >> 32) * n) >> 32.  Bootstrap row t of a tree = bounded(draw(seed, tree, 0, t), N);
 *     the features of node v = the first mtry entries of a Fisher-Yates shuffle of 0..M-1 whose
 *     s-th swap partner is s + bounded(draw(seed, tree, 1 + v, s), M - s);
 *   - nodes are numbered breadth first in creation order, leaves 0..L-1 in node order;
 *   - rows are weighted by their in-bag count; split scores are compared exactly (integer
 *     cross-multiplication); candidates in feature draw order, then ascending threshold, a later
 *     one wins only if strictly better; if no drawn feature takes two values in a node the other
 *     features are tried in index order and the first that does is used; if none does the node is
 *     a leaf with the class of largest weight (lowest class on ties).
 *   X [device] float32 [N][M] without NaN;  y [device] int32 [N] in 0..n_classes-1;
 *   1 <= N < 2^20, 1 <= mtry <= min(M, 64), n_classes <= 64.
 * The result lives on the host.  rfx_grown_sizes reports the node total, the largest number of
 * leaves in a tree, the number of level passes made and the number of (row, feature) pairs that were
 * sorted and scored over all levels (each output nullable); rfx_grown_export fills caller arrays in the layout of
 * rfx_forest_desc (host; node arrays of length total_nodes, node_offset [B+1], n_leaves [B]) plus,
 * all nullable, depth [nodes], inbag uint16 [B][N] and leaf_class int32 [B][max_leaves] (-1 past a
 * tree's last leaf), ready for rfx_forest_create, rfx_prox_oob and rfx_oob_vote.  Synchronous.
 * Errors: RFX_ERR_NULL, RFX_ERR_INVALID_ARG, RFX_ERR_OOM, RFX_ERR_HIP. */
typedef struct rfx_grown rfx_grown;
int rfx_forest_grow(const float* X, const int32_t* y, int64_t N, int32_t M, int32_t n_classes, int32_t first_tree,
                    int32_t n_trees, int32_t mtry, uint64_t seed, rfx_grown** out, void* stream);
int rfx_grown_sizes(const rfx_grown* grown, int64_t* total_nodes, int32_t* max_leaves, int32_t* levels,
                    int64_t* sorted_pairs);
int rfx_grown_export(const rfx_grown* grown, int64_t* node_offset, int32_t* feature, float* threshold, int32_t* left,
                     int32_t* right, int32_t* leaf_id, int32_t* depth, int32_t* n_leaves, uint16_t* inbag,
                     int32_t* leaf_class);
int rfx_grown_destroy(rfx_grown* grown);
/* The counter-based 64-bit draw defined above, evaluated on the host (the same function the
 * kernels call); lets a caller reproduce the bootstrap samples and feature draws of a tree. */
uint64_t rfx_growth_draw(uint64_t seed, uint64_t tree, uint64_t a, uint64_t b);

/* Leaf assignment: leaf[b*N + i] = dense leaf index of sample i in tree b, for every tree and
 * every sample, in-bag or not (CPU Proximity Computation; traversal rule: "Threshold-based
 * Splits").
 *   X    [device] float32 [N][M] row-major samples, M == forest n_features
 *   leaf [device] uint32 [B][N] out
 * Asynchronous.  Errors: RFX_ERR_NULL, RFX_ERR_INVALID_ARG (N < 1, M mismatch). */
int rfx_leaf_assign(const rfx_forest* forest, const float* X, int64_t N, int32_t M, uint32_t* leaf,
                    void* stream);

/* Measurement aids (not part of the proximity path).  rfx_probe_valu runs a dependency-free loop
 * of the two vector operations the compare-and-count kernel is made of (3-input boolean op,
 * population count with accumulate) on every CU for `rounds` rounds (1..2^20) and reports the
 * lane-operations per second reached; rfx_probe_copy copies `bytes` (2^20..2^36) of device
 * memory with a plain kernel and reports bytes read + written per second (best of 3).  All probes
 * allocate their own buffers and are synchronous.  Errors: RFX_ERR_NULL, RFX_ERR_INVALID_ARG,
 * RFX_ERR_OOM. */
int rfx_probe_valu(int32_t rounds, double* lane_ops_per_s, void* stream);
int rfx_probe_copy(int64_t bytes, double* bytes_per_s, void* stream);
/* rfx_probe_gather: the access pattern of the implicit product with everything else taken away.  Waves read
 * `gathers` rows of k float32 (k = 16, 32, 64, 128, 192 or 256) at pseudo-random indices of a table of table_rows rows
 * (64..2^26), eight row loads in flight per wave, and add them up; reports row bytes read per second (best of 3).  A
 * table smaller than the 4 MB second-level cache of an XCD measures gathers that hit it, one of tens of MB gathers
 * served by the last-level cache, one of GBs gathers from HBM.  xcd_local = 1 lets every workgroup draw from the eighth
 * of the table that belongs to the XCD running it.
 * rfx_probe_chase: the access pattern of tree traversal.  Every thread of two 1,024-thread workgroups per CU advances
 * walks_per_thread (1, 2 or 4) independent chains of `steps` dependent 8-byte loads through a table of table_bytes
 * (4 KiB..16 GiB) of pseudo-randomly linked records; with_lds = 1 puts a dependent 4-byte LDS read between two loads,
 * as the feature lookup of a node does.  Reports chain steps per second over all walks (best of 2). */
int rfx_probe_gather(int64_t table_rows, int32_t k, int64_t gathers, int32_t xcd_local, double* bytes_per_s, void* stream);
int rfx_probe_chase(int64_t table_bytes, int32_t walks_per_thread, int32_t steps, int32_t with_lds, double* steps_per_s,
                    void* stream);

/* Dense proximity (equation p(i,j) = (1/B) sum_b I(node_b(i) = node_b(j)), "Proximity
 * Matrices").
 *   leaf        [device] uint32 [B][N], every entry < leaf_bound
 *   leaf_bound  exclusive upper bound on the leaf ids, 1..2^24; ids >= leaf_bound give wrong
 *               counts (never a memory fault)
 *   count_dtype RFX_U16 (requires B <= 65535) or RFX_U32
 *   layout      RFX_FULL or RFX_UPPER_PACKED, applies to both outputs
 *   counts      [device] nullable; cnt(i,j) = #{b : leaf_b(i) = leaf_b(j)}; diagonal = B
 *   prox        [device] nullable float32; cnt / B in IEEE float32 division; diagonal = 1
 * At least one of counts / prox must be given.
 * rfx_prox_workspace_bytes: scratch of every rfx_prox_*_ws call for this N, B, leaf_bound (the
 * leaf ids transposed into bit planes, 4 * ceil(B/32) * roundup(N, 256) * roundup4(bits + 1)
 * bytes, plus 16 N bytes of per-sample sums and a counter).  1 <= N <= 3,000,000.
 * rfx_prox_dense_ws: asynchronous.  rfx_prox_dense: synchronous convenience.
 * Errors: RFX_ERR_NULL, RFX_ERR_INVALID_ARG, RFX_ERR_OVERFLOW, RFX_ERR_CAPACITY, RFX_ERR_OOM. */
int rfx_prox_workspace_bytes(int64_t N, int32_t B, int32_t leaf_bound, int64_t* bytes);
int rfx_prox_dense_ws(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int count_dtype, int layout,
                      void* counts, float* prox, void* workspace, int64_t workspace_bytes, void* stream);
int rfx_prox_dense(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int count_dtype, int layout,
                   void* counts, float* prox, void* stream);

/* rfx_prox_dense for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc).  Same arguments, outputs and errors as rfx_prox_dense,
 * but the bit-plane scratch is a 16 MiB array inside the library (one copy per GPU, held until the
 * process ends), so the call allocates nothing, frees nothing, creates no events (the timing aid does not
 * cover it) and is asynchronous.  Limit: 4 * ceil(B/32) * roundup(N, 256) * roundup4(bits + 1) <= 16 MiB
 * with bits = max(8, ceil(log2(leaf_bound))), e.g. N = 10,000 with B = 500 and leaf_bound <= 2048, or
 * N = 4,096 with B = 1,000 and leaf_bound <= 32,768; a larger problem returns RFX_ERR_CAPACITY and
 * launches nothing.  Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU
 * (different streams or threads) race on it; calls on one stream are ordered and safe.  The array needs no
 * clearing between calls (every word a call reads it has written first). */
int rfx_prox_dense_noalloc(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int count_dtype, int layout,
                           void* counts, float* prox, void* stream);

/* Out-of-bag-only proximity.  With c_b(i) the bootstrap in-bag count of sample i in tree b
 * and OOB_i = {b : c_b(i) = 0} ("Case-wise Bootstrap Tracking"):
 *   num(i,j) = #{b in OOB_i and OOB_j : leaf_b(i) = leaf_b(j)},  den(i,j) = |OOB_i and OOB_j|,
 *   prox(i,j) = num/den in IEEE float32 division, 0 where den = 0, 1 on the diagonal.
 *   inbag [device] uint16 [B][N];  num, den, prox [device] nullable (at least one given);
 *   other arguments as rfx_prox_dense.  Diagonal of num and den in RFX_FULL = |OOB_i|.
 * B <= 65535 (numerator and denominator share one 32-bit counter), else RFX_ERR_UNSUPPORTED.
 * rfx_prox_oob_ws: asynchronous, scratch of rfx_prox_workspace_bytes.  rfx_prox_oob: synchronous. */
int rfx_prox_oob_ws(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int32_t leaf_bound,
                    int count_dtype, int layout, void* num, void* den, float* prox, void* workspace,
                    int64_t workspace_bytes, void* stream);
int rfx_prox_oob(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int32_t leaf_bound,
                 int count_dtype, int layout, void* num, void* den, float* prox, void* stream);

/* Plain and out-of-bag proximity in one pass over the trees (the two share the per-tree leaf
 * comparison, so the fused pass does about 40 % less work than the two calls).  Outputs and their
 * meaning exactly as rfx_prox_dense (counts, prox, in `layout`) and rfx_prox_oob (num, den,
 * prox_oob, in `oob_layout`); at least one output of each kind must be given.  The three counts
 * of a pair share one 32-bit counter, so B <= 1023, else RFX_ERR_UNSUPPORTED (use the two calls).
 * rfx_prox_dense_oob_ws: asynchronous, scratch of rfx_prox_workspace_bytes.  rfx_prox_dense_oob:
 * synchronous. */
int rfx_prox_dense_oob_ws(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int32_t leaf_bound,
                          int count_dtype, int layout, void* counts, float* prox, int oob_layout, void* num, void* den,
                          float* prox_oob, void* workspace, int64_t workspace_bytes, void* stream);
int rfx_prox_dense_oob(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int32_t leaf_bound,
                       int count_dtype, int layout, void* counts, float* prox, int oob_layout, void* num, void* den,
                       float* prox_oob, void* stream);

/* Thresholded sparse proximity ("CPU TriBlock Proximity": only pairs i < j are kept, and only
 * those whose proximity reaches a threshold; values below it are implicit zeros).  The threshold is
 * given as a count, p >= tau <=> cnt >= min_count = ceil(tau B); min_count = 1 keeps every non-zero
 * pair, so the list is then an exact representation of the matrix.
 *   leaf, leaf_bound, count_dtype  as rfx_prox_dense
 *   min_count  >= 1
 *   capacity   entries the output arrays can hold; 0 = only count the qualifying pairs
 *   rows, cols [device] uint32 [capacity]: i and j of each kept pair, i < j
 *   counts     [device] nullable, [capacity] of count_dtype: cnt(i,j), exact
 *   prox       [device] nullable float32 [capacity]: cnt / B in IEEE float32 division
 *   nnz        [host] out: number of qualifying pairs, also when it exceeds the capacity
 * The order of the entries is unspecified (it varies from call to call); every qualifying pair
 * appears exactly once.  B < 2^20, else RFX_ERR_UNSUPPORTED.
 * rfx_prox_sparse (synchronous): when nnz > capacity > 0 the call returns RFX_ERR_CAPACITY and the
 * arrays hold an unspecified subset.
 * rfx_prox_sparse_ws (asynchronous, scratch of rfx_prox_workspace_bytes): nnz is a [device]
 * uint64, 8-byte aligned, that the call clears and the kernels count in; the caller reads it
 * after synchronising and compares it with the capacity itself.
 * Errors: RFX_ERR_NULL, RFX_ERR_INVALID_ARG, RFX_ERR_OVERFLOW, RFX_ERR_OOM, RFX_ERR_CAPACITY. */
int rfx_prox_sparse_ws(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int32_t min_count,
                       int count_dtype, int64_t capacity, uint32_t* rows, uint32_t* cols, void* counts, float* prox,
                       uint64_t* nnz, void* workspace, int64_t workspace_bytes, void* stream);
int rfx_prox_sparse(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int32_t min_count, int count_dtype,
                    int64_t capacity, uint32_t* rows, uint32_t* cols, void* counts, float* prox, int64_t* nnz,
                    void* stream);

/* The same list computed row by row from the samples grouped by leaf instead of by testing all pairs: for every
 * sample i and tree b the members j > i of i's leaf are counted into a row of 16-bit counters, sum over trees and
 * leaves of s (s - 1) / 2 increments in all instead of N^2 B / 2 tests, which pays on deep forests whose leaves are
 * small (N = 500,000, B = 1,000: three orders of magnitude fewer).  Arguments, outputs and errors as rfx_prox_sparse;
 * the entries come out grouped by row.  B <= 4096, B * N < 2^32 and B * leaf_bound < 2^32, else RFX_ERR_UNSUPPORTED.
 * Builds and destroys a grouping (rfx_pv_plan) and 4 B N bytes of scratch inside the call.  Synchronous.
 * rfx_prox_sparse itself chooses between the two by their estimated cost. */
int rfx_prox_sparse_rows(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int32_t min_count,
                         int count_dtype, int64_t capacity, uint32_t* rows, uint32_t* cols, void* counts, float* prox,
                         int64_t* nnz, void* stream);

/* The row-by-row list from an existing grouping (the plan of the implicit product, see rfx_pv_plan_create below), for
 * callers that keep one anyway: no grouping is built and nothing is allocated.  Asynchronous.
 *   plan       built for the leaf ids in question; the call marks entries of its member lists while it runs and takes
 *              the marks out again at the end, so until the call has finished on `stream` the plan must not be used by
 *              work on other streams; work queued on `stream` afterwards finds it as before.
 *   nnz        [device] uint64, 8-byte aligned: cleared by the call, counts every qualifying pair (the caller reads it
 *              after synchronising and compares it with the capacity; beyond the capacity nothing is written).
 *   workspace  [device] rfx_prox_sparse_plan_workspace_bytes (4 B N) bytes, 256-byte aligned.
 * Other arguments and outputs as rfx_prox_sparse_rows.
 * Errors: RFX_ERR_NULL, RFX_ERR_INVALID_ARG, RFX_ERR_UNSUPPORTED (B > 4096), RFX_ERR_CAPACITY (workspace too small). */
typedef struct rfx_pv_plan rfx_pv_plan; /* the grouping of the samples by tree and leaf, see rfx_pv_plan_create */
int rfx_prox_sparse_plan_workspace_bytes(const rfx_pv_plan* plan, int64_t* bytes);
int rfx_prox_sparse_plan(rfx_pv_plan* plan, int32_t min_count, int count_dtype, int64_t capacity, uint32_t* rows,
                         uint32_t* cols, void* counts, float* prox, uint64_t* nnz, void* workspace, int64_t workspace_bytes,
                         void* stream);

/* Case-wise outlier measures from the proximity rows ("Case-wise Proximity"), computed tile by
 * tile without storing the matrix.  With p(i,j) = cnt(i,j) / B:
 *   printed[i] = (1/(N-1)) sum_{j != i, p(i,j) > 0} 1 / p(i,j)^2   the paper's equation; pairs with
 *                p = 0, whose term is undefined, are skipped;
 *   classic[i] = N / sum_{j != i, labels[j] = labels[i]} p(i,j)^2  Breiman and Cutler's raw measure
 *                (all j != i when labels is null); +inf when the sum is 0.
 *   leaf, leaf_bound as rfx_prox_dense;  labels [device] nullable int32 [N];
 *   printed, classic [device] nullable float64 [N] (at least one given).
 * The sum of squares is accumulated as an exact integer; the sum of inverse squares in float64
 * with atomics, so its last bits can differ from call to call.  N >= 2, B < 2^20.
 * rfx_prox_outlier_ws: asynchronous, scratch of rfx_prox_workspace_bytes.  rfx_prox_outlier:
 * synchronous.
 * Errors: RFX_ERR_NULL, RFX_ERR_INVALID_ARG, RFX_ERR_UNSUPPORTED, RFX_ERR_CAPACITY, RFX_ERR_OOM. */
int rfx_prox_outlier_ws(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, const int32_t* labels,
                        double* printed, double* classic, void* workspace, int64_t workspace_bytes, void* stream);
int rfx_prox_outlier(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, const int32_t* labels,
                     double* printed, double* classic, void* stream);

/* Out-of-bag vote ("OOB Error Estimation"): sample i is predicted by the trees whose bootstrap
 * sample missed it (inbag = 0), each voting for the class label of the leaf that holds i;
 * pred[i] = the class with most votes (the lowest class on ties), -1 if i was never out-of-bag.
 *   leaf        [device] uint32 [B][N]
 *   inbag       [device] uint16 [B][N] bootstrap in-bag counts
 *   leaf_class  [device] int32 [B][leaf_stride]: class label of leaf l of tree b at [b][l];
 *               a leaf id >= leaf_stride or a label outside 0..n_classes-1 casts no vote
 *   n_classes   1..128
 *   y           [device] nullable int32 [N] true labels (needed for `wrong`)
 *   votes       [device] nullable uint32 [N][n_classes] out
 *   pred        [device] int32 [N] out
 *   wrong       [host] nullable out: samples with a prediction that differs from y
 *   voted       [host] nullable out: samples that have a prediction
 * The error rate is wrong / voted (the paper's (1/n) sum when every sample was out-of-bag at
 * least once).  Synchronous.  Errors: RFX_ERR_NULL, RFX_ERR_INVALID_ARG, RFX_ERR_OOM. */
int rfx_oob_vote(const uint32_t* leaf, const uint16_t* inbag, const int32_t* leaf_class, int64_t N, int32_t B,
                 int32_t leaf_stride, int32_t n_classes, const int32_t* y, uint32_t* votes, int32_t* pred,
                 int64_t* wrong, int64_t* voted, void* stream);

/* Implicit product Y = P V = (1/B) sum_b Z_b (Z_b^T V), Z_b the N x L_b one-hot leaf
 * membership of tree b, i.e. Y[i,:] = (1/B) sum_b sum_{j : leaf_b(j) = leaf_b(i)} V[j,:];
 * P is never formed.  A plan holds the per-tree grouping of samples by leaf (built once per
 * forest) and the scratch for the per-leaf sums.
 *   rfx_pv_plan_create: leaf [device] uint32 [B][N] (read during the call only), ids < leaf_bound.
 *                       B <= 65535, B * N < 2^32 and B * leaf_bound < 2^32, else
 *                       RFX_ERR_UNSUPPORTED.  Synchronous (it reports a leaf id >= leaf_bound).
 *   rfx_pv_plan_rebuild: regroups an existing plan for new leaf ids of the same N, B and leaf_bound
 *                       without allocating (the plan keeps the scratch of its grouping: 4 B leaf_bound
 *                       min(16, N/4096) bytes).  Synchronous; applications of the old grouping must have
 *                       finished.  After a failed rebuild the plan refuses applications until one succeeds.
 *   rfx_pv_plan_reserve: sizes the per-leaf sums for rank k now (4 B leaf_bound k bytes; waits for
 *                       the device when it has to replace a smaller buffer), so that every later
 *                       application of rank <= k is asynchronous.
 *   rfx_pv_plan_info:   N, B and the rank reserved so far ([host] out, each nullable).
 *   rfx_pv_apply:       V [device] float32 [N][k] in, Y [device] float32 [N][k] out, 1 <= k <= 256,
 *                       V and Y must not overlap.  Asynchronous once the plan's scratch has
 *                       been sized for k (a call with a larger k reserves first).  Part of the work
 *                       runs on a stream the plan owns, forked from and joined back into `stream`
 *                       with events, so work queued on `stream` afterwards sees Y complete; calls
 *                       on one plan from several streams at once race on its scratch.
 *   rfx_prox_matvec:    one-shot convenience: create plan, apply, destroy.  Synchronous. */
int rfx_pv_plan_create(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, rfx_pv_plan** out,
                       void* stream);
int rfx_pv_plan_destroy(rfx_pv_plan* plan);
int rfx_pv_plan_rebuild(rfx_pv_plan* plan, const uint32_t* leaf, void* stream);
int rfx_pv_plan_reserve(rfx_pv_plan* plan, int32_t k);
int rfx_pv_plan_info(const rfx_pv_plan* plan, int64_t* N, int32_t* B, int32_t* k_reserved);
int rfx_pv_apply(rfx_pv_plan* plan, const float* V, int32_t k, float* Y, void* stream);
int rfx_prox_matvec(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, const float* V, int32_t k,
                    float* Y, void* stream);

/* Rank-k factorisation of P by block power iteration, then INT8 factors.
 * P is symmetric positive semi-definite, so the paper's P ~ Q U^T ("QLORA", "Low-Rank
 * Factorization and Quantization Trade-offs") is taken in its symmetric form P ~ A A^T with
 * A = V diag(sqrt(lambda)).  Steps: V <- orth(V0); iters-1 times V <- orth(P V); then
 * Y = P V, H = sym(V^T Y), H = W diag(theta) W^T (theta descending), V <- V W: exactly
 * `iters` applications of P.  Each column of V is then signed so that its largest-magnitude
 * entry is positive, and quantised: s_c = max_i |A_ic| / 127 (1 if the column is zero),
 * Q_ic = clamp(round-half-even(A_ic / s_c), -127, 127), all in float32.
 *   V0      [device] float32 [N][k] start block (full column rank)
 *   eigvals [device] float32 [k] out, descending Ritz values
 *   V       [device] float32 [N][k] out, orthonormal Ritz vectors (before quantisation)
 *   Q       [device] int8 [N][k] out, nullable together with scales
 *   scales  [device] float32 [k] out
 * 1 <= k <= 128, k <= N, iters >= 1.
 * rfx_prox_lowrank (synchronous): builds a plan for the call and destroys it; a block that lost
 * rank (start block or P of rank < k) returns RFX_ERR_INVALID_ARG after the outputs were written.
 * rfx_prox_lowrank_plan (asynchronous): the same on an existing plan whose sums were reserved for
 * rank >= k (rfx_pv_plan_reserve), with scratch of rfx_lowrank_workspace_bytes(N, k);
 *   status  [device] nullable int32 out: 1 if a block lost rank, else 0. */
int rfx_lowrank_workspace_bytes(int64_t N, int32_t k, int64_t* bytes);
int rfx_prox_lowrank_plan(rfx_pv_plan* plan, int32_t k, int32_t iters, const float* V0, float* eigvals, float* V,
                          int8_t* Q, float* scales, int32_t* status, void* workspace, int64_t workspace_bytes,
                          void* stream);
int rfx_prox_lowrank(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int32_t k, int32_t iters,
                     const float* V0, float* eigvals, float* V, int8_t* Q, float* scales, void* stream);

/* The quantisation step of rfx_prox_lowrank on its own (same arithmetic).  Asynchronous. */
int rfx_quantise_int8(const float* V, const float* eigvals, int64_t N, int32_t k, int8_t* Q, float* scales,
                      void* stream);

/* Other encodings of the factor A = V diag(sqrt(lambda)) ("Low-Rank Factorization and Quantization
 * Trade-offs": NF4 (4-bit), INT8 (8-bit), FP16 (16-bit), FP32 (32-bit)).
 *   RFX_ENC_INT8  as rfx_quantise_int8: codes int8 [N][k], scales float32 [k].
 *   RFX_ENC_FP16  codes IEEE binary16 [N][k], round-to-nearest-even; no scales.
 *   RFX_ENC_FP32  codes float32 [N][k]; no scales.
 *   RFX_ENC_NF4   the 4-bit NormalFloat type of the QLoRA paper: 16 fixed levels in [-1, 1] applied to
 *                 values normalised by their block's absolute maximum.  Blocks are 64 consecutive rows
 *                 of one column.  codes uint8 [ceil(N/2)][k]: rows 2i and 2i+1 of a column in the low and
 *                 high nibble (a missing last row holds the zero level); scales float32 [ceil(N/64)][k]
 *                 = block maxima of |A| (1 for an all-zero block).  The nearest level is decided in
 *                 float32 by counting the midpoints of adjacent levels below the normalised value.
 * rfx_factor_sizes: bytes of `codes` and number of floats of `scales` for an encoding ([host] out).
 * rfx_quantise_factor / rfx_dequantise_factor: V, eigvals as rfx_quantise_int8; codes, scales, A
 * [device]; A float32 [N][k] out.  Asynchronous. */
#define RFX_ENC_INT8 0
#define RFX_ENC_FP16 1
#define RFX_ENC_NF4 2
#define RFX_ENC_FP32 3
int rfx_factor_sizes(int encoding, int64_t N, int32_t k, int64_t* code_bytes, int64_t* n_scales);
int rfx_quantise_factor(const float* V, const float* eigvals, int64_t N, int32_t k, int encoding, void* codes,
                        float* scales, void* stream);
int rfx_dequantise_factor(const void* codes, const float* scales, int64_t N, int32_t k, int encoding, float* A,
                          void* stream);

/* 3-D scaling coordinates from the INT8 factors ("GPU-Accelerated 3D MDS from Low-Rank
 * Proximity Matrices", Steps 1-4).  With A^ = Q diag(scales), P^ = A^ A^^T and D = 1 - P^ (the
 * paper's max P - P with max P = 1): G = -1/2 H D2 H, H = I - 11^T/N, D2 = D o D
 * (RFX_MDS_SQUARED) or D (RFX_MDS_LINEAR).  G is applied through the factors only
 * (u = H v, z = D2 u, w = H z, G v = -w/2); the INT8 codes are decoded where they are read.
 * The three algebraically largest eigenpairs are found by simultaneous power iteration on a
 * block of m vectors with a Rayleigh-Ritz step (the power method with deflation of Step 3, done
 * for all vectors at once).  In RFX_MDS_SQUARED mode G can have negative eigenvalues; the
 * iteration runs on G + sigma I with sigma = the largest -theta_min any Rayleigh-Ritz step has
 * seen (0 while every Ritz value of the block is non-negative), which never exceeds
 * |lambda_min(G)| and makes the iteration converge to the largest eigenvalues rather than the
 * largest magnitudes; the reported eigenvalues are those of G.  Coordinates are
 * x_i = (sqrt(l1) v1_i, sqrt(l2) v2_i, sqrt(l3) v3_i), a non-positive eigenvalue giving a zero
 * column; each column is signed so that its largest-magnitude entry is positive.  A block whose
 * rank is below m (G of rank < m, k < m in RFX_MDS_LINEAR mode, dependent columns of x0) is not
 * an error: dependent directions are dropped and their Ritz values are 0.
 *   Q [device] int8 [N][k], scales [device] float32 [k], 1 <= k <= 128
 *   m          block width, 3..32, m <= N (extra vectors speed up convergence)
 *   x0         [device] nullable float32 [N][m] start block; null: the m leading columns of the
 *              factor (the columns of the largest eigenvalues of P nearly span the subspace wanted, so
 *              few applications are left to do), filled up with fixed pseudo-random columns where m > k
 *   coords     [device] float32 [N][3] out;  eigvals [device] float32 [3] out
 * rfx_mds3d (synchronous): max_iters >= 1; tol >= 0: the host looks at the iteration every 2
 *   applications of G and stops when, in the last one, the three leading Ritz values changed by
 *   at most tol * |value|;  iters_done [host] nullable out: applications of G performed.
 * rfx_mds3d_ws (asynchronous, scratch of rfx_mds3d_workspace_bytes(N, k, m, dissim_mode)):
 *   exactly `iters` applications of G;  rel_change [device] nullable float32 out: the largest
 *   relative change of the three leading Ritz values in the last application (inf for iters = 1),
 *   for the caller to judge convergence. */
int rfx_mds3d_workspace_bytes(int64_t N, int32_t k, int32_t m, int dissim_mode, int64_t* bytes);
int rfx_mds3d_ws(const int8_t* Q, const float* scales, int64_t N, int32_t k, int dissim_mode, int32_t m, int32_t iters,
                 const float* x0, float* coords, float* eigvals, float* rel_change, void* workspace,
                 int64_t workspace_bytes, void* stream);
int rfx_mds3d(const int8_t* Q, const float* scales, int64_t N, int32_t k, int dissim_mode, int32_t m,
              int32_t max_iters, float tol, const float* x0, float* coords, float* eigvals,
              int32_t* iters_done, void* stream);
/* The same from a float32 factor A [device] [N][k] (any encoding after rfx_dequantise_factor). */
int rfx_mds3d_factor(const float* A, int64_t N, int32_t k, int dissim_mode, int32_t m, int32_t max_iters, float tol,
                     const float* x0, float* coords, float* eigvals, int32_t* iters_done, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RFX_H */
