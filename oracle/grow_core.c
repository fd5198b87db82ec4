/* CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain sequential growth of Breiman-Cutler classification trees, written from the paper's
 * description (Methodology: bootstrap sample per tree, a random subset of mtry features per node,
 * the split that maximises the Gini impurity decrease
 *     dI = I(parent) - nL/n I(left) - nR/n I(right),
 * thresholds taken from the values present in the node with x <= tau going left ("Threshold-based
 * Splits"), trees grown until the nodes are pure).  Shares no code with the HIP library.
 *
 * What the paper leaves open is fixed as follows:
 *   - Random numbers come from a counter-based generator, so that they do not depend on the order
 *     in which nodes are processed: draw(seed, tree, a, b) = mix(mix(mix(seed ^ (tree+1) K) ^ a) ^ b)
 *     with mix = the output function of splitmix64 and K = 0x9e3779b97f4a7c15; an integer below n
 *     is ((draw >> 32) * n) >> 32.
 *   - Bootstrap: sample t of the tree is row bounded(draw(seed, tree, 0, t), N), t = 0..N-1; a row's
 *     weight is the number of times it was drawn; rows never drawn do not influence growth.
 *   - Nodes are numbered in creation order, breadth first: the children of node v get the next two
 *     numbers when v is split, and nodes are split in numerical order.
 *   - Features of node v: the first mtry entries of a Fisher-Yates shuffle of 0..M-1 whose s-th
 *     swap partner is s + bounded(draw(seed, tree, 1 + v, s), M - s).
 *   - Maximising dI is maximising  sum_c wL_c^2 / nL + sum_c wR_c^2 / nR  (w = class weights of the
 *     two sides); the two sides of a comparison are fractions of integers and are compared exactly
 *     by cross-multiplication, so no rounding decides a split.
 *   - Candidates: every value of the feature present in the node except the largest, in ascending
 *     order, features in draw order; a candidate replaces the best so far only if strictly better.
 *   - If none of the drawn features takes two values in the node, the remaining features are tried
 *     in index order and the first that does is used (with its best threshold); if no feature does,
 *     the node becomes a leaf although it is impure.
 *   - A threshold that is a zero is stored as +0 (x <= tau does not distinguish the two zeros, so the
 *     value present in the node may be either).
 *   - Leaves are numbered 0..L-1 in node order; a leaf's class is the class of largest weight
 *     (lowest class on ties).
 *
 * Build: gcc -O2 -std=c99 -fopenmp -shared -fPIC grow_core.c -o liboracle_grow.so
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef unsigned __int128 u128;

static uint64_t mix(uint64_t z) {
    z += 0x9e3779b97f4a7c15ull;
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}

uint64_t orc_draw(uint64_t seed, uint64_t tree, uint64_t a, uint64_t b) {
    uint64_t h = mix(seed ^ ((tree + 1) * 0x9e3779b97f4a7c15ull));
    h = mix(h ^ a);
    return mix(h ^ b);
}

static uint32_t bounded(uint64_t r, uint32_t n) { return (uint32_t)(((r >> 32) * (uint64_t)n) >> 32); }

typedef struct {
    int64_t n_nodes;
    int32_t n_leaves;
    int32_t* feature;
    float* threshold;
    int32_t* left;
    int32_t* right;
    int32_t* leaf_id;
    int32_t* depth;
    int32_t* leaf_class; /* by leaf id */
    uint16_t* inbag;     /* [N] */
    int32_t* train_leaf; /* [N], -1 for rows not in the bootstrap sample */
} tree_t;

typedef struct {
    int32_t n_trees;
    int64_t N;
    tree_t* trees;
} grown_t;

typedef struct {
    float x;
    int32_t cls;
    uint32_t w;
} item_t;

static int cmp_item(const void* a, const void* b) {
    float xa = ((const item_t*)a)->x, xb = ((const item_t*)b)->x;
    return (xa > xb) - (xa < xb);
}

/* Best threshold of one feature inside a node.  items are sorted by value.  Returns 1 and the
 * best candidate's score (as num / den) and threshold if the feature takes at least two values. */
static int best_of_feature(const item_t* it, int64_t n, int32_t C, uint64_t* wl, uint64_t* wr, u128* best_num,
                           u128* best_den, float* best_thr) {
    int found = 0;
    uint64_t nl = 0, nr = 0;
    for (int32_t c = 0; c < C; ++c) {
        wl[c] = 0;
        wr[c] = 0;
    }
    for (int64_t p = 0; p < n; ++p) {
        wr[it[p].cls] += it[p].w;
        nr += it[p].w;
    }
    for (int64_t p = 0; p + 1 < n; ++p) {
        wl[it[p].cls] += it[p].w;
        wr[it[p].cls] -= it[p].w;
        nl += it[p].w;
        nr -= it[p].w;
        if (!(it[p].x < it[p + 1].x)) continue; /* not the last row of its value */
        uint64_t a = 0, b = 0;
        for (int32_t c = 0; c < C; ++c) {
            a += wl[c] * wl[c];
            b += wr[c] * wr[c];
        }
        /* a / nl + b / nr = (a nr + b nl) / (nl nr) */
        u128 num = (u128)a * nr + (u128)b * nl;
        u128 den = (u128)nl * nr;
        if (!found || num * *best_den > *best_num * den) {
            found = 1;
            *best_num = num;
            *best_den = den;
            *best_thr = it[p].x + 0.0f; /* a zero threshold is stored as +0 */
        }
    }
    return found;
}

static int grow_tree(const float* X, int64_t N, int32_t M, const int32_t* y, int32_t C, int32_t mtry, uint64_t seed,
                     int32_t tree, tree_t* T) {
    int64_t cap = 2 * N + 1;
    T->feature = malloc(sizeof(int32_t) * cap);
    T->threshold = malloc(sizeof(float) * cap);
    T->left = malloc(sizeof(int32_t) * cap);
    T->right = malloc(sizeof(int32_t) * cap);
    T->leaf_id = malloc(sizeof(int32_t) * cap);
    T->depth = malloc(sizeof(int32_t) * cap);
    T->leaf_class = malloc(sizeof(int32_t) * cap);
    T->inbag = calloc(N, sizeof(uint16_t));
    T->train_leaf = malloc(sizeof(int32_t) * N);
    int64_t* start = malloc(sizeof(int64_t) * cap);
    int64_t* count = malloc(sizeof(int64_t) * cap);
    int64_t* rows = malloc(sizeof(int64_t) * N);
    int64_t* tmp = malloc(sizeof(int64_t) * N);
    item_t* items = malloc(sizeof(item_t) * N);
    int32_t* perm = malloc(sizeof(int32_t) * M);
    uint64_t* wl = malloc(sizeof(uint64_t) * C);
    uint64_t* wr = malloc(sizeof(uint64_t) * C);
    uint64_t* tot = malloc(sizeof(uint64_t) * C);
    if (!T->feature || !T->threshold || !T->left || !T->right || !T->leaf_id || !T->depth || !T->leaf_class || !T->inbag ||
        !T->train_leaf || !start || !count || !rows || !tmp || !items || !perm || !wl || !wr || !tot)
        return -1;

    for (int64_t t = 0; t < N; ++t) T->inbag[bounded(orc_draw(seed, tree, 0, t), (uint32_t)N)] += 1;
    int64_t n_in = 0;
    for (int64_t i = 0; i < N; ++i) {
        T->train_leaf[i] = -1;
        if (T->inbag[i]) rows[n_in++] = i;
    }
    int64_t n_nodes = 1;
    int32_t n_leaves = 0;
    start[0] = 0;
    count[0] = n_in;
    T->depth[0] = 0;
    for (int64_t v = 0; v < n_nodes; ++v) {
        const int64_t s = start[v], n = count[v];
        for (int32_t c = 0; c < C; ++c) tot[c] = 0;
        for (int64_t p = 0; p < n; ++p) tot[y[rows[s + p]]] += T->inbag[rows[s + p]];
        int32_t n_present = 0, top = 0;
        for (int32_t c = 0; c < C; ++c) {
            n_present += tot[c] > 0;
            if (tot[c] > tot[top]) top = c;
        }
        int have = 0, best_f = -1;
        float best_thr = 0.0f;
        if (n_present > 1) {
            for (int32_t f = 0; f < M; ++f) perm[f] = f;
            for (int32_t q = 0; q < mtry; ++q) {
                int32_t j = q + (int32_t)bounded(orc_draw(seed, tree, 1 + (uint64_t)v, q), (uint32_t)(M - q));
                int32_t sw = perm[q];
                perm[q] = perm[j];
                perm[j] = sw;
            }
            u128 best_num = 0, best_den = 1;
            for (int32_t q = 0; q < mtry; ++q) {
                const int32_t f = perm[q];
                for (int64_t p = 0; p < n; ++p) {
                    items[p].x = X[rows[s + p] * M + f];
                    items[p].cls = y[rows[s + p]];
                    items[p].w = T->inbag[rows[s + p]];
                }
                qsort(items, n, sizeof(item_t), cmp_item);
                u128 num = 0, den = 1;
                float thr = 0.0f;
                if (best_of_feature(items, n, C, wl, wr, &num, &den, &thr) && (!have || num * best_den > best_num * den)) {
                    have = 1;
                    best_num = num;
                    best_den = den;
                    best_thr = thr;
                    best_f = f;
                }
            }
            if (!have) {
                /* the features that were not drawn, in index order: the first that can split */
                for (int32_t f = 0; f < M && !have; ++f) {
                    int drawn = 0;
                    for (int32_t q = 0; q < mtry; ++q) drawn |= perm[q] == f;
                    if (drawn) continue;
                    for (int64_t p = 0; p < n; ++p) {
                        items[p].x = X[rows[s + p] * M + f];
                        items[p].cls = y[rows[s + p]];
                        items[p].w = T->inbag[rows[s + p]];
                    }
                    qsort(items, n, sizeof(item_t), cmp_item);
                    u128 num = 0, den = 1;
                    if (best_of_feature(items, n, C, wl, wr, &num, &den, &best_thr)) {
                        have = 1;
                        best_f = f;
                    }
                }
            }
        }
        if (!have) {
            T->feature[v] = -1;
            T->threshold[v] = 0.0f;
            T->left[v] = -1;
            T->right[v] = -1;
            T->leaf_id[v] = n_leaves;
            T->leaf_class[n_leaves] = top;
            for (int64_t p = 0; p < n; ++p) T->train_leaf[rows[s + p]] = n_leaves;
            ++n_leaves;
            continue;
        }
        /* stable partition: rows with x <= tau first */
        int64_t nl = 0, nr = 0;
        for (int64_t p = 0; p < n; ++p) {
            if (X[rows[s + p] * M + best_f] <= best_thr)
                rows[s + nl++] = rows[s + p];
            else
                tmp[nr++] = rows[s + p];
        }
        memcpy(rows + s + nl, tmp, sizeof(int64_t) * nr);
        T->feature[v] = best_f;
        T->threshold[v] = best_thr;
        T->leaf_id[v] = -1;
        T->left[v] = (int32_t)n_nodes;
        T->right[v] = (int32_t)n_nodes + 1;
        start[n_nodes] = s;
        count[n_nodes] = nl;
        start[n_nodes + 1] = s + nl;
        count[n_nodes + 1] = nr;
        T->depth[n_nodes] = T->depth[n_nodes + 1] = T->depth[v] + 1;
        n_nodes += 2;
    }
    T->n_nodes = n_nodes;
    T->n_leaves = n_leaves;
    free(start);
    free(count);
    free(rows);
    free(tmp);
    free(items);
    free(perm);
    free(wl);
    free(wr);
    free(tot);
    return 0;
}

static void free_tree(tree_t* T) {
    free(T->feature);
    free(T->threshold);
    free(T->left);
    free(T->right);
    free(T->leaf_id);
    free(T->depth);
    free(T->leaf_class);
    free(T->inbag);
    free(T->train_leaf);
}

void orc_grown_free(void* h) {
    grown_t* g = h;
    if (!g) return;
    for (int32_t b = 0; b < g->n_trees; ++b) free_tree(&g->trees[b]);
    free(g->trees);
    free(g);
}

/* Grows trees first_tree .. first_tree + n_trees - 1 (the tree number enters the random draws).
 * X [N][M] row-major, y [N] in 0..C-1, 1 <= mtry <= M, N < 2^20.  Returns a handle or NULL. */
void* orc_grow(const float* X, int64_t N, int32_t M, const int32_t* y, int32_t C, int32_t first_tree, int32_t n_trees,
               int32_t mtry, uint64_t seed) {
    if (N < 1 || N >= (1 << 20) || M < 1 || C < 1 || n_trees < 1 || mtry < 1 || mtry > M) return NULL;
    for (int64_t i = 0; i < N; ++i)
        if (y[i] < 0 || y[i] >= C) return NULL;
    grown_t* g = calloc(1, sizeof(grown_t));
    if (!g) return NULL;
    g->n_trees = n_trees;
    g->N = N;
    g->trees = calloc(n_trees, sizeof(tree_t));
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
    for (int32_t b = 0; b < n_trees; ++b) bad |= grow_tree(X, N, M, y, C, mtry, seed, first_tree + b, &g->trees[b]) != 0;
    if (bad) {
        orc_grown_free(g);
        return NULL;
    }
    return g;
}

int64_t orc_grown_total_nodes(const void* h) {
    const grown_t* g = h;
    int64_t n = 0;
    for (int32_t b = 0; b < g->n_trees; ++b) n += g->trees[b].n_nodes;
    return n;
}

int32_t orc_grown_max_leaves(const void* h) {
    const grown_t* g = h;
    int32_t m = 0;
    for (int32_t b = 0; b < g->n_trees; ++b) m = g->trees[b].n_leaves > m ? g->trees[b].n_leaves : m;
    return m;
}

/* node arrays concatenated over trees; leaf_class [B][max_leaves] (-1 past a tree's last leaf) */
void orc_grown_export(const void* h, int64_t* node_offset, int32_t* feature, float* threshold, int32_t* left,
                      int32_t* right, int32_t* leaf_id, int32_t* depth, int32_t* n_leaves, uint16_t* inbag,
                      int32_t* train_leaf, int32_t* leaf_class) {
    const grown_t* g = h;
    const int32_t ml = orc_grown_max_leaves(h);
    int64_t off = 0;
    for (int32_t b = 0; b < g->n_trees; ++b) {
        const tree_t* T = &g->trees[b];
        node_offset[b] = off;
        memcpy(feature + off, T->feature, sizeof(int32_t) * T->n_nodes);
        memcpy(threshold + off, T->threshold, sizeof(float) * T->n_nodes);
        memcpy(left + off, T->left, sizeof(int32_t) * T->n_nodes);
        memcpy(right + off, T->right, sizeof(int32_t) * T->n_nodes);
        memcpy(leaf_id + off, T->leaf_id, sizeof(int32_t) * T->n_nodes);
        memcpy(depth + off, T->depth, sizeof(int32_t) * T->n_nodes);
        n_leaves[b] = T->n_leaves;
        memcpy(inbag + (int64_t)b * g->N, T->inbag, sizeof(uint16_t) * g->N);
        memcpy(train_leaf + (int64_t)b * g->N, T->train_leaf, sizeof(int32_t) * g->N);
        for (int32_t l = 0; l < ml; ++l) leaf_class[(int64_t)b * ml + l] = l < T->n_leaves ? T->leaf_class[l] : -1;
        off += T->n_nodes;
    }
    node_offset[g->n_trees] = off;
}
