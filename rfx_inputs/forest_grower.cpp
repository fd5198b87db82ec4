// Seeded input generator: grows a Breiman-Cutler classification forest on the CPU.
//
// This file produces INPUTS (flattened trees, in-bag counts) that both the CPU
// oracle and the HIP library consume.  It holds none of the proximity path's
// arithmetic (no traversal of finished trees, no pair counting, no products).
//
// What the paper fixes (Methodology: "Classification", "Threshold-based
// Splits", "Case-wise Bootstrap Tracking", "GPU vs. CPU Random Number
// Generation"):
//   * every tree is grown on a with-replacement bootstrap sample of the rows;
//   * at each node a random subset of mtry features is tried and the split
//     with the largest Gini impurity decrease
//         dI = I(parent) - nL/n I(left) - nR/n I(right)
//     is taken, the threshold being one of the feature values present in the
//     node, rows with x <= tau going left and rows with x > tau going right;
//   * the CPU generator is the 32-bit Mersenne Twister and tree b is seeded
//     with iseed + b.
// Readings where the paper is silent: features are drawn without replacement;
// rows are weighted by their in-bag count; the first best split wins (strict
// ">" in draw order, then ascending threshold); if no drawn feature varies in
// the node the remaining features are scanned in index order; a node whose
// rows are identical in every feature becomes a (possibly impure) leaf; trees
// are grown until every leaf is pure.
//
// Build: g++ -O2 -fopenmp -shared -fPIC forest_grower.cpp -o libforest_grower.so
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <random>
#include <vector>
#include <omp.h>

namespace {

struct Tree {
    std::vector<int32_t> feature, left, right, leaf_id, depth;
    std::vector<float> threshold;
    int32_t n_leaves = 0;
};

struct Forest {
    int64_t N = 0;
    int32_t M = 0, B = 0;
    std::vector<Tree> trees;
    std::vector<uint16_t> inbag;       // [B][N]
    std::vector<int32_t> train_leaf;   // [B][N], -1 for out-of-bag rows
};

// Unbiased integer in [0, n) from raw 32-bit generator outputs
// (multiply-shift with rejection), so the stream does not depend on the
// standard library's distribution classes.
inline uint32_t rand_below(std::mt19937& g, uint32_t n) {
    uint64_t m = (uint64_t)g() * n;
    uint32_t lo = (uint32_t)m;
    if (lo < n) {
        uint32_t t = (uint32_t)(-n) % n;
        while (lo < t) {
            m = (uint64_t)g() * n;
            lo = (uint32_t)m;
        }
    }
    return (uint32_t)(m >> 32);
}

struct ValIdx {
    float v;
    int32_t i;
};

struct Split {
    bool found = false;
    double gain = 0.0;
    int32_t feature = -1;
    float tau = 0.0f;
};

double gini(const std::vector<double>& cnt, double n) {
    if (n <= 0.0) return 0.0;
    double s = 0.0;
    for (double c : cnt) s += (c / n) * (c / n);
    return 1.0 - s;
}

// Best threshold of one feature inside one node; updates `best` only on a
// strictly larger gain.  Returns whether the feature varies in the node.
bool scan_feature(const float* X, int32_t M, const int32_t* y, const uint16_t* w, int32_t C,
                  const int32_t* rows, int64_t n_rows, int32_t f, const std::vector<double>& parent_cnt,
                  double parent_n, double parent_gini, std::vector<ValIdx>& buf, std::vector<double>& lcnt,
                  std::vector<double>& rcnt, Split& best) {
    buf.resize(n_rows);
    for (int64_t t = 0; t < n_rows; ++t) buf[t] = {X[(int64_t)rows[t] * M + f], rows[t]};
    std::sort(buf.begin(), buf.end(), [](const ValIdx& a, const ValIdx& b) {
        return a.v < b.v || (a.v == b.v && a.i < b.i);
    });
    if (!(buf.front().v < buf.back().v)) return false;
    std::fill(lcnt.begin(), lcnt.end(), 0.0);
    double nl = 0.0;
    for (int64_t t = 0; t + 1 < n_rows; ++t) {
        int32_t i = buf[t].i;
        lcnt[y[i]] += w[i];
        nl += w[i];
        if (buf[t].v < buf[t + 1].v) {
            double nr = parent_n - nl;
            for (int32_t c = 0; c < C; ++c) rcnt[c] = parent_cnt[c] - lcnt[c];
            double gain = parent_gini - nl / parent_n * gini(lcnt, nl) - nr / parent_n * gini(rcnt, nr);
            if (!best.found || gain > best.gain) {
                best.found = true;
                best.gain = gain;
                best.feature = f;
                best.tau = buf[t].v;
            }
        }
    }
    return true;
}

void grow_tree(const float* X, int64_t N, int32_t M, const int32_t* y, int32_t C, int32_t mtry, uint32_t seed,
               Tree& T, uint16_t* inbag, int32_t* train_leaf) {
    std::mt19937 gen(seed);
    std::memset(inbag, 0, sizeof(uint16_t) * N);
    for (int64_t t = 0; t < N; ++t) inbag[rand_below(gen, (uint32_t)N)]++;
    for (int64_t i = 0; i < N; ++i) train_leaf[i] = -1;

    std::vector<int32_t> rows;
    rows.reserve(N);
    for (int64_t i = 0; i < N; ++i)
        if (inbag[i]) rows.push_back((int32_t)i);

    auto new_node = [&](int32_t d) {
        T.feature.push_back(-1);
        T.left.push_back(-1);
        T.right.push_back(-1);
        T.leaf_id.push_back(-1);
        T.threshold.push_back(0.0f);
        T.depth.push_back(d);
        return (int32_t)T.feature.size() - 1;
    };
    struct Work {
        int32_t node;
        int64_t lo, hi;  // rows[lo, hi)
    };
    std::vector<Work> stack;
    stack.push_back({new_node(0), 0, (int64_t)rows.size()});

    std::vector<int32_t> fperm(M);
    for (int32_t f = 0; f < M; ++f) fperm[f] = f;
    std::vector<double> pcnt(C), lcnt(C), rcnt(C);
    std::vector<ValIdx> buf;
    std::vector<int32_t> tmp;

    while (!stack.empty()) {
        Work wk = stack.back();
        stack.pop_back();
        const int32_t* r = rows.data() + wk.lo;
        int64_t n_rows = wk.hi - wk.lo;
        std::fill(pcnt.begin(), pcnt.end(), 0.0);
        double pn = 0.0;
        for (int64_t t = 0; t < n_rows; ++t) {
            pcnt[y[r[t]]] += inbag[r[t]];
            pn += inbag[r[t]];
        }
        int32_t n_present = 0;
        for (int32_t c = 0; c < C; ++c) n_present += pcnt[c] > 0.0;

        Split best;
        if (n_present > 1) {
            double pg = gini(pcnt, pn);
            // mtry distinct features: partial Fisher-Yates on a persistent permutation.
            for (int32_t t = 0; t < mtry; ++t) {
                uint32_t j = t + rand_below(gen, (uint32_t)(M - t));
                std::swap(fperm[t], fperm[j]);
            }
            for (int32_t t = 0; t < mtry; ++t)
                scan_feature(X, M, y, inbag, C, r, n_rows, fperm[t], pcnt, pn, pg, buf, lcnt, rcnt, best);
            if (!best.found) {
                // None of the drawn features varies here: take the first other one that does.
                std::vector<int32_t> rest(fperm.begin() + mtry, fperm.end());
                std::sort(rest.begin(), rest.end());
                for (int32_t f : rest) {
                    scan_feature(X, M, y, inbag, C, r, n_rows, f, pcnt, pn, pg, buf, lcnt, rcnt, best);
                    if (best.found) break;
                }
            }
        }
        if (!best.found) {
            int32_t id = T.n_leaves++;
            T.leaf_id[wk.node] = id;
            for (int64_t t = 0; t < n_rows; ++t) train_leaf[r[t]] = id;
            continue;
        }
        // Stable partition with the stored float32 threshold: x <= tau goes left.
        tmp.clear();
        int64_t nl = 0;
        int32_t* rw = rows.data() + wk.lo;
        for (int64_t t = 0; t < n_rows; ++t) {
            int32_t i = rw[t];
            if (X[(int64_t)i * M + best.feature] <= best.tau)
                rw[nl++] = i;
            else
                tmp.push_back(i);
        }
        std::copy(tmp.begin(), tmp.end(), rw + nl);
        int32_t d = T.depth[wk.node];
        int32_t L = new_node(d + 1);
        int32_t R = new_node(d + 1);
        T.feature[wk.node] = best.feature;
        T.threshold[wk.node] = best.tau;
        T.left[wk.node] = L;
        T.right[wk.node] = R;
        stack.push_back({R, wk.lo + nl, wk.hi});
        stack.push_back({L, wk.lo, wk.lo + nl});
    }
}

}  // namespace

extern "C" {

// Grows B trees (tree b seeded iseed + b).  X is row-major [N][M] float32, y
// holds class labels in [0, C).  Returns an opaque handle, or null on bad
// arguments.  n_threads <= 0 uses every core.
void* fg_grow(const float* X, int64_t N, int32_t M, const int32_t* y, int32_t C, int32_t B, int32_t mtry,
              uint32_t iseed, int32_t n_threads) {
    if (!X || !y || N <= 0 || N > 0x7fffffff || M <= 0 || C <= 0 || B <= 0 || mtry <= 0 || mtry > M)
        return nullptr;
    for (int64_t i = 0; i < N; ++i)
        if (y[i] < 0 || y[i] >= C) return nullptr;
    Forest* F = new Forest;
    F->N = N;
    F->M = M;
    F->B = B;
    F->trees.resize(B);
    F->inbag.resize((size_t)B * N);
    F->train_leaf.resize((size_t)B * N);
    if (n_threads <= 0) n_threads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
    for (int32_t b = 0; b < B; ++b)
        grow_tree(X, N, M, y, C, mtry, iseed + (uint32_t)b, F->trees[b], F->inbag.data() + (size_t)b * N,
                  F->train_leaf.data() + (size_t)b * N);
    return F;
}

int64_t fg_total_nodes(const void* h) {
    const Forest* F = (const Forest*)h;
    int64_t s = 0;
    for (const Tree& t : F->trees) s += (int64_t)t.feature.size();
    return s;
}

// Copies the forest into caller-allocated arrays (sizes: node_offset B+1,
// per-node arrays fg_total_nodes(), n_leaves B, inbag and train_leaf B*N).
void fg_export(const void* h, int64_t* node_offset, int32_t* feature, float* threshold, int32_t* left,
               int32_t* right, int32_t* leaf_id, int32_t* depth, int32_t* n_leaves, uint16_t* inbag,
               int32_t* train_leaf) {
    const Forest* F = (const Forest*)h;
    int64_t off = 0;
    for (int32_t b = 0; b < F->B; ++b) {
        const Tree& t = F->trees[b];
        size_t n = t.feature.size();
        node_offset[b] = off;
        std::memcpy(feature + off, t.feature.data(), n * sizeof(int32_t));
        std::memcpy(threshold + off, t.threshold.data(), n * sizeof(float));
        std::memcpy(left + off, t.left.data(), n * sizeof(int32_t));
        std::memcpy(right + off, t.right.data(), n * sizeof(int32_t));
        std::memcpy(leaf_id + off, t.leaf_id.data(), n * sizeof(int32_t));
        std::memcpy(depth + off, t.depth.data(), n * sizeof(int32_t));
        n_leaves[b] = t.n_leaves;
        off += (int64_t)n;
    }
    node_offset[F->B] = off;
    std::memcpy(inbag, F->inbag.data(), F->inbag.size() * sizeof(uint16_t));
    std::memcpy(train_leaf, F->train_leaf.data(), F->train_leaf.size() * sizeof(int32_t));
}

void fg_free(void* h) { delete (Forest*)h; }

}  // extern "C"
