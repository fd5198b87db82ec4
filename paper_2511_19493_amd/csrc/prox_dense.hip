// Dense proximity: cnt(i,j) = #{b : leaf_b(i) = leaf_b(j)} and its out-of-bag-only variant
// (paper, "Proximity Matrices", p(i,j) = (1/B) sum_b I(node_b(i) = node_b(j)); out-of-bag sets
// from "Case-wise Bootstrap Tracking").
//
// The N^2 B / 2 equality tests are integer-ALU bound, so the leaf ids are first transposed
// into bit planes: for a group of 32 trees and a sample, word p holds bit p of the sample's
// 32 leaf ids (one tree per bit lane).  Two samples differ in tree t iff some plane differs in
// bit t, so one 3-input boolean op per plane (t | (a ^ b)) followed by one population count
// tests 32 trees at once: (P + 1) / 32 vector ops per test for P-bit leaf ids, against 2 ops per
// test for a compare-and-add on 32-bit ids.  Matches = B - mismatches; padding trees and
// padding samples have all planes zero and never mismatch.
//
// Work decomposition: a wave owns 256 "a" samples (4 consecutive per lane, their planes in
// vector registers, reloaded per tree group) and J "b" samples whose planes are wave-uniform
// and therefore come in through the scalar data path as SGPR operands; the R x J mismatch
// counters live in vector registers for the whole tree loop and are written once.  Four waves
// of a workgroup share the a samples (L1 hits) and take consecutive b ranges.  Only tile pairs
// on or below the diagonal are launched.
//
// The same tile loop also feeds a thresholded sparse output (paper, "CPU TriBlock Proximity":
// strict upper triangle, only values that reach a threshold): instead of writing its tile, a wave
// compacts the pairs whose count reaches min_count and appends them to a coordinate list.
#include <algorithm>
#include <mutex>
#include <optional>

#include "common.h"

namespace {

#ifndef RFX_R
#define RFX_R 4
#endif
#ifndef RFX_B_PREFETCH
#define RFX_B_PREFETCH 1
#endif
constexpr int kR = RFX_R;       // a samples per lane
constexpr int kATile = 64 * kR; // a samples per wave / workgroup
constexpr int kWaves = 4;

__host__ __device__ constexpr int plane_stride(int P) { return (P + 1 + 3) & ~3; }  // words per (group, sample)

// ---------------------------------------------------------------------------------------------
// leaf[B][N] (+ inbag[B][N]) -> planes[G][Npad][PS]; word P of a sample is its out-of-bag mask.
__global__ __launch_bounds__(256) void pack_planes_kernel(const uint32_t* __restrict__ leaf,
                                                         const uint16_t* __restrict__ inbag, int64_t N, int32_t B,
                                                         int64_t Npad, int32_t P, int32_t PS,
                                                         uint32_t* __restrict__ planes) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int g = blockIdx.y;
    if (i >= Npad) return;
    uint32_t w[25];
#pragma unroll
    for (int p = 0; p < 25; ++p) w[p] = 0;
    uint32_t oob = 0;
    if (i < N) {
        const int nb = min(32, B - g * 32);
        for (int t = 0; t < nb; ++t) {
            const int64_t at = (int64_t)(g * 32 + t) * N + i;
            const uint32_t id = leaf[at];
#pragma unroll
            for (int p = 0; p < 25; ++p) w[p] |= ((id >> p) & 1u) << t;
            if (inbag) oob |= (inbag[at] == 0 ? 1u : 0u) << t;
        }
    }
    uint32_t* dst = planes + ((int64_t)g * Npad + i) * PS;
#pragma unroll
    for (int p = 0; p < 25; ++p)
        if (p < P) dst[p] = w[p];
    dst[P] = oob;
    for (int p = P + 1; p < PS; ++p) dst[p] = 0;
}

struct TileOut {
    void* counts;  // plain: counts; out-of-bag: num
    void* den;     // out-of-bag only
    float* prox;
    int64_t N;
    int32_t B;
    int32_t u16;     // counts / num / den are uint16
    int32_t packed;  // strict-upper packed layout
    int32_t use_tab; // quotient table in LDS (set by the launcher)
    // sparse output: coordinate triplets appended at *sp_cursor; counts / prox are indexed by entry
    uint32_t* sp_rows;
    uint32_t* sp_cols;
    unsigned long long* sp_cursor;
    unsigned long long sp_capacity;
    uint32_t sp_min_count;
    // outlier sums, per sample: sum over the other samples of (B / cnt)^2 where cnt > 0, and of cnt^2
    // over the other samples with the same label (all others when there are no labels)
    double* o_inv;
    unsigned long long* o_sq;
    const int32_t* o_labels;
};

__device__ __forceinline__ int64_t packed_index(int64_t i, int64_t j, int64_t N) {
    return i * N - i * (i + 1) / 2 + (j - i - 1);
}

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// The outputs are written once and never read back by the kernel: streaming (non-temporal) stores
// keep them from displacing the bit planes in L2.
#ifndef RFX_NT_STORES
#define RFX_NT_STORES 1
#endif
template <class T>
__device__ __forceinline__ void stream_store(T* p, T v) {
#if RFX_NT_STORES
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

__device__ __forceinline__ void store_count(void* base, int32_t u16, int64_t at, uint32_t v) {
    if (u16)
        stream_store(static_cast<uint16_t*>(base) + at, (uint16_t)v);
    else
        stream_store(static_cast<uint32_t*>(base) + at, v);
}

// 4 consecutive counts at base[at .. at+3]; `at` is a multiple of 4 and the row start is 16-byte aligned
__device__ __forceinline__ void store4_count(void* base, int32_t u16, int64_t at, const uint32_t (&v)[4]) {
    if (u16)
        stream_store(reinterpret_cast<u32x2_t*>(static_cast<uint16_t*>(base) + at), u32x2_t{v[0] | (v[1] << 16), v[2] | (v[3] << 16)});
    else
        stream_store(reinterpret_cast<u32x4_t*>(static_cast<uint32_t*>(base) + at), u32x4_t{v[0], v[1], v[2], v[3]});
}

__device__ __forceinline__ void store4_float(float* base, int64_t at, const float (&p)[4]) {
    stream_store(reinterpret_cast<f32x4_t*>(base + at), f32x4_t{p[0], p[1], p[2], p[3]});
}

// Writes one wave tile.  acc[r][j] belongs to the pair (a_tile + 4*lane + r, b0 + j): the mismatch
// count (plain), or the out-of-bag numerator in bits 0..15 and denominator in bits 16..31.  `tr` is
// this wave's LDS transposition buffer: 64 rows of J + 4 words.
// (x << kShift) + y in one vector instruction
template <int kShift>
__device__ __forceinline__ uint32_t shift_add(uint32_t x, uint32_t y) {
    uint32_t d;
    asm("v_lshl_add_u32 %0, %1, %2, %3" : "=v"(d) : "v"(x), "n"(kShift), "v"(y));
    return d;
}

// What a raw counter means.  kField 0: the mismatch count (plain), or out-of-bag numerator | denominator
// << 16.  The fused kernel keeps three 10-bit fields in one counter (mismatches | numerator << 10 |
// denominator << 20); kField 1 reads its plain part, kField 2 its out-of-bag part.
template <bool kOob, int kField>
__device__ __forceinline__ uint32_t count_of(uint32_t raw, uint32_t B) {
    if (kField == 1) return B - (raw & 1023u);
    if (kField == 2) return (raw >> 10) & 1023u;
    return kOob ? (raw & 0xffffu) : B - raw;
}
template <bool kOob, int kField>
__device__ __forceinline__ uint32_t den_of(uint32_t raw) {
    if (kField == 2) return raw >> 20;
    return kOob ? (raw >> 16) : 0u;
}

template <int J, bool kOob, bool kTab, int kField = 0>
__device__ __forceinline__ void write_tile(const TileOut& out, const float* tab, uint32_t* tr, int lane, int64_t a_tile,
                                           int64_t b0, const uint32_t (&acc)[kR][J]) {
    static_assert(kR == 4 && J % 4 == 0 && 256 % J == 0, "tile shape assumed by the vector stores");
    const int64_t N = out.N;
    const float Bf = (float)out.B;
    const int64_t a0 = a_tile + kR * lane;
    // proximity value of a plain count: exact IEEE quotient, from the LDS table when there is one
    auto quotient = [&](uint32_t c) -> float { return kTab ? tab[c] : (float)c / Bf; };
    auto oob_quotient = [&](uint32_t c, uint32_t d, bool diag) -> float {
        return diag ? 1.0f : (d ? (float)c / (float)d : 0.0f);
    };

    if (!out.packed && (N & 3) == 0 && b0 + J <= N) {
        // Full layout, interior tile.  Row b of the output takes this lane's 4 consecutive a values as
        // one 16-byte (8-byte for uint16) store, contiguous across lanes.
        if (a0 < N) {
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const int64_t at = (b0 + j) * N + a0;
                uint32_t c[kR], d[kR];
                float p[kR];
#pragma unroll
                for (int r = 0; r < kR; ++r) {
                    c[r] = count_of<kOob, kField>(acc[r][j], (uint32_t)out.B);
                    d[r] = den_of<kOob, kField>(acc[r][j]);
                    p[r] = kOob ? oob_quotient(c[r], d[r], a0 + r == b0 + j) : quotient(c[r]);
                }
                if (out.counts) store4_count(out.counts, out.u16, at, c);
                if (kOob && out.den) store4_count(out.den, out.u16, at, d);
                if (out.prox) store4_float(out.prox, at, p);
                __builtin_amdgcn_sched_barrier(0);  // keep each store's address arithmetic next to it
            }
        }
        // Mirrored entries: row a takes J consecutive values.  They are transposed through LDS, one r
        // at a time, so that J/4 adjacent lanes write one row's J values as a contiguous run instead of
        // every lane writing 16-byte pieces of a row of its own.
        constexpr int TS = J + 4;     // LDS words per source lane
        constexpr int LPR = J / 4;    // lanes per row when reading back
        constexpr int RPI = 64 / LPR; // rows per read instruction
#pragma unroll
        for (int r = 0; r < kR; ++r) {
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int q = 0; q < J / 4; ++q)
                *reinterpret_cast<uint4*>(tr + lane * TS + 4 * q) =
                    make_uint4(acc[r][4 * q], acc[r][4 * q + 1], acc[r][4 * q + 2], acc[r][4 * q + 3]);
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int q = 0; q < J / 4; ++q) {
                const int row = q * RPI + lane / LPR;  // source lane whose values this lane writes out
                const int col = 4 * (lane % LPR);
                const int64_t a = a_tile + kR * row + r;
                const uint4 v = *reinterpret_cast<const uint4*>(tr + row * TS + col);
                if (a < N) {
                    const int64_t mt = a * N + b0 + col;
                    const uint32_t raw[4] = {v.x, v.y, v.z, v.w};
                    uint32_t c[4], d[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        c[e] = count_of<kOob, kField>(raw[e], (uint32_t)out.B);
                        d[e] = den_of<kOob, kField>(raw[e]);
                    }
                    if (out.counts) store4_count(out.counts, out.u16, mt, c);
                    if (kOob && out.den) store4_count(out.den, out.u16, mt, d);
                    if (out.prox) {
                        float p[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            p[e] = kOob ? oob_quotient(c[e], d[e], a == b0 + col + e) : quotient(c[e]);
                        store4_float(out.prox, mt, p);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        return;
    }

    if (out.packed && b0 + J <= a_tile && a_tile + kATile <= N) {
        // Packed layout, tile strictly below the diagonal and inside the matrix.  Row b of the packed
        // triangle holds this wave's 256 a values as one contiguous run, but the run starts at an
        // arbitrary element offset.  With phi = offset mod 4, every lane builds the aligned group of 4
        // that starts phi elements before its own values from its left neighbour's last phi values and
        // its own first 4 - phi, and stores it as one vector; lane 0 writes only its own part of the
        // first group and lane 63 appends the last phi values one by one.
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int64_t b = b0 + j;
            const int64_t o = packed_index(b, a_tile, N);  // packed position of (b, a_tile)
            const int phi = (int)(o & 3);
            uint32_t c[kR], d[kR];
            float p[kR];
#pragma unroll
            for (int r = 0; r < kR; ++r) {
                c[r] = count_of<kOob, kField>(acc[r][j], (uint32_t)out.B);
                d[r] = den_of<kOob, kField>(acc[r][j]);
                p[r] = kOob ? oob_quotient(c[r], d[r], false) : quotient(c[r]);
            }
            // w[e] = element at aligned position 4*lane + e of the run shifted right by phi
            auto shifted = [&](const uint32_t (&own)[kR], uint32_t (&w)[kR]) {
                uint32_t prev[kR];
#pragma unroll
                for (int r = 0; r < kR; ++r) prev[r] = __shfl_up(own[r], 1);
#pragma unroll
                for (int e = 0; e < kR; ++e) {
                    // candidates for phi = 0, 1, 2, 3: own[e], then one further to the left each time
                    const uint32_t s0 = own[e];
                    const uint32_t s1 = e >= 1 ? own[e - 1] : prev[3 + e];
                    const uint32_t s2 = e >= 2 ? own[e - 2] : prev[2 + e];
                    const uint32_t s3 = e >= 3 ? own[e - 3] : prev[1 + e];
                    w[e] = phi == 0 ? s0 : (phi == 1 ? s1 : (phi == 2 ? s2 : s3));
                }
            };
            auto emit = [&](auto* base, const uint32_t (&own)[kR], auto store4, auto store1) {
                uint32_t w[kR];
                shifted(own, w);
                const int64_t at = o - phi + 4 * lane;  // aligned group of this lane
                if (lane > 0 || phi == 0) {
                    store4(base, at, w);
                } else {
#pragma unroll
                    for (int e = 0; e < kR; ++e)
                        if (e >= phi) store1(base, at + e, w[e]);
                }
                if (lane == 63) {
#pragma unroll
                    for (int e = 0; e < kR - 1; ++e)
                        if (e < phi) store1(base, at + 4 + e, own[kR - phi + e]);
                }
            };
            auto count4 = [&](void* base, int64_t at, const uint32_t (&w)[kR]) { store4_count(base, out.u16, at, w); };
            auto count1 = [&](void* base, int64_t at, uint32_t v) { store_count(base, out.u16, at, v); };
            if (out.counts) emit(out.counts, c, count4, count1);
            if (kOob && out.den) emit(out.den, d, count4, count1);
            if (out.prox) {
                uint32_t bits[kR];
#pragma unroll
                for (int r = 0; r < kR; ++r) bits[r] = __float_as_uint(p[r]);
                auto float4s = [&](float* base, int64_t at, const uint32_t (&w)[kR]) {
                    const float f[4] = {__uint_as_float(w[0]), __uint_as_float(w[1]), __uint_as_float(w[2]), __uint_as_float(w[3])};
                    store4_float(base, at, f);
                };
                auto float1 = [&](float* base, int64_t at, uint32_t v) { stream_store(base + at, __uint_as_float(v)); };
                emit(out.prox, bits, float4s, float1);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        return;
    }

    // Ragged edge tiles, tiles on the diagonal of the packed layout, or N not a multiple of 4:
    // element-wise stores.
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int64_t b = b0 + j;
        if (b >= N) break;
#pragma unroll
        for (int r = 0; r < kR; ++r) {
            const int64_t a = a0 + r;
            if (a >= N) continue;
            uint32_t c = count_of<kOob, kField>(acc[r][j], (uint32_t)out.B);
            uint32_t d = kOob ? den_of<kOob, kField>(acc[r][j]) : (uint32_t)out.B;
            float p;
            if (a == b)
                p = 1.0f;
            else if (kOob)
                p = d ? (float)c / (float)d : 0.0f;
            else
                p = quotient(c);
            if (out.packed) {
                if (b < a) {
                    const int64_t at = packed_index(b, a, N);
                    if (out.counts) store_count(out.counts, out.u16, at, c);
                    if (kOob && out.den) store_count(out.den, out.u16, at, d);
                    if (out.prox) stream_store(out.prox + at, p);
                }
            } else {
                const int64_t at = b * N + a, mt = a * N + b;
                if (out.counts) {
                    store_count(out.counts, out.u16, at, c);
                    store_count(out.counts, out.u16, mt, c);
                }
                if (kOob && out.den) {
                    store_count(out.den, out.u16, at, d);
                    store_count(out.den, out.u16, mt, d);
                }
                if (out.prox) {
                    stream_store(out.prox + at, p);
                    stream_store(out.prox + mt, p);
                }
            }
        }
    }
}

// Sparse epilogue.  Keeps the pairs (i = b, j = a) of this wave's tile with i < j < N whose count
// reaches sp_min_count and appends (i, j, count[, count / B]) to the coordinate list.  One 64-bit
// atomic per wave reserves the run; the kept pairs are then compacted through the wave's LDS
// buffer, 4 b samples at a time (at most 1024 pairs, one word each: count << 12 | j_local << 8 |
// a_local), and copied out with contiguous stores.  A run that would pass the capacity is counted
// but not stored.
template <int J>
__device__ __forceinline__ void emit_tile(const TileOut& out, uint32_t* tr, int lane, int64_t a_tile, int64_t b0,
                                          const uint32_t (&acc)[kR][J]) {
    static_assert(kR == 4 && J == 16, "one keep bit per pair held by a lane; 8-bit a_local, 4-bit j_local");
    const int64_t N = out.N;
    const int64_t a0 = a_tile + kR * lane;
    uint64_t keep = 0;  // bit 4*j + r
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int r = 0; r < kR; ++r) {
            const uint32_t c = (uint32_t)out.B - acc[r][j];
            const bool k = a0 + r < N && b0 + j < a0 + r && c >= out.sp_min_count;
            keep |= (uint64_t)(k ? 1u : 0u) << (4 * j + r);
        }
    auto wave_scan = [&](uint32_t n, uint32_t& excl, uint32_t& total) {
        uint32_t incl = n;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t t = __shfl_up(incl, off);
            if (lane >= off) incl += t;
        }
        excl = incl - n;
        total = __shfl(incl, 63);
    };
    uint32_t excl, total;
    wave_scan((uint32_t)__builtin_popcountll(keep), excl, total);
    if (total == 0) return;
    unsigned long long base = 0;
    if (lane == 0) base = atomicAdd(out.sp_cursor, (unsigned long long)total);
    base = ((unsigned long long)(uint32_t)__shfl((int)(base >> 32), 0) << 32) | (uint32_t)__shfl((int)(uint32_t)base, 0);
    if (base + total > out.sp_capacity) return;
    const float Bf = (float)out.B;
#pragma unroll
    for (int q = 0; q < J / 4; ++q) {
        const uint32_t kq = (uint32_t)(keep >> (16 * q)) & 0xffffu;
        uint32_t exq, totq;
        wave_scan((uint32_t)__builtin_popcount(kq), exq, totq);
        __builtin_amdgcn_wave_barrier();
        uint32_t pos = exq;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int r = 0; r < kR; ++r)
                if ((kq >> (4 * jj + r)) & 1u) {
                    const uint32_t c = (uint32_t)out.B - acc[r][4 * q + jj];
                    tr[pos++] = (c << 12) | (uint32_t)((4 * q + jj) << 8) | (uint32_t)(kR * lane + r);
                }
        __builtin_amdgcn_wave_barrier();
        for (uint32_t t = lane; t < totq; t += 64) {
            const uint32_t w = tr[t];
            const unsigned long long e = base + t;
            const uint32_t c = w >> 12;
            stream_store(out.sp_rows + e, (uint32_t)(b0 + ((w >> 8) & 15u)));
            stream_store(out.sp_cols + e, (uint32_t)(a_tile + (w & 255u)));
            if (out.counts) store_count(out.counts, out.u16, (int64_t)e, c);
            if (out.prox) stream_store(out.prox + e, (float)c / Bf);
        }
        base += totq;
    }
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
__device__ __forceinline__ unsigned long long wave_sum(unsigned long long v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// Outlier epilogue (paper, "Case-wise Proximity": per-sample sums over the proximity row).  Every
// pair i < j of the tile adds f(cnt) to both of its samples: the b side is summed over the wave and
// added by one lane, the a side is first combined over the workgroup's four waves in LDS.  The sum of
// squares is an exact integer; the sum of inverse squares is float64 and its rounding depends on
// the order in which the workgroups' atomics arrive.
template <int J>
__device__ __forceinline__ void outlier_tile(const TileOut& out, uint32_t* lds, int lane, int wave, int64_t a_tile,
                                             int64_t b0, const uint32_t (&acc)[kR][J]) {
    const int64_t N = out.N;
    const int64_t a0 = a_tile + kR * lane;
    const double Bd = (double)out.B;
    int32_t la[kR];
#pragma unroll
    for (int r = 0; r < kR; ++r) la[r] = (out.o_labels && a0 + r < N) ? out.o_labels[a0 + r] : 0;
    double inv_a[kR];
    unsigned long long sq_a[kR];
#pragma unroll
    for (int r = 0; r < kR; ++r) {
        inv_a[r] = 0.0;
        sq_a[r] = 0;
    }
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int64_t b = b0 + j;
        const int32_t lb = (out.o_labels && b < N) ? out.o_labels[b] : 0;
        double inv_b = 0.0;
        unsigned long long sq_b = 0;
#pragma unroll
        for (int r = 0; r < kR; ++r) {
            const int64_t a = a0 + r;
            const uint32_t c = (uint32_t)out.B - acc[r][j];
            if (a < N && b < a && c > 0) {
                if (out.o_inv) {
                    const double q = Bd / (double)c;
                    inv_a[r] += q * q;
                    inv_b += q * q;
                }
                if (out.o_sq && (!out.o_labels || la[r] == lb)) {
                    const unsigned long long sq = (unsigned long long)c * c;
                    sq_a[r] += sq;
                    sq_b += sq;
                }
            }
        }
        inv_b = wave_sum(inv_b);
        sq_b = wave_sum(sq_b);
        if (lane == 0 && b < N) {
            if (out.o_inv && inv_b != 0.0) unsafeAtomicAdd(out.o_inv + b, inv_b);
            if (out.o_sq && sq_b != 0) atomicAdd(out.o_sq + b, sq_b);
        }
    }
    double* l_inv = reinterpret_cast<double*>(lds);                                               // [kWaves][kATile]
    unsigned long long* l_sq = reinterpret_cast<unsigned long long*>(lds) + kWaves * kATile;   // [kWaves][kATile]
#pragma unroll
    for (int r = 0; r < kR; ++r) {
        l_inv[wave * kATile + kR * lane + r] = inv_a[r];
        l_sq[wave * kATile + kR * lane + r] = sq_a[r];
    }
    __syncthreads();
    const int t = threadIdx.x;  // one a sample per thread: kATile == 64 * kWaves
    double si = 0.0;
    unsigned long long ss = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        si += l_inv[w * kATile + t];
        ss += l_sq[w * kATile + t];
    }
    const int64_t a = a_tile + t;
    if (a < N) {
        if (out.o_inv && si != 0.0) unsafeAtomicAdd(out.o_inv + a, si);
        if (out.o_sq && ss != 0) atomicAdd(out.o_sq + a, ss);
    }
}

__global__ __launch_bounds__(256) void outlier_finalise_kernel(const double* __restrict__ inv,
                                                              const unsigned long long* __restrict__ sq, int64_t N,
                                                              int32_t B, double* __restrict__ printed,
                                                              double* __restrict__ classic) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    if (printed) printed[i] = inv[i] / (double)(N - 1);
    if (classic) classic[i] = sq[i] ? (double)N * ((double)B * (double)B) / (double)sq[i] : __builtin_inf();
}

#ifndef RFX_PLAIN_WAVES
#define RFX_PLAIN_WAVES 4
#endif
// Waves per SIMD the register allocation aims for.  The main loop fits 128 VGPRs up to 14 planes (12 with an in-bag
// word per sample as well); beyond that the compiler spills a few registers.  Measured at N = 60,000, B = 512: three
// waves without spills beat four with them for the plain pass at 15 and 16 planes (18.6 -> 17.9 ms, 20.5 -> 17.0 ms)
// and for the fused pass at 16 (22.8 -> 21.3 ms); everywhere else four waves stay ahead (sparse pass at 16 planes:
// 14.7 ms against 16.7 ms).
#define RFX_MIN_WAVES(planes, mode) \
    ((((mode) == 0 && (planes) >= 15) || ((mode) == 4 && (planes) >= 16)) ? 3 : RFX_PLAIN_WAVES)

// P = number of leaf-id bit planes, J = b samples per wave, kMode = what is counted and how it leaves.
enum { kModePlain = 0, kModeOob = 1, kModeSparse = 2, kModeOutlier = 3, kModeBoth = 4 };
// Off: measured at N = 100,000, B = 1,000 it cuts the plane traffic between L2 and the fabric from 80 to 21 GB per launch
// and costs 5 % (fused pass 78.2 -> 82.0 ms, plain 57.8 -> 61.6 ms): the four waves then read four different a tiles per
// group of trees from L2 instead of sharing one through the first-level cache, and no registers are left to request
// them a group ahead.  The traffic does not bind (1 TB/s), the vector pipes do.
#ifndef RFX_TILE_SHARE_B
#define RFX_TILE_SHARE_B 0
#endif
constexpr bool tile_shares_b(int mode) { return RFX_TILE_SHARE_B != 0 && mode != kModeOutlier; }
template <int P, int J, int kMode>
__global__ __launch_bounds__(64 * kWaves, RFX_MIN_WAVES(P, kMode)) void prox_tile_kernel(const uint32_t* __restrict__ planes, int64_t Npad,
                                                                 int32_t G, int32_t n_tile_rows, TileOut out, TileOut out2) {
    constexpr bool kOob = kMode == kModeOob;
    constexpr bool kBoth = kMode == kModeBoth;  // plain and out-of-bag counts in one pass; out2 takes the latter
    constexpr int PS = plane_stride(P);
    constexpr int PL = (kOob || kBoth) ? P + 1 : P;  // words of a sample actually used
    constexpr int PV = (PL + 3) / 4;         // 16-byte loads per a sample
    // The four waves of a workgroup either share their a samples and take four consecutive groups of J b samples
    // (outlier sums: the a side is combined over the waves), or share their J b samples and take four consecutive
    // a tiles: then they ask for the same b planes at the same time and the scalar cache hands one fetch to all four,
    // a quarter of the plane traffic between L2 and the fabric.
    constexpr bool kShareB = tile_shares_b(kMode);
    constexpr int kARow = kShareB ? kATile * kWaves : kATile;  // a samples of a workgroup
    constexpr int kBTile = kShareB ? J : J * kWaves;           // b samples of a workgroup
    constexpr int kRatio = kARow / kBTile;                     // b tiles per tile row

    // Tile index.  A tile row `ta` (kARow a samples) pairs with b tiles 0 .. (ta+1)*kRatio - 1.
    // Consecutive workgroup ids go to the 8 XCDs in turn, so XCD x = id % 8 is given the tile rows
    // ta = x, x+8, x+16, ... and walks each of them from b tile 0 upwards: the workgroups an XCD runs
    // at any moment share their a planes in that XCD's L2 and write neighbouring column ranges of the
    // same output rows.  Before row number m of an XCD's list it has done
    // kRatio * (m*(x+1) + 4*m*(m-1)) tiles.
    const int64_t x = blockIdx.x & 7, l = blockIdx.x >> 3;
    auto before = [&](int64_t m) { return (int64_t)kRatio * (m * (x + 1) + 4 * m * (m - 1)); };
    int64_t m = (int64_t)((-(double)(x - 3) + sqrt((double)((x - 3) * (x - 3)) + 16.0 * (double)l / kRatio)) / 8.0);
    if (m < 0) m = 0;
    while (before(m + 1) <= l) ++m;
    while (m > 0 && before(m) > l) --m;
    const int64_t ta = x + 8 * m;
    const int64_t tb = l - before(m);
    if (ta >= n_tile_rows) return;  // the XCDs' lists differ in length; the grid covers the longest

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // this wave's 256 a samples and J b samples
    const int64_t ta_w = kShareB ? ta * kWaves + wave : ta;
    const int64_t a0 = ta_w * kATile + lane * kR;
    const int64_t b0 = __builtin_amdgcn_readfirstlane((int)(tb * kBTile + (kShareB ? 0 : wave * J)));
    // with shared b samples a wave may have nothing to do: its a tile lies past the data, or wholly above the diagonal
    // (every b of the tile >= every a of the wave)
    const bool active = !kShareB || (ta_w * kATile < Npad && b0 < (ta_w + 1) * kATile);

    // LDS: per-wave transposition buffers for the epilogue, then the table of the quotients c / B,
    // c = 0..B (plain variant with a float32 output only)
    extern __shared__ __align__(16) uint32_t lds[];
    constexpr int kTrWords = 64 * (J + 4);
    uint32_t* tr = lds + wave * kTrWords;
    float* tab = reinterpret_cast<float*>(lds + kWaves * kTrWords);
    if (out.use_tab) {
        for (int c = threadIdx.x; c <= out.B; c += 64 * kWaves) tab[c] = (float)c / (float)out.B;
        __syncthreads();
    }

    // per pair: mismatching trees (plain), or out-of-bag numerator | denominator << 16
    uint32_t acc[kR][J];
#pragma unroll
    for (int r = 0; r < kR; ++r)
#pragma unroll
        for (int j = 0; j < J; ++j) acc[r][j] = 0;

    const int n_groups = active ? G : 0;
    for (int g = 0; g < n_groups; ++g) {
        const uint4* pa = reinterpret_cast<const uint4*>(planes + ((int64_t)g * Npad + a0) * PS);
        uint32_t xa[kR][PV * 4];
#pragma unroll
        for (int r = 0; r < kR; ++r)
#pragma unroll
            for (int v = 0; v < PV; ++v) {
                uint4 q = pa[r * (PS / 4) + v];
                xa[r][v * 4 + 0] = q.x;
                xa[r][v * 4 + 1] = q.y;
                xa[r][v * 4 + 2] = q.z;
                xa[r][v * 4 + 3] = q.w;
            }
        const uint32_t* __restrict__ pb = planes + ((int64_t)g * Npad + b0) * PS;  // wave-uniform
#if RFX_B_PREFETCH
        // The planes of b sample j + 1 are requested while those of sample j are being used: scalar loads return in any
        // order, so the only wait there is waits for all of them, and a request must therefore go out after the wait for
        // the previous one and before the vector work that hides it.  The empty asm statements pin that order (they
        // consume the words of sample j, which places the wait), the scheduling barriers keep the compiler from moving
        // the requests back down to their first use.
        uint32_t xq[2][PL];
#pragma unroll
        for (int p = 0; p < PL; ++p) xq[0][p] = pb[p];
#endif
#pragma unroll
        for (int j = 0; j < J; ++j) {
            uint32_t xb[PL];
#if RFX_B_PREFETCH
#pragma unroll
            for (int p = 0; p < PL; ++p) xb[p] = xq[j & 1][p];
            asm volatile("" ::"s"(xb[0]), "s"(xb[PL - 1]), "s"(xb[PL / 2]));
            __builtin_amdgcn_sched_barrier(0);
            if (j + 1 < J) {
#pragma unroll
                for (int p = 0; p < PL; ++p) xq[(j + 1) & 1][p] = pb[(j + 1) * PS + p];
            }
            __builtin_amdgcn_sched_barrier(0);
#else
#pragma unroll
            for (int p = 0; p < PL; ++p) xb[p] = pb[j * PS + p];  // uniform address: scalar loads into SGPRs
#endif
#pragma unroll
            for (int r = 0; r < kR; ++r) {
                uint32_t t = xa[r][0] ^ xb[0];
#pragma unroll
                for (int p = 1; p < P; ++p) t = __builtin_amdgcn_bitop3_b32(t, xa[r][p], xb[p], 0xf6);  // t | (a ^ b)
                if (kBoth) {
                    // three 10-bit fields (B <= 1023): mismatches | numerator << 10 | denominator << 20
                    const uint32_t both_same = __builtin_amdgcn_bitop3_b32(t, xa[r][P], xb[P], 0x08);
                    const uint32_t both = xa[r][P] & xb[P];
                    // (two shift-and-add instructions; left to itself the compiler shifts both counts and adds the three
                    // terms, one instruction more per pair and group of trees)
                    acc[r][j] += __builtin_popcount(t);
                    acc[r][j] = shift_add<10>((uint32_t)__builtin_popcount(both_same), acc[r][j]);
                    acc[r][j] = shift_add<20>((uint32_t)__builtin_popcount(both), acc[r][j]);
                } else if (kOob) {
                    // trees where both are out-of-bag and the leaves agree: ~t & oa & ob
                    const uint32_t both_same = __builtin_amdgcn_bitop3_b32(t, xa[r][P], xb[P], 0x08);
                    const uint32_t both = xa[r][P] & xb[P];
                    acc[r][j] += __builtin_popcount(both_same);
                    acc[r][j] = shift_add<16>((uint32_t)__builtin_popcount(both), acc[r][j]);
                } else {
                    acc[r][j] += __builtin_popcount(t);
                }
            }
        }
    }

    if (!active) return;  // (no barrier follows: only the outlier sums have one, and there every wave is active)
    const int64_t a_tile = ta_w * kATile;
    if (kBoth) {
        if (out.use_tab)
            write_tile<J, false, true, 1>(out, tab, tr, lane, a_tile, b0, acc);
        else
            write_tile<J, false, false, 1>(out, tab, tr, lane, a_tile, b0, acc);
        __builtin_amdgcn_wave_barrier();
        write_tile<J, true, false, 2>(out2, tab, tr, lane, a_tile, b0, acc);
    } else if (kMode == kModeSparse)
        emit_tile<J>(out, tr, lane, a_tile, b0, acc);
    else if (kMode == kModeOutlier)
        outlier_tile<J>(out, lds, lane, wave, a_tile, b0, acc);
    else if (out.use_tab)
        write_tile<J, kOob, true>(out, tab, tr, lane, a_tile, b0, acc);
    else
        write_tile<J, kOob, false>(out, tab, tr, lane, a_tile, b0, acc);
}

template <int P, int J, int kMode>
int launch_tiles(const uint32_t* planes, int64_t Npad, int32_t G, const TileOut& out, const TileOut& out2, hipStream_t st,
                 bool timing) {
    constexpr bool kShareB = tile_shares_b(kMode);
    constexpr int kARow = kShareB ? kATile * kWaves : kATile;
    constexpr int kRatio = kARow / (kShareB ? J : J * kWaves);
    const int64_t rows = rfx::ceil_div(Npad, kARow);
    // XCD x works through tile rows x, x+8, ...; the last XCD that has `cnt` rows has the longest list
    int64_t longest = 0;
    for (int64_t x = 0; x < 8 && x < rows; ++x) {
        const int64_t cnt = (rows - x + 7) / 8;
        longest = std::max(longest, (int64_t)kRatio * (cnt * (x + 1) + 4 * cnt * (cnt - 1)));
    }
    const int64_t blocks = 8 * longest;
    if (blocks > 0x7fffffffLL) return rfx::fail(RFX_ERR_INVALID_ARG, "proximity: N too large for one launch");
    constexpr bool kOob = kMode == kModeOob;
    TileOut o = out;
    o.use_tab = ((kMode == kModePlain || kMode == kModeBoth) && out.prox && out.B < 8192) ? 1 : 0;
    static_assert(sizeof(uint32_t) * kWaves * 64 * (J + 4) >= 16 * kWaves * kATile, "outlier sums reuse the transposition buffers");
    const size_t lds = sizeof(uint32_t) * kWaves * 64 * (J + 4) +
                       (o.use_tab ? sizeof(float) * (size_t)(out.B + 1) : 0);
    // the event pair of the timing aid is created only when a caller may allocate
    std::optional<rfx::TimedLaunch> timed;
    if (timing)
        timed.emplace(kMode == kModeBoth ? "prox_tile_kernel_both" : kOob ? "prox_tile_kernel_oob" : (kMode == kModeSparse ? "prox_tile_kernel_sparse" : (kMode == kModeOutlier ? "prox_tile_kernel_outlier" : "prox_tile_kernel")), st);
    hipLaunchKernelGGL((prox_tile_kernel<P, J, kMode>), dim3((unsigned)blocks), dim3(64 * kWaves), lds, st, planes, Npad, G,
                       (int32_t)rows, o, out2);
    RFX_LAUNCH_CHECK("prox_tile_kernel");
    return RFX_OK;
}

template <int kMode>
int dispatch_planes(int P, const uint32_t* planes, int64_t Npad, int32_t G, const TileOut& out, const TileOut& out2,
                    hipStream_t st, bool timing) {
#ifndef RFX_J_PLAIN
#define RFX_J_PLAIN 16
#endif
    constexpr int J = RFX_J_PLAIN;
    switch (P) {
#define RFX_CASE(p) \
    case p:         \
        return launch_tiles<p, J, kMode>(planes, Npad, G, out, out2, st, timing);
#ifdef RFX_ONLY_P  // development builds: a single plane count compiles in seconds
        RFX_CASE(RFX_ONLY_P)
#else
        RFX_CASE(8) RFX_CASE(9) RFX_CASE(10) RFX_CASE(11) RFX_CASE(12) RFX_CASE(13) RFX_CASE(14) RFX_CASE(15)
        RFX_CASE(16) RFX_CASE(18) RFX_CASE(20) RFX_CASE(22) RFX_CASE(24)
#endif
#undef RFX_CASE
    }
    return rfx::fail(RFX_ERR_INVALID_ARG, "proximity: %d bit planes", P);
}

int check_common(const char* who, const void* leaf, int64_t N, int32_t B, int32_t leaf_bound, int count_dtype,
                 int layout) {
    if (!leaf) return rfx::fail(RFX_ERR_NULL, "%s: leaf is null", who);
    if (N < 1 || N > 3000000) return rfx::fail(RFX_ERR_INVALID_ARG, "%s: N=%lld outside 1..3000000", who, (long long)N);
    if (B < 1) return rfx::fail(RFX_ERR_INVALID_ARG, "%s: B=%d", who, B);
    if (leaf_bound < 1 || leaf_bound > (1 << 24))
        return rfx::fail(RFX_ERR_INVALID_ARG, "%s: leaf_bound=%d outside 1..2^24", who, leaf_bound);
    if (count_dtype != RFX_U16 && count_dtype != RFX_U32)
        return rfx::fail(RFX_ERR_INVALID_ARG, "%s: count_dtype=%d", who, count_dtype);
    if (layout != RFX_FULL && layout != RFX_UPPER_PACKED) return rfx::fail(RFX_ERR_INVALID_ARG, "%s: layout=%d", who, layout);
    if (count_dtype == RFX_U16 && B > 65535)
        return rfx::fail(RFX_ERR_OVERFLOW, "%s: %d trees do not fit uint16 counts", who, B);
    return RFX_OK;
}

// Number of bit planes used for ids below leaf_bound: the exact width from 9 to 16 bits, at least 8
// (narrower ids are rare and extra zero planes never mismatch), even above 16.  One kernel
// instantiation exists per value returned here.
int planes_for(int32_t leaf_bound) {
    int P = 1;
    while ((1 << P) < leaf_bound) ++P;
    if (P < 8) return 8;
    return P <= 16 ? P : (P + 1) & ~1;
}

// Scratch of one call, carved from a caller's workspace: the bit planes, then (outlier pass) the two per-sample
// sums, then (sparse pass) the 64-bit cursor.  Every part starts on a 256-byte boundary.
struct ProxScratch {
    size_t plane_bytes, sums_off, cursor_off, total;
};
ProxScratch prox_scratch(int64_t N, int32_t B, int32_t leaf_bound) {
    const int P = planes_for(leaf_bound);
    const int PS = plane_stride(P);
    const size_t G = (size_t)((B + 31) / 32);
    const size_t Npad = (size_t)(rfx::ceil_div(N, kATile) * kATile);
    ProxScratch s;
    s.plane_bytes = sizeof(uint32_t) * G * Npad * (size_t)PS;
    s.sums_off = (s.plane_bytes + 255) & ~(size_t)255;
    s.cursor_off = s.sums_off + ((16 * (size_t)N + 255) & ~(size_t)255);
    s.total = s.cursor_off + 256;
    return s;
}

int check_workspace(const char* who, const void* workspace, int64_t workspace_bytes, const ProxScratch& need) {
    if (!workspace) return rfx::fail(RFX_ERR_NULL, "%s: workspace is null", who);
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return rfx::fail(RFX_ERR_INVALID_ARG, "%s: workspace is not 256-byte aligned", who);
    if (workspace_bytes < 0 || (size_t)workspace_bytes < need.total)
        return rfx::fail(RFX_ERR_CAPACITY, "%s: workspace of %lld bytes, %zu needed", who, (long long)workspace_bytes, need.total);
    return RFX_OK;
}

__global__ void zero_words_kernel(uint32_t* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}
int zero_words(void* p, size_t bytes, hipStream_t st) {
    const int64_t n = (int64_t)(bytes / 4);
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)rfx::ceil_div(n, 256)), dim3(256), 0, st, static_cast<uint32_t*>(p), n);
    RFX_LAUNCH_CHECK("zero_words_kernel");
    return RFX_OK;
}

// Enqueues the transposition into bit planes and the tile pass on `st`; `planes` is scratch of
// prox_scratch(...).plane_bytes bytes that must stay untouched until the kernels have run.  No allocation, no
// synchronisation.
template <int kMode>
int enqueue(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int32_t leaf_bound, const TileOut& out,
            hipStream_t st, uint32_t* planes, const TileOut& out2 = TileOut{}, bool timing = true) {
    const int P = planes_for(leaf_bound);
    const int PS = plane_stride(P);
    const int32_t G = (B + 31) / 32;
    const int64_t Npad = rfx::ceil_div(N, kATile) * kATile;
    hipLaunchKernelGGL(pack_planes_kernel, dim3((unsigned)rfx::ceil_div(Npad, 256), (unsigned)G), dim3(256), 0, st, leaf,
                       inbag, N, B, Npad, P, PS, planes);
    RFX_LAUNCH_CHECK("pack_planes_kernel");
    return dispatch_planes<kMode>(P, planes, Npad, G, out, out2, st, timing);
}

// The synchronous conveniences: scratch allocated for the call, the asynchronous variant, a wait, the scratch freed.
template <class Call>
int with_own_workspace(const char* who, int64_t N, int32_t B, int32_t leaf_bound, hipStream_t st, Call&& call) {
    const ProxScratch need = prox_scratch(N, B, leaf_bound);
    rfx::DevBuf ws;
    RFX_HIP(ws.alloc(need.total));
    int rc = call(ws.p, (int64_t)need.total);
    hipError_t e = hipStreamSynchronize(st);  // the scratch is freed on return
    if (rc != RFX_OK) return rc;
    if (e != hipSuccess) return rfx::fail(RFX_ERR_HIP, "%s: kernels failed: %s", who, hipGetErrorString(e));
    return RFX_OK;
}

}  // namespace

// RFX_TILE_MODE (0..4), when defined, compiles the entry points of one mode only, so that the build can
// compile the five sets of kernel instantiations side by side.
#if !defined(RFX_TILE_MODE) || RFX_TILE_MODE == 0
// Bit-plane scratch of rfx_prox_dense_noalloc: one array per GPU for the life of the process.
constexpr size_t kStaticPlaneWords = (size_t)4 << 20;  // 16 MiB
static __device__ __align__(256) uint32_t scratch[kStaticPlaneWords];

namespace {
// Device address of `scratch` on the current device (the host-side symbol is not an address a kernel can use).
int static_planes(uint32_t** out) {
    static std::mutex mu;
    static uint32_t* addr[64] = {};
    int dev = 0;
    RFX_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return rfx::fail(RFX_ERR_UNSUPPORTED, "rfx_prox_dense_noalloc: device %d", dev);
    std::lock_guard<std::mutex> lk(mu);
    if (!addr[dev]) {
        void* p = nullptr;
        RFX_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        addr[dev] = static_cast<uint32_t*>(p);
    }
    *out = addr[dev];
    return RFX_OK;
}
}  // namespace
#endif

extern "C" {

#if !defined(RFX_TILE_MODE) || RFX_TILE_MODE == 0
int rfx_prox_workspace_bytes(int64_t N, int32_t B, int32_t leaf_bound, int64_t* bytes) {
    if (!bytes) return rfx::fail(RFX_ERR_NULL, "rfx_prox_workspace_bytes: bytes is null");
    int rc = check_common("rfx_prox_workspace_bytes", bytes, N, B, leaf_bound, RFX_U32, RFX_FULL);
    if (rc != RFX_OK) return rc;
    *bytes = (int64_t)prox_scratch(N, B, leaf_bound).total;
    return RFX_OK;
}

static int check_dense(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int count_dtype, int layout,
                       const void* counts, const float* prox) {
    int rc = check_common("rfx_prox_dense", leaf, N, B, leaf_bound, count_dtype, layout);
    if (rc != RFX_OK) return rc;
    if (!counts && !prox) return rfx::fail(RFX_ERR_NULL, "rfx_prox_dense: neither counts nor prox given");
    return RFX_OK;
}

int rfx_prox_dense_ws(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int count_dtype, int layout,
                      void* counts, float* prox, void* workspace, int64_t workspace_bytes, void* stream) {
    int rc = check_dense(leaf, N, B, leaf_bound, count_dtype, layout, counts, prox);
    if (rc != RFX_OK) return rc;
    if ((rc = check_workspace("rfx_prox_dense", workspace, workspace_bytes, prox_scratch(N, B, leaf_bound))) != RFX_OK) return rc;
    TileOut out{counts, nullptr, prox, N, B, count_dtype == RFX_U16, layout == RFX_UPPER_PACKED, 0, nullptr, nullptr, nullptr, 0, 0, nullptr, nullptr, nullptr};
    return enqueue<kModePlain>(leaf, nullptr, N, B, leaf_bound, out, rfx::as_stream(stream), static_cast<uint32_t*>(workspace));
}

int rfx_prox_dense(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int count_dtype, int layout,
                   void* counts, float* prox, void* stream) {
    int rc = check_dense(leaf, N, B, leaf_bound, count_dtype, layout, counts, prox);
    if (rc != RFX_OK) return rc;
    return with_own_workspace("rfx_prox_dense", N, B, leaf_bound, rfx::as_stream(stream), [&](void* ws, int64_t bytes) {
        return rfx_prox_dense_ws(leaf, N, B, leaf_bound, count_dtype, layout, counts, prox, ws, bytes, stream);
    });
}

int rfx_prox_dense_noalloc(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int count_dtype, int layout,
                           void* counts, float* prox, void* stream) {
    int rc = check_dense(leaf, N, B, leaf_bound, count_dtype, layout, counts, prox);
    if (rc != RFX_OK) return rc;
    const ProxScratch need = prox_scratch(N, B, leaf_bound);
    if (need.plane_bytes > sizeof(uint32_t) * kStaticPlaneWords)
        return rfx::fail(RFX_ERR_CAPACITY,
                         "rfx_prox_dense_noalloc: N=%lld, B=%d, leaf_bound=%d need %zu bytes of bit planes, the built-in "
                         "scratch holds %zu (use rfx_prox_dense or rfx_prox_dense_ws)",
                         (long long)N, B, leaf_bound, need.plane_bytes, sizeof(uint32_t) * kStaticPlaneWords);
    uint32_t* planes = nullptr;
    if ((rc = static_planes(&planes)) != RFX_OK) return rc;
    TileOut out{counts, nullptr, prox, N, B, count_dtype == RFX_U16, layout == RFX_UPPER_PACKED, 0, nullptr, nullptr, nullptr, 0, 0, nullptr, nullptr, nullptr};
    return enqueue<kModePlain>(leaf, nullptr, N, B, leaf_bound, out, rfx::as_stream(stream), planes, TileOut{}, /*timing=*/false);
}
#endif

#if !defined(RFX_TILE_MODE) || RFX_TILE_MODE == 1
static int check_oob(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int32_t leaf_bound, int count_dtype,
                     int layout, const void* num, const void* den, const float* prox) {
    int rc = check_common("rfx_prox_oob", leaf, N, B, leaf_bound, count_dtype, layout);
    if (rc != RFX_OK) return rc;
    if (!inbag) return rfx::fail(RFX_ERR_NULL, "rfx_prox_oob: inbag is null");
    if (B > 65535) return rfx::fail(RFX_ERR_UNSUPPORTED, "rfx_prox_oob: more than 65535 trees");
    if (!num && !den && !prox) return rfx::fail(RFX_ERR_NULL, "rfx_prox_oob: no output given");
    return RFX_OK;
}

int rfx_prox_oob_ws(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int32_t leaf_bound, int count_dtype,
                    int layout, void* num, void* den, float* prox, void* workspace, int64_t workspace_bytes, void* stream) {
    int rc = check_oob(leaf, inbag, N, B, leaf_bound, count_dtype, layout, num, den, prox);
    if (rc != RFX_OK) return rc;
    if ((rc = check_workspace("rfx_prox_oob", workspace, workspace_bytes, prox_scratch(N, B, leaf_bound))) != RFX_OK) return rc;
    TileOut out{num, den, prox, N, B, count_dtype == RFX_U16, layout == RFX_UPPER_PACKED, 0, nullptr, nullptr, nullptr, 0, 0, nullptr, nullptr, nullptr};
    return enqueue<kModeOob>(leaf, inbag, N, B, leaf_bound, out, rfx::as_stream(stream), static_cast<uint32_t*>(workspace));
}

int rfx_prox_oob(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int32_t leaf_bound,
                 int count_dtype, int layout, void* num, void* den, float* prox, void* stream) {
    int rc = check_oob(leaf, inbag, N, B, leaf_bound, count_dtype, layout, num, den, prox);
    if (rc != RFX_OK) return rc;
    return with_own_workspace("rfx_prox_oob", N, B, leaf_bound, rfx::as_stream(stream), [&](void* ws, int64_t bytes) {
        return rfx_prox_oob_ws(leaf, inbag, N, B, leaf_bound, count_dtype, layout, num, den, prox, ws, bytes, stream);
    });
}
#endif

#if !defined(RFX_TILE_MODE) || RFX_TILE_MODE == 2
static int check_sparse(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int32_t min_count, int count_dtype,
                        int64_t capacity, const uint32_t* rows, const uint32_t* cols, const void* nnz) {
    int rc = check_common("rfx_prox_sparse", leaf, N, B, leaf_bound, count_dtype, RFX_UPPER_PACKED);
    if (rc != RFX_OK) return rc;
    if (!nnz) return rfx::fail(RFX_ERR_NULL, "rfx_prox_sparse: nnz is null");
    if (min_count < 1) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse: min_count=%d below 1", min_count);
    if (capacity < 0) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse: capacity=%lld", (long long)capacity);
    if (capacity > 0 && (!rows || !cols)) return rfx::fail(RFX_ERR_NULL, "rfx_prox_sparse: rows / cols are null");
    if (B >= (1 << 20)) return rfx::fail(RFX_ERR_UNSUPPORTED, "rfx_prox_sparse: 2^20 trees or more");
    return RFX_OK;
}

int rfx_prox_sparse_ws(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int32_t min_count, int count_dtype,
                       int64_t capacity, uint32_t* rows, uint32_t* cols, void* counts, float* prox, uint64_t* nnz,
                       void* workspace, int64_t workspace_bytes, void* stream) {
    int rc = check_sparse(leaf, N, B, leaf_bound, min_count, count_dtype, capacity, rows, cols, nnz);
    if (rc != RFX_OK) return rc;
    if (reinterpret_cast<uintptr_t>(nnz) % 8 != 0) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_sparse: nnz is not 8-byte aligned");
    if ((rc = check_workspace("rfx_prox_sparse", workspace, workspace_bytes, prox_scratch(N, B, leaf_bound))) != RFX_OK) return rc;
    hipStream_t st = rfx::as_stream(stream);
    if ((rc = zero_words(nnz, sizeof(uint64_t), st)) != RFX_OK) return rc;
    TileOut out{counts, nullptr, prox, N, B, count_dtype == RFX_U16, 1, 0, rows, cols, reinterpret_cast<unsigned long long*>(nnz),
                (unsigned long long)capacity, (uint32_t)min_count, nullptr, nullptr, nullptr};
    return enqueue<kModeSparse>(leaf, nullptr, N, B, leaf_bound, out, st, static_cast<uint32_t*>(workspace));
}

int rfx_prox_sparse(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, int32_t min_count, int count_dtype,
                    int64_t capacity, uint32_t* rows, uint32_t* cols, void* counts, float* prox, int64_t* nnz,
                    void* stream) {
    int rc = check_sparse(leaf, N, B, leaf_bound, min_count, count_dtype, capacity, rows, cols, nnz);
    if (rc != RFX_OK) return rc;
    // deep forests with small leaves: far fewer counter increments than pair tests
    bool by_rows = false;
    if ((rc = rfx::sparse_rows_cheaper(leaf, N, B, leaf_bound, rfx::as_stream(stream), &by_rows)) != RFX_OK) return rc;
    if (by_rows)
        return rfx_prox_sparse_rows(leaf, N, B, leaf_bound, min_count, count_dtype, capacity, rows, cols, counts, prox, nnz, stream);
    const ProxScratch need = prox_scratch(N, B, leaf_bound);
    unsigned long long total = 0;
    rc = with_own_workspace("rfx_prox_sparse", N, B, leaf_bound, rfx::as_stream(stream), [&](void* ws, int64_t bytes) {
        uint64_t* cursor = reinterpret_cast<uint64_t*>(static_cast<char*>(ws) + need.cursor_off);
        int r = rfx_prox_sparse_ws(leaf, N, B, leaf_bound, min_count, count_dtype, capacity, rows, cols, counts, prox, cursor,
                                   ws, bytes, stream);
        if (r != RFX_OK) return r;
        RFX_HIP(hipMemcpyAsync(&total, cursor, sizeof(total), hipMemcpyDeviceToHost, rfx::as_stream(stream)));
        return RFX_OK;
    });
    if (rc != RFX_OK) return rc;
    *nnz = (int64_t)total;
    if (total > (unsigned long long)capacity && capacity > 0)
        return rfx::fail(RFX_ERR_CAPACITY, "rfx_prox_sparse: %llu pairs reach the threshold, capacity is %lld", total,
                         (long long)capacity);
    return RFX_OK;
}
#endif

#if !defined(RFX_TILE_MODE) || RFX_TILE_MODE == 4
static int check_both(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int32_t leaf_bound, int count_dtype,
                      int layout, const void* counts, const float* prox, int oob_layout, const void* num, const void* den,
                      const float* prox_oob) {
    int rc = check_common("rfx_prox_dense_oob", leaf, N, B, leaf_bound, count_dtype, layout);
    if (rc != RFX_OK) return rc;
    if (oob_layout != RFX_FULL && oob_layout != RFX_UPPER_PACKED)
        return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_dense_oob: oob_layout=%d", oob_layout);
    if (!inbag) return rfx::fail(RFX_ERR_NULL, "rfx_prox_dense_oob: inbag is null");
    if (B > 1023) return rfx::fail(RFX_ERR_UNSUPPORTED, "rfx_prox_dense_oob: more than 1023 trees");
    if ((!counts && !prox) || (!num && !den && !prox_oob))
        return rfx::fail(RFX_ERR_NULL, "rfx_prox_dense_oob: an output of each kind is required");
    return RFX_OK;
}

int rfx_prox_dense_oob_ws(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int32_t leaf_bound,
                          int count_dtype, int layout, void* counts, float* prox, int oob_layout, void* num, void* den,
                          float* prox_oob, void* workspace, int64_t workspace_bytes, void* stream) {
    int rc = check_both(leaf, inbag, N, B, leaf_bound, count_dtype, layout, counts, prox, oob_layout, num, den, prox_oob);
    if (rc != RFX_OK) return rc;
    if ((rc = check_workspace("rfx_prox_dense_oob", workspace, workspace_bytes, prox_scratch(N, B, leaf_bound))) != RFX_OK) return rc;
    TileOut plain{counts, nullptr, prox, N, B, count_dtype == RFX_U16, layout == RFX_UPPER_PACKED, 0, nullptr, nullptr, nullptr, 0, 0, nullptr, nullptr, nullptr};
    TileOut oob{num, den, prox_oob, N, B, count_dtype == RFX_U16, oob_layout == RFX_UPPER_PACKED, 0, nullptr, nullptr, nullptr, 0, 0, nullptr, nullptr, nullptr};
    return enqueue<kModeBoth>(leaf, inbag, N, B, leaf_bound, plain, rfx::as_stream(stream), static_cast<uint32_t*>(workspace), oob);
}

int rfx_prox_dense_oob(const uint32_t* leaf, const uint16_t* inbag, int64_t N, int32_t B, int32_t leaf_bound,
                       int count_dtype, int layout, void* counts, float* prox, int oob_layout, void* num, void* den,
                       float* prox_oob, void* stream) {
    int rc = check_both(leaf, inbag, N, B, leaf_bound, count_dtype, layout, counts, prox, oob_layout, num, den, prox_oob);
    if (rc != RFX_OK) return rc;
    return with_own_workspace("rfx_prox_dense_oob", N, B, leaf_bound, rfx::as_stream(stream), [&](void* ws, int64_t bytes) {
        return rfx_prox_dense_oob_ws(leaf, inbag, N, B, leaf_bound, count_dtype, layout, counts, prox, oob_layout, num, den,
                                     prox_oob, ws, bytes, stream);
    });
}
#endif

#if !defined(RFX_TILE_MODE) || RFX_TILE_MODE == 3
static int check_outlier(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, const double* printed,
                         const double* classic) {
    int rc = check_common("rfx_prox_outlier", leaf, N, B, leaf_bound, RFX_U32, RFX_FULL);
    if (rc != RFX_OK) return rc;
    if (!printed && !classic) return rfx::fail(RFX_ERR_NULL, "rfx_prox_outlier: neither output given");
    if (N < 2) return rfx::fail(RFX_ERR_INVALID_ARG, "rfx_prox_outlier: needs at least 2 samples");
    if (B >= (1 << 20)) return rfx::fail(RFX_ERR_UNSUPPORTED, "rfx_prox_outlier: 2^20 trees or more");
    return RFX_OK;
}

int rfx_prox_outlier_ws(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, const int32_t* labels,
                        double* printed, double* classic, void* workspace, int64_t workspace_bytes, void* stream) {
    int rc = check_outlier(leaf, N, B, leaf_bound, printed, classic);
    if (rc != RFX_OK) return rc;
    const ProxScratch need = prox_scratch(N, B, leaf_bound);
    if ((rc = check_workspace("rfx_prox_outlier", workspace, workspace_bytes, need)) != RFX_OK) return rc;
    hipStream_t st = rfx::as_stream(stream);
    // inv [N] float64, then sq [N] uint64
    double* inv = reinterpret_cast<double*>(static_cast<char*>(workspace) + need.sums_off);
    unsigned long long* sq = reinterpret_cast<unsigned long long*>(inv + N);
    if ((rc = zero_words(inv, 16 * (size_t)N, st)) != RFX_OK) return rc;
    TileOut out{nullptr, nullptr, nullptr, N, B, 0, 0, 0, nullptr, nullptr, nullptr, 0, 0, printed ? inv : nullptr,
                classic ? sq : nullptr, labels};
    rc = enqueue<kModeOutlier>(leaf, nullptr, N, B, leaf_bound, out, st, static_cast<uint32_t*>(workspace));
    if (rc != RFX_OK) return rc;
    hipLaunchKernelGGL(outlier_finalise_kernel, dim3((unsigned)rfx::ceil_div(N, 256)), dim3(256), 0, st, inv, sq, N, B,
                       printed, classic);
    RFX_LAUNCH_CHECK("outlier_finalise_kernel");
    return RFX_OK;
}

int rfx_prox_outlier(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, const int32_t* labels,
                     double* printed, double* classic, void* stream) {
    int rc = check_outlier(leaf, N, B, leaf_bound, printed, classic);
    if (rc != RFX_OK) return rc;
    return with_own_workspace("rfx_prox_outlier", N, B, leaf_bound, rfx::as_stream(stream), [&](void* ws, int64_t bytes) {
        return rfx_prox_outlier_ws(leaf, N, B, leaf_bound, labels, printed, classic, ws, bytes, stream);
    });
}
#endif
}  // extern "C"
