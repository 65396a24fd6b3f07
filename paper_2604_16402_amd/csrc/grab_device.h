// Device-side helpers shared by the search and append kernels (gfx950 only): queue keys,
// wave reductions and the gathered fp32 distance with its fixed summation order.
#pragma once
#include <type_traits>

#include "grab_internal.h"

namespace {

typedef unsigned long long u64;
constexpr u64 SENT = ~0ull;  // empty queue entry; sorts last

// order-preserving image of an fp32 value in uint32
__device__ __forceinline__ uint32_t dist_image(float d) {
    uint32_t b = __float_as_uint(d);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float image_dist(uint32_t m) {
    return __uint_as_float((m & 0x80000000u) ? (m & 0x7FFFFFFFu) : ~m);
}
// queue key: distance image | slot | expanded flag.  Keys of different slots never tie.
__device__ __forceinline__ u64 make_key(float d, uint32_t slot) { return ((u64)dist_image(d) << 32) | ((u64)slot << 1); }
__device__ __forceinline__ uint32_t key_slot(u64 k) { return (uint32_t)(k & 0xFFFFFFFFull) >> 1; }

// number of set bits of m below the caller's lane (m the same in every lane): the caller's place
// among the lanes that a ballot marked
__device__ __forceinline__ int lanes_below(u64 m) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) v += __shfl_xor(v, m);
    return v;
}

// ---- lane exchanges that stay out of LDS ------------------------------------------------------
// DPP moves cover the partners at distance 1, 2, 4 and 8 (quad permutes, the half-row mirror
// followed by a quad reversal, a rotation by 8 inside a row of 16); the row and half-wave swaps
// of gfx950 cover distance 16 and 32.  A dependent chain of these costs a few cycles per step
// where a ds_bpermute round trip costs on the order of a hundred.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
// value of lane (lane ^ J)
template <int J>
__device__ __forceinline__ uint32_t xchg32(uint32_t x, int lane) {
    static_assert(J == 1 || J == 2 || J == 4 || J == 8 || J == 16 || J == 32, "partner distance");
    if constexpr (J == 1) return dpp_u32<0xB1>(x);                    // quad_perm [1,0,3,2]
    else if constexpr (J == 2) return dpp_u32<0x4E>(x);               // quad_perm [2,3,0,1]
    else if constexpr (J == 4) return dpp_u32<0x1B>(dpp_u32<0x141>(x));  // i -> 7-i, then reverse the quad
    else if constexpr (J == 8) return dpp_u32<0x128>(x);              // row_ror:8
    else if constexpr (J == 16) {
        auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);  // odd rows of [0] <-> even rows of [1]
        return (lane & 16) ? r[0] : r[1];
    } else {
        auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);  // upper half of [0] <-> lower half of [1]
        return (lane & 32) ? r[0] : r[1];
    }
}
template <int J>
__device__ __forceinline__ u64 xchg64(u64 k, int lane) {
    return ((u64)xchg32<J>((uint32_t)(k >> 32), lane) << 32) | (u64)xchg32<J>((uint32_t)k, lane);
}
// value of lane src, the same src in every lane
__device__ __forceinline__ u64 read_lane64(u64 k, int src) {
    return ((u64)(uint32_t)__builtin_amdgcn_readlane((int)(k >> 32), src) << 32) |
           (u64)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)k, src);
}
__device__ __forceinline__ u64 shfl_xor64(u64 k, int m) {
    return ((u64)(uint32_t)__shfl_xor((int)(k >> 32), m) << 32) | (u64)(uint32_t)__shfl_xor((int)(k & 0xFFFFFFFFull), m);
}

// maximum / minimum over the wavefront, in every lane, by lane exchanges that stay out of LDS
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x, int lane) {
    uint32_t o;
    o = xchg32<1>(x, lane); x = x > o ? x : o;
    o = xchg32<2>(x, lane); x = x > o ? x : o;
    o = xchg32<4>(x, lane); x = x > o ? x : o;
    o = xchg32<8>(x, lane); x = x > o ? x : o;
    o = xchg32<16>(x, lane); x = x > o ? x : o;
    o = xchg32<32>(x, lane); x = x > o ? x : o;
    return x;
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x, int lane) { return ~wave_max_u32(~x, lane); }

// value of lane (lane ^ (K-1)): the mirror image inside aligned blocks of K lanes
template <int K>
__device__ __forceinline__ uint32_t mirror32(uint32_t x, int lane) {
    if constexpr (K == 2) return dpp_u32<0xB1>(x);
    else if constexpr (K == 4) return dpp_u32<0x1B>(x);           // quad_perm [3,2,1,0]
    else if constexpr (K == 8) return dpp_u32<0x141>(x);          // row_half_mirror
    else if constexpr (K == 16) return dpp_u32<0x140>(x);         // row_mirror
    else if constexpr (K == 32) return xchg32<16>(dpp_u32<0x140>(x), lane);
    else return xchg32<32>(xchg32<16>(dpp_u32<0x140>(x), lane), lane);
}
template <int K>
__device__ __forceinline__ u64 mirror64(u64 k, int lane) {
    return ((u64)mirror32<K>((uint32_t)(k >> 32), lane) << 32) | (u64)mirror32<K>((uint32_t)k, lane);
}
__device__ __forceinline__ u64 reverse64(u64 k, int lane) { return mirror64<64>(k, lane); }

// compare-exchange with the lane at distance J: the lower lane of a pair keeps the smaller key
template <int J>
__device__ __forceinline__ u64 cmpx(u64 key, int lane) {
    const u64 o = xchg64<J>(key, lane);
    return ((key < o) == ((lane & J) == 0)) ? key : o;
}
// the steps J, J/2, ..., 1 that sort a bitonic run of 2J lanes ascending
template <int J>
__device__ __forceinline__ u64 bitonic_merge(u64 key, int lane) {
    key = cmpx<J>(key, lane);
    if constexpr (J > 1) key = bitonic_merge<J / 2>(key, lane);
    return key;
}
// two sorted runs of K/2 lanes -> one sorted run of K lanes.  The first step pairs each lane with
// its mirror image in the block, so every step orders its pair the same way and the whole
// network needs one lane mask per distance
template <int K>
__device__ __forceinline__ u64 merge_runs(u64 key, int lane) {
    const u64 o = mirror64<K>(key, lane);
    key = ((key < o) == ((lane & (K / 2)) == 0)) ? key : o;
    if constexpr (K >= 4) key = bitonic_merge<K / 4>(key, lane);
    return key;
}
// ascending sort of the keys of lanes [0,P), P a power of two (the same in every lane); lanes
// beyond hold SENT and stay put
__device__ __forceinline__ u64 sort_lanes(u64 key, int P, int lane) {
    key = merge_runs<2>(key, lane);
    if (P >= 4) key = merge_runs<4>(key, lane);
    if (P >= 8) key = merge_runs<8>(key, lane);
    if (P >= 16) key = merge_runs<16>(key, lane);
    if (P >= 32) key = merge_runs<32>(key, lane);
    if (P >= 64) key = merge_runs<64>(key, lane);
    return key;
}

// The candidate queue: M keys per lane in registers, position p = 64*r + lane of register r,
// sorted ascending over p.  Strides of 64 and more are compare-exchanges between registers of
// the same lane; smaller strides are lane exchanges applied to every register.
template <int M>
struct LaneQueue {
    u64 k[M];

    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int r = 0; r < M; ++r) k[r] = SENT;
    }
    // queue <- the 64*M smallest of queue and ck (sorted over the lanes, SENT-padded), cut to beam:
    // min against the reversed newcomers turns the sorted queue into a bitonic sequence that holds
    // exactly the survivors; a bitonic merge sorts it again
    __device__ __forceinline__ void merge(u64 ck, int beam, int lane) {
        const u64 rv = reverse64(ck, lane);
        k[M - 1] = k[M - 1] < rv ? k[M - 1] : rv;
#pragma unroll
        for (int s = M / 2; s >= 1; s >>= 1)
#pragma unroll
            for (int r = 0; r < M; ++r)
                if ((r & s) == 0) {
                    const u64 x = k[r], y = k[r + s];
                    k[r] = x < y ? x : y;
                    k[r + s] = x < y ? y : x;
                }
#pragma unroll
        for (int r = 0; r < M; ++r) k[r] = bitonic_merge<32>(k[r], lane);
#pragma unroll
        for (int r = 0; r < M; ++r)
            if (64 * r + lane >= beam) k[r] = SENT;
    }
    // key at position p (same p in every lane)
    __device__ __forceinline__ u64 at(int p) const {
        u64 t = SENT;
#pragma unroll
        for (int r = 0; r < M; ++r)
            if ((p >> 6) == r) t = k[r];
        return read_lane64(t, p & 63);
    }
};

template <int NCH>
struct EvalShape {
    // pieces of a row held in registers at once, and rows per lane group in flight
    static constexpr int CB = NCH <= 8 ? NCH
                              : (NCH % 10 == 0 ? 10 : (NCH % 8 == 0 ? 8 : (NCH % 6 == 0 ? 6 : (NCH % 4 == 0 ? 4 : (NCH % 3 == 0 ? 3 : (NCH % 2 == 0 ? 2 : 1))))));
    static constexpr int R0 = 16 / CB;
    static constexpr int R = R0 < 1 ? 1 : (R0 > 8 ? 8 : R0);
    static constexpr bool QREG = NCH <= 8;
};

// lane exchanges inside groups of eight lanes without touching LDS: DPP quad permutes give
// xor 1 and xor 2, the half-row mirror pairs lane i with lane 7-i of its group
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

// acc plus the four products of one 16-byte piece under the metric, in index order.  The metric is a
// template argument so that a caller decides it once per batch of rows and not once per piece: a
// branch between every four multiplications keeps the compiler from interleaving the rows' chains.
template <bool L2>
__device__ __forceinline__ float fma_piece(const float4 qv, const float4 x, float acc) {
    if constexpr (L2) {
        const float dx = qv.x - x.x, dy = qv.y - x.y, dz = qv.z - x.z, dw = qv.w - x.w;
        acc = __builtin_fmaf(dx, dx, acc);
        acc = __builtin_fmaf(dy, dy, acc);
        acc = __builtin_fmaf(dz, dz, acc);
        acc = __builtin_fmaf(dw, dw, acc);
    } else {
        acc = __builtin_fmaf(qv.x, x.x, acc);
        acc = __builtin_fmaf(qv.y, x.y, acc);
        acc = __builtin_fmaf(qv.z, x.z, acc);
        acc = __builtin_fmaf(qv.w, x.w, acc);
    }
    return acc;
}
// f(std::true_type) under squared L2, f(std::false_type) under the inner product
#define GRAB_WITH_METRIC(metric, f)            \
    do {                                       \
        if ((metric) == GRAB_L2SQ) f(std::true_type{}); \
        else f(std::false_type{});             \
    } while (0)

// Gathered distances (Algorithm 2, ComputeDistance) for up to 8*R slots L[base..]: eight lanes
// share a row, lane `sub` of a group takes the 16-byte pieces 8c+sub (one 128-byte line per
// piece index across the group) and accumulates them in index order with fused multiply-adds;
// the eight partial sums are combined pairwise (lanes 0+1, 2+3, ..., then pairs, then halves).
// This fixed order makes the fp32 result reproducible bit for bit.  All loads of the batch are
// issued before the first multiply.  Every lane of a group ends with the row's distance in
// s[r]; v[r] is the row's slot and act[r] tells whether round r had a row for this group.
template <int NCH, int RA>
__device__ __forceinline__ void eval_batch_rows(const float *__restrict__ X, const float4 *qreg, const float *qlds,
                                           const uint32_t *L, int base, int n, int lane, int metric,
                                           float (&s)[EvalShape<NCH>::R], uint32_t (&v)[EvalShape<NCH>::R],
                                           bool (&act)[EvalShape<NCH>::R]) {
    constexpr int CB = EvalShape<NCH>::CB, R = EvalShape<NCH>::R;
    constexpr int D4 = NCH * 8;  // 16-byte pieces per row
    const int sub = lane & 7, grp = lane >> 3;
    float acc[RA];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (r < RA) {
            int idx = base + r * 8 + grp;
            act[r] = idx < n;
            v[r] = act[r] ? L[idx] : 0u;
            acc[r] = 0.0f;
        } else {
            act[r] = false; v[r] = 0u; s[r] = 0.0f;
        }
    }
#pragma unroll
    for (int c0 = 0; c0 < NCH; c0 += CB) {
        float4 buf[RA][CB];
#pragma unroll
        for (int r = 0; r < RA; ++r) {
            const float4 *row = reinterpret_cast<const float4 *>(X) + (size_t)v[r] * D4 + sub;
#pragma unroll
            for (int cc = 0; cc < CB; ++cc)
                buf[r][cc] = act[r] ? row[(c0 + cc) * 8] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        auto products = [&](auto l2) __attribute__((always_inline)) {
#pragma unroll
            for (int cc = 0; cc < CB; ++cc) {
                float4 qv;
                if constexpr (EvalShape<NCH>::QREG) qv = qreg[c0 + cc];
                else qv = reinterpret_cast<const float4 *>(qlds)[(c0 + cc) * 8 + sub];
#pragma unroll
                for (int r = 0; r < RA; ++r) acc[r] = fma_piece<decltype(l2)::value>(qv, buf[r][cc], acc[r]);
            }
        };
        GRAB_WITH_METRIC(metric, products);
    }
#pragma unroll
    for (int r = 0; r < RA; ++r) {
        float t = acc[r];
        t += dpp_move<0xB1>(t);   // quad_perm [1,0,3,2]: lane ^ 1
        t += dpp_move<0x4E>(t);   // quad_perm [2,3,0,1]: lane ^ 2
        t += dpp_move<0x141>(t);  // row_half_mirror: the other half of the group of eight
        s[r] = metric == GRAB_L2SQ ? t : -t;
    }
}

// eval_batch_rows for as many rounds as the batch has rows for: a batch that fills a quarter, half or
// three quarters of the 8 R slots skips the loads and the arithmetic of the rounds that would have no
// row in any group
template <int NCH>
__device__ __forceinline__ void eval_batch(const float *__restrict__ X, const float4 *qreg, const float *qlds,
                                           const uint32_t *L, int base, int n, int lane, int metric,
                                           float (&s)[EvalShape<NCH>::R], uint32_t (&v)[EvalShape<NCH>::R],
                                           bool (&act)[EvalShape<NCH>::R]) {
    constexpr int R = EvalShape<NCH>::R;
    const int rounds = (n - base + 7) >> 3;
    if constexpr (R >= 4) {
        if (rounds * 4 <= R) { eval_batch_rows<NCH, R / 4>(X, qreg, qlds, L, base, n, lane, metric, s, v, act); return; }
    }
    if constexpr (R >= 2) {
        if (rounds * 2 <= R) { eval_batch_rows<NCH, R / 2>(X, qreg, qlds, L, base, n, lane, metric, s, v, act); return; }
    }
    if constexpr (R == 4) {
        if (rounds == 3) { eval_batch_rows<NCH, 3>(X, qreg, qlds, L, base, n, lane, metric, s, v, act); return; }
    }
    eval_batch_rows<NCH, R>(X, qreg, qlds, L, base, n, lane, metric, s, v, act);
}

// distances of the n slots in L to the query, written to dist_out[0..n)
template <int NCH>
__device__ __forceinline__ void eval_rows(const float *__restrict__ X, const float4 *qreg, const float *qlds,
                                          const uint32_t *L, int n, int lane, int metric, float *dist_out) {
    constexpr int R = EvalShape<NCH>::R;
    for (int base = 0; base < n; base += 8 * R) {
        float s[R];
        uint32_t v[R];
        bool act[R];
        eval_batch<NCH>(X, qreg, qlds, L, base, n, lane, metric, s, v, act);
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (act[r] && (lane & 7) == 0) dist_out[base + r * 8 + (lane >> 3)] = s[r];
    }
}

// Distances of slots to up to G query rows at once: the rows are read once and every query
// (qs[g][dim] in LDS, used iff bit g of qmask is set) is applied to them while they sit in
// registers, each (query, row) pair in the summation order of eval_batch.  The three steps are
// separate so that a caller can issue the row loads before its query rows have reached LDS.
template <int NCH>
struct RowRegs {
    float4 buf[EvalShape<NCH>::R][EvalShape<NCH>::CB];
    uint32_t v[EvalShape<NCH>::R];
    bool act[EvalShape<NCH>::R];
};
// which rows this lane group takes in the batch that starts at L[base]
template <int NCH>
__device__ __forceinline__ void rows_pick(const uint32_t *L, int base, int n, int lane, RowRegs<NCH> &rr) {
#pragma unroll
    for (int r = 0; r < EvalShape<NCH>::R; ++r) {
        const int idx = base + r * 8 + (lane >> 3);
        rr.act[r] = idx < n;
        rr.v[r] = rr.act[r] ? L[idx] : 0u;
    }
}
// loads pieces c0 .. c0 + CB of those rows
template <int NCH>
__device__ __forceinline__ void rows_issue(const float *__restrict__ X, int c0, int lane, RowRegs<NCH> &rr) {
    constexpr int CB = EvalShape<NCH>::CB, R = EvalShape<NCH>::R, D4 = NCH * 8;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float4 *row = reinterpret_cast<const float4 *>(X) + (size_t)rr.v[r] * D4 + (lane & 7);
#pragma unroll
        for (int cc = 0; cc < CB; ++cc)
            rr.buf[r][cc] = rr.act[r] ? row[(c0 + cc) * 8] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}
template <int NCH, int G>
__device__ __forceinline__ void rows_fma(const RowRegs<NCH> &rr, const float *qs, unsigned qmask, int c0, int lane, int metric,
                                         float (&acc)[G][EvalShape<NCH>::R]) {
    constexpr int CB = EvalShape<NCH>::CB, R = EvalShape<NCH>::R, D4 = NCH * 8;
    const float4 *q4 = reinterpret_cast<const float4 *>(qs);
    auto products = [&](auto l2) __attribute__((always_inline)) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (!((qmask >> g) & 1u)) continue;
#pragma unroll
            for (int cc = 0; cc < CB; ++cc) {
                const float4 qv = q4[g * D4 + (c0 + cc) * 8 + (lane & 7)];
#pragma unroll
                for (int r = 0; r < R; ++r) acc[g][r] = fma_piece<decltype(l2)::value>(qv, rr.buf[r][cc], acc[g][r]);
            }
        }
    };
    GRAB_WITH_METRIC(metric, products);
}
// out[g * 64 + j] = dist(query g, L[j]) for the rows of the batch at `base`
template <int NCH, int G>
__device__ __forceinline__ void rows_store(const RowRegs<NCH> &rr, float (&acc)[G][EvalShape<NCH>::R], unsigned qmask, int base,
                                           int lane, int metric, float *out) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (!((qmask >> g) & 1u)) continue;
#pragma unroll
        for (int r = 0; r < EvalShape<NCH>::R; ++r) {
            float t = acc[g][r];
            t += dpp_move<0xB1>(t);
            t += dpp_move<0x4E>(t);
            t += dpp_move<0x141>(t);
            if (rr.act[r] && (lane & 7) == 0) out[g * 64 + base + r * 8 + (lane >> 3)] = metric == GRAB_L2SQ ? t : -t;
        }
    }
}
// all batches from L[base0] on; n <= 64.  Callers synchronise before qs is written and after out is read.
template <int NCH, int G>
__device__ __forceinline__ void eval_rows_multi(const float *__restrict__ X, const float *qs, unsigned qmask,
                                                const uint32_t *L, int base0, int n, int lane, int metric, float *out) {
    constexpr int CB = EvalShape<NCH>::CB, R = EvalShape<NCH>::R;
    for (int base = base0; base < n; base += 8 * R) {
        RowRegs<NCH> rr;
        rows_pick<NCH>(L, base, n, lane, rr);
        float acc[G][R];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int r = 0; r < R; ++r) acc[g][r] = 0.0f;
#pragma unroll
        for (int c0 = 0; c0 < NCH; c0 += CB) {
            rows_issue<NCH>(X, c0, lane, rr);
            rows_fma<NCH, G>(rr, qs, qmask, c0, lane, metric, acc);
        }
        rows_store<NCH, G>(rr, acc, qmask, base, lane, metric, out);
    }
}

// dist(query row in LDS, L[j]) for n <= 8 slots, one per group of eight lanes, in the summation
// order of eval_batch; out[j] receives it
template <int NCH>
__device__ __forceinline__ void eval_rows_few(const float *__restrict__ X, const float *q, const uint32_t *L, int n, int lane,
                                              int metric, float *out) {
    constexpr int CB = EvalShape<NCH>::CB, D4 = NCH * 8;
    const int sub = lane & 7, grp = lane >> 3;
    const bool act = grp < n;
    const uint32_t v = act ? L[grp] : 0u;
    const float4 *row = reinterpret_cast<const float4 *>(X) + (size_t)v * D4 + sub;
    const float4 *q4 = reinterpret_cast<const float4 *>(q);
    float acc = 0.0f;
#pragma unroll
    for (int c0 = 0; c0 < NCH; c0 += CB) {
        float4 buf[CB];
#pragma unroll
        for (int cc = 0; cc < CB; ++cc) buf[cc] = act ? row[(c0 + cc) * 8] : make_float4(0.f, 0.f, 0.f, 0.f);
        auto products = [&](auto l2) __attribute__((always_inline)) {
#pragma unroll
            for (int cc = 0; cc < CB; ++cc) acc = fma_piece<decltype(l2)::value>(q4[(c0 + cc) * 8 + sub], buf[cc], acc);
        };
        GRAB_WITH_METRIC(metric, products);
    }
    float t = acc;
    t += dpp_move<0xB1>(t);
    t += dpp_move<0x4E>(t);
    t += dpp_move<0x141>(t);
    if (act && sub == 0) out[grp] = metric == GRAB_L2SQ ? t : -t;
}

// dist(query row qa, row qb), both dim floats in LDS, by one group of eight lanes in the summation
// order of eval_batch; every lane of the group returns it
template <int NCH>
__device__ __forceinline__ float dist_lds_rows(const float *qa, const float *qb, int lane, int metric) {
    const int sub = lane & 7;
    const float4 *a4 = reinterpret_cast<const float4 *>(qa), *b4 = reinterpret_cast<const float4 *>(qb);
    float acc = 0.0f;
    auto products = [&](auto l2) __attribute__((always_inline)) {
#pragma unroll 4
        for (int c = 0; c < NCH; ++c) acc = fma_piece<decltype(l2)::value>(a4[c * 8 + sub], b4[c * 8 + sub], acc);
    };
    GRAB_WITH_METRIC(metric, products);
    float t = acc;
    t += dpp_move<0xB1>(t);
    t += dpp_move<0x4E>(t);
    t += dpp_move<0x141>(t);
    return metric == GRAB_L2SQ ? t : -t;
}

// Distances from the row held by each group of eight lanes (mine: piece 8c+sub of that group's
// row) to the rows rows[0..n), the same list for every group, in the summation order of
// eval_batch with `mine` in the place of the query.  f(j, s) is called by every lane of a group
// with the distance s between its row and rows[j].
// `done()` is asked after every batch of rows (the same answer in every lane): true ends the scan early.
template <int NCH, typename F, typename S>
__device__ __forceinline__ void group_vs_rows(const float *__restrict__ X, const float4 (&mine)[NCH], const uint32_t *rows,
                                              int n, int lane, int metric, F &&f, S &&done) {
    constexpr int RR = NCH <= 2 ? 8 : (NCH <= 4 ? 4 : 2);   // rows in flight
    constexpr int D4 = NCH * 8;
    const int sub = lane & 7;
    for (int j0 = 0; j0 < n; j0 += RR) {
        float4 buf[RR][NCH];
#pragma unroll
        for (int r = 0; r < RR; ++r) {
            const uint32_t v = j0 + r < n ? rows[j0 + r] : rows[j0];
            const float4 *row = reinterpret_cast<const float4 *>(X) + (size_t)v * D4 + sub;
#pragma unroll
            for (int c = 0; c < NCH; ++c) buf[r][c] = row[c * 8];
        }
        float acc[RR];
        auto products = [&](auto l2) __attribute__((always_inline)) {
#pragma unroll
            for (int r = 0; r < RR; ++r) {
                acc[r] = 0.0f;
#pragma unroll
                for (int c = 0; c < NCH; ++c) acc[r] = fma_piece<decltype(l2)::value>(mine[c], buf[r][c], acc[r]);
            }
        };
        GRAB_WITH_METRIC(metric, products);
#pragma unroll
        for (int r = 0; r < RR; ++r) {
            float t = acc[r];
            t += dpp_move<0xB1>(t);
            t += dpp_move<0x4E>(t);
            t += dpp_move<0x141>(t);
            if (j0 + r < n) f(j0 + r, metric == GRAB_L2SQ ? t : -t);
        }
        if (done()) break;
    }
}

// Remote edge selection (Section 4.3, Remote Edge Construction) for one node per wavefront.
// gs[0..ng) / gd: candidate slots and distances ordered by (distance, slot), GRAB_EMPTY-padded.
// A candidate is proximal iff its attribute differs from attr_u by at most `window`.  pk[0..kp)
// receives the first kp proximal candidates, pk[kp..kr) the first kr - kp others, pkd their
// distances; GRAB_EMPTY where a class runs out.  pk / pkd are LDS; every lane of the workgroup
// (one wavefront) must call.
__device__ __forceinline__ void select_remote_wave(const uint32_t *__restrict__ gs, const float *__restrict__ gd, int ng,
                                                   const int32_t *__restrict__ attr, int32_t attr_u, int64_t window,
                                                   int kp, int kr, int lane, uint32_t *pk, float *pkd) {
    for (int j = lane; j < kr; j += 64) { pk[j] = GRAB_EMPTY; pkd[j] = 0.0f; }
    __syncthreads();
    const u64 lt_mask = (1ull << lane) - 1ull;
    int np = 0, ngl = 0;
    for (int c0 = 0; c0 < ng && (np < kp || ngl < kr - kp); c0 += 64) {
        const int t = c0 + lane;
        const uint32_t c = t < ng ? gs[t] : GRAB_EMPTY;
        const bool valid = c != GRAB_EMPTY;
        bool prox = false;
        if (valid) {
            long long diff = (long long)attr[c] - (long long)attr_u;
            if (diff < 0) diff = -diff;
            prox = diff <= window;
        }
        const u64 mp = __ballot(valid && prox), mg = __ballot(valid && !prox);
        if (valid && prox) {
            const int r = np + __popcll(mp & lt_mask);
            if (r < kp) { pk[r] = c; pkd[r] = gd[t]; }
        }
        if (valid && !prox) {
            const int r = ngl + __popcll(mg & lt_mask);
            if (r < kr - kp) { pk[kp + r] = c; pkd[kp + r] = gd[t]; }
        }
        np += __popcll(mp);
        ngl += __popcll(mg);
    }
    __syncthreads();
}

// what the freshness bias of Eq. 3 scales: the distance itself for squared L2; for minus the inner
// product, which is negative for similar vectors, max(0, 1 + d): half the squared Euclidean
// distance on unit vectors
__device__ __forceinline__ float bias_base(float d, int metric) {
    if (metric == GRAB_L2SQ) return d;
    const float s = 1.0f + d;
    return s > 0.0f ? s : 0.0f;
}

// the "query" side of eval_rows from a row in memory: registers for rows up to 256 floats,
// LDS (qlds, dim floats) beyond; callers synchronise before the next eval_rows
template <int NCH>
__device__ __forceinline__ void load_query(const float *__restrict__ row, float4 *qreg, float *qlds, int lane) {
    const float4 *src = reinterpret_cast<const float4 *>(row);
    if constexpr (EvalShape<NCH>::QREG) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) qreg[c] = src[c * 8 + (lane & 7)];
    } else {
        for (int i = lane; i < NCH * 8; i += 64) reinterpret_cast<float4 *>(qlds)[i] = src[i];
    }
}

}  // namespace
