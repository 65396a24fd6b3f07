// Device-side helpers shared by the search and append kernels (gfx950 only): queue keys,
// wave reductions and the gathered fp32 distance with its fixed summation order.
#pragma once

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

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) v += __shfl_xor(v, m);
    return v;
}

// ---- a 64-entry queue held one key per lane, sorted and merged with lane exchanges ----------
__device__ __forceinline__ u64 shfl64(u64 k, int src) {
    return ((u64)(uint32_t)__shfl((int)(k >> 32), src) << 32) | (u64)(uint32_t)__shfl((int)(k & 0xFFFFFFFFull), src);
}
__device__ __forceinline__ u64 shfl_xor64(u64 k, int m) {
    return ((u64)(uint32_t)__shfl_xor((int)(k >> 32), m) << 32) | (u64)(uint32_t)__shfl_xor((int)(k & 0xFFFFFFFFull), m);
}
// ascending bitonic sort of the keys of lanes [0,P); lanes beyond hold SENT and stay put
__device__ __forceinline__ u64 sort_lanes(u64 key, int P, int lane) {
    for (int k = 2; k <= P; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            u64 o = shfl_xor64(key, j);
            bool take_min = ((lane & j) == 0) == ((lane & k) == 0);
            bool less = key < o;
            key = (less == take_min) ? key : o;
        }
    return key;
}
// queue (sorted, one key per lane) <- the 64 smallest of queue and ck (sorted), cut to beam
__device__ __forceinline__ u64 merge_lanes(u64 qk, u64 ck, int beam, int lane) {
    u64 r = shfl64(ck, 63 - lane);
    u64 m = qk < r ? qk : r;
#pragma unroll
    for (int j = 32; j > 0; j >>= 1) {
        u64 o = shfl_xor64(m, j);
        bool take_min = (lane & j) == 0;
        bool less = m < o;
        m = (less == take_min) ? m : o;
    }
    return lane < beam ? m : SENT;
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
        const u64 rv = shfl64(ck, 63 - lane);
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
        for (int j = 32; j > 0; j >>= 1) {
            const bool take_min = (lane & j) == 0;
#pragma unroll
            for (int r = 0; r < M; ++r) {
                const u64 o = shfl_xor64(k[r], j);
                const bool less = k[r] < o;
                k[r] = (less == take_min) ? k[r] : o;
            }
        }
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
        return shfl64(t, p & 63);
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
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}

// Gathered distances (Algorithm 2, ComputeDistance) for up to 8*R slots L[base..]: eight lanes
// share a row, lane `sub` of a group takes the 16-byte pieces 8c+sub (one 128-byte line per
// piece index across the group) and accumulates them in index order with fused multiply-adds;
// the eight partial sums are combined pairwise (lanes 0+1, 2+3, ..., then pairs, then halves).
// This fixed order makes the fp32 result reproducible bit for bit.  All loads of the batch are
// issued before the first multiply.  Every lane of a group ends with the row's distance in
// s[r]; v[r] is the row's slot and act[r] tells whether round r had a row for this group.
template <int NCH>
__device__ __forceinline__ void eval_batch(const float *__restrict__ X, const float4 *qreg, const float *qlds,
                                           const uint32_t *L, int base, int n, int lane, int metric,
                                           float (&s)[EvalShape<NCH>::R], uint32_t (&v)[EvalShape<NCH>::R],
                                           bool (&act)[EvalShape<NCH>::R]) {
    constexpr int CB = EvalShape<NCH>::CB, R = EvalShape<NCH>::R;
    constexpr int D4 = NCH * 8;  // 16-byte pieces per row
    const int sub = lane & 7, grp = lane >> 3;
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int idx = base + r * 8 + grp;
        act[r] = idx < n;
        v[r] = act[r] ? L[idx] : 0u;
        acc[r] = 0.0f;
    }
#pragma unroll
    for (int c0 = 0; c0 < NCH; c0 += CB) {
        float4 buf[R][CB];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float4 *row = reinterpret_cast<const float4 *>(X) + (size_t)v[r] * D4 + sub;
#pragma unroll
            for (int cc = 0; cc < CB; ++cc)
                buf[r][cc] = act[r] ? row[(c0 + cc) * 8] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int cc = 0; cc < CB; ++cc) {
            float4 qv;
            if constexpr (EvalShape<NCH>::QREG) qv = qreg[c0 + cc];
            else qv = reinterpret_cast<const float4 *>(qlds)[(c0 + cc) * 8 + sub];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                float4 x = buf[r][cc];
                if (metric == GRAB_L2SQ) {
                    float dx = qv.x - x.x, dy = qv.y - x.y, dz = qv.z - x.z, dw = qv.w - x.w;
                    acc[r] = __builtin_fmaf(dx, dx, acc[r]);
                    acc[r] = __builtin_fmaf(dy, dy, acc[r]);
                    acc[r] = __builtin_fmaf(dz, dz, acc[r]);
                    acc[r] = __builtin_fmaf(dw, dw, acc[r]);
                } else {
                    acc[r] = __builtin_fmaf(qv.x, x.x, acc[r]);
                    acc[r] = __builtin_fmaf(qv.y, x.y, acc[r]);
                    acc[r] = __builtin_fmaf(qv.z, x.z, acc[r]);
                    acc[r] = __builtin_fmaf(qv.w, x.w, acc[r]);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float t = acc[r];
        t += dpp_move<0xB1>(t);   // quad_perm [1,0,3,2]: lane ^ 1
        t += dpp_move<0x4E>(t);   // quad_perm [2,3,0,1]: lane ^ 2
        t += dpp_move<0x141>(t);  // row_half_mirror: the other half of the group of eight
        s[r] = metric == GRAB_L2SQ ? t : -t;
    }
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
