// Exact nearest neighbours inside a bucket for the construction (Section 4.3, local k-NN graph and
// nearest node of a target bucket), as a matrix-core filter followed by an exact re-rank.
//
// All pairwise inner products of a bucket are one dense contraction, the only one in this library,
// so they run on the matrix cores: every fp32 value x is split into two bf16 terms h + m with
// |x - h - m| <= 2^-18 |x|, and u.v is taken as uh.vh + uh.vm + um.vh by 32x32x16 bf16 MFMAs with
// fp32 accumulation.  That gives every (source, target) pair a score s~ = |v|^2 / 2 - u.v (minus
// the inner product under that metric) whose distance from the score of the library's fixed-order
// fp32 distance is at most W = kappa (|u| + max |v|)^2 (file comment of the margin below).  Scores
// only FILTER: a source keeps, in a list of its own, every target whose score is within 2 W of the
// P-th smallest score seen so far, which provably contains its P nearest targets under the
// canonical distance; those few candidates are then evaluated with the canonical distance itself
// and ordered by (distance, slot), so the output is bit for bit what the all-fp32 kernel gives.
//
// Margin.  Let tau~ be the P-th smallest score of a source.  P targets have s~ <= tau~, hence
// canonical score <= tau~ + W, hence the P-th smallest canonical score is <= tau~ + W, hence each of
// the P nearest targets has canonical score <= tau~ + W and s~ <= tau~ + 2 W.  W bounds, with room to
// spare, the split (3 * 2^-18 |u||v|), the fp32 accumulation of 3 dim products whatever its
// rounding (3 dim 2^-23 |u||v|), the rounding of |v|^2 / 2 and the rounding of the canonical sum
// (dim 2^-24 of the distance): kappa = 2^-14 + dim 2^-21.
#include <new>

#include "grab_device.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int FT = 128;        // source rows, and targets per step, of a workgroup (2 x 4 wavefronts of 64 x 32)
// A step stages 16 * KS floats of every row; rows are cut so that a pass over a row takes an even
// number of steps (two register sets take turns fetching ahead, without any copying between them)
template <int NCH>
struct StepShape {
    static constexpr int KS = NCH % 2 == 0 ? 2 : NCH;             // 16-float pieces per step: 32, 96 and 160 floats go in two steps
    static constexpr int KC = 16 * KS;                             // floats per step
    static constexpr int STEPS = NCH * 32 / KC;                    // steps per row, even
    static constexpr int PITCH = KC + 8;                           // bf16 per staged row: 16 bytes of padding (conflict-free 16-byte reads)
    static constexpr int PIECES = FT * 2 * KS;                     // 16-byte pieces per matrix and term and step
    static constexpr int NPT = (PIECES + 511) / 512;               // of them per thread
};
constexpr int FT_CAP = 512;    // entries of a source's candidate list
constexpr int FT_OUT = 256;    // most candidates a source may hand to the exact re-rank

__device__ __forceinline__ uint16_t bf16_rn(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_val(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// x = h + m (+ at most 2^-18 |x|); half the squared norm (zero under the inner-product metric), the
// norm, and the largest norm of the index.  One wavefront per 16 rows.
constexpr int SPLIT_ROWS = 16;
__global__ __launch_bounds__(256) void k_split_rows(const float *__restrict__ X, int64_t n_slots, int32_t D, int32_t metric,
                                                    uint16_t *__restrict__ Xh, uint16_t *__restrict__ Xm,
                                                    float *__restrict__ hn, float *__restrict__ nrm, uint32_t *__restrict__ maxnorm) {
    __shared__ uint32_t wg_max;
    if (threadIdx.x == 0) wg_max = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int64_t row0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * SPLIT_ROWS;
    float biggest = 0.0f;
    for (int64_t row = row0; row < row0 + SPLIT_ROWS && row < n_slots; ++row) {
        float ss = 0.0f;
        for (int k = 2 * lane; k < D; k += 128) {
            const float2 x = *reinterpret_cast<const float2 *>(X + row * D + k);
            const uint16_t h0 = bf16_rn(x.x), h1 = bf16_rn(x.y);
            const uint16_t m0 = bf16_rn(x.x - bf16_val(h0)), m1 = bf16_rn(x.y - bf16_val(h1));
            *reinterpret_cast<uint32_t *>(Xh + row * D + k) = (uint32_t)h0 | ((uint32_t)h1 << 16);
            *reinterpret_cast<uint32_t *>(Xm + row * D + k) = (uint32_t)m0 | ((uint32_t)m1 << 16);
            ss = __builtin_fmaf(x.x, x.x, ss);
            ss = __builtin_fmaf(x.y, x.y, ss);
        }
#pragma unroll
        for (int sft = 32; sft > 0; sft >>= 1) ss += __shfl_xor(ss, sft);
        const float n = __builtin_sqrtf(ss) * 1.000001f;
        if (lane == 0) {
            hn[row] = metric == GRAB_L2SQ ? 0.5f * ss : 0.0f;
            nrm[row] = n;
        }
        biggest = n > biggest ? n : biggest;
    }
    if (lane == 0) atomicMax(&wg_max, __float_as_uint(biggest));   // non-negative floats order like their bit patterns
    __syncthreads();
    if (threadIdx.x == 0) atomicMax(maxnorm, wg_max);
}

struct FilterArgs {
    const uint16_t *Xh, *Xm;   // [n_slots][D] bf16 terms
    const float *hn, *nrm;
    const uint32_t *maxnorm;
    const float *X;
    const int32_t *table, *tgt;
    const int32_t *blk_start;  // [B + 1]: first work item of each source bucket (items = blocks of FT rows)
    int32_t B, n_items;
    uint32_t *out_s;
    float *out_d;
    int64_t out_stride, out_off, n_slots;
    int32_t P, metric, exclude_self;
    u64 *lists;                // [gridDim.x][FT][FT_CAP]: score image << 32 | target slot
    uint32_t *cand;            // [n_slots][FT_OUT]: the candidates of every row after the last cut
    int32_t *n_cand;           // [n_slots]
    const uint32_t *slot2id;
    uint32_t *overflow;        // set when a list could not be cut below its capacity (the pass is then void)
    float kappa;
};

// Cuts the list of source row r (of this workgroup) to the entries within w2 of its P-th smallest
// score and sets the row's threshold to that bound; the entries kept are also returned in k[]
// (SENT elsewhere), their number in the return value.  One wavefront; every lane calls.
__device__ __forceinline__ int prune_row(const FilterArgs &a, u64 *list, int r, int lane, float *thr, const float *w2, int *cnt,
                                         u64 (&k)[FT_CAP / 64]) {
    int n = cnt[r];
    if (n > FT_CAP) { n = FT_CAP; if (lane == 0) atomicExch(a.overflow, 1u); }
#pragma unroll
    for (int j = 0; j < FT_CAP / 64; ++j) k[j] = j * 64 + lane < n ? list[(size_t)r * FT_CAP + j * 64 + lane] : SENT;
    float bound = __builtin_inff();
    if (n > a.P) {
        // the P-th smallest score image, bit by bit from the top
        uint32_t prefix = 0;
        int want = a.P;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t hi_mask = bit == 31 ? 0u : (0xFFFFFFFFu << (bit + 1));
            int zeros = 0;
#pragma unroll
            for (int j = 0; j < FT_CAP / 64; ++j) {
                if (j * 64 >= n) continue;   // the same in every lane
                const uint32_t img = (uint32_t)(k[j] >> 32);
                zeros += __popcll(__ballot(k[j] != SENT && (img & hi_mask) == prefix && !((img >> bit) & 1u)));
            }
            if (want > zeros) { want -= zeros; prefix |= 1u << bit; }
        }
        bound = image_dist(prefix) + w2[r];
    }
    int kept = 0;
#pragma unroll
    for (int j = 0; j < FT_CAP / 64; ++j) {
        const bool keep = k[j] != SENT && image_dist((uint32_t)(k[j] >> 32)) <= bound;
        const u64 m = __ballot(keep);
        if (keep) list[(size_t)r * FT_CAP + kept + __popcll(m & ((1ull << lane) - 1ull))] = k[j];
        else k[j] = SENT;
        kept += __popcll(m);
    }
    if (lane == 0) {
        cnt[r] = kept;
        thr[r] = bound;
        if (kept > FT_CAP - FT) atomicExch(a.overflow, 1u);
    }
    return kept;
}

// One step (16 KS floats from float kc * KC on) of the workgroup's 128 source rows (from slot src0)
// and of 128 target rows (from slot tgt0), both terms, into registers: 16-byte pieces, NPT per thread
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a plain vector: stays in registers where HIP's uint4 class does not
template <int NPT>
struct StepRegs { u32x4 ah[NPT], am[NPT], bh[NPT], bm[NPT]; };
template <int NCH, bool ARES>
__device__ __forceinline__ void fetch_step(const FilterArgs &a, int64_t src0, int64_t tgt0, int kc, int tid,
                                           StepRegs<StepShape<NCH>::NPT> &g) {
    typedef StepShape<NCH> S;
    constexpr int D = NCH * 32;
#pragma unroll
    for (int i = 0; i < S::NPT; ++i) {
        const int idx = tid + 512 * i;
        const int row = (S::PIECES % 512 != 0 && idx >= S::PIECES) ? 0 : idx / (2 * S::KS), q = (S::PIECES % 512 != 0 && idx >= S::PIECES) ? 0 : idx - row * (2 * S::KS);
        int64_t sa = src0 + row, sbv = tgt0 + row;
        if (sa >= a.n_slots) sa = a.n_slots - 1;
        if (sbv >= a.n_slots) sbv = a.n_slots - 1;
        const size_t ga = (size_t)sa * D + kc * S::KC + 8 * q, gb = (size_t)sbv * D + kc * S::KC + 8 * q;
        if constexpr (!ARES) {
            g.ah[i] = *reinterpret_cast<const u32x4 *>(a.Xh + ga);
            g.am[i] = *reinterpret_cast<const u32x4 *>(a.Xm + ga);
        }
        g.bh[i] = *reinterpret_cast<const u32x4 *>(a.Xh + gb);
        g.bm[i] = *reinterpret_cast<const u32x4 *>(a.Xm + gb);
    }
}

// Workgroup barrier that orders LDS traffic only: the global loads fetched ahead stay in flight
// across it (__syncthreads would wait for them too)
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Workgroup of eight wavefronts, 2 x 4: wavefront (wr, wc) owns the scores of source rows
// 64 wr .. 64 wr + 63 against targets 32 wc .. 32 wc + 31 of the current 128.
template <int NCH>
__global__ __launch_bounds__(512) void k_knn_filter(FilterArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    // Rows of up to 128 floats: the workgroup's source rows stay in LDS, whole, for all of its work on
    // them (fetched again for every 128 targets they were most of the traffic, and the traffic, not
    // the matrix cores, set the pace); longer rows are staged 32 floats at a time like the targets.
    typedef StepShape<NCH> S;
    constexpr int D = NCH * 32;
    constexpr bool ARES = NCH <= 4;
    constexpr int APITCH = ARES ? D + 8 : S::PITCH;                // bf16 per source row in LDS
    constexpr int FT_PITCH = S::PITCH;
    uint16_t *sA = reinterpret_cast<uint16_t *>(smem);             // [2 terms][FT][APITCH]
    uint16_t *sB = sA + 2 * FT * APITCH;                           // [2 terms][FT][FT_PITCH]
    unsigned char *tail = smem + (size_t)2 * FT * (APITCH + FT_PITCH) * 2;
    float *thr = reinterpret_cast<float *>(tail);                  // [FT] a target is listed iff its score <= thr
    float *w2 = thr + FT;                                          // [FT] twice the margin of the row
    int *cnt = reinterpret_cast<int *>(w2 + FT);                   // [FT] entries in the row's list
    int *flags = cnt + FT;                                         // [0]: some list is nearly full
    float *sc = reinterpret_cast<float *>(flags + 4) + (size_t)(threadIdx.x >> 6) * 1024;   // per wavefront: the scores of one block
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, wr = w >> 2, wc = w & 3;
    const int lrow = lane & 31, lhalf = lane >> 5;
    u64 *list = a.lists + (size_t)blockIdx.x * FT * FT_CAP;
    const float maxn = __uint_as_float(*a.maxnorm);
    // a list is cut to what can still matter when it has grown to a few times P (early cuts make the
    // threshold tight early), at the latest where the next 128 targets could overflow it
    const int trigger = 3 * a.P + 61 < FT_CAP - FT ? 3 * a.P + 61 : FT_CAP - FT;

    for (int item = blockIdx.x; item < a.n_items; item += gridDim.x) {
        // source bucket of the item: the last b with blk_start[b] <= item
        int b = 0;
        {
            int l = 0, r = a.B;
            while (r - l > 1) { const int m = (l + r) >> 1; if (a.blk_start[m] <= item) l = m; else r = m; }
            b = l;
        }
        const int sb = a.table[T_COLS * b + T_BASE], sn = a.table[T_COLS * b + T_NTOT];
        const int i0 = (item - a.blk_start[b]) * FT;
        const int t = a.tgt[b];
        const int tb = t >= 0 ? a.table[T_COLS * t + T_BASE] : 0, tn = t >= 0 ? a.table[T_COLS * t + T_NTOT] : 0;
        __syncthreads();   // the previous item is done with the shared arrays
        if (tid < FT) {
            const bool valid = i0 + tid < sn;
            const float nu = valid ? a.nrm[sb + i0 + tid] : 0.0f;
            thr[tid] = valid ? __builtin_inff() : -__builtin_inff();
            w2[tid] = 2.0f * a.kappa * (nu + maxn) * (nu + maxn);
            cnt[tid] = 0;
        }
        if (tid == 0) flags[0] = 0;
        __syncthreads();

        // ---------------------------------------------------------------- filter: scores on the matrix cores
        // Every step stages 32 floats of the 128 source and 128 target rows through LDS.  Two register
        // sets take turns, each asked for the step after next as soon as it has been written to LDS,
        // so a fetch has two steps of matrix work to arrive.
        if constexpr (ARES) {
            if (tn > 0) {
                for (int idx = tid; idx < FT * (D / 8); idx += 512) {
                    const int row = idx / (D / 8), q = idx - row * (D / 8);
                    int64_t sa = (int64_t)sb + i0 + row;
                    if (sa >= a.n_slots) sa = a.n_slots - 1;
                    *reinterpret_cast<u32x4 *>(sA + row * APITCH + 8 * q) = *reinterpret_cast<const u32x4 *>(a.Xh + (size_t)sa * D + 8 * q);
                    *reinterpret_cast<u32x4 *>(sA + FT * APITCH + row * APITCH + 8 * q) = *reinterpret_cast<const u32x4 *>(a.Xm + (size_t)sa * D + 8 * q);
                }
            }
        }
        StepRegs<S::NPT> g0, g1;
        const int n_steps = tn > 0 ? ((tn + FT - 1) / FT) * S::STEPS : 0;
        if (n_steps > 0) {
            fetch_step<NCH, ARES>(a, sb + i0, tb, 0, tid, g0);
            fetch_step<NCH, ARES>(a, sb + i0, tb, 1, tid, g1);
        }
        int step = 0;
        for (int j0 = 0; j0 < tn; j0 += FT) {
            f32x16 acc[2];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[rb][i] = 0.0f;
            const int col = 32 * wc + lrow;
            const bool validc = j0 + col < tn;
            const uint32_t tslot = (uint32_t)(tb + j0 + col);
            const float hnv = validc ? a.hn[tb + j0 + col] : 0.0f;
            // one step: the registers fetched two steps ago go to LDS, the same registers are asked for
            // the step after next, then the matrix cores take this step from LDS
            auto do_step = [&](StepRegs<S::NPT> &g, int kc) {
                lds_barrier();
#pragma unroll
                for (int i = 0; i < S::NPT; ++i) {
                    const int idx = tid + 512 * i;
                    if (S::PIECES % 512 != 0 && idx >= S::PIECES) continue;
                    const int row = idx / (2 * S::KS), q = idx - row * (2 * S::KS);
                    const int lo = row * FT_PITCH + 8 * q;
                    if constexpr (!ARES) {
                        *reinterpret_cast<u32x4 *>(sA + lo) = g.ah[i];
                        *reinterpret_cast<u32x4 *>(sA + FT * FT_PITCH + lo) = g.am[i];
                    }
                    *reinterpret_cast<u32x4 *>(sB + lo) = g.bh[i];
                    *reinterpret_cast<u32x4 *>(sB + FT * FT_PITCH + lo) = g.bm[i];
                }
                lds_barrier();
                {
                    // the step after next: the same place in this pass over the rows, or in the next 128
                    // targets.  Asked for without condition (past the end the row numbers are clamped and the
                    // data never used): a conditional load would make every later wait a wait for all loads.
                    const int kn = kc + 2 < S::STEPS ? kc + 2 : kc + 2 - S::STEPS;
                    fetch_step<NCH, ARES>(a, sb + i0, tb + j0 + (kc + 2 < S::STEPS ? 0 : FT), kn, tid, g);
                }
#pragma unroll
                for (int ks = 0; ks < S::KS; ++ks) {
                    bf16x8 ah[2], am[2];
                    const int co = (32 * wc + lrow) * FT_PITCH + 16 * ks + 8 * lhalf;
                    const bf16x8 bh = *reinterpret_cast<const bf16x8 *>(sB + co);
                    const bf16x8 bm = *reinterpret_cast<const bf16x8 *>(sB + FT * FT_PITCH + co);
#pragma unroll
                    for (int x = 0; x < 2; ++x) {
                        const int ro = (64 * wr + 32 * x + lrow) * APITCH + (ARES ? kc * S::KC : 0) + 16 * ks + 8 * lhalf;
                        ah[x] = *reinterpret_cast<const bf16x8 *>(sA + ro);
                        am[x] = *reinterpret_cast<const bf16x8 *>(sA + FT * APITCH + ro);
                    }
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb) {
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[rb], bh, acc[rb], 0, 0, 0);
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[rb], bm, acc[rb], 0, 0, 0);
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am[rb], bh, acc[rb], 0, 0, 0);
                    }
                }
                ++step;
            };
#pragma unroll 1
            for (int kc = 0; kc < S::STEPS; kc += 2) {
                do_step(g0, kc);
                do_step(g1, kc + 1);
            }
            // element i of a block in lane l: row (i / 4) * 8 + (l / 32) * 4 + i % 4, column l % 32
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                // thresholds of the sixteen rows this lane sees in the block: four runs of four consecutive rows
                float4 t4[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) t4[g] = *reinterpret_cast<const float4 *>(thr + 64 * wr + 32 * rb + 8 * g + 4 * lhalf);
                // which of its sixteen elements are at or below their rows' thresholds: mostly none once
                // the lists have filled
                uint32_t hits = 0;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float tv = (i & 3) == 0 ? t4[i >> 2].x : ((i & 3) == 1 ? t4[i >> 2].y : ((i & 3) == 2 ? t4[i >> 2].z : t4[i >> 2].w));
                    hits |= (hnv - acc[rb][i] <= tv ? 1u : 0u) << i;
                }
                if (!validc) hits = 0;
                if (__ballot(hits != 0) == 0) continue;
                // The block's scores go through LDS so that a lane can walk its own hits in an ordinary
                // loop (unrolled over the sixteen elements it doubles the kernel's register count).  Each hit
                // claims its place in its row's list by itself: the order inside a list is of no
                // consequence, lists are cut by value and the survivors are ordered by their exact keys.
#pragma unroll
                for (int i = 0; i < 16; ++i) sc[i * 64 + lane] = hnv - acc[rb][i];
                while (hits) {
                    const int i = __builtin_ctz(hits);
                    hits &= hits - 1;
                    const int row = 64 * wr + 32 * rb + (i >> 2) * 8 + (i & 3) + 4 * lhalf;
                    if (a.exclude_self && tslot == (uint32_t)(sb + i0 + row)) continue;
                    const float s = sc[i * 64 + lane];
                    const int pos = atomicAdd(&cnt[row], 1);
                    if (pos < FT_CAP) list[(size_t)row * FT_CAP + pos] = ((u64)dist_image(s) << 32) | (u64)tslot;
                    if (pos >= trigger) flags[0] = 1;
                }
            }
            lds_barrier();   // the fetches for the next 128 targets stay in flight
            if (flags[0]) {
                // lists that have grown are cut to what can still matter (their entries were written by
                // several wavefronts: wait for those stores)
                __syncthreads();
                u64 k[FT_CAP / 64];
                for (int r = w; r < FT; r += 8)
                    if (cnt[r] > trigger) (void)prune_row(a, list, r, lane, thr, w2, cnt, k);
                __syncthreads();
                if (tid == 0) flags[0] = 0;
            }
        }
        __syncthreads();

        // ---------------------------------------------------------------- final cut: the candidates of every row
        for (int r = w; r < FT; r += 8) {
            if (i0 + r >= sn) continue;
            const int64_t slot_u = (int64_t)sb + i0 + r;
            u64 k[FT_CAP / 64];
            const int nc = tn > 0 ? prune_row(a, list, r, lane, thr, w2, cnt, k) : 0;
            if (nc > FT_OUT) { if (lane == 0) atomicExch(a.overflow, 1u); continue; }
            int at = 0;
            if (nc > 0) {
#pragma unroll
                for (int j = 0; j < FT_CAP / 64; ++j) {
                    const bool keep = k[j] != SENT;
                    const u64 m = __ballot(keep);
                    if (keep) a.cand[slot_u * FT_OUT + at + __popcll(m & ((1ull << lane) - 1ull))] = (uint32_t)(k[j] & 0xFFFFFFFFull);
                    at += __popcll(m);
                }
            }
            if (lane == 0) a.n_cand[slot_u] = nc;
        }
    }
}

// Exact distances of a row's candidates in the library's fixed summation order, ordered by
// (distance, slot); the first P are the row's nearest targets.  One wavefront per row.
template <int NCH, int PM>
__global__ __launch_bounds__(64) void k_knn_rerank(FilterArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int D = NCH * 32;
    uint32_t *mycand = reinterpret_cast<uint32_t *>(smem);
    float *mydist = reinterpret_cast<float *>(mycand + FT_OUT);
    float *qlds = mydist + FT_OUT;
    const int lane = threadIdx.x;
    const int64_t slot_u = blockIdx.x;
    if (a.slot2id[slot_u] == GRAB_EMPTY) return;
    const int nc = a.n_cand[slot_u];
    LaneQueue<PM> q;
    q.clear();
    if (nc > 0) {
        for (int x = lane; x < nc; x += 64) mycand[x] = a.cand[slot_u * FT_OUT + x];
        float4 qreg[EvalShape<NCH>::QREG ? NCH : 1];
        load_query<NCH>(a.X + (size_t)slot_u * D, qreg, qlds, lane);
        __syncthreads();
        eval_rows<NCH>(a.X, qreg, qlds, mycand, nc, lane, a.metric, mydist);
        __syncthreads();
        for (int c0 = 0; c0 < nc; c0 += 64) {
            u64 key = c0 + lane < nc ? make_key(mydist[c0 + lane], mycand[c0 + lane]) : SENT;
            key = sort_lanes(key, 64, lane);
            q.merge(key, a.P, lane);
        }
    }
    if (a.P == 1) {
        const u64 best = q.at(0);
        if (lane == 0) a.out_s[slot_u * a.out_stride + a.out_off] = best == SENT ? GRAB_EMPTY : key_slot(best);
    } else {
#pragma unroll
        for (int m = 0; m < PM; ++m) {
            const int pos = 64 * m + lane;
            if (pos < a.P) {
                const u64 kk = q.k[m];
                const bool has = kk != SENT;
                a.out_s[slot_u * a.P + pos] = has ? key_slot(kk) : GRAB_EMPTY;
                a.out_d[slot_u * a.P + pos] = has ? image_dist((uint32_t)(kk >> 32)) : __builtin_inff();
            }
        }
    }
}

template <int NCH>
grab_status launch_filter_t(grab_index *ix, const FilterArgs &a, unsigned grid) {
    const size_t lds = (size_t)2 * FT * ((NCH <= 4 ? NCH * 32 + 8 : StepShape<NCH>::PITCH) + StepShape<NCH>::PITCH) * 2 + (size_t)FT * 12 + 16 + (size_t)8 * 1024 * 4;
    k_knn_filter<NCH><<<dim3(grid), dim3(512), lds, ix->stream>>>(a);
    GRAB_HIP(ix, hipGetLastError());
    const size_t lds2 = (size_t)FT_OUT * 8 + (EvalShape<NCH>::QREG ? 0 : (size_t)NCH * 32 * 4);
    if (a.P > 64) k_knn_rerank<NCH, 2><<<dim3((unsigned)a.n_slots), dim3(64), lds2, ix->stream>>>(a);
    else k_knn_rerank<NCH, 1><<<dim3((unsigned)a.n_slots), dim3(64), lds2, ix->stream>>>(a);
    GRAB_HIP(ix, hipGetLastError());
    return GRAB_OK;
}

}  // namespace

struct KnnFilter {
    uint16_t *Xh = nullptr, *Xm = nullptr;
    float *hn = nullptr, *nrm = nullptr;
    uint32_t *maxnorm = nullptr, *overflow = nullptr;
    int32_t *blk_start = nullptr;
    u64 *lists = nullptr;
    uint32_t *cand = nullptr;
    int32_t *n_cand = nullptr;
    int32_t n_items = 0;
    unsigned grid = 0;
};

void grab_knn_release(KnnFilter *f) {
    if (!f) return;
    (void)hipFree(f->Xh); (void)hipFree(f->Xm); (void)hipFree(f->hn); (void)hipFree(f->nrm);
    (void)hipFree(f->maxnorm); (void)hipFree(f->blk_start); (void)hipFree(f->lists); (void)hipFree(f->cand); (void)hipFree(f->n_cand);
    delete f;
}

// Splits the rows of the index into their bf16 terms and sets up the work list (one item per 128
// rows of a bucket) and the candidate lists of the filter.  GRAB_ENOMEM leaves *out null: the
// caller then uses the all-fp32 kernel.
grab_status grab_knn_prepare(grab_index *ix, KnnFilter **out) {
    *out = nullptr;
    KnnFilter *f = new (std::nothrow) KnnFilter;
    if (!f) return grab_fail(ix, GRAB_ENOMEM, "host allocation failed");
    const int64_t N = ix->n_slots;
    const int32_t B = ix->B, D = ix->dim;
    std::vector<int32_t> h((size_t)B + 1, 0);
    for (int b = 0; b < B; ++b) h[b + 1] = h[b] + (ix->h_table[T_COLS * b + T_NTOT] + FT - 1) / FT;
    f->n_items = h[B];
    f->grid = (unsigned)(f->n_items < 512 ? (f->n_items > 0 ? f->n_items : 1) : 512);
    hipError_t e = hipSuccess;
    auto alloc = [&](void **p, size_t bytes) { if (e == hipSuccess) e = hipMalloc(p, bytes ? bytes : 16); };
    alloc((void **)&f->Xh, (size_t)N * D * 2); alloc((void **)&f->Xm, (size_t)N * D * 2);
    alloc((void **)&f->hn, (size_t)N * 4); alloc((void **)&f->nrm, (size_t)N * 4);
    alloc((void **)&f->maxnorm, 16);
    alloc((void **)&f->blk_start, ((size_t)B + 1) * 4);
    alloc((void **)&f->lists, (size_t)f->grid * FT * FT_CAP * 8);
    alloc((void **)&f->cand, (size_t)N * FT_OUT * 4);
    alloc((void **)&f->n_cand, (size_t)N * 4);
    if (e != hipSuccess) { grab_knn_release(f); return grab_fail(ix, GRAB_ENOMEM, "construction filter needs more device memory: %s", hipGetErrorString(e)); }
    f->overflow = f->maxnorm + 1;
    hipStream_t st = ix->stream;
    if ((e = hipMemsetAsync(f->maxnorm, 0, 16, st)) == hipSuccess)
        e = hipMemcpyAsync(f->blk_start, h.data(), h.size() * 4, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) {
        k_split_rows<<<dim3((unsigned)((N + 4 * SPLIT_ROWS - 1) / (4 * SPLIT_ROWS))), dim3(256), 0, st>>>(ix->X, N, D, ix->metric, f->Xh, f->Xm, f->hn, f->nrm, f->maxnorm);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);   // blk_start's host copy goes out of scope
    if (e != hipSuccess) { grab_knn_release(f); return grab_fail(ix, GRAB_EHIP, "construction filter set-up failed: %s", hipGetErrorString(e)); }
    *out = f;
    return GRAB_OK;
}

// One pass: for every object the P nearest objects of its bucket's target bucket (d_tgt[b], -1: none),
// written as the all-fp32 kernel writes them.  *overflow = true: a candidate list could not be kept
// below its capacity (many equal distances); the outputs are then not valid and the caller
// repeats the pass with the all-fp32 kernel.  Waits for the pass.
grab_status grab_knn_pass(grab_index *ix, KnnFilter *f, const int32_t *d_tgt, uint32_t *out_s, float *out_d, int64_t out_stride,
                          int64_t out_off, int32_t P, int32_t exclude_self, bool *overflow) {
    *overflow = false;
    if (f->n_items == 0) return GRAB_OK;
    FilterArgs a;
    a.Xh = f->Xh; a.Xm = f->Xm; a.hn = f->hn; a.nrm = f->nrm; a.maxnorm = f->maxnorm; a.X = ix->X;
    a.table = ix->table; a.tgt = d_tgt; a.blk_start = f->blk_start; a.B = ix->B; a.n_items = f->n_items;
    a.out_s = out_s; a.out_d = out_d; a.out_stride = out_stride; a.out_off = out_off; a.n_slots = ix->n_slots;
    a.P = P; a.metric = ix->metric; a.exclude_self = exclude_self;
    a.lists = f->lists; a.overflow = f->overflow; a.cand = f->cand; a.n_cand = f->n_cand; a.slot2id = ix->slot2id;
    a.kappa = 6.103515625e-05f + (float)ix->dim * 4.76837158203125e-07f;
    GRAB_HIP(ix, hipMemsetAsync(f->overflow, 0, 4, ix->stream));
    GRAB_HIP(ix, hipMemsetAsync(f->n_cand, 0, (size_t)ix->n_slots * 4, ix->stream));
    grab_status rc = GRAB_EINVAL;
    switch (ix->dim / 32) {
#define GRAB_CASE(N) case N: rc = launch_filter_t<N>(ix, a, f->grid); break;
        GRAB_FOR_EACH_NCH(GRAB_CASE)
#undef GRAB_CASE
        default:
            return grab_fail(ix, GRAB_EINVAL, "dim %d has no construction kernel", ix->dim);
    }
    if (rc != GRAB_OK) return rc;
    uint32_t h = 0;
    GRAB_HIP(ix, hipMemcpyAsync(&h, f->overflow, 4, hipMemcpyDeviceToHost, ix->stream));
    GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    *overflow = h != 0;
    return GRAB_OK;
}
