// Batched insertion (Section 4.4) for gfx950: append at the bucket tails without moving any
// slot, candidate search against the pre-batch graph, forward selection by the diversity rule
// (Eq. 2) and reverse rewiring with the freshness bias (Eq. 3).
//
// The paper claims slots with an atomic counter and fills a request buffer atomically; both
// orders are irreproducible.  Here slots come from a stable sort of (bucket, batch position)
// and reverse requests are sorted by (target, kind, distance, source) and applied serially
// per target by one wavefront, so that the same batch always yields the same bytes.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_select.hpp>
#include <rocprim/iterator/counting_iterator.hpp>
#include <rocprim/iterator/transform_iterator.hpp>

#include "grab_device.h"

namespace {

constexpr int TPB = 256;
inline unsigned blocks_for(int64_t work) { return (unsigned)((work + TPB - 1) / TPB); }

// Bucket of a new attribute x against the pre-batch table: the run of buckets with
// min <= x <= max, spread by external id; else the first bucket with max >= x (else the last).
__global__ void k_assign_bucket(const int32_t *__restrict__ table, int32_t B, const int32_t *__restrict__ attrs,
                                int64_t m, int64_t n_prev, int32_t *__restrict__ bucket, uint32_t *__restrict__ keys,
                                uint32_t *__restrict__ idx) {
    int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= m) return;
    const int32_t x = attrs[i];
    int l = 0, r = B;  // e0 = number of buckets with max < x
    while (l < r) { int mid = (l + r) >> 1; if (table[T_COLS * mid + T_MAX] < x) l = mid + 1; else r = mid; }
    const int e0 = l;
    l = 0; r = B;      // e1 + 1 = number of buckets with min <= x
    while (l < r) { int mid = (l + r) >> 1; if (table[T_COLS * mid + T_MIN] <= x) l = mid + 1; else r = mid; }
    const int e1 = l - 1;
    int b;
    if (e0 <= e1) b = e0 + (int)((uint64_t)(n_prev + i) % (uint64_t)(e1 - e0 + 1));
    else b = e0 < B ? e0 : B - 1;
    bucket[i] = b;
    keys[i] = (uint32_t)b;
    idx[i] = (uint32_t)i;
}

// per bucket: first position and count of its items in the bucket-sorted batch
__global__ void k_bucket_spans(const uint32_t *__restrict__ sorted_keys, int64_t m, int32_t B,
                               int32_t *__restrict__ starts, int32_t *__restrict__ counts) {
    int b = blockIdx.x * TPB + threadIdx.x;
    if (b >= B) return;
    int64_t l = 0, r = m;
    while (l < r) { int64_t mid = (l + r) >> 1; if (sorted_keys[mid] < (uint32_t)b) l = mid + 1; else r = mid; }
    const int64_t s = l;
    r = m;
    while (l < r) { int64_t mid = (l + r) >> 1; if (sorted_keys[mid] <= (uint32_t)b) l = mid + 1; else r = mid; }
    starts[b] = (int32_t)s;
    counts[b] = (int32_t)(l - s);
}

// slot = base + n_total + rank among the batch items of the same bucket, in batch order
__global__ void k_assign_slots(const uint32_t *__restrict__ sorted_keys, const uint32_t *__restrict__ sorted_idx,
                               int64_t m, const int32_t *__restrict__ starts, const int32_t *__restrict__ table,
                               uint32_t *__restrict__ slot) {
    int64_t p = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (p >= m) return;
    const uint32_t b = sorted_keys[p];
    const int32_t *t = table + T_COLS * b;
    slot[sorted_idx[p]] = (uint32_t)(t[T_BASE] + t[T_NTOT] + (int32_t)(p - starts[b]));
}

__global__ void k_fill_range(int32_t *__restrict__ lo, int32_t *__restrict__ hi, int64_t m) {
    int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < m) { lo[i] = INT32_MIN; hi[i] = INT32_MAX; }
}

// scope of the global-scope candidate search: every slot outside the object's own bucket
__global__ void k_scope_outside(const int32_t *__restrict__ bucket, int64_t m, int32_t *__restrict__ scope) {
    int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < m) scope[i] = -2 - bucket[i];
}

// feature row, attribute and id maps of the new objects (one thread per 16-byte piece)
__global__ void k_write_new(const float4 *__restrict__ vecs, const int32_t *__restrict__ attrs,
                            const uint32_t *__restrict__ slot, int64_t m, int64_t n_prev, int32_t row_f4,
                            float4 *__restrict__ X, int32_t *__restrict__ attr_s, uint32_t *__restrict__ slot2id,
                            uint32_t *__restrict__ id2slot) {
    int64_t t = (int64_t)blockIdx.x * TPB + threadIdx.x;
    int64_t i = t / row_f4;
    if (i >= m) return;
    int32_t c = (int32_t)(t - i * row_f4);
    const uint32_t s = slot[i];
    X[(int64_t)s * row_f4 + c] = vecs[i * row_f4 + c];
    if (c == 0) {
        attr_s[s] = attrs[i];
        slot2id[s] = (uint32_t)(n_prev + i);
        id2slot[n_prev + i] = s;
    }
}

// min / max of the new attributes per bucket: reduced in LDS first, so that a bucket's table entry
// sees one atomic pair per workgroup instead of one per object
#define WIDEN_PER_BLOCK 4096
__global__ __launch_bounds__(TPB) void k_widen(const int32_t *__restrict__ attrs, const int32_t *__restrict__ bucket, int64_t m,
                                               int32_t B, int32_t *__restrict__ table) {
    __shared__ int32_t mn[GRAB_MAX_BUCKETS], mx[GRAB_MAX_BUCKETS];
    for (int b = threadIdx.x; b < B; b += TPB) { mn[b] = INT32_MAX; mx[b] = INT32_MIN; }
    __syncthreads();
    const int64_t i0 = (int64_t)blockIdx.x * WIDEN_PER_BLOCK, i1 = i0 + WIDEN_PER_BLOCK < m ? i0 + WIDEN_PER_BLOCK : m;
    for (int64_t i = i0 + threadIdx.x; i < i1; i += TPB) {
        const int b = bucket[i];
        const int32_t x = attrs[i];
        atomicMin(&mn[b], x);
        atomicMax(&mx[b], x);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += TPB)
        if (mn[b] <= mx[b]) {
            int32_t *t = table + T_COLS * b;
            atomicMin(&t[T_MIN], mn[b]);
            atomicMax(&t[T_MAX], mx[b]);
        }
}

__global__ void k_grow(int32_t *__restrict__ table, const int32_t *__restrict__ counts, int32_t B) {
    int b = blockIdx.x * TPB + threadIdx.x;
    if (b < B) table[T_COLS * b + T_NTOT] += counts[b];
}

__global__ void k_iota(uint32_t *__restrict__ a, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < n) a[i] = (uint32_t)i;
}

// Work counters of one insertion call (device, 64-bit), reported by grab_get_append_stats
enum { ST_REQ_LOCAL = 0, ST_REQ_REMOTE, ST_GROUPS_LOCAL, ST_GROUPS_REMOTE, ST_APPLIED_LOCAL, ST_APPLIED_REMOTE, ST_SCANNED,
       ST_REMOTE_ROWS, ST_LOCAL_PASS, ST_SEARCH_EVALS, ST_SEARCH_PARENTS, ST_SPARE, ST_N };

__global__ void k_zero_stats(u64 *__restrict__ stats) {
    if (threadIdx.x < ST_N) stats[threadIdx.x] = 0;
}

// distance evaluations and expanded parents of a candidate search, summed over its queries
__global__ __launch_bounds__(TPB) void k_sum_search_counters(const uint32_t *__restrict__ counters, int64_t nq, u64 *__restrict__ stats) {
    __shared__ u64 acc[2];
    if (threadIdx.x < 2) acc[threadIdx.x] = 0;
    __syncthreads();
    u64 ev = 0, pa = 0;
    for (int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x; i < nq; i += (int64_t)gridDim.x * TPB) {
        pa += counters[i * 8 + 1];
        ev += counters[i * 8 + 2];
    }
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) { ev += shfl_xor64(ev, m); pa += shfl_xor64(pa, m); }
    if ((threadIdx.x & 63) == 0) { atomicAdd(&acc[0], ev); atomicAdd(&acc[1], pa); }
    __syncthreads();
    if (threadIdx.x == 0) { atomicAdd(&stats[ST_SEARCH_EVALS], acc[0]); atomicAdd(&stats[ST_SEARCH_PARENTS], acc[1]); }
}

struct ForwardArgs {
    const float *X;
    uint32_t *A;
    const float *vecs;          // the new vectors, batch order
    const uint32_t *slot;
    const uint32_t *cand_s;     // local candidate search results: slots [m][beam]
    const float *cand_d;        //                                 distances to the new vector
    u64 *key1, *key2;           // request keys, one per row entry
    float *reqd;
    const uint32_t *by_bucket;  // batch positions in bucket order: the order the workgroups take them in
    int64_t m;
    int32_t beam, kl, kr, metric;
    // proximal / global reading of the remote part (mode 1)
    int32_t mode, kp, remote_cands;
    int64_t window;
    const uint32_t *gcand_s;    // global-scope candidate search results: slots [m][beam]
    const float *gcand_d;
    const int32_t *attr;        // attributes of the index, by slot
    const int32_t *new_attr;    // attributes of the new objects, batch order
    uint32_t *node_out;         // [m][2]: candidates examined by the Eq. 2 scan, rows evaluated for the remote part
};

// Forward edges of one new node per wavefront (Section 4.4 step 2).  Local part (Eq. 2): scan the
// candidates in (distance, slot) order, keep c iff dist(q,c) < dist(c,n) for every kept n, stop
// at K_local, back-fill with the earliest rejected ones.  Remote part: entry j is the nearest to
// the new vector among the j-th remote entries of its local candidates.  Writes the new adjacency
// row [local | remote] and one reverse request per written edge.
template <int NCH>
__global__ __launch_bounds__(64) void k_forward(ForwardArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int D = NCH * 32;
    const int lane = threadIdx.x;
    // new nodes of one bucket read the same candidate rows and the same remote target buckets: the
    // workgroups take the batch in bucket order, one contiguous run of it per XCD
    const int64_t chunk = (a.m + 7) / 8;
    const int64_t pos = (int64_t)(blockIdx.x % 8) * chunk + blockIdx.x / 8;
    if (pos >= a.m) return;
    const int64_t i = a.by_bucket[pos];
    const int K = a.kl + a.kr;
    uint32_t *cs = reinterpret_cast<uint32_t *>(smem);          // local candidates
    float *cd = reinterpret_cast<float *>(cs + a.beam);
    uint32_t *rs = reinterpret_cast<uint32_t *>(cd + a.beam);   // remote candidates of one entry
    float *rd = reinterpret_cast<float *>(rs + a.beam);
    uint32_t *kept = reinterpret_cast<uint32_t *>(rd + a.beam);
    float *keptd = reinterpret_cast<float *>(kept + 64);
    uint32_t *rej = reinterpret_cast<uint32_t *>(keptd + 64);
    float *rejd = reinterpret_cast<float *>(rej + 64);
    float *dtmp = rejd + 64;
    uint32_t *alive = reinterpret_cast<uint32_t *>(dtmp + 64);  // rows of the chunk's candidates not hidden by a kept row,
    uint32_t *alive_g = alive + 8;                              // and their places in the chunk
    uint32_t *pk = alive_g + 8;                                 // mode 1: remote picks,
    float *pkd = reinterpret_cast<float *>(pk + 64);            //         their distances,
    uint32_t *rowl = reinterpret_cast<uint32_t *>(pkd + 64);    //         the local part of the new row,
    uint32_t *ul = rowl + 64;                                   //         local candidates not in it
    uint32_t *uniq = ul + 64;                                   // set of distinct remote candidates
    const int uniq_words = (2 * a.beam + 3) & ~3;    // keeps the query row behind it 16-byte aligned
    float *qlds = reinterpret_cast<float *>(uniq + uniq_words);
    float4 qreg[EvalShape<NCH>::QREG ? NCH : 1];
    const uint32_t self = a.slot[i];
    const u64 lt_mask = (1ull << lane) - 1ull;
    // ---- local part
    int nc = 0;
    for (int c0 = 0; c0 < a.beam; c0 += 64) {
        const int idx = c0 + lane;
        uint32_t s = idx < a.beam ? a.cand_s[i * a.beam + idx] : GRAB_EMPTY;
        bool ok = s != GRAB_EMPTY;
        u64 m = __ballot(ok);
        if (ok) { int pos = nc + __popcll(m & lt_mask); cs[pos] = s; cd[pos] = a.cand_d[i * a.beam + idx]; }
        nc += __popcll(m);
    }
    __syncthreads();
    int nk = 0, nrej = 0;
    unsigned scanned = 0, remote_rows = 0;   // candidates examined by the Eq. 2 scan; rows evaluated for the remote part
    if constexpr (EvalShape<NCH>::QREG) {
        // eight candidates at a time, one per lane group: their rows are loaded together, each is
        // compared with every row kept so far and with the other seven, and the chunk is then
        // resolved in candidate order exactly as a one-by-one scan would
        const int sub = lane & 7, grp = lane >> 3;
        for (int t0 = 0; t0 < nc && nk < a.kl; t0 += 8) {
            const int G = min(8, nc - t0);
            const int mt = t0 + grp < nc ? t0 + grp : t0;
            const float mydq = cd[mt];
            float4 mine[NCH];
            {
                const float4 *row = reinterpret_cast<const float4 *>(a.X) + (size_t)cs[mt] * (NCH * 8) + sub;
#pragma unroll
                for (int c = 0; c < NCH; ++c) mine[c] = row[c * 8];
            }
            // a candidate is out as soon as one kept row hides it: the scan of the kept rows ends when
            // every candidate of the chunk is out
            bool hid = t0 + grp >= nc;
            group_vs_rows<NCH>(a.X, mine, kept, nk, lane, a.metric, [&](int, float s) { hid |= !(mydq < s); },
                               [&]() { return __ballot(!hid) == 0; });
            const u64 hm = __ballot(hid);
            // candidates of the chunk still in: only they can be kept, so only their rows can hide a
            // later one of them
            int na = 0;
            for (int g = 0; g < G; ++g)
                if (((hm >> (8 * g)) & 1ull) == 0) { if (lane == 0) alive[na] = cs[t0 + g]; if (lane == 0) alive_g[na] = (uint32_t)g; ++na; }
            __syncthreads();
            if (na > 1)
                group_vs_rows<NCH>(a.X, mine, alive, na, lane, a.metric, [&](int h, float s) { if (sub == 0) dtmp[grp * 8 + alive_g[h]] = s; },
                                   []() { return false; });
            __syncthreads();
            uint32_t keptmask = 0;
            for (int g = 0; g < G && nk < a.kl; ++g) {
                const float dqc = cd[t0 + g];
                bool ok = ((hm >> (8 * g)) & 1ull) == 0;
                for (int h = 0; h < g; ++h)
                    if ((keptmask >> h) & 1u) ok = ok && (dqc < dtmp[g * 8 + h]);
                if (lane == 0) {
                    if (ok) { kept[nk] = cs[t0 + g]; keptd[nk] = dqc; }
                    else if (nrej < 64) { rej[nrej] = cs[t0 + g]; rejd[nrej] = dqc; }
                }
                if (ok) { ++nk; keptmask |= 1u << g; } else if (nrej < 64) ++nrej;
                ++scanned;
            }
            __syncthreads();
        }
    } else {
        for (int t = 0; t < nc && nk < a.kl; ++t) {
            const uint32_t c = cs[t];
            const float dqc = cd[t];
            bool ok = true;
            if (nk > 0) {
                load_query<NCH>(a.X + (size_t)c * D, qreg, qlds, lane);
                __syncthreads();
                eval_rows<NCH>(a.X, qreg, qlds, kept, nk, lane, a.metric, dtmp);
                __syncthreads();
                bool hidden = lane < nk && !(dqc < dtmp[lane]);
                ok = __ballot(hidden) == 0;
            }
            if (lane == 0) {
                if (ok) { kept[nk] = c; keptd[nk] = dqc; }
                else if (nrej < 64) { rej[nrej] = c; rejd[nrej] = dqc; }
            }
            if (ok) ++nk; else if (nrej < 64) ++nrej;
            ++scanned;
            __syncthreads();
        }
    }
    auto flush_stats = [&]() __attribute__((always_inline)) {
        if (lane == 0) { a.node_out[2 * i] = scanned; a.node_out[2 * i + 1] = remote_rows; }
    };
    for (int j = lane; j < a.kl; j += 64) {
        uint32_t v = GRAB_EMPTY;
        float d = 0.0f;
        if (j < nk) { v = kept[j]; d = keptd[j]; }
        else if (j - nk < nrej) { v = rej[j - nk]; d = rejd[j - nk]; }
        a.A[(size_t)self * (uint32_t)K + j] = v;
        rowl[j] = v;
        const int64_t r = i * K + j;
        a.key1[r] = v == GRAB_EMPTY ? ~0ull : ((u64)v << 1);
        a.key2[r] = ((u64)dist_image(d) << 32) | (u64)self;
        a.reqd[r] = d;
    }
    // ---- remote part, proximal / global reading: picks from the global-scope candidates; a position
    // without a pick takes the nearest local candidate not yet in the row (a redundant local edge,
    // which makes no reverse request)
    if (a.mode == 1) {
        if (a.kr == 0) { flush_stats(); return; }
        __syncthreads();
        select_remote_wave(a.gcand_s + i * a.beam, a.gcand_d + i * a.beam, a.beam, a.attr, a.new_attr[i], a.window, a.kp,
                           a.kr, lane, pk, pkd);
        int nu = 0;
        for (int c0 = 0; c0 < nc && nu < a.kr; c0 += 64) {
            const int t = c0 + lane;
            bool un = t < nc;
            const uint32_t c = un ? cs[t] : GRAB_EMPTY;
            if (un)
                for (int x = 0; x < a.kl; ++x) un = un && rowl[x] != c;
            const u64 mu = __ballot(un);
            if (un) {
                const int r = nu + __popcll(mu & lt_mask);
                if (r < a.kr) ul[r] = c;
            }
            nu += __popcll(mu);
        }
        nu = min(nu, a.kr);
        __syncthreads();
        const bool has = lane < a.kr;
        uint32_t v = GRAB_EMPTY;
        float d = 0.0f;
        if (has) { v = pk[lane]; d = pkd[lane]; }
        const bool pick = has && v != GRAB_EMPTY;
        const u64 mless = __ballot(has && !pick);
        if (has && !pick) {
            const int r = __popcll(mless & lt_mask);
            v = r < nu ? ul[r] : GRAB_EMPTY;
        }
        if (has) {
            a.A[(size_t)self * (uint32_t)K + a.kl + lane] = v;
            const int64_t r = i * K + a.kl + lane;
            a.key1[r] = pick ? (((u64)v << 1) | 1ull) : ~0ull;
            a.key2[r] = ((u64)dist_image(d) << 32) | (u64)self;
            a.reqd[r] = d;
        }
        flush_stats();
        return;
    }
    // ---- remote part, by target bucket
    // the candidates' j-th remote entries are requested one j ahead, so that the request flies while the
    // rows of entry j - 1 are evaluated
    constexpr int MAXC = 8;   // candidates per lane: queues of up to 512
    const int nrc = a.remote_cands > 0 && a.remote_cands < nc ? a.remote_cands : nc;   // the nearest candidates only
    uint32_t ahead[MAXC];
    auto request = [&](int j) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int t = 64 * c + lane;
            ahead[c] = GRAB_EMPTY;
            if (64 * c < nrc && t < nrc) ahead[c] = a.A[(size_t)cs[t] * (uint32_t)K + a.kl + j];
        }
    };
    if (a.kr > 0) {
        request(0);
        load_query<NCH>(a.vecs + (size_t)i * D, qreg, qlds, lane);
        __syncthreads();
    }
    for (int j = 0; j < a.kr; ++j) {
        // neighbouring candidates mostly share their j-th remote entry: each distinct slot is
        // evaluated once (the minimum below does not depend on repeats)
        for (int x = lane; x < uniq_words; x += 64) uniq[x] = GRAB_EMPTY;
        uint32_t now[MAXC];
#pragma unroll
        for (int c = 0; c < MAXC; ++c) now[c] = ahead[c];
        if (j + 1 < a.kr) request(j + 1);
        __syncthreads();
        int nr = 0;
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            if (64 * c >= nrc) break;
            const uint32_t r = now[c];
            bool ok = false;
            if (r != GRAB_EMPTY) {
                uint32_t h = (uint32_t)(((u64)(r * 0x9E3779B1u) * (u64)uniq_words) >> 32);
                for (int probe = 0; probe < uniq_words; ++probe) {
                    const uint32_t old = atomicCAS(&uniq[h], GRAB_EMPTY, r);
                    if (old == GRAB_EMPTY) { ok = true; break; }
                    if (old == r) break;
                    h = h + 1 == (uint32_t)uniq_words ? 0u : h + 1;
                }
            }
            u64 m = __ballot(ok);
            if (ok) rs[nr + __popcll(m & lt_mask)] = r;
            nr += __popcll(m);
        }
        __syncthreads();
        remote_rows += (unsigned)nr;
        u64 best = ~0ull;
        if (nr > 0) {
            eval_rows<NCH>(a.X, qreg, qlds, rs, nr, lane, a.metric, rd);
            __syncthreads();
            for (int t = lane; t < nr; t += 64) {
                u64 k = ((u64)dist_image(rd[t]) << 32) | (u64)rs[t];
                best = k < best ? k : best;
            }
#pragma unroll
            for (int sft = 32; sft > 0; sft >>= 1) {
                uint32_t hi = __shfl_xor((uint32_t)(best >> 32), sft), lo = __shfl_xor((uint32_t)best, sft);
                u64 other = ((u64)hi << 32) | lo;
                best = other < best ? other : best;
            }
        }
        if (lane == 0) {
            const uint32_t v = best == ~0ull ? GRAB_EMPTY : (uint32_t)(best & 0xFFFFFFFFull);
            const float d = best == ~0ull ? 0.0f : image_dist((uint32_t)(best >> 32));
            a.A[(size_t)self * (uint32_t)K + a.kl + j] = v;
            const int64_t r = i * K + a.kl + j;
            a.key1[r] = v == GRAB_EMPTY ? ~0ull : (((u64)v << 1) | 1ull);
            a.key2[r] = ((u64)dist_image(d) << 32) | (u64)self;
            a.reqd[r] = d;
        }
        __syncthreads();
    }
    flush_stats();
}

struct RewireArgs {
    const float *X;
    uint32_t *A;
    const int32_t *table;
    const u64 *key1s;       // sorted (target << 1 | kind); ~0 for "no request"
    const uint4 *rec;       // by sorted position: {source slot, dist(target, source) bits, source bucket, source attribute}
    const u64 *heads;       // per (target, kind) group, in sorted order: position of its first request << 32 | key; one workgroup each
    int64_t nreq;
    uint32_t n_heads;
    uint32_t *big_heads, *n_big;   // groups of more than 64 requests, left to a second launch
    int32_t kl, kr, metric, B;
    float a;                // alpha squared: the bias acts on squared distances (see bias_base)
    // proximal / global reading of the remote part (mode 1)
    int32_t mode, kp;
    int64_t window;
    const int32_t *attr;
    uint32_t *grp_out;      // per group, in the order of `heads`: requests applied | passed << 16
};

__device__ __forceinline__ int bucket_of_slot_dev(const int32_t *__restrict__ table, int32_t B, uint32_t slot) {
    int l = 0, r = B;  // last bucket whose base <= slot
    while (r - l > 1) {
        int m = (l + r) >> 1;
        if ((uint32_t)table[T_COLS * m + T_BASE] <= slot) l = m; else r = m;
    }
    return l;
}

// sorted position -> (position << 32 | key): what a group head is listed as, so that the wavefront
// of a group knows its target before it has read anything else
struct HeadEntry {
    const u64 *key1s;
    __host__ __device__ u64 operator()(uint32_t p) const { return ((u64)p << 32) | (key1s[p] & 0xFFFFFFFFull); }
};

// Bucket of a slot (the same slot in every lane): the last bucket whose slab base is <= slot,
// counted 64 buckets at a time, one base per lane
__device__ __forceinline__ int wave_bucket_of(const int32_t *__restrict__ table, int32_t B, uint32_t slot, int lane) {
    int c = 0;
    for (int b0 = 0; b0 < B; b0 += 64)
        c += __popcll(__ballot(b0 + lane < B && (uint32_t)table[T_COLS * (b0 + lane) + T_BASE] <= slot));
    return c - 1;
}

// what the rewiring needs of each request, in sorted order, so that a group finds its requests
// without chasing the sort permutation: source slot, distance, bucket and attribute of the source
// (a new object: request index / K is its position in the batch); marks the group heads
__global__ void k_request_records(const u64 *__restrict__ key1s, const uint32_t *__restrict__ order, const u64 *__restrict__ key2,
                                  const float *__restrict__ reqd, const int32_t *__restrict__ bucket,
                                  const int32_t *__restrict__ new_attr, int32_t K, int64_t nreq, uint4 *__restrict__ rec,
                                  unsigned char *__restrict__ head, uint32_t *__restrict__ n_valid) {
    const int64_t p = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (p >= nreq) return;
    const u64 key = key1s[p];
    head[p] = key != ~0ull && (p == 0 || key1s[p - 1] != key);
    if (p == 0) n_valid[1] = 0;   // the rewiring's count of groups left to its second launch
    // the "no request" keys sort last: the real requests are the positions before the first of them
    if (key == ~0ull) { if (p == 0) *n_valid = 0; return; }
    if (p + 1 == nreq || key1s[p + 1] == ~0ull) *n_valid = (uint32_t)(p + 1);
    const uint32_t ridx = order[p];
    const uint32_t i = ridx / (uint32_t)K;
    rec[p] = make_uint4((uint32_t)(key2[ridx] & 0xFFFFFFFFull), __float_as_uint(reqd[ridx]), (uint32_t)bucket[i], (uint32_t)new_attr[i]);
}

// Lane, among those with `in` set (at least one), whose (image, slot) pair is the largest; every
// lane returns it.  Two 32-bit reductions: the largest image first, the slot only among its ties.
__device__ __forceinline__ int farthest_lane(bool in, uint32_t image, uint32_t slot, int lane) {
    const uint32_t m = wave_max_u32(in ? image : 0u, lane);
    u64 tie = __ballot(in && image == m);
    if (__popcll(tie) > 1) {
        const uint32_t sm = wave_max_u32(in && image == m ? slot : 0u, lane);
        tie = __ballot(in && image == m && slot == sm);
    }
    return __ffsll((long long)tie) - 1;
}

// requests of a local group evaluated per pass over the target's neighbour rows (the target itself
// rides along in the first pass); bounded by the LDS the staged query rows take
template <int NCH>
struct RewireShape {
    static constexpr int G = NCH <= 4 ? 5 : (NCH <= 8 ? 3 : (NCH <= 32 ? 2 : 1));
};

// Reverse rewiring (Section 4.4 step 3): the wavefront that sits on the first request of a
// (target, kind) group applies the whole group in order.
// Local kind: Eq. 2 with Eq. 3's effective distance decides whether the newcomer may enter; it
// then fills an empty entry or overwrites, among the entries it points to itself, the one
// farthest from the target (the target still reaches it through the newcomer).  The rows of the
// target's neighbours are read once per pass: the target and up to G requesting nodes are staged in
// LDS and all their distances to those rows are taken while the rows sit in registers; an entry
// rewritten by an earlier request of the same pass is a new node whose row is staged too, so the
// later requests get their distance to it from LDS.  Remote kind: the entry of the target's remote
// part that lies in the newcomer's bucket is overwritten iff the newcomer's biased distance to the
// target is smaller.
// The next requests of a group in (distance image, source slot) order, written to rq / rd / rb / ra;
// returns how many.  BIG = false: the whole group (at most 64 requests, held one per lane in rc)
// is ranked by counting.  BIG = true: the 64 smallest keys above `last`, found by a pass over all
// requests of the group; what a request carries besides its key is read again from its source.
template <bool BIG>
__device__ __forceinline__ int next_requests(const RewireArgs &a, int64_t p0, int gt, const uint4 *raw, u64 &last, int lane,
                                             uint32_t *rq, float *rd, int32_t *rb, int32_t *ra) {
    int nb;
    if constexpr (!BIG) {
        const uint4 rc = raw[lane];
        const u64 mykey = lane < gt ? (((u64)dist_image(__uint_as_float(rc.y)) << 32) | (u64)rc.x) : SENT;
        int rank = 0;
        for (int j = 0; j < gt; ++j) rank += read_lane64(mykey, j) < mykey ? 1 : 0;
        if (lane < gt) { rq[rank] = rc.x; rd[rank] = __uint_as_float(rc.y); rb[rank] = (int32_t)rc.z; ra[rank] = (int32_t)rc.w; }
        nb = gt;
    } else {
        LaneQueue<1> best;
        best.clear();
        for (int64_t pp = p0; pp < p0 + gt; pp += 64) {
            u64 ck = SENT;
            if (pp + lane < p0 + gt) {
                const uint4 r = a.rec[pp + lane];
                const u64 k2 = ((u64)dist_image(__uint_as_float(r.y)) << 32) | (u64)r.x;
                if (k2 > last) ck = k2;
            }
            ck = sort_lanes(ck, 64, lane);
            best.merge(ck, 64, lane);
        }
        const u64 bk = best.k[0];
        nb = __popcll(__ballot(bk != SENT));
        const uint32_t src = (uint32_t)(bk & 0xFFFFFFFFull);
        if (lane < nb) { rq[lane] = src; rd[lane] = image_dist((uint32_t)(bk >> 32)); ra[lane] = a.attr[src]; }
        for (int j = 0; j < nb; ++j) {
            const int bj = wave_bucket_of(a.table, a.B, (uint32_t)(read_lane64(bk, j) & 0xFFFFFFFFull), lane);
            if (lane == j) rb[j] = bj;
        }
        last = read_lane64(bk, nb - 1);
    }
    __syncthreads();
    return nb;
}

// BIG = false: one workgroup per group; a group of more than 64 requests is only noted in
// a.big_heads.  BIG = true: a few workgroups share out the noted groups (a second launch).
template <int NCH, bool BIG>
__global__ __launch_bounds__(64, 4) void k_rewire(RewireArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int D = NCH * 32, D4 = NCH * 8, G = RewireShape<NCH>::G;
    constexpr bool WHOLE = EvalShape<NCH>::CB == NCH;   // a whole row fits the register batch
    const int lane = threadIdx.x;
    for (uint32_t hi = blockIdx.x; hi < (BIG ? *a.n_big : a.n_heads); hi += BIG ? gridDim.x : a.n_heads) {
    // one wavefront per (target, kind) group, which it applies in (distance, source) order
    const uint32_t head_index = BIG ? a.big_heads[hi] : hi;
    const u64 head = a.heads[head_index];
    const int64_t p0 = (int64_t)(head >> 32);
    const u64 key = head & 0xFFFFFFFFull;
    // the first 64 positions from the head on (requests of the group are contiguous, in no order)
    const bool in_first = p0 + lane < a.nreq && a.key1s[p0 + lane] == key;
    unsigned st_applied = 0, st_pass = 0;
    const uint32_t v = (uint32_t)(key >> 1);
    const int kind = (int)(key & 1ull);
    const int K = a.kl + a.kr, off = kind ? a.kl : 0, len = kind ? a.kr : a.kl;
    uint32_t *R = reinterpret_cast<uint32_t *>(smem);   // current part of v's row
    uint32_t *Rl = R + 64;                                // same with empty entries pointing at row 0
    float *Dall = reinterpret_cast<float *>(Rl + 64);     // [0]: dist(v, R[j]); [1 + k]: dist(request k of the pass, R[j])
    uint32_t *qrow = reinterpret_cast<uint32_t *>(Dall + (G + 1) * 64);   // the requesting nodes' own rows, 128 entries each
    uint32_t *rq = qrow + G * 128;                        // sources of up to 64 requests of the group, in order,
    float *rd = reinterpret_cast<float *>(rq + 64);       // their distances to v,
    int32_t *rb = reinterpret_cast<int32_t *>(rd + 64);   // their buckets
    int32_t *ra = rb + 64;                                // and attributes
    float *qs = reinterpret_cast<float *>(ra + 64);       // staged rows: v, then the requesting nodes of the pass
    float *dq = Dall;                                     // remote kind: dist(v, R[j])
    uint4 *raw = reinterpret_cast<uint4 *>(qs + (size_t)(G + 1) * D);   // the records of those positions as they come
    raw[lane] = p0 + lane < a.nreq ? a.rec[p0 + lane] : make_uint4(0u, 0u, 0u, 0u);
    if (lane < len) {
        uint32_t e = a.A[(size_t)v * (uint32_t)K + off + lane];
        R[lane] = e;
        Rl[lane] = e == GRAB_EMPTY ? 0u : e;
    }
    // size of the group
    int gt;
    {
        const u64 same = __ballot(in_first);
        gt = same == ~0ull ? 64 : __ffsll((long long)~same) - 1;
        if (gt == 64)
            for (int64_t pp = p0 + 64;; pp += 64) {
                const u64 more = __ballot(pp + lane < a.nreq && a.key1s[pp + lane] == key);
                const int g = more == ~0ull ? 64 : __ffsll((long long)~more) - 1;
                gt += g;
                if (g < 64) break;
            }
    }
    if constexpr (!BIG) {
        if (gt > 64) {
            if (lane == 0) a.big_heads[atomicAdd(a.n_big, 1u)] = head_index;
            continue;
        }
    }
    __syncthreads();   // the previous group of this workgroup is done with the arrays below
    bool changed = false;
    u64 last = 0;   // groups beyond 64 requests: the largest (distance, source) key applied so far
    int done = 0;
    __syncthreads();
    if (kind == 1) {
        // distances of the row's entries to v, and the bucket of the entry each lane looks after
        for (int t = lane; t < D4; t += 64) reinterpret_cast<float4 *>(qs)[t] = reinterpret_cast<const float4 *>(a.X)[(size_t)v * D4 + t];
        __syncthreads();
        if (len <= 8) eval_rows_few<NCH>(a.X, qs, Rl, len, lane, a.metric, Dall);   // dist(v, R[j])
        else eval_rows_multi<NCH, 1>(a.X, qs, 1u, Rl, 0, len, lane, a.metric, Dall);
        const int32_t attr_v = a.mode == 1 ? a.attr[v] : 0;
        uint32_t mine_r = lane < len ? R[lane] : GRAB_EMPTY;
        const int bv = a.mode == 1 ? wave_bucket_of(a.table, a.B, v, lane) : 0;
        int bmine = -1;
        for (int j = 0; j < len; ++j) {
            const uint32_t e = (uint32_t)__builtin_amdgcn_readlane((int)mine_r, j);
            const int be = e != GRAB_EMPTY ? wave_bucket_of(a.table, a.B, e, lane) : -1;
            if (lane == j) bmine = be;
        }
        __syncthreads();
        do {
            const int nb = next_requests<BIG>(a, p0, gt, raw, last, lane, rq, rd, rb, ra);
            for (int t = 0; t < nb; ++t) {
                const uint32_t q = rq[t];
                const float dvq = rd[t];
                const float lhs = a.a * bias_base(dvq, a.metric);
                int at = -1;
                if (a.mode == 1) {
                    // q competes for the positions of its class; an empty one or one holding a node of
                    // v's own bucket (a redundant local edge) is taken at once, else the farthest gives way
                    long long diff = (long long)ra[t] - (long long)attr_v;
                    if (diff < 0) diff = -diff;
                    const int j0 = diff <= a.window ? 0 : a.kp, j1 = diff <= a.window ? a.kp : len;
                    const bool inc = lane >= j0 && lane < j1;
                    const u64 free_m = __ballot(inc && (mine_r == GRAB_EMPTY || bmine == bv));
                    if (free_m) {
                        at = __ffsll((long long)free_m) - 1;
                    } else if (j1 > j0) {
                        const int far = farthest_lane(inc, dist_image(dq[lane]), mine_r, lane);
                        if (lhs < bias_base(dq[far], a.metric)) at = far;
                    }
                } else {
                    const int bq = rb[t];
                    const bool inb = mine_r != GRAB_EMPTY && bmine == bq;
                    if (__ballot(inb)) {
                        const int far = farthest_lane(inb, dist_image(dq[lane]), mine_r, lane);
                        if (lhs < bias_base(dq[far], a.metric)) at = far;
                    } else {
                        const u64 empties = __ballot(lane < len && mine_r == GRAB_EMPTY);
                        if (empties) at = __ffsll((long long)empties) - 1;
                    }
                }
                __syncthreads();
                if (at >= 0) {
                    if (lane == at) { R[at] = q; dq[at] = dvq; mine_r = q; bmine = rb[t]; }
                    changed = true;
                    ++st_applied;
                }
                __syncthreads();
            }
            done += nb;
        } while (BIG && done < gt);
    } else {
        const float4 *X4 = reinterpret_cast<const float4 *>(a.X);
        float4 *qs4 = reinterpret_cast<float4 *>(qs);
        const int sub = lane & 7, grp = lane >> 3;
        const int K8 = (K + 7) & ~7;
        bool first = true;
        do {
            const int nb = next_requests<BIG>(a, p0, gt, raw, last, lane, rq, rd, rb, ra);
            for (int c0 = 0; c0 < nb; c0 += G) {
                const int ng = min(G, nb - c0);
                const unsigned qmask = (first ? 1u : 0u) | (((1u << ng) - 1u) << 1);
                // the neighbour rows are on their way while the query rows are staged
                RowRegs<NCH> rr;
                if constexpr (WHOLE) {
                    rows_pick<NCH>(Rl, 0, len, lane, rr);
                    rows_issue<NCH>(a.X, 0, lane, rr);
                }
                for (int t = lane; t < (G + 1) * D4; t += 64) {
                    const int g = t / D4, c = t - g * D4;
                    if ((qmask >> g) & 1u) qs4[t] = X4[(size_t)(g == 0 ? v : rq[c0 + g - 1]) * D4 + c];
                }
                // the requesting nodes' rows, padded to whole groups of eight entries with a value no slot has
                for (int k = 0; k < ng; ++k)
                    for (int x = lane; x < K8; x += 64)
                        qrow[k * 128 + x] = x < K ? a.A[(size_t)rq[c0 + k] * (uint32_t)K + x] : 0xFFFFFFFEu;
                __syncthreads();
                if constexpr (WHOLE) {
                    float acc[G + 1][EvalShape<NCH>::R];
#pragma unroll
                    for (int g = 0; g <= G; ++g)
#pragma unroll
                        for (int r = 0; r < EvalShape<NCH>::R; ++r) acc[g][r] = 0.0f;
                    rows_fma<NCH, G + 1>(rr, qs, qmask, 0, lane, a.metric, acc);
                    rows_store<NCH, G + 1>(rr, acc, qmask, 0, lane, a.metric, Dall);
                    eval_rows_multi<NCH, G + 1>(a.X, qs, qmask, Rl, 8 * EvalShape<NCH>::R, len, lane, a.metric, Dall);
                } else {
                    eval_rows_multi<NCH, G + 1>(a.X, qs, qmask, Rl, 0, len, lane, a.metric, Dall);
                }
                __syncthreads();
                first = false;
                for (int k = 0; k < ng; ++k) {
                    const uint32_t q = rq[c0 + k];
                    const float dvq = rd[c0 + k];
                    const float lhs = a.a * bias_base(dvq, a.metric);
                    const uint32_t mine = lane < len ? R[lane] : GRAB_EMPTY;
                    const float dql = Dall[(1 + k) * 64 + lane], dvl = Dall[lane];
                    const bool blocked = lane < len && mine != GRAB_EMPTY && !(lhs < bias_base(dql, a.metric));
                    int at = -1;
                    if (__ballot(blocked) == 0) {
                        ++st_pass;
                        const u64 empties = __ballot(lane < len && mine == GRAB_EMPTY);
                        if (empties) {
                            at = __ffsll((long long)empties) - 1;
                        } else {
                            // victim: among the entries q points to itself (v still reaches them through q),
                            // the one farthest from v (ties: smaller slot)
                            bool covered = false;
                            if (len <= 32) {
                                // two lanes per entry, each compares it with one half of q's row
                                const uint32_t e = (lane & 31) < len ? R[lane & 31] : GRAB_EMPTY;
                                const uint4 *h4 = reinterpret_cast<const uint4 *>(qrow + k * 128) + (lane >> 5) * (K8 >> 3);
                                bool c = false;
                                for (int x = 0; x < (K8 >> 3); ++x) {
                                    const uint4 w = h4[x];
                                    c |= w.x == e || w.y == e || w.z == e || w.w == e;
                                }
                                const u64 cm = __ballot(c);
                                covered = lane < len && (((cm | (cm >> 32)) >> lane) & 1ull);
                            } else if (lane < len) {
                                for (int x = 0; x < K; ++x) covered |= qrow[k * 128 + x] == mine;
                            }
                            if (__ballot(covered)) {
                                // farthest from v, ties to the smaller slot
                                const uint32_t img = dist_image(dvl);
                                const uint32_t m = wave_max_u32(covered ? img : 0u, lane);
                                u64 tie = __ballot(covered && img == m);
                                if (__popcll(tie) > 1) {
                                    const uint32_t sm = wave_min_u32(covered && img == m ? mine : GRAB_EMPTY, lane);
                                    tie = __ballot(covered && img == m && mine == sm);
                                }
                                at = __ffsll((long long)tie) - 1;
                            }
                        }
                    }
                    __syncthreads();
                    if (at >= 0) {
                        if (lane == at) { R[at] = q; Rl[at] = q; Dall[at] = dvq; }
                        // entry `at` now holds q: the later requests of this pass take their distance to it
                        // from the staged rows, one request per group of eight lanes
                        const int kk = k + 1 + grp;
                        if (kk < ng) {
                            const float d = dist_lds_rows<NCH>(qs + (size_t)(1 + kk) * D, qs + (size_t)(1 + k) * D, lane, a.metric);
                            if (sub == 0) Dall[(1 + kk) * 64 + at] = d;
                        }
                        changed = true;
                        ++st_applied;
                    }
                    __syncthreads();
                }
            }
            done += nb;
        } while (BIG && done < gt);
    }
    if (changed && lane < len) a.A[(size_t)v * (uint32_t)K + off + lane] = R[lane];
    if (lane == 0) a.grp_out[head_index] = st_applied | (st_pass << 16);
    }
}

// Work counters of the call from what the kernels left behind: requests and groups by kind from
// the list of group heads (a group ends where the next one starts), applied / passed requests from
// what each group's wavefront reported, scan lengths from the new nodes
__global__ __launch_bounds__(TPB) void k_reduce_stats(const u64 *__restrict__ heads, const uint32_t *__restrict__ grp_out, uint32_t n_heads,
                                                      const uint32_t *__restrict__ n_valid, const uint32_t *__restrict__ node_out,
                                                      int64_t m, u64 *__restrict__ stats) {
    __shared__ u64 acc[ST_N];
    if (threadIdx.x < ST_N) acc[threadIdx.x] = 0;
    __syncthreads();
    u64 v[ST_SEARCH_EVALS];
#pragma unroll
    for (int x = 0; x < ST_SEARCH_EVALS; ++x) v[x] = 0;
    const int64_t stride = (int64_t)gridDim.x * TPB, t0 = (int64_t)blockIdx.x * TPB + threadIdx.x;
    for (int64_t h = t0; h < n_heads; h += stride) {
        const u64 e = heads[h];
        const uint32_t pos = (uint32_t)(e >> 32), end = h + 1 < n_heads ? (uint32_t)(heads[h + 1] >> 32) : *n_valid;
        const int kind = (int)(e & 1ull);
        const uint32_t g = grp_out[h];
        v[ST_REQ_LOCAL + kind] += end - pos;
        v[ST_GROUPS_LOCAL + kind] += 1;
        v[ST_APPLIED_LOCAL + kind] += g & 0xFFFFu;
        v[ST_LOCAL_PASS] += g >> 16;
    }
    for (int64_t i = t0; i < m; i += stride) { v[ST_SCANNED] += node_out[2 * i]; v[ST_REMOTE_ROWS] += node_out[2 * i + 1]; }
#pragma unroll
    for (int x = 0; x < ST_SEARCH_EVALS; ++x) {
        u64 t = v[x];
#pragma unroll
        for (int sft = 32; sft > 0; sft >>= 1) t += shfl_xor64(t, sft);
        if ((threadIdx.x & 63) == 0 && t) atomicAdd(&acc[x], t);
    }
    __syncthreads();
    if (threadIdx.x < ST_SEARCH_EVALS && acc[threadIdx.x]) atomicAdd(&stats[threadIdx.x], acc[threadIdx.x]);
}

template <int NCH>
grab_status launch_append_t(grab_index *ix, const ForwardArgs &f, const RewireArgs &r, int64_t m, int phase) {
    const size_t qbytes = EvalShape<NCH>::QREG ? 0 : (size_t)ix->dim * 4;
    if (phase == 0) {
        size_t lds = (size_t)f.beam * 16 + 64 * 4 * 9 + 64 + (size_t)((2 * f.beam + 3) & ~3) * 4 + qbytes;
        k_forward<NCH><<<dim3((unsigned)((m + 7) / 8 * 8)), dim3(64), lds, ix->stream>>>(f);
    } else {
        constexpr int G = RewireShape<NCH>::G;
        size_t lds = 64 * 4 * (2 + (G + 1) + 4) + (size_t)G * 128 * 4 + (size_t)(G + 1) * ix->dim * 4 + 64 * 16;
        if (r.n_heads > 0) {
            k_rewire<NCH, false><<<dim3(r.n_heads), dim3(64), lds, ix->stream>>>(r);
            k_rewire<NCH, true><<<dim3(r.n_heads < 2048u ? r.n_heads : 2048u), dim3(64), lds, ix->stream>>>(r);
        }
    }
    GRAB_HIP(ix, hipGetLastError());
    return GRAB_OK;
}

grab_status launch_append(grab_index *ix, const ForwardArgs &f, const RewireArgs &r, int64_t m, int phase) {
    if (!(phase == 0 ? f.node_out : r.grp_out)) return grab_fail(ix, GRAB_EINVAL, "insertion kernels need their counter arrays");
    switch (ix->dim / 32) {
#define GRAB_CASE(N) case N: return launch_append_t<N>(ix, f, r, m, phase);
        GRAB_FOR_EACH_NCH(GRAB_CASE)
#undef GRAB_CASE
        default:
            return grab_fail(ix, GRAB_EINVAL, "dim %d has no append kernel", ix->dim);
    }
}

}  // namespace

// Runs the whole insertion for m new objects whose vectors/attributes are already on the device.
grab_status grab_append_device(grab_index *ix, const float *d_vecs, const int32_t *d_attrs, int64_t m,
                               const SearchLaunch &proto) {
    hipStream_t st = ix->stream;
    const int32_t B = ix->B, kl = ix->kl, kr = ix->kr, K = kl + kr, beam = proto.beam;
    const int64_t nreq = m * K;
    grab_status rc;
    // ---- arena
    enum { A_BUCKET, A_KEYS, A_IDX, A_KEYS_S, A_IDX_S, A_STARTS, A_COUNTS, A_SLOT, A_LO, A_HI, A_CL_S, A_CL_D, A_KEY1, A_KEY2, A_REQD, A_ORD0, A_ORD1, A_ORD2, A_K2S, A_K1G, A_K1S, A_TMP, A_CG_S, A_CG_D, A_SCOPE, A_NODE_OUT, A_GRP_OUT, A_REC, A_HEAD, A_HEADS, A_NHEADS, A_N };
    size_t need[A_N];
    for (size_t &x : need) x = 0;
    need[A_BUCKET] = need[A_KEYS] = need[A_IDX] = need[A_KEYS_S] = need[A_IDX_S] = need[A_SLOT] = need[A_LO] = need[A_HI] = (size_t)m * 4;
    need[A_STARTS] = need[A_COUNTS] = (size_t)B * 4;
    need[A_CL_S] = need[A_CL_D] = (size_t)m * beam * 4;
    need[A_NODE_OUT] = (size_t)m * 8;
    need[A_GRP_OUT] = (size_t)nreq * 4;
    need[A_HEADS] = (size_t)nreq * 8;
    need[A_REC] = (size_t)nreq * 16;
    need[A_HEAD] = (size_t)nreq;
    need[A_NHEADS] = 16;
    const RemoteRule rule = grab_remote_rule(ix, kr);
    if (rule.mode == 1) {
        need[A_CG_S] = need[A_CG_D] = (size_t)m * beam * 4;
        need[A_SCOPE] = (size_t)m * 4;
    }
    need[A_KEY1] = need[A_KEY2] = need[A_K1S] = (size_t)nreq * 8;
    need[A_REQD] = need[A_ORD0] = need[A_ORD2] = (size_t)nreq * 4;
    size_t tmp1 = 0, tmp2 = 0;
    GRAB_HIP(ix, rocprim::radix_sort_pairs(nullptr, tmp1, (uint32_t *)nullptr, (uint32_t *)nullptr, (uint32_t *)nullptr,
                                           (uint32_t *)nullptr, (size_t)m, 0, 32, st));
    GRAB_HIP(ix, rocprim::radix_sort_pairs(nullptr, tmp2, (u64 *)nullptr, (u64 *)nullptr, (uint32_t *)nullptr,
                                           (uint32_t *)nullptr, (size_t)nreq, 0, 64, st));
    size_t tmp3 = 0;
    if (nreq >= (int64_t)1 << 31) return grab_fail(ix, GRAB_EINVAL, "batch of %lld objects is too large for one call", (long long)m);
    typedef rocprim::transform_iterator<rocprim::counting_iterator<uint32_t>, HeadEntry, u64> HeadIt;
    GRAB_HIP(ix, rocprim::select(nullptr, tmp3, HeadIt(rocprim::counting_iterator<uint32_t>(0), HeadEntry{nullptr}), (unsigned char *)nullptr,
                                 (u64 *)nullptr, (uint32_t *)nullptr, (size_t)nreq, st));
    need[A_TMP] = (tmp1 > tmp2 ? (tmp1 > tmp3 ? tmp1 : tmp3) : (tmp2 > tmp3 ? tmp2 : tmp3)) + 16;
    if ((int)ix->app.size() < A_N) ix->app.resize(A_N);
    for (int i = 0; i < A_N; ++i)
        if ((rc = grab_reserve(ix, ix->app[i], need[i])) != GRAB_OK) return rc;
    if ((rc = grab_reserve(ix, ix->app_stats, ST_N * 8)) != GRAB_OK) return rc;
    u64 *stats = (u64 *)ix->app_stats.p;
    auto P = [&](int i) { return ix->app[i].p; };
    auto mark = [&](int i) { if (ix->profile) (void)hipEventRecord(ix->app_ev[i], st); };
    int32_t *bucket = (int32_t *)P(A_BUCKET), *starts = (int32_t *)P(A_STARTS), *counts = (int32_t *)P(A_COUNTS);
    uint32_t *slot = (uint32_t *)P(A_SLOT);

    // ---- 1, 2: bucket and slot of every new object (pre-batch table), capacity check on the host
    k_assign_bucket<<<blocks_for(m), TPB, 0, st>>>(ix->table, B, d_attrs, m, ix->n, bucket, (uint32_t *)P(A_KEYS), (uint32_t *)P(A_IDX));
    int bucket_bits = 1;
    while ((1 << bucket_bits) < B) ++bucket_bits;
    GRAB_HIP(ix, rocprim::radix_sort_pairs(P(A_TMP), tmp1, (uint32_t *)P(A_KEYS), (uint32_t *)P(A_KEYS_S), (uint32_t *)P(A_IDX),
                                           (uint32_t *)P(A_IDX_S), (size_t)m, 0, bucket_bits, st));
    k_bucket_spans<<<blocks_for(B), TPB, 0, st>>>((uint32_t *)P(A_KEYS_S), m, B, starts, counts);
    k_assign_slots<<<blocks_for(m), TPB, 0, st>>>((uint32_t *)P(A_KEYS_S), (uint32_t *)P(A_IDX_S), m, starts, ix->table, slot);
    GRAB_HIP(ix, hipGetLastError());
    // the per-bucket counts travel to pinned host memory while the candidate search, which writes
    // nothing into the index, is already queued behind them; the host looks at them after queueing it
    int32_t *h_counts = ix->h_table + (size_t)T_COLS * B;
    uint32_t *h_nheads = (uint32_t *)(h_counts + B);
    if (!ix->sync_ev) GRAB_HIP(ix, hipEventCreateWithFlags(&ix->sync_ev, hipEventDisableTiming));
    GRAB_HIP(ix, hipMemcpyAsync(h_counts, counts, (size_t)B * 4, hipMemcpyDeviceToHost, st));
    GRAB_HIP(ix, hipEventRecord(ix->sync_ev, st));
    // ---- 3: local candidate search against the pre-batch index (new rows are not visible yet)
    k_zero_stats<<<1, 64, 0, st>>>(stats);
    mark(0);
    k_fill_range<<<blocks_for(m), TPB, 0, st>>>((int32_t *)P(A_LO), (int32_t *)P(A_HI), m);
    if ((rc = grab_reserve(ix, ix->plans, m * sizeof(QueryPlan))) != GRAB_OK) return rc;
    if ((rc = grab_reserve(ix, ix->seeds, (size_t)m * proto.n_seeds * 4)) != GRAB_OK) return rc;
    if ((rc = grab_reserve(ix, ix->counters, (size_t)m * 8 * 4)) != GRAB_OK) return rc;
    SearchLaunch s = proto;
    s.queries = d_vecs; s.lo = (const int32_t *)P(A_LO); s.hi = (const int32_t *)P(A_HI); s.nq = m;
    s.plans = (QueryPlan *)ix->plans.p; s.seeds = (uint32_t *)ix->seeds.p; s.counters = (uint32_t *)ix->counters.p;
    s.out_slots = true;
    s.only_bucket = bucket; s.out_ids = (uint32_t *)P(A_CL_S); s.out_dist = (float *)P(A_CL_D);
    if ((rc = grab_plan_order(ix, s)) != GRAB_OK) return rc;
    s.sorted_queries = (const uint32_t *)P(A_IDX_S);   // the batch in bucket order: the launch order needs no counting
    if ((rc = grab_launch_select(ix, s)) != GRAB_OK) return rc;
    if ((rc = grab_launch_beam(ix, s)) != GRAB_OK) return rc;
    k_sum_search_counters<<<dim3(64), TPB, 0, st>>>(s.counters, m, stats);
    ix->last_nq = 0;
    if (rule.mode == 1 && kr > 0) {
        // ---- 3': the same search over every other bucket (Section 4.4: candidates from the global scope)
        k_scope_outside<<<blocks_for(m), TPB, 0, st>>>(bucket, m, (int32_t *)P(A_SCOPE));
        s.only_bucket = (const int32_t *)P(A_SCOPE); s.out_ids = (uint32_t *)P(A_CG_S); s.out_dist = (float *)P(A_CG_D);
        if ((rc = grab_launch_select(ix, s)) != GRAB_OK) return rc;
        if ((rc = grab_launch_beam(ix, s)) != GRAB_OK) return rc;
        k_sum_search_counters<<<dim3(64), TPB, 0, st>>>(s.counters, m, stats);
    }
    mark(1);
    // ---- capacity check (nothing has been written so far)
    GRAB_HIP(ix, hipEventSynchronize(ix->sync_ev));
    for (int b = 0; b < B; ++b)
        if (ix->h_table[T_COLS * b + T_NTOT] + h_counts[b] > ix->h_table[T_COLS * b + T_CAP])
            return grab_fail(ix, GRAB_EFULL, "bucket %d holds %d of %d slots and the batch adds %d", b,
                             ix->h_table[T_COLS * b + T_NTOT], ix->h_table[T_COLS * b + T_CAP], h_counts[b]);
    // ---- 4: forward selection, new adjacency rows, reverse requests
    ForwardArgs f;
    f.X = ix->X; f.A = ix->A; f.vecs = d_vecs; f.slot = slot;
    f.cand_s = (const uint32_t *)P(A_CL_S); f.cand_d = (const float *)P(A_CL_D);
    f.key1 = (u64 *)P(A_KEY1); f.key2 = (u64 *)P(A_KEY2); f.reqd = (float *)P(A_REQD);
    f.by_bucket = (const uint32_t *)P(A_IDX_S); f.m = m;
    f.beam = beam; f.kl = kl; f.kr = kr; f.metric = ix->metric;
    f.mode = rule.mode; f.kp = rule.n_proximal; f.window = rule.window; f.remote_cands = ix->prm.append_remote_cands;
    f.gcand_s = (const uint32_t *)P(A_CG_S); f.gcand_d = (const float *)P(A_CG_D);
    f.attr = ix->attr; f.new_attr = d_attrs; f.node_out = (uint32_t *)P(A_NODE_OUT);
    RewireArgs r;
    memset(&r, 0, sizeof(r));
    if ((rc = launch_append(ix, f, r, m, 0)) != GRAB_OK) return rc;
    mark(2);
    // ---- the new objects themselves
    const int32_t row_f4 = ix->dim / 4;
    k_write_new<<<blocks_for(m * row_f4), TPB, 0, st>>>((const float4 *)d_vecs, d_attrs, slot, m, ix->n, row_f4, (float4 *)ix->X,
                                                        ix->attr, ix->slot2id, ix->id2slot);
    // ---- 5: requests grouped by (target, kind): one radix sort over the 33 bits of (target << 1 | kind);
    // the "no request" key has them all set and sorts last.  Inside a group the rewiring itself
    // puts the requests in (distance, source) order.
    k_iota<<<blocks_for(nreq), TPB, 0, st>>>((uint32_t *)P(A_ORD0), nreq);
    GRAB_HIP(ix, rocprim::radix_sort_pairs(P(A_TMP), tmp2, (u64 *)P(A_KEY1), (u64 *)P(A_K1S), (uint32_t *)P(A_ORD0),
                                           (uint32_t *)P(A_ORD2), (size_t)nreq, 0, 33, st));
    // per sorted position what the rewiring needs of the request; the positions where a group starts
    k_request_records<<<blocks_for(nreq), TPB, 0, st>>>((const u64 *)P(A_K1S), (const uint32_t *)P(A_ORD2), (const u64 *)P(A_KEY2),
                                                        (const float *)P(A_REQD), bucket, d_attrs, K, nreq, (uint4 *)P(A_REC),
                                                        (unsigned char *)P(A_HEAD), (uint32_t *)P(A_NHEADS) + 1);
    GRAB_HIP(ix, rocprim::select(P(A_TMP), tmp3, HeadIt(rocprim::counting_iterator<uint32_t>(0), HeadEntry{(const u64 *)P(A_K1S)}),
                                 (unsigned char *)P(A_HEAD), (u64 *)P(A_HEADS), (uint32_t *)P(A_NHEADS), (size_t)nreq, st));
    GRAB_HIP(ix, hipMemcpyAsync(h_nheads, P(A_NHEADS), 4, hipMemcpyDeviceToHost, st));
    GRAB_HIP(ix, hipStreamSynchronize(st));
    const uint32_t n_heads = *h_nheads;
    r.X = ix->X; r.A = ix->A; r.key1s = (const u64 *)P(A_K1S); r.rec = (const uint4 *)P(A_REC);
    r.heads = (const u64 *)P(A_HEADS); r.n_heads = n_heads; r.nreq = nreq;
    r.big_heads = (uint32_t *)P(A_ORD0); r.n_big = (uint32_t *)P(A_NHEADS) + 2;
    r.kl = kl; r.kr = kr; r.metric = ix->metric; r.table = ix->table; r.B = B;
    r.mode = rule.mode; r.kp = rule.n_proximal; r.window = rule.window; r.attr = ix->attr; r.grp_out = (uint32_t *)P(A_GRP_OUT);
    r.a = ix->prm.alpha * ix->prm.alpha;
    mark(3);
    if ((rc = launch_append(ix, f, r, m, 1)) != GRAB_OK) return rc;
    mark(4);
    k_reduce_stats<<<dim3(256), TPB, 0, st>>>(r.heads, r.grp_out, n_heads, (const uint32_t *)P(A_NHEADS) + 1, f.node_out, m, stats);
    // ---- 6: table
    k_widen<<<dim3((unsigned)((m + WIDEN_PER_BLOCK - 1) / WIDEN_PER_BLOCK)), TPB, 0, st>>>(d_attrs, bucket, m, B, ix->table);
    k_grow<<<blocks_for(B), TPB, 0, st>>>(ix->table, counts, B);
    GRAB_HIP(ix, hipGetLastError());
    GRAB_HIP(ix, hipMemcpyAsync(ix->h_table, ix->table, sizeof(int32_t) * T_COLS * B, hipMemcpyDeviceToHost, st));
    GRAB_HIP(ix, hipStreamSynchronize(st));
    ix->n += m;
    ix->app_timed = ix->profile;
    ix->app_has_stats = true;
    return GRAB_OK;
}
