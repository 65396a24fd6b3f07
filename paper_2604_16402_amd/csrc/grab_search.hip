// Range-constrained graph search (Algorithm 2) for gfx950: a bucket-select + seeding kernel
// and a beam-search kernel that runs one query per 64-lane wavefront.
//
// Data movement per query: the query row once, one 128-byte-aligned feature row per
// distance evaluation (8 lanes x 16 B per 128-byte line, all lines of up to 8*R rows in
// flight at once), one adjacency row per expanded parent.  The candidate queue lives in
// registers, the waiting new keys, the slot list and the visited set in LDS.  The scalar
// pre-check is decided from slot intervals prepared by the select kernel, so only slots in
// the appended tails of the two edge buckets cost an attribute read.
#include "grab_device.h"
#include <type_traits>

namespace {

// integer finaliser used for the seed jitter (the public-domain MurmurHash3 finaliser)
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x85ebca6bu; x ^= x >> 13; x *= 0xc2b2ae35u; x ^= x >> 16;
    return x;
}

// ---- half a wavefront per query ------------------------------------------------------------------
// Bucket selection and seeding are a chain of memory round trips with little work between them, so
// two queries share a wavefront: lanes 0-31 serve one, lanes 32-63 the other, and a batch of
// 10,000 queries fits the device in one round of wavefronts.
__device__ __forceinline__ int half_sum(int v) {
#pragma unroll
    for (int m = 16; m > 0; m >>= 1) v += __shfl_xor(v, m);
    return v;
}
// the 32 bits of a ballot that belong to the caller's half
__device__ __forceinline__ uint32_t half_ballot(bool p, int half) { return (uint32_t)(__ballot(p) >> (32 * half)); }

// Two searches per half-wave in lockstep, so that their memory round trips overlap:
// r1 = first index i of sorted a1[0..n1) with a1[i] >= key1, r2 = first index of sorted a2[0..n2)
// with a2[i] > key2.  A 128-way search: each step probes 128 evenly spaced positions, four per
// lane, which settles 16,384 entries in two round trips.  `on` = this half searches at all; the
// loop runs until both halves are done.
__device__ void half_bound2(const int32_t *__restrict__ a1, int n1, int key1, const int32_t *__restrict__ a2, int n2, int key2,
                            bool on, int half, int hl, int &r1, int &r2) {
    int lo1 = 0, hi1 = on ? n1 : 0, lo2 = 0, hi2 = on ? n2 : 0;
    while (__any(hi1 > lo1 || hi2 > lo2)) {
        const int ch1 = (hi1 - lo1 + 127) >> 7, ch2 = (hi2 - lo2 + 127) >> 7;
        int x1[4], x2[4];
        bool act1[4], act2[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {      // probe i = 4 * hl + j of the step
            const int p1 = lo1 + (4 * hl + j) * ch1, p2 = lo2 + (4 * hl + j) * ch2;
            act1[j] = p1 < hi1; act2[j] = p2 < hi2;
            x1[j] = 0; x2[j] = 0;
            if (act1[j]) x1[j] = a1[p1];
            if (act2[j]) x2[j] = a2[p2];
        }
        int c1 = 0, c2 = 0;     // sorted input: the first c probes are below
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            c1 += __popc(half_ballot(act1[j] && x1[j] < key1, half));
            c2 += __popc(half_ballot(act2[j] && x2[j] <= key2, half));
        }
        if (hi1 > lo1) {
            if (c1 == 0) {
                hi1 = lo1;
            } else {
                const int nhi = lo1 + c1 * ch1;
                lo1 = lo1 + (c1 - 1) * ch1 + 1;
                hi1 = nhi < hi1 ? nhi : hi1;
            }
        }
        if (hi2 > lo2) {
            if (c2 == 0) {
                hi2 = lo2;
            } else {
                const int nhi = lo2 + c2 * ch2;
                lo2 = lo2 + (c2 - 1) * ch2 + 1;
                hi2 = nhi < hi2 ? nhi : hi2;
            }
        }
    }
    r1 = lo1;
    r2 = lo2;
}

// ----------------------------------------------------------------------------- select + seed
// Algorithm 2 lines 1-2: the run of buckets whose [min,max] meets [lo,hi]; the valid part of
// the sorted prefix of the two edge buckets by search; the seed population (valid sorted part
// then appended tail of every selected bucket, in bucket order) and one stratified, jittered
// seed per stratum.  Half a wavefront per query (workgroup w: queries 2w and 2w + 1).  The bucket
// table is read once, into LDS; the two searches of a query run in lockstep.
//
// The same launch files the query for the launch order (q_bin non-null): queries that select
// the same buckets read the same vectors, so the search runs them grouped by first selected
// bucket, each XCD taking contiguous runs of that order (see k_order).  bin of a query = its first
// selected bucket (the bucket it is scoped to, for a candidate search); bin B = nothing selected.
// This launch counts the bins and hands every query its rank inside its bin (one atomic per query,
// issued early, its answer picked up at the end); k_order turns bins and ranks into positions.
// Only the order in which queries run changes; every query's result and counters are what they
// are in any order.
__global__ __launch_bounds__(64) void k_select_seed(const int32_t *__restrict__ table, int32_t B,
                                                    const int32_t *__restrict__ attr,
                                                    const int32_t *__restrict__ lo_, const int32_t *__restrict__ hi_,
                                                    const int32_t *__restrict__ only_bucket, int64_t nq, int32_t S, uint32_t salt,
                                                    QueryPlan *__restrict__ plans, uint32_t *__restrict__ seeds,
                                                    const int32_t *__restrict__ fence, int32_t *__restrict__ q_bin,
                                                    int32_t *__restrict__ q_rank, int32_t *__restrict__ bin_count) {
    extern __shared__ int32_t sm_sel[];
    const int lane = threadIdx.x, half = lane >> 5, hl = lane & 31;
    int32_t *tbase = sm_sel, *tnsort = sm_sel + B, *tntot = sm_sel + 2 * B;
    int32_t *pre = sm_sel + 3 * B + half * (B + 1);   // pre[B + 1] of this half
    const int64_t q = 2 * (int64_t)blockIdx.x + half;
    const bool live = q < nq;
    const int lo = live ? lo_[q] : 0, hi = live ? hi_[q] : -1;
    // scope of the query: -1 = its attribute range; b >= 0 = the slab of bucket b; -2 - b = every
    // slot outside the slab of bucket b; INT32_MIN = nothing
    const int only = live ? (only_bucket ? only_bucket[q] : -1) : INT32_MIN;
    const int ex = (only <= -2 && only != INT32_MIN) ? -2 - only : -1;   // excluded bucket
    // bucket intervals are ordered, so counting gives the run: buckets entirely below lo come
    // first, buckets starting at or below hi form a prefix.  Both halves fill the shared columns
    // (with the same values).
    int below = 0, start_ok = 0;
    for (int b = hl; b < B; b += 32) {
        const int32_t *t = table + T_COLS * b;
        tbase[b] = t[T_BASE]; tnsort[b] = t[T_NSORT]; tntot[b] = t[T_NTOT];
        below += t[T_MAX] < lo;
        start_ok += t[T_MIN] <= hi;
    }
    __syncthreads();
    below = half_sum(below);
    start_ok = half_sum(start_ok);
    int b0 = 0, b1 = -1;
    if (only >= 0) {
        b0 = b1 = only;
    } else if (ex >= 0) {
        b0 = 0; b1 = B - 1;
    } else if (only == -1 && lo <= hi) {
        b0 = below;
        b1 = start_ok - 1;
        if (b1 < b0) { b0 = 0; b1 = -1; }
    }
    const bool sel = b1 >= b0;     // false also for the half that has no query
    // the query's bin and its rank inside the bin (order of arrival; the answer is not needed
    // before the end of this kernel)
    const bool filed = q_bin && live && hl == 0;
    int bin = 0, rank = 0;
    if (filed) {
        bin = only >= 0 ? only : (ex >= 0 ? ex : (sel ? b0 : B));
        if (bin < 0 || bin > B) bin = B;
        rank = atomicAdd(&bin_count[GRAB_BIN_STRIDE * bin], 1);
    }
    const int base0 = tbase[b0], ns0 = tnsort[b0], nt0 = tntot[b0];
    const int base1 = sel ? tbase[b1] : 0, ns1 = sel ? tnsort[b1] : 0, nt1 = sel ? tntot[b1] : 0;
    const bool whole = only >= 0 || ex >= 0;   // whole slabs, nothing to check: the "sorted span" is every occupied slot
    int sa0 = 0, se0 = nt0, se1 = nt1, tail0 = 0, tail1 = 0, up = 0, sa = 0;
    {
        // first the fences (contiguous, a few cache lines), then the GRAB_FENCE - 1 attributes
        // between the last fence entry below the bound and the next one
        const bool on = sel && !whole;
        int c0, c1;
        half_bound2(fence + grab_fence_offset(base0, b0), (ns0 + GRAB_FENCE - 1) / GRAB_FENCE, lo,
                    fence + grab_fence_offset(base1, sel ? b1 : 0), (ns1 + GRAB_FENCE - 1) / GRAB_FENCE, hi, on, half, hl, c0, c1);
        const int w0 = c0 > 0 ? (c0 - 1) * GRAB_FENCE + 1 : 0, w1 = c1 > 0 ? (c1 - 1) * GRAB_FENCE + 1 : 0;
        const int n0 = c0 > 0 ? min(c0 * GRAB_FENCE, ns0) - w0 : 0, n1 = c1 > 0 ? min(c1 * GRAB_FENCE, ns1) - w1 : 0;
        half_bound2(attr + base0 + w0, n0, lo, attr + base1 + w1, n1, hi, on, half, hl, sa, up);
        sa += w0;
        up += w1;
    }
    if (sel && !whole) {
        sa0 = sa;
        tail0 = nt0 - ns0;
        se1 = 0;
        if (b1 == b0) {
            se0 = up < sa0 ? sa0 : up;
        } else {
            se0 = ns0;
            se1 = up;
            tail1 = nt1 - ns1;
        }
    }
    // population count per selected bucket, exclusive prefix in LDS
    const int nb = sel ? b1 - b0 + 1 : 0;
    int carry = 0;
    for (int i0 = 0; i0 < nb; i0 += 32) {
        int i = i0 + hl, c = 0;
        if (i < nb) {
            int b = b0 + i;
            if (b == ex) c = 0;
            else if (b == b0) c = (se0 - sa0) + tail0;
            else if (b == b1) c = se1 + tail1;
            else c = tntot[b];
        }
        int inc = c;
#pragma unroll
        for (int d = 1; d < 32; d <<= 1) {
            int upv = __shfl_up(inc, d);
            if (hl >= d) inc += upv;
        }
        if (i < nb) pre[i] = carry + inc - c;
        carry += __shfl(inc, 32 * half + 31);
    }
    if (hl == 0) pre[nb] = carry;
    __syncthreads();
    const int V = carry;
    const int count = V < S ? V : S;
    const uint32_t stride = (V > S) ? (uint32_t)(V / S) : 1u;
    // floor(j V / S) = j floor(V / S) + floor(j (V mod S) / S); for S <= 4096 the last quotient is
    // of numbers below 2^24, which one float multiplication finds to within one
    const int vrem = V > S ? V - (int)stride * S : 0;
    const float rcp_s = 1.0f / (float)S;
    if (live)
        for (int j = hl; j < S; j += 32) {
            uint32_t slot = GRAB_EMPTY;
            if (j < count) {
                int pos = j;       // below V
                if (V > S) {
                    if (S <= 4096) {
                        const int x = j * vrem;
                        int qt = (int)((float)x * rcp_s);
                        const int rm = x - qt * S;
                        qt += (rm >= S) - (rm < 0);
                        pos = j * (int)stride + qt;
                    } else {
                        pos = (int)(((int64_t)j * V) / S);
                    }
                    pos += (int)(mix32((uint32_t)j ^ salt) % stride);
                }
                int l = 0, r = nb;  // last selected bucket whose prefix <= pos
                while (r - l > 1) {
                    int m = (l + r) >> 1;
                    if (pre[m] <= pos) l = m; else r = m;
                }
                int off = pos - pre[l];
                int b = b0 + l;
                if (b == b0) slot = off < se0 - sa0 ? base0 + sa0 + off : base0 + ns0 + (off - (se0 - sa0));
                else if (b == b1) slot = off < se1 ? base1 + off : base1 + ns1 + (off - se1);
                else slot = tbase[b] + off;
            }
            seeds[q * S + j] = slot;
        }
    if (live && hl == 0) {
        QueryPlan p;
        p.b0 = b0; p.b1 = b1; p.V = V; p.n_seeds = count;
        p.s0 = p.e0 = p.t0s = p.t0e = p.ms = p.e1 = p.t1s = p.t1e = 0;
        p.first_valid = p.end_valid = 0; p.pad0 = p.pad1 = 0;
        if (sel) {
            if (ex >= 0) {
                // everything before the excluded slab, and everything after it
                const int32_t *te = table + T_COLS * ex;
                p.s0 = base0; p.e0 = te[T_BASE];
                p.ms = te[T_BASE] + te[T_CAP]; p.e1 = base1 + table[T_COLS * b1 + T_CAP];
                if (V == 0) { p.b0 = 0; p.b1 = -1; }     // nothing lies outside the only bucket
            } else {
                p.s0 = base0 + sa0; p.e0 = base0 + se0;
                p.t0s = base0 + ns0; p.t0e = base0 + ns0 + tail0;
                if (b1 > b0) {
                    p.ms = tbase[b0 + 1];
                    p.e1 = base1 + se1;
                    p.t1s = base1 + ns1; p.t1e = base1 + ns1 + tail1;
                }
            }
            p.first_valid = p.s0;
            p.end_valid = b1 > b0 ? p.e1 : p.e0;
        }
        plans[q] = p;
    }
    if (filed) { q_bin[q] = bin; q_rank[q] = rank; }
}

// ------------------------------------------------------------------------------ launch order
#define GRAB_ORDER_RUN 256   // short run length, see k_order
// Counters of the launch order: bin i has its own 128-byte line (atomics to one line are served
// one after another, and a batch sends thousands at once), word 0 of the line = queries in the
// bin (counted by k_select_seed).  A block of counters must be zero when a call starts counting:
// an index keeps two blocks and uses them in turn, and the k_order of a call clears the block of
// the call before; k_order_reset clears when that is in doubt (fresh memory, a launch that failed
// in between) or when there is only one block.
__global__ void k_order_reset(int32_t *__restrict__ bin_count, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) bin_count[i] = 0;
}

// Places the queries in the launch order: position in bucket order = start of the bin + rank;
// workgroup w of the search kernel runs query order[w] (GRAB_EMPTY: none).
// Runs of `run` consecutive positions go round the XCDs: the i-th workgroup of XCD c (w = 8 i + c)
// takes element i % run of run (i / run) * 8 + c.  Evenly filled bins: runs_per_xcd long runs per
// XCD (one gives the most sharing).  When one bin holds a large share of the batch, what a query
// costs follows its bin (a query that starts in the last bucket cannot be wide), and long runs
// would leave some XCDs with all the expensive queries: short runs then.
// One thread per entry of `order`: it marks its own entry empty if no position maps there, and
// files query t (t < nq).  bin_clear (may be null): the counter block to zero for a later call.
__global__ __launch_bounds__(256) void k_order(const int32_t *__restrict__ q_bin, const int32_t *__restrict__ q_rank,
                                               const int32_t *__restrict__ bin_count, int32_t *__restrict__ bin_clear, int nbins,
                                               int64_t nq, uint32_t *__restrict__ order, int64_t order_len, int runs_per_xcd) {
    __shared__ int32_t start[GRAB_MAX_BUCKETS + 2];
    __shared__ int s_biggest;
    const int tid = threadIdx.x, lane = tid & 63;
    const int64_t t = (int64_t)blockIdx.x * 256 + tid;
    int bin = -1, rank = 0;
    if (t < nq) { bin = q_bin[t]; rank = q_rank[t]; }
    if (tid < 64) {   // exclusive prefix of the bin counts (every workgroup recomputes it: at most 1025 words)
        int carry = 0, biggest = 0;
        for (int i0 = 0; i0 < nbins; i0 += 64) {
            const int i = i0 + lane;
            const int c = i < nbins ? bin_count[GRAB_BIN_STRIDE * i] : 0;
            biggest = max(biggest, c);
            int inc = c;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                int up = __shfl_up(inc, d);
                if (lane >= d) inc += up;
            }
            if (i < nbins) start[i] = carry + inc - c;
            carry += __shfl(inc, 63);
        }
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) biggest = max(biggest, __shfl_xor(biggest, d));
        if (lane == 0) s_biggest = biggest;
    }
    if (bin_clear && t < nbins) bin_clear[GRAB_BIN_STRIDE * t] = 0;
    __syncthreads();
    const int64_t parts = 8 * (int64_t)runs_per_xcd;
    const int64_t run = (int64_t)s_biggest * 16 > nq ? GRAB_ORDER_RUN : (nq + parts - 1) / parts;
    if (t < order_len) {   // the position that maps to entry t
        const int64_t i = t / 8, c = t % 8;
        const int64_t pos = ((i / run) * 8 + c) * run + i % run;
        if (pos >= nq) order[t] = GRAB_EMPTY;
    }
    if (bin >= 0 && bin < nbins) {
        const int64_t pos = (int64_t)start[bin] + rank;      // position in bucket order
        if (pos >= 0 && pos < nq) {
            const int64_t g = pos / run, e = pos % run;
            const int64_t w = ((g / 8) * run + e) * 8 + g % 8;
            if (w < order_len) order[w] = (uint32_t)t;
        }
    }
}

// The launch order read off a list of the queries that is already in bin order (a batch sorted by
// the bucket each query is scoped to): entry t of `order` takes the query at the position that
// k_order would map there, with runs_per_xcd long runs per XCD.
__global__ __launch_bounds__(256) void k_order_sorted(const uint32_t *__restrict__ sorted, int64_t nq, uint32_t *__restrict__ order,
                                                      int64_t order_len, int runs_per_xcd) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= order_len) return;
    const int64_t parts = 8 * (int64_t)runs_per_xcd;
    const int64_t run = (nq + parts - 1) / parts;
    const int64_t i = t / 8, c = t % 8;
    const int64_t pos = ((i / run) * 8 + c) * run + i % run;
    order[t] = pos < nq ? sorted[pos] : GRAB_EMPTY;
}

// ------------------------------------------------------------------------------- beam search
struct BeamArgs {
    const float *X;
    const int32_t *attr;
    const uint32_t *A;
    const uint32_t *slot2id;
    const float *queries;
    const int32_t *lo, *hi;
    const QueryPlan *plans;
    const uint32_t *seeds;
    uint32_t *counters;
    uint32_t *out_ids;
    float *out_dist;
    const uint32_t *order;   // query of each workgroup, or nullptr: workgroup i runs query i
    int64_t nq;
    int32_t K, k, beam, QP, width, max_iter, S, visited_cap, hsize, maxc, metric, out_slots;
};

// scalar pre-check (Algorithm 2, the range test ahead of ComputeDistance) from slot
// intervals; reads the attribute only for slots in the appended tail of an edge bucket
__device__ __forceinline__ bool precheck(const QueryPlan &p, uint32_t v, const int32_t *__restrict__ attr, int lo,
                                         int hi, bool &tail) {
    // every interval of the plan has start <= end < 2^31, so one unsigned comparison tests membership
    // (and fails for the empty entry 0xFFFFFFFF); no branch unless the edge buckets have appended tails
    bool ok = (v - (uint32_t)p.s0 < (uint32_t)(p.e0 - p.s0)) | (v - (uint32_t)p.ms < (uint32_t)(p.e1 - p.ms));
    tail = false;
    if (p.t0e != p.t0s || p.t1e != p.t1s) {   // the same for every lane
        tail = !ok && ((v - (uint32_t)p.t0s < (uint32_t)(p.t0e - p.t0s)) | (v - (uint32_t)p.t1s < (uint32_t)(p.t1e - p.t1s)));
        if (tail) {
            const int a = attr[v];
            ok = a >= lo && a <= hi;
        }
    }
    return ok;
}

// Pre-check and exact visited set for NV slots per lane at once.  The visited set is open
// addressing over H words of LDS (any multiple of 64, at most 80 % full when the capacity rule
// stops the search) with linear probing, one compare-and-swap per probe; the NV probe sequences
// of a lane advance together, so a round costs one LDS round trip, not NV.  Slots that pass both
// tests are appended to L (entry order, lanes ascending); returns the new length of L.
// Which copy of a slot that occurs twice is the one admitted does not matter: queue keys are
// unique per slot and the queue is a set.
template <int NV>
__device__ __forceinline__ int admit(const QueryPlan &p, const uint32_t (&v)[NV], const int32_t *__restrict__ attr,
                                     int lo, int hi, uint32_t *tab, uint32_t H, uint32_t *L, int n_c,
                                     uint32_t &c_rej, uint32_t &c_tail) {
    bool pend[NV], fresh[NV];
    uint32_t h[NV];
    bool any = false;
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        bool tail = false, ok = false;
        const bool live = v[u] != GRAB_EMPTY;
        ok = precheck(p, v[u], attr, lo, hi, tail);   // false for an empty entry
        c_rej += __popcll(__ballot(live && !ok));
        c_tail += __popcll(__ballot(tail));
        pend[u] = ok;
        fresh[u] = false;
        any |= ok;
        h[u] = (uint32_t)(((u64)(v[u] * 0x9E3779B1u) * (u64)H) >> 32);
    }
    for (uint32_t probe = 0; probe < H && __ballot(any) != 0; ++probe) {
        any = false;
#pragma unroll
        for (int u = 0; u < NV; ++u)
            if (pend[u]) {
                const uint32_t old = atomicCAS(&tab[h[u]], GRAB_EMPTY, v[u]);
                fresh[u] = old == GRAB_EMPTY;
                pend[u] = old != GRAB_EMPTY && old != v[u];
                h[u] = h[u] + 1 == H ? 0u : h[u] + 1;
                any |= pend[u];
            }
    }
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const u64 m = __ballot(fresh[u]);
        if (fresh[u]) L[n_c + lanes_below(m)] = v[u];
        n_c += __popcll(m);
    }
    return n_c;
}

// f(integral constant N, args...) with the smallest N in 1..4 such that 64 N lanes-entries cover `left`
// entries (4 if none does): a pass over few entries does not pay for four per lane
#define GRAB_FOR_LANE_LOADS(f, left, ...)                                         \
    do {                                                                          \
        const int left__ = (left);                                                \
        if (left__ <= 64) f(std::integral_constant<int, 1>{}, __VA_ARGS__);       \
        else if (left__ <= 128) f(std::integral_constant<int, 2>{}, __VA_ARGS__); \
        else if (left__ <= 192) f(std::integral_constant<int, 3>{}, __VA_ARGS__); \
        else f(std::integral_constant<int, 4>{}, __VA_ARGS__);                    \
    } while (0)

// One query per wavefront; the queue of up to 64*M keys stays in registers for the whole search.
// New keys wait in a 64-entry LDS buffer, are sorted with a lane-exchange bitonic network sized
// to their number and merged into the queue.  A new key is dropped at once when it is not
// smaller than the worst key of a full queue: it could never enter.
// (four waves per SIMD wherever the registers of the gathered rows leave room for it)
template <int NCH, int M>
__global__ __launch_bounds__(64, (NCH != 8 && M <= 4) ? 4 : 1) void k_beam_search(BeamArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int D = NCH * 32;
    constexpr int R = EvalShape<NCH>::R;
    constexpr int NV = 4;
    const int lane = threadIdx.x;
    const int64_t q = a.order ? (int64_t)a.order[blockIdx.x] : (int64_t)blockIdx.x;
    if (q >= a.nq) return;   // a hole of the launch order (GRAB_EMPTY)
    const int H = a.hsize;
    u64 *C = reinterpret_cast<u64 *>(smem);                 // keys waiting to be merged
    uint32_t *hash = reinterpret_cast<uint32_t *>(C + 64);
    uint32_t *L = hash + H;                                 // slots to evaluate
    uint32_t *par = L + a.maxc;                             // parent slots
    float *qlds = reinterpret_cast<float *>(par + 16);

    const QueryPlan p = a.plans[q];
    const int lo = a.lo[q], hi = a.hi[q];
    uint32_t c_iters = 0, c_par = 0, c_evals = 0, c_seed = 0, c_rej = 0, c_tail = 0, c_vis = 0, c_stop = 0;

    // query row -> registers (or LDS for long rows), in the piece order eval_batch uses
    float4 qreg[EvalShape<NCH>::QREG ? NCH : 1];
    load_query<NCH>(a.queries + q * D, qreg, qlds, lane);
    for (int i = lane; i < H / 4; i += 64) reinterpret_cast<uint4 *>(hash)[i] = make_uint4(~0u, ~0u, ~0u, ~0u);
    __syncthreads();

    LaneQueue<M> Q;
    Q.clear();
    u64 thr = SENT;   // worst key of a full queue, SENT while it has room
    int cnt = 0;      // keys waiting in C

    // merge the cnt keys waiting in C into the queue
    auto flush = [&]() __attribute__((always_inline)) {
        if (cnt == 0) return;
        int P = 2;
        while (P < cnt) P <<= 1;
        u64 ck = lane < cnt ? C[lane] : SENT;
        ck = sort_lanes(ck, P, lane);
        Q.merge(ck, a.beam, lane);
        thr = Q.at(a.beam - 1);
        cnt = 0;
        __syncthreads();
    };
    // ComputeDistance + UpdateQueue for the n slots in L
    auto evaluate = [&](int n) __attribute__((always_inline)) {
        const int sub = lane & 7;
        for (int base = 0; base < n; base += 8 * R) {
            if (cnt + 8 * R > 64) flush();
            float s[R];
            uint32_t v[R];
            bool act[R];
            eval_batch<NCH>(a.X, qreg, qlds, L, base, n, lane, a.metric, s, v, act);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (base + 8 * r >= n) break;   // no group has a row in this round
                u64 key = make_key(s[r], v[r]);
                bool keep = act[r] && sub == 0 && key < thr;
                u64 m = __ballot(keep);
                if (keep) C[cnt + lanes_below(m)] = key;
                cnt += __popcll(m);
            }
            __syncthreads();
        }
        flush();
    };

    if (p.b1 < p.b0) {
        c_stop = 3;
    } else {
        // ---- seeds (Algorithm 2, lines 2-3), in chunks of maxc
        const uint32_t *sd = a.seeds + q * a.S;
        for (int s0 = 0; s0 < p.n_seeds; s0 += a.maxc) {
            const int lim = min(p.n_seeds, s0 + a.maxc);
            int n_c = 0;
            // entries e0 .. of the chunk, N per lane
            auto admit_seeds = [&](auto nvc, int e0) __attribute__((always_inline)) {
                constexpr int N = decltype(nvc)::value;
                uint32_t sv[N];
#pragma unroll
                for (int u = 0; u < N; ++u) {
                    const int e = e0 + 64 * u + lane;
                    sv[u] = e < lim ? sd[e] : GRAB_EMPTY;
                }
                uint32_t unused = 0;
                n_c = admit<N>(p, sv, a.attr, lo, hi, hash, (uint32_t)H, L, n_c, unused, c_tail);
            };
            for (int e0 = s0; e0 < lim; e0 += 64 * NV) GRAB_FOR_LANE_LOADS(admit_seeds, lim - e0, e0);
            __syncthreads();
            c_vis += n_c; c_evals += n_c; c_seed += n_c;
            evaluate(n_c);
        }
        // ---- greedy expansion (Algorithm 2, the while loop)
        const uint32_t recipK = (65536u + (uint32_t)a.K - 1u) / (uint32_t)a.K;
        while (true) {
            if ((int)c_iters == a.max_iter) { c_stop = 1; break; }
            // PopUnvisited: first `width` queue entries not yet expanded
            int np = 0;
            u64 chosen[M];
#pragma unroll
            for (int r = 0; r < M; ++r) {
                chosen[r] = 0;
                u64 m = __ballot(Q.k[r] != SENT && !(Q.k[r] & 1ull));
                while (m && np < a.width) {
                    int b = __ffsll((long long)m) - 1;
                    m &= m - 1;
                    chosen[r] |= 1ull << b;
                    if (lane == b) par[np] = key_slot(Q.k[r]);
                    ++np;
                }
            }
            if (np == 0) break;
            if ((int)c_vis + np * a.K > a.visited_cap) { c_stop = 2; break; }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < M; ++r)
                if ((chosen[r] >> lane) & 1ull) Q.k[r] |= 1ull;
            c_iters += 1; c_par += np;
            // GatherNeighbors + pre-check + visited test, all parents' rows at once
            const int total = np * a.K;
            int n_c = 0;
            auto admit_neighbours = [&](auto nvc, int e0) __attribute__((always_inline)) {
                constexpr int N = decltype(nvc)::value;
                uint32_t nv[N];   // the adjacency loads of up to 64*N entries are in flight together
#pragma unroll
                for (int u = 0; u < N; ++u) {
                    const int e = e0 + 64 * u + lane;
                    nv[u] = GRAB_EMPTY;
                    if (e < total) {
                        uint32_t pi = __umul24((uint32_t)e, recipK) >> 16;      // e < 512, recipK <= 65,536
                        uint32_t j = (uint32_t)e - __umul24(pi, (uint32_t)a.K);
                        nv[u] = a.A[(size_t)par[pi] * (uint32_t)a.K + j];
                    }
                }
                n_c = admit<N>(p, nv, a.attr, lo, hi, hash, (uint32_t)H, L, n_c, c_rej, c_tail);
            };
            for (int e0 = 0; e0 < total; e0 += 64 * NV) GRAB_FOR_LANE_LOADS(admit_neighbours, total - e0, e0);
            __syncthreads();
            c_vis += n_c; c_evals += n_c;
            evaluate(n_c);
        }
    }
    // ---- Top-k from the queue
#pragma unroll
    for (int r = 0; r < M; ++r) {
        const int j = 64 * r + lane;
        if (j < a.k) {
            const u64 key = Q.k[r];
            uint32_t id = GRAB_EMPTY;
            float d = __builtin_inff();
            if (key != SENT) {
                uint32_t slot = key_slot(key);
                id = a.out_slots ? slot : a.slot2id[slot];
                d = image_dist((uint32_t)(key >> 32));
            }
            a.out_ids[q * a.k + j] = id;
            a.out_dist[q * a.k + j] = d;
        }
    }
    if (lane < 8) {
        uint32_t val = lane == 0 ? c_iters : lane == 1 ? c_par : lane == 2 ? c_evals : lane == 3 ? c_seed
                     : lane == 4 ? c_rej : lane == 5 ? c_tail : lane == 6 ? c_vis : c_stop;
        a.counters[q * 8 + lane] = val;
    }
}

template <int NCH, int M>
grab_status launch_beam_tm(grab_index *ix, const BeamArgs &a, int64_t nq, size_t lds) {
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_beam_search<NCH, M>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return grab_fail(ix, GRAB_EHIP, "LDS request of %zu bytes refused: %s", lds, hipGetErrorString(e));
    }
    k_beam_search<NCH, M><<<dim3((unsigned)nq), dim3(64), lds, ix->stream>>>(a);
    GRAB_HIP(ix, hipGetLastError());
    return GRAB_OK;
}

template <int NCH>
grab_status launch_beam_t(grab_index *ix, const BeamArgs &a, int64_t nq, int H) {
    size_t lds = 64 * 8 + (size_t)H * 4 + (size_t)a.maxc * 4 + 16 * 4;
    if (!EvalShape<NCH>::QREG) lds += (size_t)ix->dim * 4;
    switch (a.QP / 64) {
        case 1: return launch_beam_tm<NCH, 1>(ix, a, nq, lds);
        case 2: return launch_beam_tm<NCH, 2>(ix, a, nq, lds);
        case 4: return launch_beam_tm<NCH, 4>(ix, a, nq, lds);
        default: return launch_beam_tm<NCH, 8>(ix, a, nq, lds);
    }
}

inline int pow2_at_least(int x, int floor_) {
    int p = floor_;
    while (p < x) p <<= 1;
    return p;
}

// Measurement aid: every group of eight lanes reads whole rows of the index at pseudo-random
// slots, with the access shape of eval_batch and nothing else to do.  Its rate is what the memory
// system delivers for random rows of this size over this footprint, the practical ceiling of the
// gathered distance evaluation.
template <int NCH>
__global__ __launch_bounds__(64) void k_gather_probe(const float *__restrict__ X, uint32_t n_slots, int batches,
                                                     float *sink) {
    constexpr int CB = EvalShape<NCH>::CB, R = EvalShape<NCH>::R, D4 = NCH * 8;
    const int lane = threadIdx.x, sub = lane & 7, grp = lane >> 3;
    float acc = 0.f;
    for (int it = 0; it < batches; ++it) {
        uint32_t v[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t h = mix32((blockIdx.x * 0x9E3779B1u) ^ ((uint32_t)((it * R + r) * 8 + grp) * 0x85EBCA6Bu));
            v[r] = (uint32_t)(((u64)h * n_slots) >> 32);
        }
#pragma unroll
        for (int c0 = 0; c0 < NCH; c0 += CB) {
            float4 buf[R][CB];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float4 *row = reinterpret_cast<const float4 *>(X) + (size_t)v[r] * D4 + sub;
#pragma unroll
                for (int cc = 0; cc < CB; ++cc) buf[r][cc] = row[(c0 + cc) * 8];
            }
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int cc = 0; cc < CB; ++cc) acc += (buf[r][cc].x + buf[r][cc].y) + (buf[r][cc].z + buf[r][cc].w);
        }
    }
    if (acc == 1.2345678e-30f) sink[0] = acc;   // keeps the loads alive; practically never taken
}

template <int NCH>
grab_status launch_probe_t(grab_index *ix, int64_t waves, int32_t batches, float *sink, double *bytes) {
    k_gather_probe<NCH><<<dim3((unsigned)waves), dim3(64), 0, ix->stream>>>(ix->X, (uint32_t)ix->n_slots, batches, sink);
    GRAB_HIP(ix, hipGetLastError());
    *bytes = (double)waves * batches * 8 * EvalShape<NCH>::R * (double)ix->dim * 4.0;
    return GRAB_OK;
}

}  // namespace

grab_status grab_launch_gather_probe(grab_index *ix, int64_t waves, int32_t batches, float *sink, double *bytes) {
    switch (ix->dim / 32) {
#define GRAB_CASE(N) case N: return launch_probe_t<N>(ix, waves, batches, sink, bytes);
        GRAB_FOR_EACH_NCH(GRAB_CASE)
#undef GRAB_CASE
        default:
            return grab_fail(ix, GRAB_EINVAL, "dim %d has no search kernel", ix->dim);
    }
}

int64_t grab_order_len(int64_t nq) { return (nq + 8 * GRAB_ORDER_RUN - 1) / (8 * GRAB_ORDER_RUN) * (8 * GRAB_ORDER_RUN); }

grab_status grab_plan_order(grab_index *ix, SearchLaunch &s) {
    s.q_bin = s.q_rank = s.bin_count = nullptr;
    s.order = nullptr;
    s.order_len = 0;
    s.order_dirty = nullptr;
    s.order_block = nullptr;
    if (s.nq < 2048) return GRAB_OK;   // a batch that does not even fill the device once gains nothing
    // room for either run length k_order may choose: nq rounded up to eight short runs
    const int64_t len = grab_order_len(s.nq);
    grab_status st;
    if ((st = grab_reserve(ix, ix->q_bin, (size_t)s.nq * 4)) != GRAB_OK) return st;
    if ((st = grab_reserve(ix, ix->q_rank, (size_t)s.nq * 4)) != GRAB_OK) return st;
    if ((st = grab_reserve(ix, ix->q_order, (size_t)len * 4)) != GRAB_OK) return st;
    const void *before = ix->bin_count.p;
    if ((st = grab_reserve(ix, ix->bin_count, 2 * GRAB_BIN_BLOCK_BYTES)) != GRAB_OK) return st;
    if (ix->bin_count.p != before) ix->order_dirty = true;    // fresh memory: counters not yet zero
    s.q_bin = (int32_t *)ix->q_bin.p; s.q_rank = (int32_t *)ix->q_rank.p; s.bin_count = (int32_t *)ix->bin_count.p;
    s.order = (uint32_t *)ix->q_order.p;
    s.order_len = len;
    s.order_dirty = &ix->order_dirty;
    s.order_block = &ix->order_block;
    return GRAB_OK;
}

grab_status grab_launch_select(grab_index *ix, const SearchLaunch &s) {
    if (s.nq == 0) return GRAB_OK;
    const int nbins = ix->B + 1;   // the last bin takes the queries whose range meets no bucket
    const size_t lds = (size_t)(5 * ix->B + 2) * 4;
    const bool counted = s.order && !s.sorted_queries;
    int32_t *count = nullptr, *clear = nullptr;
    if (counted) {
        count = s.bin_count;
        if (s.order_block) {
            count = s.bin_count + (size_t)*s.order_block * GRAB_BIN_BLOCK_WORDS;
            clear = s.bin_count + (size_t)(1 - *s.order_block) * GRAB_BIN_BLOCK_WORDS;
        }
        // the block is left zero by an earlier k_order; if that is in doubt (fresh memory, a launch
        // that failed in between, a single block) everything is cleared first
        const bool dirty = !s.order_dirty || *s.order_dirty;
        if (s.order_dirty) *s.order_dirty = true;
        if (dirty) {
            const int words = (s.order_block ? 2 : 1) * GRAB_BIN_BLOCK_WORDS;
            k_order_reset<<<dim3((unsigned)((words + 255) / 256)), dim3(256), 0, ix->stream>>>(s.bin_count, words);
            GRAB_HIP(ix, hipGetLastError());
        }
    }
    k_select_seed<<<dim3((unsigned)((s.nq + 1) / 2)), dim3(64), lds, ix->stream>>>(ix->table, ix->B, ix->attr, s.lo, s.hi,
                                                                                s.only_bucket, s.nq, s.n_seeds, s.salt, s.plans,
                                                                                s.seeds, ix->fence, counted ? s.q_bin : nullptr,
                                                                                s.q_rank, count);
    GRAB_HIP(ix, hipGetLastError());
    // measured: rows of 512 B (1M x 128) run fastest with one run per XCD (headline 481 us against
    // 502 us with four and 516 us in input order); rows of 3,840 B (1M x 960) with four (3.82 ms
    // against 4.06 ms with one and 4.19 ms in input order)
    const int runs_per_xcd = ix->dim >= 512 ? 4 : 1;
    if (s.order && s.sorted_queries) {
        k_order_sorted<<<dim3((unsigned)((s.order_len + 255) / 256)), dim3(256), 0, ix->stream>>>(s.sorted_queries, s.nq, s.order,
                                                                                               s.order_len, runs_per_xcd);
        GRAB_HIP(ix, hipGetLastError());
    }
    if (counted) {
        k_order<<<dim3((unsigned)((s.order_len + 255) / 256)), dim3(256), 0, ix->stream>>>(s.q_bin, s.q_rank, count, clear, nbins,
                                                                                        s.nq, s.order, s.order_len, runs_per_xcd);
        GRAB_HIP(ix, hipGetLastError());
        if (s.order_block) *s.order_block ^= 1;
        if (s.order_dirty) *s.order_dirty = false;
    }
    return GRAB_OK;
}

grab_status grab_launch_beam(grab_index *ix, const SearchLaunch &s) {
    if (s.nq == 0) return GRAB_OK;
    BeamArgs a;
    a.X = ix->X; a.attr = ix->attr; a.A = s.adj ? s.adj : ix->A; a.slot2id = ix->slot2id;
    a.queries = s.queries; a.lo = s.lo; a.hi = s.hi; a.plans = s.plans; a.seeds = s.seeds;
    a.counters = s.counters; a.out_ids = s.out_ids; a.out_dist = s.out_dist;
    a.order = s.order; a.nq = s.nq;
    a.K = ix->kl + ix->kr; a.k = s.k; a.beam = s.beam; a.QP = pow2_at_least(s.beam, 64);
    a.width = s.width; a.max_iter = s.max_iter; a.S = s.n_seeds; a.visited_cap = s.visited_cap;
    // visited table: the power of two above 4/3 of the capacity when that wastes little LDS (short
    // probe runs), else 5/4 of the capacity rounded up to 64 words (80 % full at the very worst)
    int H = pow2_at_least((int)(((int64_t)s.visited_cap * 4 + 2) / 3) + 1, 64);
    if ((int64_t)H * 5 > (int64_t)s.visited_cap * 8) H = (int)((((int64_t)s.visited_cap * 5 + 3) / 4 + 63) / 64 * 64);
    a.hsize = H;
    a.maxc = pow2_at_least(s.width * a.K, 64);
    a.metric = ix->metric; a.out_slots = s.out_slots ? 1 : 0;
    const int nch = ix->dim / 32;
    switch (nch) {
#define GRAB_CASE(N) case N: return launch_beam_t<N>(ix, a, s.order ? s.order_len : s.nq, H);
        GRAB_FOR_EACH_NCH(GRAB_CASE)
#undef GRAB_CASE
        default:
            return grab_fail(ix, GRAB_EINVAL, "dim %d has no search kernel", ix->dim);
    }
}
