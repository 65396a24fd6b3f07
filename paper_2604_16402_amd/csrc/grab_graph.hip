// Two-pass index construction (Section 4.3) for gfx950: exact brute-force k-NN inside every
// bucket, diversity pruning (Eq. 2 as a construction rule), reverse lists, interleaved
// forward/reverse merge into the local part of each row, and remote edges to the nearest node of
// a few other buckets.  The global candidate graph of the paper's second pass (Algorithm 1, a
// third-party pipeline) is replaced by exact nearest-node search in the target buckets.
//
// The k-NN kernel is compute-bound on the vector ALUs (no MFMA: every distance is produced
// with the library's fixed fp32 summation order so that ties and ranks are reproducible): a
// workgroup of four wavefronts owns 32 source rows; each lane of a wavefront owns one target row
// of the current 64-row tile and eight source rows, i.e. 64 partial sums; tiles are staged
// through LDS transposed so that lane reads are conflict-free and source values are broadcast.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include "grab_device.h"

namespace {

constexpr int TPB = 256;
inline unsigned blocks_for(int64_t work) { return (unsigned)((work + TPB - 1) / TPB); }

struct KnnArgs {
    const float *X;
    const int32_t *table;
    const int32_t *tgt;   // [B] target bucket of each source bucket, -1: none
    uint32_t *out_s;      // P > 1: [n_slots][P] slots;  P == 1: out_s[slot * out_stride + out_off]
    float *out_d;         // P > 1: [n_slots][P] distances
    int64_t out_stride, out_off, n_slots;
    int32_t P, metric, exclude_self;
};

template <int NCH, int PM>
__global__ __launch_bounds__(256) void k_knn(KnnArgs a) {
    constexpr int D4 = NCH * 8;
    __shared__ float Bt[32 * 65];             // target tile chunk, [float k][row], padded
    __shared__ float4 Aq[32 * 8];             // source tile chunk, [row][piece]
    __shared__ u64 scratch[4][64];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int b = blockIdx.y;
    const int sb = a.table[T_COLS * b + T_BASE], sn = a.table[T_COLS * b + T_NTOT];
    const int i0 = blockIdx.x * 32;
    if (i0 >= sn) return;
    const int t = a.tgt[b];
    uint32_t slot_i[8];
    bool valid_i[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        slot_i[r] = (uint32_t)(sb + i0 + w * 8 + r);
        valid_i[r] = i0 + w * 8 + r < sn;
    }
    if (t < 0) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (!valid_i[r]) continue;
            if (a.P == 1) { if (lane == 0) a.out_s[(int64_t)slot_i[r] * a.out_stride + a.out_off] = GRAB_EMPTY; }
            else for (int pos = lane; pos < a.P; pos += 64) { a.out_s[(int64_t)slot_i[r] * a.P + pos] = GRAB_EMPTY; a.out_d[(int64_t)slot_i[r] * a.P + pos] = __builtin_inff(); }
        }
        return;
    }
    const int tb = a.table[T_COLS * t + T_BASE], tn = a.table[T_COLS * t + T_NTOT];
    const float4 *X4 = reinterpret_cast<const float4 *>(a.X);
    const u64 lt_mask = (1ull << lane) - 1ull;
    LaneQueue<PM> qk[8];   // P > 1: the P best keys of each source row; P == 1: k[0] is a per-lane minimum
    u64 thr[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) { qk[r].clear(); thr[r] = SENT; }

    for (int j0 = 0; j0 < tn; j0 += 64) {
        float acc[8][8];
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int p = 0; p < 8; ++p) acc[r][p] = 0.0f;
        for (int c = 0; c < NCH; ++c) {
            __syncthreads();
            {   // stage the target chunk transposed: thread -> (row, two 16-byte pieces)
                const int row = tid >> 2, pp = (tid & 3) * 2;
                int64_t sj = (int64_t)tb + j0 + row;
                if (sj >= a.n_slots) sj = a.n_slots - 1;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    float4 f = X4[sj * D4 + c * 8 + pp + i];
                    const int k = (pp + i) * 4;
                    Bt[(k + 0) * 65 + row] = f.x; Bt[(k + 1) * 65 + row] = f.y;
                    Bt[(k + 2) * 65 + row] = f.z; Bt[(k + 3) * 65 + row] = f.w;
                }
                const int arow = tid >> 3, ap = tid & 7;
                int64_t si = (int64_t)sb + i0 + arow;
                if (si >= a.n_slots) si = a.n_slots - 1;
                Aq[arow * 8 + ap] = X4[si * D4 + c * 8 + ap];
            }
            __syncthreads();
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const float x0 = Bt[(4 * p + 0) * 65 + lane], x1 = Bt[(4 * p + 1) * 65 + lane];
                const float x2 = Bt[(4 * p + 2) * 65 + lane], x3 = Bt[(4 * p + 3) * 65 + lane];
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const float4 q = Aq[(w * 8 + r) * 8 + p];   // same address in every lane: broadcast
                    if (a.metric == GRAB_L2SQ) {
                        float d0 = q.x - x0, d1 = q.y - x1, d2 = q.z - x2, d3 = q.w - x3;
                        acc[r][p] = __builtin_fmaf(d0, d0, acc[r][p]);
                        acc[r][p] = __builtin_fmaf(d1, d1, acc[r][p]);
                        acc[r][p] = __builtin_fmaf(d2, d2, acc[r][p]);
                        acc[r][p] = __builtin_fmaf(d3, d3, acc[r][p]);
                    } else {
                        acc[r][p] = __builtin_fmaf(q.x, x0, acc[r][p]);
                        acc[r][p] = __builtin_fmaf(q.y, x1, acc[r][p]);
                        acc[r][p] = __builtin_fmaf(q.z, x2, acc[r][p]);
                        acc[r][p] = __builtin_fmaf(q.w, x3, acc[r][p]);
                    }
                }
            }
        }
        const uint32_t slot_j = (uint32_t)(tb + j0 + lane);
        const bool valid_j = j0 + lane < tn;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            // same pairwise combination as the gathered distance: ((p0+p1)+(p2+p3))+((p4+p5)+(p6+p7))
            float s = ((acc[r][0] + acc[r][1]) + (acc[r][2] + acc[r][3])) + ((acc[r][4] + acc[r][5]) + (acc[r][6] + acc[r][7]));
            if (a.metric != GRAB_L2SQ) s = -s;
            const u64 key = make_key(s, slot_j);
            const bool keep = valid_j && valid_i[r] && !(a.exclude_self && slot_j == slot_i[r]) && key < thr[r];
            if (a.P == 1) {
                if (keep && key < qk[r].k[0]) qk[r].k[0] = key;     // per-lane running minimum, reduced at the end
            } else {
                const u64 m = __ballot(keep);
                if (m) {
                    const int cnt = __popcll(m);
                    if (keep) scratch[w][__popcll(m & lt_mask)] = key;
                    __builtin_amdgcn_wave_barrier();
                    u64 ck = lane < cnt ? scratch[w][lane] : SENT;
                    __builtin_amdgcn_wave_barrier();
                    int Pc = 2;
                    while (Pc < cnt) Pc <<= 1;
                    ck = sort_lanes(ck, Pc, lane);
                    qk[r].merge(ck, a.P, lane);
                    thr[r] = qk[r].at(a.P - 1);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        if (a.P == 1) {
            u64 best = qk[r].k[0];
#pragma unroll
            for (int s = 32; s > 0; s >>= 1) {
                u64 o = shfl_xor64(best, s);
                best = o < best ? o : best;
            }
            if (valid_i[r] && lane == 0)
                a.out_s[(int64_t)slot_i[r] * a.out_stride + a.out_off] = best == SENT ? GRAB_EMPTY : key_slot(best);
        } else if (valid_i[r]) {
#pragma unroll
            for (int m = 0; m < PM; ++m) {
                const int pos = 64 * m + lane;
                if (pos < a.P) {
                    const u64 kk = qk[r].k[m];
                    const bool has = kk != SENT;
                    a.out_s[(int64_t)slot_i[r] * a.P + pos] = has ? key_slot(kk) : GRAB_EMPTY;
                    a.out_d[(int64_t)slot_i[r] * a.P + pos] = has ? image_dist((uint32_t)(kk >> 32)) : __builtin_inff();
                }
            }
        }
    }
}

struct PruneArgs {
    const float *X;
    const uint32_t *slot2id;
    const uint32_t *cand_s;  // [n_slots][P] ordered by (distance, slot)
    const float *cand_d;
    uint32_t *F;             // [n_slots][P] forward list: kept by Eq. 2 first, then the rejected ones
    float *Fd;
    int32_t P, metric;
};

// Eq. 2 scan for one node per wavefront: candidate t is kept iff dist(u,c_t) < dist(c_t,n) for every
// n kept before it; the kept rows are evaluated eight lanes per row against the candidate's row.
// Up to 128 candidates: lane l holds candidates l and 64 + l.
template <int NCH>
__global__ __launch_bounds__(64) void k_prune(PruneArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int D = NCH * 32;
    const int lane = threadIdx.x;
    const int64_t u = blockIdx.x;
    if (a.slot2id[u] == GRAB_EMPTY) return;
    uint32_t *kept = reinterpret_cast<uint32_t *>(smem);
    float *dtmp = reinterpret_cast<float *>(kept + 128);
    float *qlds = dtmp + 128;
    float4 qreg[EvalShape<NCH>::QREG ? NCH : 1];
    uint32_t cs[2];
    float cd[2];
    u64 validm[2], keptm[2] = {0, 0};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int t = 64 * h + lane;
        cs[h] = t < a.P ? a.cand_s[u * a.P + t] : GRAB_EMPTY;
        cd[h] = t < a.P ? a.cand_d[u * a.P + t] : 0.0f;
        validm[h] = __ballot(cs[h] != GRAB_EMPTY);
    }
    const int nc = __popcll(validm[0]) + __popcll(validm[1]);   // valid candidates form a prefix
    const u64 lt_mask = (1ull << lane) - 1ull;
    int nk = 0;
    if constexpr (EvalShape<NCH>::QREG) {
        // eight candidates at a time, one per group of eight lanes: their rows are loaded together, each
        // is compared with the rows kept so far (the scan ends as soon as all eight are hidden) and, where
        // two or more survive that, with the other survivors; the chunk is then resolved in candidate
        // order exactly as a one-by-one scan would
        uint32_t *alive = reinterpret_cast<uint32_t *>(dtmp + 128);
        uint32_t *alive_g = alive + 8;
        float *pair = reinterpret_cast<float *>(alive_g + 8);   // [8][8] distances between survivors
        const int sub = lane & 7, grp = lane >> 3;
        for (int t0 = 0; t0 < nc; t0 += 8) {
            const int G = min(8, nc - t0);
            const int mt = t0 + grp < nc ? t0 + grp : t0;
            const uint32_t myc = mt < 64 ? (uint32_t)__shfl((int)cs[0], mt) : (uint32_t)__shfl((int)cs[1], mt - 64);
            const float mydq = mt < 64 ? __shfl(cd[0], mt) : __shfl(cd[1], mt - 64);
            float4 mine[NCH];
            {
                const float4 *row = reinterpret_cast<const float4 *>(a.X) + (size_t)myc * (NCH * 8) + sub;
#pragma unroll
                for (int c = 0; c < NCH; ++c) mine[c] = row[c * 8];
            }
            bool hid = t0 + grp >= nc;
            group_vs_rows<NCH>(a.X, mine, kept, nk, lane, a.metric, [&](int, float s) { hid |= !(mydq < s); },
                               [&]() { return __ballot(!hid) == 0; });
            const u64 hm = __ballot(hid);
            int na = 0;
            for (int g = 0; g < G; ++g)
                if (((hm >> (8 * g)) & 1ull) == 0) {
                    const uint32_t cg = (uint32_t)__shfl((int)myc, 8 * g);
                    if (lane == 0) { alive[na] = cg; alive_g[na] = (uint32_t)g; }
                    ++na;
                }
            __syncthreads();
            if (na > 1)
                group_vs_rows<NCH>(a.X, mine, alive, na, lane, a.metric, [&](int h, float s) { if (sub == 0) pair[grp * 8 + alive_g[h]] = s; },
                                   []() { return false; });
            __syncthreads();
            uint32_t keptmask = 0;
            for (int g = 0; g < G; ++g) {
                const int t = t0 + g;
                const float dqc = __shfl(mydq, 8 * g);
                bool ok = ((hm >> (8 * g)) & 1ull) == 0;
                for (int h = 0; h < g; ++h)
                    if ((keptmask >> h) & 1u) ok = ok && (dqc < pair[g * 8 + h]);
                const uint32_t cg = (uint32_t)__shfl((int)myc, 8 * g);   // every lane takes part in the exchange
                if (ok) {
                    if (lane == 0) kept[nk] = cg;
                    keptm[t >> 6] |= 1ull << (t & 63);
                    keptmask |= 1u << g;
                    ++nk;
                }
            }
            __syncthreads();
        }
    } else {
    for (int t = 0; t < nc; ++t) {
        const uint32_t c = t < 64 ? (uint32_t)__shfl((int)cs[0], t) : (uint32_t)__shfl((int)cs[1], t - 64);
        const float dqc = t < 64 ? __shfl(cd[0], t) : __shfl(cd[1], t - 64);
        bool ok = true;
        if (nk > 0) {
            load_query<NCH>(a.X + (size_t)c * D, qreg, qlds, lane);
            if constexpr (!EvalShape<NCH>::QREG) __syncthreads();
            eval_rows<NCH>(a.X, qreg, qlds, kept, nk, lane, a.metric, dtmp);
            __syncthreads();
            const bool hidden = (lane < nk && !(dqc < dtmp[lane])) || (64 + lane < nk && !(dqc < dtmp[64 + lane]));
            ok = __ballot(hidden) == 0;
        }
        if (ok) {
            if (lane == 0) kept[nk] = c;
            keptm[t >> 6] |= 1ull << (t & 63);
            ++nk;
        }
        __syncthreads();
    }
    }
    const int nk0 = __popcll(keptm[0]), nr0 = __popcll(~keptm[0] & validm[0]);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int t = 64 * h + lane;
        if (t >= a.P) continue;
        uint32_t out = GRAB_EMPTY;
        float outd = __builtin_inff();
        int pos = t;
        if (t < nc) {
            const bool mine = (keptm[h] >> lane) & 1ull;
            const int kept_before = (h ? nk0 : 0) + __popcll(keptm[h] & lt_mask);
            const int rej_before = (h ? nr0 : 0) + __popcll(~keptm[h] & validm[h] & lt_mask);
            pos = mine ? kept_before : nk + rej_before;
            out = cs[h]; outd = cd[h];
        }
        a.F[u * a.P + pos] = out;
        a.Fd[u * a.P + pos] = outd;
    }
}

// one thread per (node, j < kl): the reverse-graph edge F(u)[j] <- u with its two sort keys
__global__ void k_rev_keys(const uint32_t *__restrict__ F, const float *__restrict__ Fd, int64_t n_slots, int32_t P,
                           int32_t kl, uint32_t *__restrict__ key1, u64 *__restrict__ key2, uint32_t *__restrict__ idx) {
    int64_t e = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (e >= n_slots * kl) return;
    const int64_t u = e / kl;
    const int j = (int)(e - u * kl);
    const uint32_t v = F[u * P + j];
    key1[e] = v;   // empty entries (0xFFFFFFFF) sort last
    key2[e] = ((u64)dist_image(v == GRAB_EMPTY ? 0.0f : Fd[u * P + j]) << 32) | (u64)(uint32_t)u;
    idx[e] = (uint32_t)e;
}

__global__ void k_gather_u32(const uint32_t *__restrict__ src, const uint32_t *__restrict__ order, int64_t n,
                             uint32_t *__restrict__ dst) {
    int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < n) dst[i] = src[order[i]];
}

// sorted by (target, distance, source): the first kl sources of every target form its reverse list
__global__ void k_rev_fill(const uint32_t *__restrict__ key1s, const uint32_t *__restrict__ order,
                           const u64 *__restrict__ key2, int64_t ne, int32_t kl, uint32_t *__restrict__ R) {
    int64_t p = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (p >= ne) return;
    const uint32_t v = key1s[p];
    if (v == GRAB_EMPTY) return;
    int64_t l = 0, r = p;   // first position holding v
    while (l < r) { int64_t mid = (l + r) >> 1; if (key1s[mid] < v) l = mid + 1; else r = mid; }
    const int64_t rank = p - l;
    if (rank < kl) R[(int64_t)v * kl + rank] = (uint32_t)(key2[order[p]] & 0xFFFFFFFFull);
}

// F0, R0, F1, R1, ... (the reverse list ends after kl entries, the forward list goes on to P)
// without empties and repeats; the first kl survivors are the necessary local edges; with
// want = K the next ones fill the rest of the row as redundant local edges (Section 4.3, Local
// Router Construction)
__global__ void k_interleave(const uint32_t *__restrict__ F, const uint32_t *__restrict__ R,
                             const uint32_t *__restrict__ slot2id, int64_t n_slots, int32_t P, int32_t kl, int32_t K,
                             int32_t want, uint32_t *__restrict__ A) {
    int64_t u = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (u >= n_slots || slot2id[u] == GRAB_EMPTY) return;
    uint32_t *row = A + u * K;
    int w = 0;
    for (int j = 0; j < P && w < want; ++j)
        for (int side = 0; side < 2 && w < want; ++side) {
            if (side == 1 && j >= kl) continue;
            const uint32_t c = side == 0 ? F[u * P + j] : R[u * kl + j];
            if (c == GRAB_EMPTY) continue;
            bool dup = false;
            for (int x = 0; x < w; ++x) dup |= row[x] == c;
            if (!dup) row[w++] = c;
        }
}

template <int NCH>
grab_status launch_graph_t(grab_index *ix, const KnnArgs *k, const PruneArgs *p, unsigned tiles) {
    if (k) {
        if (k->P > 64) k_knn<NCH, 2><<<dim3(tiles, (unsigned)ix->B), dim3(256), 0, ix->stream>>>(*k);
        else k_knn<NCH, 1><<<dim3(tiles, (unsigned)ix->B), dim3(256), 0, ix->stream>>>(*k);
    } else {
        size_t lds = 128 * 4 * 2 + (EvalShape<NCH>::QREG ? (16 + 64) * 4 : (size_t)ix->dim * 4);
        k_prune<NCH><<<dim3((unsigned)ix->n_slots), dim3(64), lds, ix->stream>>>(*p);
    }
    GRAB_HIP(ix, hipGetLastError());
    return GRAB_OK;
}

grab_status launch_graph(grab_index *ix, const KnnArgs *k, const PruneArgs *p, unsigned tiles) {
    switch (ix->dim / 32) {
#define GRAB_CASE(N) case N: return launch_graph_t<N>(ix, k, p, tiles);
        GRAB_FOR_EACH_NCH(GRAB_CASE)
#undef GRAB_CASE
        default:
            return grab_fail(ix, GRAB_EINVAL, "dim %d has no construction kernel", ix->dim);
    }
}

// target buckets of bucket b: +-1, +-2, +-4, ... then the remaining offsets by size
int remote_targets(int b, int B, int kr, int *out) {
    int n = 0;
    for (int pass = 0; pass < 2 && n < kr; ++pass)
        for (int o = 1; o < B && n < kr; o = pass == 0 ? o * 2 : o + 1) {
            if (pass == 1 && (o & (o - 1)) == 0) continue;
            for (int sgn = 1; sgn >= -1 && n < kr; sgn -= 2) {
                int t = b + sgn * o;
                if (t >= 0 && t < B) out[n++] = t;
            }
        }
    return n;
}

}  // namespace

grab_status grab_build_graph_device(grab_index *ix, int32_t kl, int32_t kr, int32_t pool, const SearchLaunch &proto) {
    hipStream_t st = ix->stream;
    const int32_t B = ix->B, K = kl + kr;
    const int64_t N = ix->n_slots, ne = N * kl;
    int32_t max_n = 0;
    for (int b = 0; b < B; ++b) max_n = ix->h_table[T_COLS * b + T_NTOT] > max_n ? ix->h_table[T_COLS * b + T_NTOT] : max_n;
    const unsigned tiles = (unsigned)((max_n + 31) / 32);
    std::vector<void *> tmp;
    auto cleanup = [&]() { for (void *p : tmp) (void)hipFree(p); };
    grab_status rc = GRAB_OK;
#define G_ALLOC(ptr, bytes)                                                                                  \
    do {                                                                                                     \
        void *p__ = nullptr;                                                                                 \
        hipError_t e__ = hipMalloc(&p__, (bytes) ? (bytes) : 16);                                            \
        if (e__ != hipSuccess) {                                                                             \
            cleanup();                                                                                       \
            return grab_fail(ix, GRAB_ENOMEM, "construction needs %zu more bytes: %s", (size_t)(bytes), hipGetErrorString(e__)); \
        }                                                                                                    \
        tmp.push_back(p__);                                                                                  \
        ptr = reinterpret_cast<decltype(ptr)>(p__);                                                          \
    } while (0)
#define G_HIP(call)                                                                                          \
    do {                                                                                                     \
        hipError_t e__ = (call);                                                                             \
        if (e__ != hipSuccess) {                                                                             \
            cleanup();                                                                                       \
            return grab_fail(ix, GRAB_EHIP, "%s failed: %s", #call, hipGetErrorString(e__));                 \
        }                                                                                                    \
    } while (0)
    uint32_t *cand_s, *F, *R, *key1, *key1g, *key1s, *ord0, *ord1, *ord2;
    float *cand_d, *Fd;
    u64 *key2, *key2s;
    int32_t *tgt;
    G_ALLOC(cand_s, (size_t)N * pool * 4); G_ALLOC(cand_d, (size_t)N * pool * 4);
    G_ALLOC(F, (size_t)N * pool * 4); G_ALLOC(Fd, (size_t)N * pool * 4);
    G_ALLOC(R, (size_t)ne * 4);
    G_ALLOC(key1, (size_t)ne * 4); G_ALLOC(key1g, (size_t)ne * 4); G_ALLOC(key1s, (size_t)ne * 4);
    G_ALLOC(ord0, (size_t)ne * 4); G_ALLOC(ord1, (size_t)ne * 4); G_ALLOC(ord2, (size_t)ne * 4);
    G_ALLOC(key2, (size_t)ne * 8); G_ALLOC(key2s, (size_t)ne * 8);
    G_ALLOC(tgt, (size_t)B * 4);
    // pass 1 searches every bucket for its own nearest objects
    {
        std::vector<int32_t> h((size_t)B, -1);
        for (int b = 0; b < B; ++b) h[b] = b;
        G_HIP(hipMemcpyAsync(tgt, h.data(), h.size() * 4, hipMemcpyHostToDevice, st));
        G_HIP(hipStreamSynchronize(st));
    }
    G_HIP(hipMemsetAsync(ix->A, 0xFF, (size_t)N * K * 4, st));
    G_HIP(hipMemsetAsync(R, 0xFF, (size_t)ne * 4, st));
    G_HIP(hipMemsetAsync(F, 0xFF, (size_t)N * pool * 4, st));
    // pass 1: candidates, pruning, reverse lists, interleaved merge
    KnnArgs k;
    k.X = ix->X; k.table = ix->table; k.tgt = tgt; k.out_s = cand_s; k.out_d = cand_d;
    k.out_stride = pool; k.out_off = 0; k.n_slots = N; k.P = pool; k.metric = ix->metric; k.exclude_self = 1;
    {
        // scores on the matrix cores pick the few candidates whose exact distances are then taken;
        // without memory for that, or where too many distances are equal, every pair is evaluated in fp32
        KnnFilter *flt = nullptr;
        bool redo = true;
        if (grab_knn_prepare(ix, &flt) == GRAB_OK) {
            rc = grab_knn_pass(ix, flt, tgt, cand_s, cand_d, pool, 0, pool, 1, &redo);
            grab_knn_release(flt);
            if (rc != GRAB_OK) { cleanup(); return rc; }
        }
        if (redo && (rc = launch_graph(ix, &k, nullptr, tiles)) != GRAB_OK) { cleanup(); return rc; }
    }
    PruneArgs p;
    p.X = ix->X; p.slot2id = ix->slot2id; p.cand_s = cand_s; p.cand_d = cand_d; p.F = F; p.Fd = Fd; p.P = pool; p.metric = ix->metric;
    if ((rc = launch_graph(ix, nullptr, &p, tiles)) != GRAB_OK) { cleanup(); return rc; }
    if (ne > 0) {
        k_rev_keys<<<blocks_for(ne), TPB, 0, st>>>(F, Fd, N, pool, kl, key1, key2, ord0);
        size_t t1 = 0, t2 = 0;
        G_HIP(rocprim::radix_sort_pairs(nullptr, t2, key2, key2s, ord0, ord1, (size_t)ne, 0, 64, st));
        G_HIP(rocprim::radix_sort_pairs(nullptr, t1, key1g, key1s, ord1, ord2, (size_t)ne, 0, 32, st));
        void *sort_tmp;
        G_ALLOC(sort_tmp, (t1 > t2 ? t1 : t2) + 16);
        G_HIP(rocprim::radix_sort_pairs(sort_tmp, t2, key2, key2s, ord0, ord1, (size_t)ne, 0, 64, st));
        k_gather_u32<<<blocks_for(ne), TPB, 0, st>>>(key1, ord1, ne, key1g);
        G_HIP(rocprim::radix_sort_pairs(sort_tmp, t1, key1g, key1s, ord1, ord2, (size_t)ne, 0, 32, st));
        k_rev_fill<<<blocks_for(ne), TPB, 0, st>>>(key1s, ord2, key2, ne, kl, R);
    }
    k_interleave<<<blocks_for(N), TPB, 0, st>>>(F, R, ix->slot2id, N, pool, kl, K, ix->prm.remote_mode == 1 ? K : kl, ix->A);
    G_HIP(hipGetLastError());
    G_HIP(hipStreamSynchronize(st));
    cleanup();
    // pass 2: remote entries
    ix->kl = kl; ix->kr = kr;
    return grab_build_remote_device(ix, proto);
}

namespace {

// scope of construction's candidate search for the row at each slot: every slot outside the
// row's own bucket; nothing for a slot without an object
__global__ void k_scope_rows(const int32_t *__restrict__ table, int32_t B, const uint32_t *__restrict__ slot2id,
                             int64_t first, int64_t count, int32_t *__restrict__ scope) {
    int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= count) return;
    const int64_t u = first + i;
    int32_t sc = INT32_MIN;
    if (slot2id[u] != GRAB_EMPTY) {
        int l = 0, r = B;   // last bucket whose base <= slot
        while (r - l > 1) {
            int m = (l + r) >> 1;
            if ((int64_t)table[T_COLS * m + T_BASE] <= u) l = m; else r = m;
        }
        sc = -2 - l;
    }
    scope[i] = sc;
}

__global__ void k_full_range(int32_t *__restrict__ lo, int32_t *__restrict__ hi, int64_t m) {
    int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < m) { lo[i] = INT32_MIN; hi[i] = INT32_MAX; }
}

// fusion (Section 4.3, Remote Edge Construction): one wavefront per row; proximal and global picks
// from the row's global candidates overwrite the redundant positions, a position without a pick
// keeps its redundant local edge
__global__ __launch_bounds__(64) void k_fuse(const uint32_t *__restrict__ cand_s, const float *__restrict__ cand_d, int32_t beam,
                                             const int32_t *__restrict__ attr, const uint32_t *__restrict__ slot2id,
                                             int64_t first, int64_t count, int32_t kl, int32_t kr, int32_t kp, int64_t window,
                                             uint32_t *__restrict__ A) {
    __shared__ uint32_t pk[64];
    __shared__ float pkd[64];
    const int64_t i = blockIdx.x;
    const int lane = threadIdx.x;
    if (i >= count) return;
    const int64_t u = first + i;
    if (slot2id[u] == GRAB_EMPTY) return;
    select_remote_wave(cand_s + i * beam, cand_d + i * beam, beam, attr, attr[u], window, kp, kr, lane, pk, pkd);
    if (lane < kr && pk[lane] != GRAB_EMPTY) A[u * (kl + kr) + kl + lane] = pk[lane];
}

}  // namespace

grab_status grab_build_remote_device(grab_index *ix, const SearchLaunch &proto) {
    hipStream_t st = ix->stream;
    const int32_t B = ix->B, kl = ix->kl, kr = ix->kr, K = kl + kr;
    const int64_t N = ix->n_slots;
    if (kr == 0) return GRAB_OK;
    std::vector<void *> tmp;
    auto cleanup = [&]() { for (void *p : tmp) (void)hipFree(p); };
    const RemoteRule rule = grab_remote_rule(ix, kr);
    if (rule.mode == 0) {
        // entry j = the nearest object of the j-th target bucket
        int32_t max_n = 0;
        for (int b = 0; b < B; ++b) max_n = ix->h_table[T_COLS * b + T_NTOT] > max_n ? ix->h_table[T_COLS * b + T_NTOT] : max_n;
        const unsigned tiles = (unsigned)((max_n + 31) / 32);
        int32_t *tgt;
        G_ALLOC(tgt, (size_t)B * 4 * kr);
        std::vector<int32_t> h((size_t)B * kr, -1);
        std::vector<int> t(kr);
        for (int b = 0; b < B; ++b) {
            int n = remote_targets(b, B, kr, t.data());
            for (int j = 0; j < n; ++j) h[(size_t)j * B + b] = t[j];
        }
        G_HIP(hipMemcpyAsync(tgt, h.data(), h.size() * 4, hipMemcpyHostToDevice, st));
        G_HIP(hipStreamSynchronize(st));
        KnnArgs k;
        k.X = ix->X; k.table = ix->table; k.n_slots = N; k.metric = ix->metric;
        grab_status rc;
        KnnFilter *flt = nullptr;
        (void)grab_knn_prepare(ix, &flt);   // null: every pair in fp32
        for (int j = 0; j < kr; ++j) {
            k.tgt = tgt + (size_t)j * B; k.out_s = ix->A; k.out_d = nullptr;
            k.out_stride = K; k.out_off = kl + j; k.P = 1; k.exclude_self = 0;
            bool redo = true;
            if (flt && (rc = grab_knn_pass(ix, flt, k.tgt, k.out_s, nullptr, K, kl + j, 1, 0, &redo)) != GRAB_OK) {
                grab_knn_release(flt); cleanup(); return rc;
            }
            if (redo && (rc = launch_graph(ix, &k, nullptr, tiles)) != GRAB_OK) { grab_knn_release(flt); cleanup(); return rc; }
        }
        grab_knn_release(flt);
        G_HIP(hipGetLastError());
        G_HIP(hipStreamSynchronize(st));
        cleanup();
        return GRAB_OK;
    }
    // proximal / global reading: global candidates of every row from the library's own search over
    // a copy of the graph as it is now (so that no search sees a row already rewritten)
    const int64_t chunk = N < (1ll << 20) ? N : (1ll << 20);
    const int32_t beam = proto.beam;
    uint32_t *snap, *cand_s, *seeds, *counters;
    float *cand_d;
    int32_t *scope, *lo, *hi;
    QueryPlan *plans;
    G_ALLOC(snap, (size_t)N * K * 4);
    G_ALLOC(cand_s, (size_t)chunk * beam * 4); G_ALLOC(cand_d, (size_t)chunk * beam * 4);
    G_ALLOC(scope, (size_t)chunk * 4); G_ALLOC(lo, (size_t)chunk * 4); G_ALLOC(hi, (size_t)chunk * 4);
    G_ALLOC(plans, (size_t)chunk * sizeof(QueryPlan));
    G_ALLOC(seeds, (size_t)chunk * proto.n_seeds * 4);
    G_ALLOC(counters, (size_t)chunk * 8 * 4);
    G_HIP(hipMemcpyAsync(snap, ix->A, (size_t)N * K * 4, hipMemcpyDeviceToDevice, st));
    k_full_range<<<blocks_for(chunk), TPB, 0, st>>>(lo, hi, chunk);
    grab_status rc;
    for (int64_t first = 0; first < N; first += chunk) {
        const int64_t count = N - first < chunk ? N - first : chunk;
        k_scope_rows<<<blocks_for(count), TPB, 0, st>>>(ix->table, B, ix->slot2id, first, count, scope);
        SearchLaunch s = proto;
        s.queries = ix->X + (size_t)first * ix->dim; s.lo = lo; s.hi = hi; s.only_bucket = scope; s.adj = snap; s.nq = count;
        s.plans = plans; s.seeds = seeds; s.counters = counters; s.out_ids = cand_s; s.out_dist = cand_d; s.out_slots = true;
        if ((rc = grab_plan_order(ix, s)) != GRAB_OK) { cleanup(); return rc; }
        if ((rc = grab_launch_select(ix, s)) != GRAB_OK) { cleanup(); return rc; }
        if ((rc = grab_launch_beam(ix, s)) != GRAB_OK) { cleanup(); return rc; }
        k_fuse<<<dim3((unsigned)count), dim3(64), 0, st>>>(cand_s, cand_d, beam, ix->attr, ix->slot2id, first, count, kl, kr,
                                                           rule.n_proximal, rule.window, ix->A);
        G_HIP(hipGetLastError());
    }
    ix->last_nq = 0;
    G_HIP(hipStreamSynchronize(st));
#undef G_ALLOC
#undef G_HIP
    cleanup();
    return GRAB_OK;
}
