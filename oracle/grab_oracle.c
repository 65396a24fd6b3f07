/*
 * CPU oracle for range-filtered beam search and batched append over a bucketed graph
 * index (GRAB-ANNS, Sections 4.2, 4.4, 4.5; Algorithm 2; Eq. 2 and Eq. 3).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, scalar implementation that follows
 * the algorithm's steps in the paper's order.  Only tests, the smoke check and the CPU
 * baseline leg of the benchmark may call it; the product library shares no code with it.
 *
 * What the paper fixes and what this file pins by its own reading:
 *   - bucket selection by interval intersection, seeds drawn only from intersecting
 *     buckets, scalar pre-check before any distance, queue update, top-k (Algorithm 2);
 *   - the seed sampler, the convergence test, the visited-set capacity rule, the
 *     (distance, slot) tie-break and the fp32 summation order are not given by the paper;
 *     they are stated where they are implemented below ("reading:").
 *
 * Index arrays are in *slot* space (bucket-major physical rows):
 *   X[n_cap][dim] fp32, attr[n_cap] int32, A[n_cap][K] uint32 slots (0xFFFFFFFF = empty),
 *   slot2id[n_cap], table[B][6] = {base, n_sorted, n_total, cap, min_attr, max_attr}.
 * Slots [base, base+n_sorted) of a bucket hold attributes in non-decreasing order; slots
 * [base+n_sorted, base+n_total) are appended later in arrival order (unsorted tail).
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math: the fp32
 * reduction order below is part of the contract).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define EMPTY 0xFFFFFFFFu
#define T_BASE 0
#define T_NSORT 1
#define T_NTOT 2
#define T_CAP 3
#define T_MIN 4
#define T_MAX 5

typedef struct {
    int32_t dim;
    int32_t metric;      /* 0: squared L2, 1: negated inner product */
    int32_t k_local;
    int32_t k_remote;
    int32_t n_buckets;
    int32_t pad_;
    int64_t n_cap;
    float *X;
    int32_t *attr;
    uint32_t *A;
    uint32_t *slot2id;
    int32_t *table;
} oracle_index;

typedef struct {
    int32_t search_width; /* parents expanded per iteration                    */
    int32_t max_iter;     /* hard cap on iterations                            */
    int32_t n_seeds;      /* S                                                 */
    int32_t visited_cap;  /* search stops before the visited set could pass it */
    uint32_t seed_salt;
} oracle_params;

/* ------------------------------------------------------------------ distance (A6)
 * Algorithm 2 line "ComputeDistance"; Table 2 names Euclidean.  Returned value is the
 * squared L2 distance (ranking-equivalent) or minus the inner product.
 * reading: fp32 with a fixed summation tree, so that any other fp32 implementation can
 * reproduce the bits: eight partial sums; partial l takes elements 4*(8c+l)..+3 for
 * c = 0,1,... in index order, each step one fused multiply-add; the partials are then
 * combined pairwise ((p0+p1)+(p2+p3))+((p4+p5)+(p6+p7)).  dim must be a multiple of 32. */
float oracle_distance(const float *q, const float *v, int32_t dim, int32_t metric) {
    float p[8];
    for (int l = 0; l < 8; ++l) p[l] = 0.0f;
    for (int c = 0; c < dim / 32; ++c)
        for (int l = 0; l < 8; ++l)
            for (int e = 0; e < 4; ++e) {
                int j = 4 * (8 * c + l) + e;
                if (metric == 0) {
                    float x = q[j] - v[j];
                    p[l] = fmaf(x, x, p[l]);
                } else {
                    p[l] = fmaf(q[j], v[j], p[l]);
                }
            }
    float s01 = p[0] + p[1], s23 = p[2] + p[3], s45 = p[4] + p[5], s67 = p[6] + p[7];
    float s = (s01 + s23) + (s45 + s67);
    return metric == 0 ? s : -s;
}

/* order-preserving image of an fp32 value in uint32 (smaller float <=> smaller image) */
static uint32_t dist_image(float d) {
    uint32_t b;
    memcpy(&b, &d, 4);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

/* ------------------------------------------------------------- bucket select (A2)
 * Algorithm 2 line 1 (GetIntersectingBuckets): the buckets whose closed attribute
 * interval [min,max] meets [lo,hi].  Bucket intervals are ordered, so the answer is a
 * run b0..b1.  Returns 0 when empty. */
static int select_buckets(const oracle_index *ix, int32_t lo, int32_t hi, int *b0, int *b1) {
    *b0 = 0;
    *b1 = -1;
    if (lo > hi) return 0;
    int first = -1, last = -1;
    for (int b = 0; b < ix->n_buckets; ++b) {
        const int32_t *t = ix->table + 6 * b;
        if (t[T_MAX] >= lo && t[T_MIN] <= hi) {
            if (first < 0) first = b;
            last = b;
        }
    }
    if (first < 0) return 0;
    *b0 = first;
    *b1 = last;
    return 1;
}

/* valid part [*a,*e) of a bucket's sorted prefix, as offsets inside the prefix */
static void sorted_span(const oracle_index *ix, int b, int32_t lo, int32_t hi, int64_t *a, int64_t *e) {
    const int32_t *t = ix->table + 6 * b;
    const int32_t *s = ix->attr + t[T_BASE];
    int64_t n = t[T_NSORT], l, r;
    l = 0; r = n;                        /* lower bound: first attr >= lo */
    while (l < r) { int64_t m = (l + r) / 2; if (s[m] < lo) l = m + 1; else r = m; }
    *a = l;
    l = 0; r = n;                        /* upper bound: first attr > hi */
    while (l < r) { int64_t m = (l + r) / 2; if (s[m] <= hi) l = m + 1; else r = m; }
    *e = l < *a ? *a : l;
}

static int bucket_of_slot(const oracle_index *ix, uint32_t slot) {
    for (int b = 0; b < ix->n_buckets; ++b) {
        const int32_t *t = ix->table + 6 * b;
        if ((int64_t)slot >= t[T_BASE] && (int64_t)slot < (int64_t)t[T_BASE] + t[T_CAP]) return b;
    }
    return -1;
}

/* 32-bit integer finaliser (the public-domain MurmurHash3 one) used to jitter seeds */
static uint32_t mix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x85ebca6bu;
    x ^= x >> 13;
    x *= 0xc2b2ae35u;
    x ^= x >> 16;
    return x;
}

/* ---------------------------------------------------------------- seeding (A3)
 * Algorithm 2 line 2 (SampleSeedsFrom(B_valid)).
 * reading: the seed population P is, over the selected buckets in order, the valid part
 * of the sorted prefix followed by the whole appended tail; V = |P|.  If V <= S every
 * member is a seed.  Otherwise seed j is P[floor(j*V/S) + mix32(j ^ salt) mod floor(V/S)]:
 * one seed per stratum with an integer jitter.  `only_bucket` >= 0 restricts P to that
 * bucket's whole slab contents (used by append).
 * Writes seed slots to seeds[0..S) (EMPTY-padded); returns the count; *V_out = V;
 * span[0] = first valid sorted slot of b0, span[1] = end of valid sorted slots of b1. */
static int64_t population_member(const oracle_index *ix, int b0, int b1, const int64_t *sa,
                                 const int64_t *se, int64_t i) {
    for (int b = b0; b <= b1; ++b) {
        const int32_t *t = ix->table + 6 * b;
        int64_t ns = se[b - b0] - sa[b - b0];
        if (i < ns) return t[T_BASE] + sa[b - b0] + i;
        i -= ns;
        int64_t nt = t[T_NTOT] - t[T_NSORT];
        if (i < nt) return (int64_t)t[T_BASE] + t[T_NSORT] + i;
        i -= nt;
    }
    return -1;
}

static int64_t make_seeds(const oracle_index *ix, int32_t lo, int32_t hi, int only_bucket,
                          const oracle_params *pr, uint32_t *seeds, int64_t *V_out,
                          int *b0_out, int *b1_out, int64_t span[2]) {
    int b0, b1;
    int64_t S = pr->n_seeds;
    for (int64_t j = 0; j < S; ++j) seeds[j] = EMPTY;
    *V_out = 0;
    span[0] = span[1] = 0;
    if (only_bucket >= 0) {
        b0 = b1 = only_bucket;
    } else if (!select_buckets(ix, lo, hi, &b0, &b1)) {
        *b0_out = 0;
        *b1_out = -1;
        return 0;
    }
    *b0_out = b0;
    *b1_out = b1;
    int nb = b1 - b0 + 1;
    int64_t *sa = (int64_t *)malloc(sizeof(int64_t) * nb), *se = (int64_t *)malloc(sizeof(int64_t) * nb);
    int64_t V = 0;
    for (int b = b0; b <= b1; ++b) {
        const int32_t *t = ix->table + 6 * b;
        if (only_bucket >= 0) {
            sa[b - b0] = 0;
            se[b - b0] = t[T_NSORT];
        } else {
            sorted_span(ix, b, lo, hi, &sa[b - b0], &se[b - b0]);
        }
        V += (se[b - b0] - sa[b - b0]) + (t[T_NTOT] - t[T_NSORT]);
    }
    span[0] = ix->table[6 * b0 + T_BASE] + sa[0];
    span[1] = ix->table[6 * b1 + T_BASE] + se[nb - 1];
    *V_out = V;
    int64_t count = 0;
    if (V <= S) {
        for (int64_t i = 0; i < V; ++i) seeds[count++] = (uint32_t)population_member(ix, b0, b1, sa, se, i);
    } else {
        uint64_t stride = (uint64_t)(V / S);
        for (int64_t j = 0; j < S; ++j) {
            uint64_t pos = ((uint64_t)j * (uint64_t)V) / (uint64_t)S + (uint64_t)mix32((uint32_t)j ^ pr->seed_salt) % stride;
            seeds[count++] = (uint32_t)population_member(ix, b0, b1, sa, se, (int64_t)pos);
        }
    }
    free(sa);
    free(se);
    return count;
}

/* debug/parity view of selection and seeding for one query:
 * info = {b0, b1, V, first valid sorted slot in b0, end valid sorted slot in b1, n_seeds} */
void oracle_select(const oracle_index *ix, const oracle_params *pr, int32_t lo, int32_t hi,
                   int64_t info[6], uint32_t *seeds) {
    int b0, b1;
    int64_t V, span[2];
    int64_t c = make_seeds(ix, lo, hi, -1, pr, seeds, &V, &b0, &b1, span);
    info[0] = b0; info[1] = b1; info[2] = V; info[3] = span[0]; info[4] = span[1]; info[5] = c;
}

/* ------------------------------------------------------------------ search (A4-A7) */
typedef struct {
    uint32_t img;   /* dist_image(dist) */
    uint32_t slot;
    float dist;
    int expanded;
} entry;

static int entry_cmp(const void *a, const void *b) {
    const entry *x = (const entry *)a, *y = (const entry *)b;
    if (x->img != y->img) return x->img < y->img ? -1 : 1;
    if (x->slot != y->slot) return x->slot < y->slot ? -1 : 1;
    return 0;
}

typedef struct {
    uint8_t *seen;      /* one byte per slot: the exact visited set */
    uint32_t *touched;  /* slots to clear afterwards */
    int64_t n_touched;
    entry *Q;           /* beam + scratch */
    uint32_t *seeds;
    int64_t cap_touched, cap_Q, cap_seeds;
} scratch;

static scratch *scratch_new(int64_t n_cap) {
    scratch *s = (scratch *)calloc(1, sizeof(scratch));
    s->seen = (uint8_t *)calloc((size_t)n_cap, 1);
    return s;
}
static void scratch_free(scratch *s) {
    free(s->seen); free(s->touched); free(s->Q); free(s->seeds); free(s);
}
static void scratch_fit(scratch *s, int64_t touched, int64_t q, int64_t seeds) {
    if (touched > s->cap_touched) { s->touched = (uint32_t *)realloc(s->touched, 4 * (size_t)touched); s->cap_touched = touched; }
    if (q > s->cap_Q) { s->Q = (entry *)realloc(s->Q, sizeof(entry) * (size_t)q); s->cap_Q = q; }
    if (seeds > s->cap_seeds) { s->seeds = (uint32_t *)realloc(s->seeds, 4 * (size_t)seeds); s->cap_seeds = seeds; }
}

/* counters per query: 0 iterations, 1 parents expanded, 2 distance evaluations (seeds
 * included), 3 seed evaluations, 4 neighbours rejected by the pre-check, 5 slots (seeds and
 * neighbours) lying in the appended tail of bucket b0 or b1, 6 visited-set size at the
 * end, 7 stop reason (0 no unexpanded entry, 1 max_iter, 2 visited capacity, 3 empty range) */
enum { C_ITERS, C_PARENTS, C_EVALS, C_SEED_EVALS, C_REJECTS, C_TAIL, C_VISITED, C_STOP };

static int in_edge_tail(const oracle_index *ix, int b0, int b1, uint32_t v) {
    for (int pass = 0; pass < 2; ++pass) {
        int b = pass == 0 ? b0 : b1;
        if (pass == 1 && b1 == b0) break;
        const int32_t *t = ix->table + 6 * b;
        if ((int64_t)v >= (int64_t)t[T_BASE] + t[T_NSORT] && (int64_t)v < (int64_t)t[T_BASE] + t[T_NTOT]) return 1;
    }
    return 0;
}

/* One query.  Algorithm 2 with these readings of what it leaves open:
 *  - seeds pass the same scalar pre-check as any candidate (only tail seeds can fail);
 *  - PopUnvisited takes the first `search_width` entries of the sorted queue not yet expanded;
 *  - "converged" = no unexpanded entry, or max_iter iterations, or the next iteration
 *    could push the visited set past visited_cap (checked before expanding);
 *  - a neighbour is pre-checked first, then looked up in the visited set, then evaluated;
 *    rejected neighbours are not recorded as visited;
 *  - the queue keeps the best `beam` entries ordered by (distance, slot).
 * `only_bucket` >= 0 (append's local candidate search) replaces the attribute test by
 * "slot lies in that bucket's slab".  Leaves the final queue in sc->Q, returns its length. */
static int64_t search_one(const oracle_index *ix, const oracle_params *pr, const float *q,
                          int32_t lo, int32_t hi, int only_bucket, int32_t beam, scratch *sc,
                          uint32_t *ctr) {
    const int K = ix->k_local + ix->k_remote;
    const int w = pr->search_width;
    int b0, b1;
    int64_t V, span[2];
    uint32_t c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    scratch_fit(sc, (int64_t)pr->visited_cap + 1, (int64_t)beam + (int64_t)w * K + pr->n_seeds, pr->n_seeds);
    int64_t ns = make_seeds(ix, lo, hi, only_bucket, pr, sc->seeds, &V, &b0, &b1, span);
    entry *Q = sc->Q;
    int64_t nQ = 0;
    sc->n_touched = 0;
    if (b1 < b0) c[C_STOP] = 3;
    for (int64_t j = 0; j < ns; ++j) {
        uint32_t v = sc->seeds[j];
        if (only_bucket < 0) {
            if (in_edge_tail(ix, b0, b1, v)) c[C_TAIL]++;
            if (ix->attr[v] < lo || ix->attr[v] > hi) continue;
        }
        sc->seen[v] = 1;
        sc->touched[sc->n_touched++] = v;
        float d = oracle_distance(q, ix->X + (size_t)v * ix->dim, ix->dim, ix->metric);
        Q[nQ].img = dist_image(d); Q[nQ].slot = v; Q[nQ].dist = d; Q[nQ].expanded = 0;
        nQ++;
        c[C_EVALS]++;
        c[C_SEED_EVALS]++;
    }
    qsort(Q, (size_t)nQ, sizeof(entry), entry_cmp);
    if (nQ > beam) nQ = beam;

    int iter = 0;
    while (c[C_STOP] == 0) {
        if (iter == pr->max_iter) { c[C_STOP] = 1; break; }
        int parents[64], np = 0;
        for (int64_t i = 0; i < nQ && np < w; ++i)
            if (!Q[i].expanded) parents[np++] = (int)i;
        if (np == 0) break;
        if (sc->n_touched + (int64_t)np * K > pr->visited_cap) { c[C_STOP] = 2; break; }
        uint32_t pslot[64];
        for (int i = 0; i < np; ++i) { Q[parents[i]].expanded = 1; pslot[i] = Q[parents[i]].slot; }
        iter++;
        c[C_PARENTS] += np;
        int64_t nC = nQ;   /* new candidates are appended after the current queue */
        for (int i = 0; i < np; ++i)
            for (int j = 0; j < K; ++j) {
                uint32_t v = ix->A[(size_t)pslot[i] * K + j];
                if (v == EMPTY) continue;
                if (only_bucket >= 0) {
                    if (bucket_of_slot(ix, v) != only_bucket) { c[C_REJECTS]++; continue; }
                } else {
                    if (in_edge_tail(ix, b0, b1, v)) c[C_TAIL]++;
                    if (ix->attr[v] < lo || ix->attr[v] > hi) { c[C_REJECTS]++; continue; }
                }
                if (sc->seen[v]) continue;
                sc->seen[v] = 1;
                sc->touched[sc->n_touched++] = v;
                float d = oracle_distance(q, ix->X + (size_t)v * ix->dim, ix->dim, ix->metric);
                Q[nC].img = dist_image(d); Q[nC].slot = v; Q[nC].dist = d; Q[nC].expanded = 0;
                nC++;
                c[C_EVALS]++;
            }
        qsort(Q, (size_t)nC, sizeof(entry), entry_cmp);
        nQ = nC < beam ? nC : beam;
    }
    c[C_ITERS] = (uint32_t)iter;
    c[C_VISITED] = (uint32_t)sc->n_touched;
    for (int64_t i = 0; i < sc->n_touched; ++i) sc->seen[sc->touched[i]] = 0;
    if (ctr) memcpy(ctr, c, sizeof(c));
    return nQ;
}

/* Batched search.  Results per query: first k queue entries as (external id, distance),
 * ascending by (distance, slot); missing entries are (0xFFFFFFFF, +inf).  out_slots may be
 * NULL.  Queries are independent; `threads` > 1 runs them under OpenMP, one per thread. */
int oracle_search(const oracle_index *ix, const oracle_params *pr, const float *queries,
                  const int32_t *lo, const int32_t *hi, int64_t nq, int32_t k, int32_t beam,
                  uint32_t *out_ids, float *out_dist, uint32_t *counters, int32_t threads) {
    if (ix->dim % 32 != 0 || k < 1 || k > beam || pr->search_width < 1 || pr->search_width > 64 ||
        pr->n_seeds < 1 || pr->n_seeds > pr->visited_cap) return 1;
#ifdef _OPENMP
    if (threads < 1) threads = 1;
#pragma omp parallel num_threads(threads)
#endif
    {
        scratch *sc = scratch_new(ix->n_cap);
#ifdef _OPENMP
#pragma omp for schedule(static)
#endif
        for (int64_t qi = 0; qi < nq; ++qi) {
            int64_t nQ = search_one(ix, pr, queries + (size_t)qi * ix->dim, lo[qi], hi[qi], -1, beam, sc,
                                    counters ? counters + 8 * qi : NULL);
            for (int j = 0; j < k; ++j) {
                if (j < nQ) {
                    out_ids[qi * k + j] = ix->slot2id[sc->Q[j].slot];
                    out_dist[qi * k + j] = sc->Q[j].dist;
                } else {
                    out_ids[qi * k + j] = EMPTY;
                    out_dist[qi * k + j] = INFINITY;
                }
            }
        }
        scratch_free(sc);
    }
    return 0;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
