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

uint32_t oracle_mix32(uint32_t x) { return mix32(x); }   /* for the test that pins it on published values */

/* ---------------------------------------------------------------- seeding (A3)
 * Algorithm 2 line 2 (SampleSeedsFrom(B_valid)).
 * reading: the seed population P is, over the selected buckets in order, the valid part
 * of the sorted prefix followed by the whole appended tail; V = |P|.  If V <= S every
 * member is a seed.  Otherwise seed j is P[floor(j*V/S) + mix32(j ^ salt) mod floor(V/S)]:
 * one seed per stratum with an integer jitter.  `scope` (see search_one) >= 0 restricts P to that
 * bucket's whole contents; scope <= -2 makes P the whole contents of every bucket but one, in
 * bucket order (both used by append and by the construction's second pass).
 * Writes seed slots to seeds[0..S) (EMPTY-padded); returns the count; *V_out = V;
 * span[0] = first valid sorted slot of b0, span[1] = end of valid sorted slots of b1. */
static int64_t population_member(const oracle_index *ix, int b0, int b1, int skip, const int64_t *sa,
                                 const int64_t *se, int64_t i) {
    for (int b = b0; b <= b1; ++b) {
        if (b == skip) continue;
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

static int64_t make_seeds(const oracle_index *ix, int32_t lo, int32_t hi, int scope,
                          const oracle_params *pr, uint32_t *seeds, int64_t *V_out,
                          int *b0_out, int *b1_out, int64_t span[2]) {
    int b0, b1;
    int64_t S = pr->n_seeds;
    for (int64_t j = 0; j < S; ++j) seeds[j] = EMPTY;
    *V_out = 0;
    span[0] = span[1] = 0;
    const int skip = scope <= -2 ? -2 - scope : -1;
    if (scope >= 0) {
        b0 = b1 = scope;
    } else if (skip >= 0) {
        b0 = 0;
        b1 = ix->n_buckets - 1;
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
        if (scope >= 0 || skip >= 0) {
            sa[b - b0] = 0;
            se[b - b0] = t[T_NSORT];
        } else {
            sorted_span(ix, b, lo, hi, &sa[b - b0], &se[b - b0]);
        }
        if (b != skip) V += (se[b - b0] - sa[b - b0]) + (t[T_NTOT] - t[T_NSORT]);
    }
    span[0] = ix->table[6 * b0 + T_BASE] + sa[0];
    span[1] = ix->table[6 * b1 + T_BASE] + se[nb - 1];
    *V_out = V;
    if (V == 0 && skip >= 0) {   /* nothing outside the only bucket: an empty selection */
        *b0_out = 0;
        *b1_out = -1;
        free(sa);
        free(se);
        return 0;
    }
    int64_t count = 0;
    if (V <= S) {
        for (int64_t i = 0; i < V; ++i) seeds[count++] = (uint32_t)population_member(ix, b0, b1, skip, sa, se, i);
    } else {
        uint64_t stride = (uint64_t)(V / S);
        for (int64_t j = 0; j < S; ++j) {
            uint64_t pos = ((uint64_t)j * (uint64_t)V) / (uint64_t)S + (uint64_t)mix32((uint32_t)j ^ pr->seed_salt) % stride;
            seeds[count++] = (uint32_t)population_member(ix, b0, b1, skip, sa, se, (int64_t)pos);
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
 * `scope` is the scope of the search: -1 = the attribute range [lo,hi]; b >= 0 (the local
 * candidate search of an insertion) replaces the attribute test by "slot lies in bucket b's
 * slab"; -2 - b (the global-scope candidate search) by "slot lies outside bucket b's slab".
 * Leaves the final queue in sc->Q, returns its length. */
static int64_t search_one(const oracle_index *ix, const oracle_params *pr, const float *q,
                          int32_t lo, int32_t hi, int scope, int32_t beam, scratch *sc,
                          uint32_t *ctr) {
    const int K = ix->k_local + ix->k_remote;
    const int w = pr->search_width;
    int b0, b1;
    int64_t V, span[2];
    uint32_t c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    scratch_fit(sc, (int64_t)pr->visited_cap + 1, (int64_t)beam + (int64_t)w * K + pr->n_seeds, pr->n_seeds);
    int64_t ns = make_seeds(ix, lo, hi, scope, pr, sc->seeds, &V, &b0, &b1, span);
    entry *Q = sc->Q;
    int64_t nQ = 0;
    sc->n_touched = 0;
    if (b1 < b0) c[C_STOP] = 3;
    for (int64_t j = 0; j < ns; ++j) {
        uint32_t v = sc->seeds[j];
        if (scope == -1) {
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
                if (scope >= 0) {
                    if (bucket_of_slot(ix, v) != scope) { c[C_REJECTS]++; continue; }
                } else if (scope <= -2) {
                    if (bucket_of_slot(ix, v) == -2 - scope) { c[C_REJECTS]++; continue; }
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

/* The candidate searches of insertion and construction, exposed for tests: query i runs with
 * scope[i] (see search_one) and leaves its whole final queue, `beam` entries as slots and
 * distances ordered by (distance, slot), padded with (0xFFFFFFFF, +inf). */
int oracle_search_scoped(const oracle_index *ix, const oracle_params *pr, const float *queries, const int32_t *scope,
                         int64_t nq, int32_t beam, uint32_t *out_slots, float *out_dist) {
    scratch *sc = scratch_new(ix->n_cap);
    for (int64_t qi = 0; qi < nq; ++qi) {
        int64_t nQ = search_one(ix, pr, queries + (size_t)qi * ix->dim, 0, 0, scope[qi], beam, sc, NULL);
        for (int j = 0; j < beam; ++j) {
            out_slots[qi * beam + j] = j < nQ ? sc->Q[j].slot : EMPTY;
            out_dist[qi * beam + j] = j < nQ ? sc->Q[j].dist : INFINITY;
        }
    }
    scratch_free(sc);
    return 0;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ============================================================== batched append (Section 4.4)
 * The paper gives the stages (append at the tail, logical assignment, candidate search in the
 * target bucket and globally, forward selection by heuristic pruning, reverse rewiring from a
 * request buffer) and two rules (Eq. 2 diversity, Eq. 3 freshness bias).  It gives no candidate
 * counts, no eviction choice and no order for conflicting updates, and it claims slots with
 * an atomic counter whose order is not reproducible.  reading (normative for this build):
 *
 *  0. Snapshot: every decision below about existing nodes uses the index as it was before
 *     the batch; new nodes are not candidates for each other.
 *  1. Bucket of a new attribute x: the buckets with min <= x <= max form a run [e0,e1]; take
 *     e0 + (external id mod run length).  If the run is empty take the first bucket with
 *     max >= x (the last bucket if none); its interval is widened after the batch.
 *  2. Slot: base + n_total + (number of earlier batch items sent to the same bucket), i.e. a
 *     stable counting sort in batch order.  If any bucket would pass its capacity the call
 *     fails (status 3) and nothing is written.  External id = n_prev + position in the batch.
 *     Existing slots never move.
 *  3. Local candidates: one run of the search above with the new vector as query, restricted to
 *     the target bucket's slab, beam = append_beam.  The whole final queue is the candidate
 *     list, ordered by (distance, slot).
 *  4. Forward selection.  Local part (Eq. 2): scan the list in order; keep c iff
 *     dist(q,c) < dist(c,n) for every n kept so far; stop when K_local are kept; then back-fill
 *     with the earliest rejected candidates; still short -> empty entries.  Remote part: entry j
 *     is the nearest to q (ties: smaller slot) among the j-th remote entries of the local
 *     candidates, empty if they have none.  In a graph built by the two-pass construction the
 *     j-th remote entry of every node of a bucket points into the same target bucket, so the new
 *     row keeps that structure: it is the online form of the remote wiring (Section 4.3 pass 2,
 *     "proximal" and "global" remote edges), found through graph locality instead of a scan.
 *     `remote_cands` > 0 looks at the remote entries of the nearest remote_cands candidates only
 *     (the nearest candidates' remote neighbours are the ones near q; 0 = all candidates).
 *     (Section 4.4 has the candidate search also look outside the target bucket; nearest-anywhere candidates
 *     gave new nodes remote edges into arbitrary far buckets, which a range filter rejects, and
 *     recall of the dynamic workload decayed with every batch.)
 *  5. Reverse requests: one per written edge q->v: (v, kind, dist(v,q), q).  Sorted by
 *     (v, kind, distance image, q's slot) and applied one after another per target.  With
 *     a = alpha squared (distances here are squared, so that the test is the paper's on true
 *     Euclidean distances):
 *     local kind, R = local part of v's row:
 *       pass  = a*dist(v,q) < dist(q,n) for every n in R           (Eq. 2 with Eq. 3's d_eff)
 *       if !pass: drop.  Else if R has an empty entry: fill the first one.  Else, among the
 *       entries of R that q itself points to (anywhere in q's new row), the one farthest from v
 *       (ties: smaller slot) is overwritten; if there is none the request is dropped.  The
 *       overwritten neighbour n stays reachable from v through q, so no pathway is lost
 *       (Section 4.4, topology maintenance), and no node can lose its last in-edge: an edge x->n
 *       only disappears while q->n exists.  Among the pathways q covers, the longest edge of v is
 *       the one v needs least.  Rules tried first: evicting the farthest neighbour of all keeps
 *       only the closest ones, which the paper warns turns the graph into isolated cliques (on
 *       clustered data it removed exactly the long links and left thousands of strongly
 *       connected components); evicting the covered neighbour nearest to q kept the graph
 *       connected but rewrote half of every old row with near-duplicates of its short edges
 *       (Recall@10 0.82 after doubling a 1M index against 0.91 with the rule above and 0.93 for
 *       a bulk rebuild).
 *     remote kind, R = remote part of v's row: among the entries of R that lie in q's bucket take
 *       the one farthest from v (ties: larger slot) and overwrite it iff a*dist(v,q) < its
 *       distance to v: the entry for that bucket keeps pointing at (about) the nearest node of
 *       the bucket, with the fresh node favoured by the bias.  If no entry lies in q's bucket, q
 *       fills the first empty entry, if any.
 *     Fresh nodes already placed in R by this batch count as ordinary neighbours.
 *  6. Table: n_total grows by the bucket's batch count; min/max absorb the new attributes.
 *
 * Steps 3-5 above wire the remote part by target bucket (remote_rule.mode 0).  The paper's own wording
 * is the second reading kept here (remote_rule.mode 1; Section 4.4 "Parallel Candidate Search": candidates
 * from the target bucket and from the global scope; Section 4.3 "Remote Edge Construction": the
 * remote budget split into proximal and global candidates, redundant local edges kept where too
 * few qualify).  It differs in the remote part only:
 *  3'. A second run of the search with the new vector as query and the scope "every slot outside
 *      the target bucket's slab" (same parameters, beam = append_beam): the global candidates,
 *      ordered by (distance, slot).
 *  4'. Remote part: scan the global candidates in order.  A candidate whose attribute differs from
 *      the new object's by at most `window` is proximal, any other one global.  The first
 *      n_proximal proximal ones fill remote positions 0.., the first K_remote - n_proximal global
 *      ones the positions n_proximal..; no diversity test (Section 4.3 filters and ranks).  A
 *      position left without a pick takes the nearest local candidate not yet in the row (the
 *      redundant local edge that Section 4.3 keeps rather than leave an entry empty), else stays
 *      empty.  Only picks that leave the bucket make a reverse request.
 *  5'. Remote request at v: q is proximal to v iff |attr(q) - attr(v)| <= window, and competes
 *      for the remote positions of its class only.  It takes the first of them that is empty or
 *      holds a node of v's own bucket (a redundant local edge is there to be overwritten by a
 *      remote one); if there is none, the entry of these positions farthest from v (ties: larger
 *      slot) gives way iff a*dist(v,q) < its distance to v: each class keeps the nearest nodes it
 *      has seen, the fresh one favoured by the bias (Eq. 3).
 *
 * Inner-product metric: Eq. 3 scales a distance, and minus the inner product is not one (it is
 * negative for similar vectors, so scaling it by alpha < 1 would push a newcomer away).  Both
 * sides of every biased comparison are therefore shifted first: s(d) = max(0, 1 + d), which for
 * unit vectors is half the squared Euclidean distance, and the bias acts as alpha^2 on it, as on
 * squared Euclidean distances.  The comparison "a*dist(x) < dist(y)" reads a*s(dist(x)) < s(dist(y)).
 */
typedef struct {
    int32_t mode;        /* 0: remote entry j belongs to the j-th target bucket; 1: proximal / global split */
    int32_t n_proximal;  /* mode 1: remote positions reserved for proximal candidates (0..K_remote) */
    int64_t window;      /* mode 1: largest attribute difference of a proximal candidate */
} remote_rule;

/* the quantity the freshness bias scales (see above): the distance itself for squared L2 */
static float bias_base(const oracle_index *ix, float d) {
    if (ix->metric == 0) return d;
    float s = 1.0f + d;
    return s > 0.0f ? s : 0.0f;
}

/* Section 4.3, remote edge selection over candidates ordered by (distance, slot): picks[0..kp) the
 * nearest proximal ones, picks[kp..kr) the nearest global ones, EMPTY where the class runs out */
static void select_remote(const oracle_index *ix, int32_t attr_u, const uint32_t *gs, const float *gd, int ng,
                          const remote_rule *rr, uint32_t *picks, float *pickd) {
    const int kr = ix->k_remote, kp = rr->n_proximal;
    int np = 0, ngl = 0;
    for (int j = 0; j < kr; ++j) { picks[j] = EMPTY; pickd[j] = 0.0f; }
    for (int t = 0; t < ng; ++t) {
        int64_t diff = (int64_t)ix->attr[gs[t]] - (int64_t)attr_u;
        if (diff < 0) diff = -diff;
        if (diff <= rr->window) {
            if (np < kp) { picks[np] = gs[t]; pickd[np] = gd[t]; np++; }
        } else if (ngl < kr - kp) {
            picks[kp + ngl] = gs[t]; pickd[kp + ngl] = gd[t]; ngl++;
        }
    }
}

typedef struct {
    uint32_t v;      /* target (existing node) slot */
    uint32_t kind;   /* 0 local, 1 remote */
    uint32_t img;    /* dist_image(dist(v,q)) */
    uint32_t q;      /* new node slot */
    float dist;
} request;

static int request_cmp(const void *a, const void *b) {
    const request *x = (const request *)a, *y = (const request *)b;
    if (x->v != y->v) return x->v < y->v ? -1 : 1;
    if (x->kind != y->kind) return x->kind < y->kind ? -1 : 1;
    if (x->img != y->img) return x->img < y->img ? -1 : 1;
    if (x->q != y->q) return x->q < y->q ? -1 : 1;
    return 0;
}

/* Eq. 2 scan over `nc` ordered candidates (slot, dist to q); writes up to `cap` slots to row,
 * returns how many were kept by the rule (the rest of the row is back-fill, then EMPTY) */
static int forward_select(const oracle_index *ix, const uint32_t *cs, const float *cd, int nc, int cap,
                          uint32_t *row, uint64_t *scanned) {
    int kept = 0, nrej = 0;
    uint32_t *rej = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(nc > 0 ? nc : 1));
    for (int t = 0; t < nc && kept < cap; ++t) {
        int ok = 1;
        ++*scanned;
        for (int j = 0; j < kept && ok; ++j) {
            float dcn = oracle_distance(ix->X + (size_t)cs[t] * ix->dim, ix->X + (size_t)row[j] * ix->dim, ix->dim, ix->metric);
            if (!(cd[t] < dcn)) ok = 0;
        }
        if (ok) row[kept++] = cs[t]; else rej[nrej++] = cs[t];
    }
    int fill = kept;
    for (int j = 0; j < nrej && fill < cap; ++j) row[fill++] = rej[j];
    for (; fill < cap; ++fill) row[fill] = EMPTY;
    free(rej);
    return kept;
}

/* stats (may be NULL) receives the work counters of the call: 0 requests made for local edges,
 * 1 for remote edges, 2 (target, kind) groups for local parts, 3 for remote parts, 4 requests that
 * rewrote an entry, local, 5 remote, 6 candidates examined by the Eq. 2 scans, 7 rows evaluated
 * for the remote parts of new rows (mode 0), 8 local requests that passed the biased test,
 * 9 distance evaluations and 10 expanded parents of the candidate searches, 11 unused.
 * Returns 0, or 3 when a bucket is out of tail room (nothing written).  `pr` holds the search
 * parameters already resolved for beam = append_beam.  id2slot has room for n_prev + m entries.
 * kept_out (may be NULL): per new node {entries kept by Eq. 2 in the local part, in the remote part}. */
int oracle_append(oracle_index *ix, const oracle_params *pr, float alpha, int32_t append_beam,
                  const float *vecs, const int32_t *attrs, int64_t m, int64_t n_prev, uint32_t *id2slot,
                  int32_t *kept_out, int32_t threads, const remote_rule *rr, uint64_t *stats, int32_t remote_cands) {
    const int B = ix->n_buckets, kl = ix->k_local, kr = ix->k_remote, K = kl + kr, dim = ix->dim;
    const int mode = rr ? rr->mode : 0;
    if (mode != 0 && (mode != 1 || rr->n_proximal < 0 || rr->n_proximal > kr || rr->window < 0)) return 1;
    int32_t *bucket = (int32_t *)malloc(sizeof(int32_t) * (size_t)m);
    uint32_t *slot = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)m);
    int64_t *count = (int64_t *)calloc((size_t)B, sizeof(int64_t));
    /* 1 */
    for (int64_t i = 0; i < m; ++i) {
        int32_t x = attrs[i];
        int e0 = -1, e1 = -1;
        for (int b = 0; b < B; ++b)
            if (ix->table[6 * b + T_MIN] <= x && x <= ix->table[6 * b + T_MAX]) { if (e0 < 0) e0 = b; e1 = b; }
        int b;
        if (e0 >= 0) {
            b = e0 + (int)((uint64_t)(n_prev + i) % (uint64_t)(e1 - e0 + 1));
        } else {
            b = B - 1;
            for (int c = 0; c < B; ++c) if (ix->table[6 * c + T_MAX] >= x) { b = c; break; }
        }
        bucket[i] = b;
    }
    /* 2 */
    for (int64_t i = 0; i < m; ++i) {
        const int32_t *t = ix->table + 6 * bucket[i];
        slot[i] = (uint32_t)((int64_t)t[T_BASE] + t[T_NTOT] + count[bucket[i]]);
        count[bucket[i]]++;
    }
    for (int b = 0; b < B; ++b)
        if (ix->table[6 * b + T_NTOT] + count[b] > ix->table[6 * b + T_CAP]) {
            free(bucket); free(slot); free(count);
            return 3;
        }
    uint64_t st[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    /* 3 + 4 on the snapshot */
    uint32_t *rows = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)m * K);
    float *rowd = (float *)malloc(sizeof(float) * (size_t)m * K);   /* dist(q, row entry) */
    uint8_t *rowk = (uint8_t *)malloc((size_t)m * K);               /* request kind: 0 local, 1 remote, 2 none */
#ifdef _OPENMP
    if (threads < 1) threads = 1;
#pragma omp parallel num_threads(threads)
#endif
    {
        scratch *sc = scratch_new(ix->n_cap);
        uint32_t *cs = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)append_beam);
        float *cd = (float *)malloc(sizeof(float) * (size_t)append_beam);
        uint32_t *gs = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)append_beam);
        float *gd = (float *)malloc(sizeof(float) * (size_t)append_beam);
        uint64_t my_scanned = 0, my_rows = 0, my_evals = 0, my_parents = 0;
        uint32_t ctr[8];
#ifdef _OPENMP
#pragma omp for schedule(static)
#endif
        for (int64_t i = 0; i < m; ++i) {
            const float *q = vecs + (size_t)i * dim;
            uint32_t *row = rows + (size_t)i * K;
            int kept[2] = {0, 0};
            /* local part: Eq. 2 selection over the candidates found in the target bucket */
            int64_t nQ = search_one(ix, pr, q, 0, 0, bucket[i], append_beam, sc, ctr);
            my_evals += ctr[C_EVALS]; my_parents += ctr[C_PARENTS];
            int nc = 0;
            for (int64_t j = 0; j < nQ; ++j) { cs[nc] = sc->Q[j].slot; cd[nc] = sc->Q[j].dist; nc++; }
            kept[0] = forward_select(ix, cs, cd, nc, kl, row, &my_scanned);
            for (int j = 0; j < kl; ++j) {
                float d = 0.0f;
                if (row[j] != EMPTY)
                    for (int t = 0; t < nc; ++t) if (cs[t] == row[j]) d = cd[t];
                rowd[(size_t)i * K + j] = d;
                rowk[(size_t)i * K + j] = 0;
            }
            if (mode == 0) {
            /* remote part: entry j is the nearest to q among the j-th remote entries of its local
             * candidates (they all lie in the j-th target bucket when the graph was built that way) */
            const int nrc = remote_cands > 0 && remote_cands < nc ? remote_cands : nc;   /* the nearest candidates only */
            for (int j = 0; j < kr; ++j) {
                uint32_t best = EMPTY, best_img = 0; float best_d = 0.0f;
                for (int t = 0; t < nrc; ++t) {
                    uint32_t r = ix->A[(size_t)cs[t] * K + kl + j];
                    if (r == EMPTY) continue;
                    int seen = 0;       /* a row several candidates share is one evaluation */
                    for (int x = 0; x < t && !seen; ++x) seen = ix->A[(size_t)cs[x] * K + kl + j] == r;
                    my_rows += !seen;
                    float d = oracle_distance(q, ix->X + (size_t)r * dim, dim, ix->metric);
                    uint32_t im = dist_image(d);
                    if (best == EMPTY || im < best_img || (im == best_img && r < best)) { best = r; best_img = im; best_d = d; }
                }
                row[kl + j] = best;
                rowd[(size_t)i * K + kl + j] = best_d;
                rowk[(size_t)i * K + kl + j] = 1;
                if (best != EMPTY) kept[1]++;
            }
            } else {
            /* 3', 4': global-scope candidates, proximal / global picks, redundant local edges elsewhere */
            int64_t nG = search_one(ix, pr, q, 0, 0, -2 - bucket[i], append_beam, sc, ctr);
            my_evals += ctr[C_EVALS]; my_parents += ctr[C_PARENTS];
            int ng = 0;
            for (int64_t j = 0; j < nG; ++j) { gs[ng] = sc->Q[j].slot; gd[ng] = sc->Q[j].dist; ng++; }
            select_remote(ix, attrs[i], gs, gd, ng, rr, row + kl, rowd + (size_t)i * K + kl);
            int next_local = 0;
            for (int j = 0; j < kr; ++j) {
                rowk[(size_t)i * K + kl + j] = 1;
                if (row[kl + j] != EMPTY) { kept[1]++; continue; }
                rowk[(size_t)i * K + kl + j] = 2;      /* no reverse request for a fallback entry */
                for (; next_local < nc; ++next_local) {
                    int used = 0;
                    for (int x = 0; x < kl; ++x) if (row[x] == cs[next_local]) used = 1;
                    if (!used) break;
                }
                if (next_local < nc) row[kl + j] = cs[next_local++];
            }
            }
            if (kept_out) { kept_out[2 * i] = kept[0]; kept_out[2 * i + 1] = kept[1]; }
        }
        free(cs); free(cd); free(gs); free(gd);
        scratch_free(sc);
#ifdef _OPENMP
#pragma omp critical
#endif
        { st[6] += my_scanned; st[7] += my_rows; st[9] += my_evals; st[10] += my_parents; }
    }
    /* write the new nodes */
    int64_t nreq = 0;
    request *req = (request *)malloc(sizeof(request) * (size_t)(m * K > 0 ? m * K : 1));
    for (int64_t i = 0; i < m; ++i) {
        uint32_t s = slot[i];
        memcpy(ix->X + (size_t)s * dim, vecs + (size_t)i * dim, sizeof(float) * (size_t)dim);
        ix->attr[s] = attrs[i];
        ix->slot2id[s] = (uint32_t)(n_prev + i);
        id2slot[n_prev + i] = s;
        memcpy(ix->A + (size_t)s * K, rows + (size_t)i * K, sizeof(uint32_t) * (size_t)K);
        for (int j = 0; j < K; ++j) {
            uint32_t v = rows[(size_t)i * K + j];
            if (v == EMPTY || rowk[(size_t)i * K + j] == 2) continue;
            float d = rowd[(size_t)i * K + j];
            req[nreq].v = v; req[nreq].kind = rowk[(size_t)i * K + j]; req[nreq].img = dist_image(d);
            req[nreq].q = s; req[nreq].dist = d;
            st[req[nreq].kind]++;
            nreq++;
        }
    }
    /* 5: requests of one target are applied in order; different targets touch different rows, so
     * the targets may be worked on in parallel without changing any result */
    qsort(req, (size_t)nreq, sizeof(request), request_cmp);
    const float a = alpha * alpha;
    int64_t ngroups = 0;
    int64_t *gstart = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nreq + 1));
    for (int64_t r = 0; r < nreq; ++r) {
        if (r == 0 || req[r].v != req[r - 1].v) gstart[ngroups++] = r;
        if (r == 0 || req[r].v != req[r - 1].v || req[r].kind != req[r - 1].kind) st[2 + req[r].kind]++;
    }
    gstart[ngroups] = nreq;
    uint64_t applied_l = 0, applied_r = 0, passed = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 64) num_threads(threads) reduction(+ : applied_l, applied_r, passed)
#endif
    for (int64_t g = 0; g < ngroups; ++g)
    for (int64_t r = gstart[g]; r < gstart[g + 1]; ++r) {
        uint32_t *R = ix->A + (size_t)req[r].v * K + (req[r].kind == 0 ? 0 : kl);
        int len = req[r].kind == 0 ? kl : kr;
        const float *xq = ix->X + (size_t)req[r].q * dim, *xv = ix->X + (size_t)req[r].v * dim;
        float lhs = a * bias_base(ix, req[r].dist);
        if (req[r].kind == 1 && mode == 0) {
            /* remote part of v: the entry that points into q's bucket keeps the nearest node of
             * that bucket, the fresh node judged by its biased distance (Eq. 3) */
            int bq = bucket_of_slot(ix, req[r].q);
            int far = -1, empty_at = -1; uint32_t far_img = 0;
            for (int j = 0; j < len; ++j) {
                if (R[j] == EMPTY) { if (empty_at < 0) empty_at = j; continue; }
                if (bucket_of_slot(ix, R[j]) != bq) continue;
                uint32_t im = dist_image(oracle_distance(xv, ix->X + (size_t)R[j] * dim, dim, ix->metric));
                if (far < 0 || im > far_img || (im == far_img && R[j] > R[far])) { far = j; far_img = im; }
            }
            if (far >= 0) {
                float dfar = oracle_distance(xv, ix->X + (size_t)R[far] * dim, dim, ix->metric);
                if (lhs < bias_base(ix, dfar)) { R[far] = req[r].q; applied_r++; }
            } else if (empty_at >= 0) {
                R[empty_at] = req[r].q; applied_r++;
            }
            continue;
        }
        if (req[r].kind == 1) {
            /* 5': q competes for the remote positions of its class (proximal or global relative to v) */
            int64_t diff = (int64_t)ix->attr[req[r].q] - (int64_t)ix->attr[req[r].v];
            if (diff < 0) diff = -diff;
            const int j0 = diff <= rr->window ? 0 : rr->n_proximal, j1 = diff <= rr->window ? rr->n_proximal : kr;
            const int bv = bucket_of_slot(ix, req[r].v);
            int take = -1, far = -1; uint32_t far_img = 0;
            for (int j = j0; j < j1 && take < 0; ++j)
                if (R[j] == EMPTY || bucket_of_slot(ix, R[j]) == bv) take = j;
            if (take >= 0) { R[take] = req[r].q; applied_r++; continue; }
            for (int j = j0; j < j1; ++j) {
                uint32_t im = dist_image(oracle_distance(xv, ix->X + (size_t)R[j] * dim, dim, ix->metric));
                if (far < 0 || im > far_img || (im == far_img && R[j] > R[far])) { far = j; far_img = im; }
            }
            if (far >= 0) {
                float dfar = oracle_distance(xv, ix->X + (size_t)R[far] * dim, dim, ix->metric);
                if (lhs < bias_base(ix, dfar)) { R[far] = req[r].q; applied_r++; }
            }
            continue;
        }
        int pass = 1, empty_at = -1;
        for (int j = 0; j < len; ++j) {
            if (R[j] == EMPTY) { if (empty_at < 0) empty_at = j; continue; }
            float dqn = oracle_distance(xq, ix->X + (size_t)R[j] * dim, dim, ix->metric);
            if (!(lhs < bias_base(ix, dqn))) pass = 0;
        }
        if (!pass) continue;
        passed++;
        if (empty_at >= 0) { R[empty_at] = req[r].q; applied_l++; continue; }
        /* the newcomer may only take the place of a neighbour it points to itself, so that the
         * pathway v -> n survives as v -> q -> n; among those the one farthest from v (ties: smaller slot) */
        int victim = -1; uint32_t victim_img = 0;
        const uint32_t *qrow = ix->A + (size_t)req[r].q * K;
        for (int j = 0; j < len; ++j) {
            int covered = 0;
            for (int x = 0; x < K; ++x) if (qrow[x] == R[j]) covered = 1;
            if (!covered) continue;
            uint32_t im = dist_image(oracle_distance(xv, ix->X + (size_t)R[j] * dim, dim, ix->metric));
            if (victim < 0 || im > victim_img || (im == victim_img && R[j] < R[victim])) { victim = j; victim_img = im; }
        }
        if (victim >= 0) { R[victim] = req[r].q; applied_l++; }
    }
    free(gstart);
    st[4] = applied_l; st[5] = applied_r; st[8] = passed;
    if (stats) memcpy(stats, st, sizeof(st));
    /* 6 */
    for (int64_t i = 0; i < m; ++i) {
        int32_t *t = ix->table + 6 * bucket[i];
        if (attrs[i] < t[T_MIN]) t[T_MIN] = attrs[i];
        if (attrs[i] > t[T_MAX]) t[T_MAX] = attrs[i];
    }
    for (int b = 0; b < B; ++b) ix->table[6 * b + T_NTOT] += (int32_t)count[b];
    free(req); free(rows); free(rowd); free(rowk); free(bucket); free(slot); free(count);
    return 0;
}

/* ============================================================ graph construction (Section 4.3)
 * The paper builds the index in two passes: (1) inside every bucket an exact brute-force k-NN
 * graph, pruned, united with its reverse graph by an interleaved merge whose leading K_local
 * entries are the necessary local edges; (2) remote edges chosen from a global candidate graph,
 * split into proximal ones (neighbouring attribute ranges) and global ones, written into the
 * remaining slots.  The global candidate graph of pass 2 is a third-party pipeline (Algorithm 1)
 * and is not rebuilt here.  reading (normative for this build):
 *
 *  1. Candidates of node u: the `pool` nearest other nodes of its bucket, ordered by
 *     (distance, slot).
 *  2. Pruning (Eq. 2 used as a construction rule): scan the candidates in order, keep c iff
 *     dist(u,c) < dist(c,n) for every n kept so far; forward list F(u) = kept ones, then the
 *     rejected ones, each in candidate order.
 *  3. Reverse list R(v): the sources u with v among the first K_local entries of F(u), ordered by
 *     (dist(u,v), slot of u), at most K_local of them.
 *  4. Interleaved merge: F0, R0, F1, R1, ... over the first K_local entries of each list; empty
 *     entries and repeats are skipped; the first K_local survivors are the local part of the row.
 *  5. Remote part: entry j is the node nearest to u in the j-th target bucket of u's bucket b.
 *     Targets are b+1, b-1, b+2, b-2, b+4, b-4, ... (doubling: adjacent attribute intervals
 *     first, then longer jumps), then the remaining offsets in order of size; targets outside
 *     [0,B) are skipped; the first K_remote distinct ones count.  Fewer than K_remote targets
 *     leave empty entries (the paper's fallback to redundant local edges is not used, so that
 *     the remote part never holds an edge that stays inside the bucket).
 *
 * Step 5 is the remote wiring by target bucket (remote_rule.mode 0).  The second reading
 * (remote_rule.mode 1) follows Section 4.3's own words, with the library's search in the place of
 * the third-party global graph as the source of cross-bucket candidates:
 *  4'. The interleaved merge goes on past K_local: after F and R are exhausted up to K_local it
 *      continues with the rest of F; the first K_local survivors are the necessary local edges,
 *      the next K_remote the redundant ones, stored in the remote part of the row.
 *  5'. For every node u, against the graph as step 4' left it (all nodes are processed against
 *      that same graph): global candidates = one run of the search (Algorithm 2) with u's vector
 *      as query and the scope "every slot outside u's bucket", beam entries, ordered by
 *      (distance, slot).  A candidate whose attribute differs from u's by at most `window` is
 *      proximal, any other global.  The first n_proximal proximal ones overwrite remote positions
 *      0.., the first K_remote - n_proximal global ones the positions n_proximal..; a position
 *      without a pick keeps its redundant local edge.
 */
typedef struct {
    uint32_t img, slot;
    float dist;
} knn_entry;

static int knn_cmp(const void *a, const void *b) {
    const knn_entry *x = (const knn_entry *)a, *y = (const knn_entry *)b;
    if (x->img != y->img) return x->img < y->img ? -1 : 1;
    if (x->slot != y->slot) return x->slot < y->slot ? -1 : 1;
    return 0;
}

/* the P nearest occupied slots of `target_bucket` to the row at `slot` (itself excluded),
 * ordered by (distance, slot); missing entries are (EMPTY, +inf) */
void oracle_knn(const oracle_index *ix, uint32_t slot, int32_t target_bucket, int32_t P, uint32_t *out_slots,
                float *out_dist) {
    const int32_t *t = ix->table + 6 * target_bucket;
    int64_t m = t[T_NTOT], n = 0;
    knn_entry *e = (knn_entry *)malloc(sizeof(knn_entry) * (size_t)(m > 0 ? m : 1));
    const float *q = ix->X + (size_t)slot * ix->dim;
    for (int64_t j = 0; j < m; ++j) {
        uint32_t s = (uint32_t)(t[T_BASE] + j);
        if (s == slot) continue;
        float d = oracle_distance(q, ix->X + (size_t)s * ix->dim, ix->dim, ix->metric);
        e[n].img = dist_image(d); e[n].slot = s; e[n].dist = d;
        n++;
    }
    qsort(e, (size_t)n, sizeof(knn_entry), knn_cmp);
    for (int j = 0; j < P; ++j) {
        out_slots[j] = j < n ? e[j].slot : EMPTY;
        out_dist[j] = j < n ? e[j].dist : INFINITY;
    }
    free(e);
}

/* target buckets of bucket b for its remote entries; returns how many (<= k_remote) */
int oracle_remote_targets(int32_t b, int32_t B, int32_t k_remote, int32_t *out) {
    int n = 0;
    for (int pass = 0; pass < 2 && n < k_remote; ++pass)
        for (int o = 1; o < B && n < k_remote; o = pass == 0 ? o * 2 : o + 1) {
            if (pass == 1 && (o & (o - 1)) == 0) continue;   /* powers of two were taken in pass 0 */
            for (int sgn = 1; sgn >= -1 && n < k_remote; sgn -= 2) {
                int t = b + sgn * o;
                if (t < 0 || t >= B) continue;
                out[n++] = t;
            }
        }
    return n;
}

/* forward list of one node: F (slots) and Fd (distances to the node), `pool` entries */
static void forward_list(const oracle_index *ix, uint32_t u, int32_t b, int32_t pool, uint32_t *F, float *Fd) {
    uint32_t *cs = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)pool), *kept = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)pool);
    float *cd = (float *)malloc(sizeof(float) * (size_t)pool);
    uint8_t *is_kept = (uint8_t *)calloc((size_t)pool, 1);
    oracle_knn(ix, u, b, pool, cs, cd);
    int nk = 0;
    for (int t = 0; t < pool && cs[t] != EMPTY; ++t) {
        int ok = 1;
        for (int j = 0; j < nk && ok; ++j) {
            float dcn = oracle_distance(ix->X + (size_t)cs[t] * ix->dim, ix->X + (size_t)kept[j] * ix->dim, ix->dim, ix->metric);
            if (!(cd[t] < dcn)) ok = 0;
        }
        if (ok) { kept[nk++] = cs[t]; is_kept[t] = 1; }
    }
    int w = 0;
    for (int pass = 1; pass >= 0; --pass)
        for (int t = 0; t < pool; ++t)
            if (cs[t] != EMPTY && is_kept[t] == pass) { F[w] = cs[t]; Fd[w] = cd[t]; w++; }
    for (; w < pool; ++w) { F[w] = EMPTY; Fd[w] = INFINITY; }
    free(cs); free(kept); free(cd); free(is_kept);
}

typedef struct {
    uint32_t v, img, u;
} rev_edge;
static int rev_cmp(const void *a, const void *b) {
    const rev_edge *x = (const rev_edge *)a, *y = (const rev_edge *)b;
    if (x->v != y->v) return x->v < y->v ? -1 : 1;
    if (x->img != y->img) return x->img < y->img ? -1 : 1;
    if (x->u != y->u) return x->u < y->u ? -1 : 1;
    return 0;
}

/* Pass 2 alone (step 5 or 5'), on whatever graph the index holds: rewrites the remote part of
 * every row.  mode 0 needs no search parameters (pr may be NULL). */
int oracle_build_remote(oracle_index *ix, const remote_rule *rr, const oracle_params *pr, int32_t beam, int32_t threads) {
    const int kl = ix->k_local, kr = ix->k_remote, K = kl + kr, B = ix->n_buckets;
    const int mode = rr ? rr->mode : 0;
    if (threads < 1) threads = 1;
    if (kr == 0) return 0;
    if (mode == 0) {
        for (int b = 0; b < B; ++b) {
            const int32_t *t = ix->table + 6 * b;
            int32_t tg[64];
            int nt = oracle_remote_targets(b, B, kr, tg);
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(threads)
#endif
            for (int64_t j = 0; j < t[T_NTOT]; ++j) {
                uint32_t u = (uint32_t)(t[T_BASE] + j);
                for (int r = 0; r < kr; ++r) ix->A[(size_t)u * K + kl + r] = EMPTY;
                for (int r = 0; r < nt; ++r) {
                    float d;
                    oracle_knn(ix, u, tg[r], 1, ix->A + (size_t)u * K + kl + r, &d);
                }
            }
        }
        return 0;
    }
    if (mode != 1 || !pr || rr->n_proximal < 0 || rr->n_proximal > kr || rr->window < 0 || beam < 1) return 1;
    /* every search runs against the graph as it is now, not against rows already rewritten */
    oracle_index snap = *ix;
    snap.A = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)ix->n_cap * K);
    memcpy(snap.A, ix->A, sizeof(uint32_t) * (size_t)ix->n_cap * K);
#ifdef _OPENMP
#pragma omp parallel num_threads(threads)
#endif
    {
        scratch *sc = scratch_new(ix->n_cap);
        uint32_t *gs = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)beam), *picks = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)kr);
        float *gd = (float *)malloc(sizeof(float) * (size_t)beam), *pickd = (float *)malloc(sizeof(float) * (size_t)kr);
        for (int b = 0; b < B; ++b) {
            const int32_t *t = ix->table + 6 * b;
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 16)
#endif
            for (int64_t j = 0; j < t[T_NTOT]; ++j) {
                uint32_t u = (uint32_t)(t[T_BASE] + j);
                int64_t nG = search_one(&snap, pr, ix->X + (size_t)u * ix->dim, 0, 0, -2 - b, beam, sc, NULL);
                int ng = 0;
                for (int64_t x = 0; x < nG; ++x) { gs[ng] = sc->Q[x].slot; gd[ng] = sc->Q[x].dist; ng++; }
                select_remote(ix, ix->attr[u], gs, gd, ng, rr, picks, pickd);
                for (int r = 0; r < kr; ++r)
                    if (picks[r] != EMPTY) ix->A[(size_t)u * K + kl + r] = picks[r];
            }
        }
        free(gs); free(gd); free(picks); free(pickd);
        scratch_free(sc);
    }
    free(snap.A);
    return 0;
}

/* Fills ix->A (all rows) for the objects currently in the index.  F_out/R_out (may be NULL)
 * receive the forward lists [n_cap][pool] and reverse lists [n_cap][k_local] for inspection. */
int oracle_build_graph(oracle_index *ix, int32_t pool, uint32_t *F_out, uint32_t *R_out, int32_t threads,
                       const remote_rule *rr, const oracle_params *pr, int32_t beam) {
    const int kl = ix->k_local, kr = ix->k_remote, K = kl + kr, B = ix->n_buckets;
    const int mode = rr ? rr->mode : 0;
    if (pool < kl || kl < 0 || kr < 0 || K < 1) return 1;
    const int64_t N = ix->n_cap;
    uint32_t *F = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N * pool);
    float *Fd = (float *)malloc(sizeof(float) * (size_t)N * pool);
    uint32_t *R = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N * (kl > 0 ? kl : 1));
    for (int64_t i = 0; i < N * pool; ++i) F[i] = EMPTY;
    for (int64_t i = 0; i < N * kl; ++i) R[i] = EMPTY;
    for (int64_t i = 0; i < N * K; ++i) ix->A[i] = EMPTY;
    if (threads < 1) threads = 1;
    for (int b = 0; b < B; ++b) {
        const int32_t *t = ix->table + 6 * b;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(threads)
#endif
        for (int64_t j = 0; j < t[T_NTOT]; ++j) {
            uint32_t u = (uint32_t)(t[T_BASE] + j);
            forward_list(ix, u, b, pool, F + (size_t)u * pool, Fd + (size_t)u * pool);
        }
    }
    /* reverse lists */
    int64_t ne = 0;
    rev_edge *E = (rev_edge *)malloc(sizeof(rev_edge) * (size_t)(N * kl > 0 ? N * kl : 1));
    for (int64_t u = 0; u < N; ++u)
        for (int j = 0; j < kl; ++j) {
            uint32_t v = F[(size_t)u * pool + j];
            if (v == EMPTY) continue;
            E[ne].v = v; E[ne].img = dist_image(Fd[(size_t)u * pool + j]); E[ne].u = (uint32_t)u;
            ne++;
        }
    qsort(E, (size_t)ne, sizeof(rev_edge), rev_cmp);
    for (int64_t p = 0, start = 0; p < ne; ++p) {
        if (p > 0 && E[p].v != E[p - 1].v) start = p;
        if (p - start < kl) R[(size_t)E[p].v * kl + (p - start)] = E[p].u;
    }
    /* interleaved merge: `want` entries per row (mode 1 also fills the redundant positions) */
    const int want = mode == 1 ? K : kl;
    for (int64_t u = 0; u < N; ++u) {
        uint32_t *row = ix->A + (size_t)u * K;
        int w = 0;
        for (int j = 0; j < pool && w < want; ++j)
            for (int side = 0; side < 2 && w < want; ++side) {
                if (side == 1 && j >= kl) continue;      /* the reverse list has K_local entries */
                uint32_t c = side == 0 ? F[(size_t)u * pool + j] : R[(size_t)u * kl + j];
                if (c == EMPTY) continue;
                int dup = 0;
                for (int x = 0; x < w; ++x) if (row[x] == c) dup = 1;
                if (!dup) row[w++] = c;
            }
    }
    if (F_out) memcpy(F_out, F, sizeof(uint32_t) * (size_t)N * pool);
    if (R_out) memcpy(R_out, R, sizeof(uint32_t) * (size_t)N * kl);
    free(F); free(Fd); free(R); free(E);
    return oracle_build_remote(ix, rr, pr, beam, threads);
}
