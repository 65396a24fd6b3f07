/*
 * grab.h - C ABI of the MI355X range-filtered graph search library (libgrab.so).
 *
 * The library holds one bucketed graph index per handle, entirely in device memory, and
 * runs every step of the search and append path in HIP kernels written for gfx950.
 * The calls follow the paper's problem statement: a data set of (vector, scalar) objects
 * and queries Q = (q, k, [l, u]) (Section 2.4, Hybrid Search definition), answered by the
 * range-constrained graph search of Algorithm 2 over the bucketed topology of Section 4.2,
 * and batches of new objects inserted as in Section 4.4.
 *
 * Conventions for every call
 *   - Returns a grab_status.  On anything but GRAB_OK the index is unchanged unless the
 *     call's comment says otherwise, and grab_last_error() gives a message.
 *   - Every pointer argument may be a device pointer (e.g. torch-allocated) or an ordinary
 *     host pointer; the library finds out with hipPointerGetAttributes.  The caller owns
 *     all input and output buffers; the library copies what it needs into arrays it owns
 *     and keeps no caller pointer after the call returns.
 *   - Work is enqueued on the HIP stream given to grab_create.  A call with device outputs
 *     returns after enqueueing; a call with host outputs (or host inputs) synchronises the
 *     stream before returning.  Calls that report GRAB_EFULL / GRAB_EINVAL from device-side
 *     checks (grab_load_graph, grab_append_batch) synchronise too.
 *   - Arguments are validated on the host before any kernel is launched.
 *   - Matrices are dense row-major.  Object ids ("external ids") are row numbers of the
 *     grab_build_buckets input and continue n, n+1, ... in append order.  "Slots" are
 *     physical row numbers of the bucket-major device arrays.
 *   - 0xFFFFFFFF marks an empty adjacency entry and a missing result.
 *   - dim must be one of 32, 64, 96, 128, 160, 192, 256, 384, 512, 640, 768, 960, 1024, 1536,
 *     2048 (rows are whole 128-byte lines, and the kernels are built per row length);
 *     grab_create refuses any other value with GRAB_EINVAL.
 *   - The queries of a batch are independent; the library runs them in an order of its own
 *     (grouped by the buckets they select) and every result is what it would be in any order.
 *   - Not thread-safe per handle; different handles are independent.
 */
#ifndef GRAB_H
#define GRAB_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct grab_index grab_index; /* opaque; owns all device arrays */

typedef enum {
    GRAB_OK = 0,
    GRAB_EINVAL = 1, /* bad argument (sizes, null pointer, k > beam, malformed graph, ...) */
    GRAB_ESTATE = 2, /* call out of order (search before load_graph, ...)                   */
    GRAB_EFULL = 3,  /* a bucket has no tail room left for an append                        */
    GRAB_ENOMEM = 4, /* device or host allocation failed                                    */
    GRAB_EHIP = 5    /* a HIP runtime call failed                                           */
} grab_status;

typedef enum {
    GRAB_L2SQ = 0, /* sum_j (q_j - v_j)^2  (Euclidean ranking, Table 2; no square root) */
    GRAB_IP = 1    /* -sum_j q_j v_j       (smaller is better)                           */
} grab_metric;

/* Tunables of Algorithm 2 and Section 4.4 (names as in Section 5's hyper-parameter study). */
typedef enum {
    GRAB_P_SEARCH_WIDTH = 0, /* parents expanded per iteration, 1..8; default 1            */
    GRAB_P_MAX_ITER = 1,     /* iteration cap; 0 = 2*beam (default)                        */
    GRAB_P_N_SEEDS = 2,      /* seeds per query; 0 = min(beam, 64) (default)               */
    GRAB_P_VISITED_CAP = 3,  /* the search stops before its visited set could exceed this;
                                default 2800, at most 24000                                */
    GRAB_P_SEED_SALT = 4,    /* moves the seed jitter; default 0                           */
    GRAB_P_ALPHA = 5,        /* freshness bias of Eq. 3, in (0, 1]; default 0.6            */
    GRAB_P_APPEND_BEAM = 6,  /* candidate queue size of the candidate searches of
                                grab_append_batch and grab_build_remote; default 64        */
    GRAB_P_PROFILE = 7,      /* 1: bracket the search kernels with HIP events on the index's
                                stream so that grab_get_timing can report them; default 0  */
    GRAB_P_REMOTE_MODE = 8,  /* how grab_build_graph, grab_build_remote and grab_append_batch wire
                                remote edges (Section 4.3, Remote Edge Construction):
                                0 (default) entry j of the remote part belongs to the j-th target
                                bucket; 1 candidates from a search over every other bucket, split
                                into proximal and global picks                              */
    GRAB_P_N_PROXIMAL = 9,   /* mode 1: remote positions kept for proximal candidates, 0..64;
                                -1 (default) = ceil(k_remote / 2)                          */
    GRAB_P_APPEND_REMOTE_CANDS = 11, /* grab_append_batch under mode 0: the remote part of a new row
                                is chosen among the remote entries of its nearest this-many local
                                candidates; 0 (default) = all GRAB_P_APPEND_BEAM of them           */
    GRAB_P_REMOTE_WINDOW = 10 /* mode 1: a candidate is proximal iff its attribute differs from the
                                node's by at most this fraction of the attribute span of the index
                                (largest minus smallest stored attribute, as int32 keys), rounded
                                down; in [0, 1], default 0.2 (the paper's example)         */
} grab_param;

/* Creates an empty index for `dim`-dimensional fp32 vectors under `metric`: the container of the
 * unified memory layout of Section 4.2.4 (feature matrix, adjacency matrix, bucket <-> index maps),
 * all of it in device memory.
 * `hip_stream` is a hipStream_t (NULL = the default stream); it must outlive the index. */
grab_status grab_create(grab_index **out, int32_t dim, int32_t metric, void *hip_stream);

/* Frees every device and host array of the index.  NULL is allowed. */
void grab_destroy(grab_index *ix);

/* Message for the last non-OK status of this handle ("" if none).  Owned by the handle. */
const char *grab_last_error(const grab_index *ix);

/* Predicate-based bucket partitioning (Section 4.2.1) into the unified device layout
 * (Section 4.2.4).  vectors[n][dim] fp32, attrs[n] int32.  Objects are ordered by
 * (attribute, id) and cut into n_buckets buckets of equal count (ranks floor(b*n/B) ..
 * floor((b+1)*n/B)); bucket b owns a contiguous slab of count_b + floor((n_cap-n)/B) slots,
 * the extra ones being tail room for grab_append_batch.  Builds the feature matrix,
 * attribute array, id<->slot maps and bucket table, and a small search aid for Algorithm 2's
 * range selection (every 128th attribute of each bucket's sorted part: slots / 128 + n_buckets
 * words); drops any graph loaded before.
 * Requires 1 <= n_buckets <= 1024, n_buckets <= n <= n_cap < 2^31.
 * Errors: GRAB_EINVAL (arguments), GRAB_ENOMEM, GRAB_EHIP; the index is empty afterwards. */
grab_status grab_build_buckets(grab_index *ix, const float *vectors, const int32_t *attrs,
                               int64_t n, int32_t n_buckets, int64_t n_cap);

/* Installs the hybrid edge topology (Section 4.2.2) with fixed degree k_local + k_remote
 * (Section 4.2.3).  local_adj[n][k_local] and remote_adj[n][k_remote] hold external ids
 * (0xFFFFFFFF = no edge), one row per object currently in the index.  Ids are translated
 * to slots and each row is stored as [local | remote].  Checked on the device: ids < n,
 * local edges stay inside the node's bucket, remote edges leave it; a violation gives
 * GRAB_EINVAL and leaves the index without a graph.  k_local + k_remote must be 1..128;
 * k_remote may be 0 (remote_adj then unused).  GRAB_ESTATE before grab_build_buckets. */
grab_status grab_load_graph(grab_index *ix, const uint32_t *local_adj, int32_t k_local,
                            const uint32_t *remote_adj, int32_t k_remote);

/* Two-pass index construction (Section 4.3) on the objects currently in the index, replacing any
 * graph loaded or built before.  Pass 1 (local router): for every object the `pool` nearest
 * objects of its bucket by exact brute force, pruned by the diversity rule (Eq. 2: a candidate is
 * kept iff it is closer to the object than to every candidate kept before it; rejected ones
 * follow the kept ones), united with the reverse graph by an interleaved merge (forward, reverse,
 * forward, ...) whose first k_local distinct entries become the local part of the row.  Pass 2
 * (remote edges): entry j of the remote part is the nearest object of the j-th target bucket;
 * targets of bucket b are b+1, b-1, b+2, b-2, b+4, b-4, ... (adjacent attribute intervals first,
 * then doubling jumps), then the remaining offsets by size, skipping buckets that do not exist.
 * The paper draws remote candidates from a global graph built by a third-party pipeline
 * (Algorithm 1); here they come from exact search in the target bucket (GRAB_P_REMOTE_MODE 0) or
 * from the library's own search over all other buckets (mode 1, see grab_build_remote).  Distances
 * use the same fixed fp32 summation order as the search, ties go to the smaller slot.  (The nearest
 * objects are found exactly: low-precision scores from the matrix cores only narrow each object's
 * targets down, with a proven margin, to the few whose fixed-order distances are then taken.)
 * pool = 0 means min(4 * k_local, 128): wide enough to reach past a node's own cluster, which is
 * what gives the graph its long links.  Requires 1 <= k_local <= 64, 0 <= k_remote <= 64,
 * k_local <= pool <= 128.  Errors: GRAB_EINVAL, GRAB_ESTATE (no layout), GRAB_ENOMEM, GRAB_EHIP;
 * on error the index is left without a graph. */
grab_status grab_build_graph(grab_index *ix, int32_t k_local, int32_t k_remote, int32_t pool);

/* Pass 2 of the construction alone (Section 4.3, Remote Edge Construction) on the graph the index
 * holds, whatever made it: rewrites the remote part of every row under the reading that
 * GRAB_P_REMOTE_MODE selects.
 *   0: entry j = the nearest object of the j-th target bucket, as in grab_build_graph.
 *   1: the paper's split.  Global candidates of a row = one run of the search (Algorithm 2) with
 *      the row's own vector as query over every slot outside the row's bucket, against the graph
 *      as it is when the call starts, with queue GRAB_P_APPEND_BEAM and the current seeds / width /
 *      visited-cap / max-iter parameters (the library's search stands where the paper has a global
 *      graph from a third-party pipeline, Algorithm 1).  A candidate is proximal iff its attribute
 *      differs from the row's by at most the window (GRAB_P_REMOTE_WINDOW), any other one global.
 *      The nearest GRAB_P_N_PROXIMAL proximal candidates overwrite remote positions 0.., the
 *      nearest k_remote - n_proximal global ones the positions after them; a position with no pick
 *      keeps what it holds.  Under this reading grab_build_graph first lets the interleaved merge
 *      of pass 1 run on into the remote part (the redundant local edges, which the paper keeps
 *      where too few remote candidates qualify), so the remote part of a row may hold edges that
 *      stay inside the bucket, and grab_load_graph accepts such rows while mode 1 is set.
 * Errors: GRAB_ESTATE (no graph), GRAB_EINVAL (n_proximal > k_remote, search parameters),
 * GRAB_ENOMEM, GRAB_EHIP; the graph may be partly rewritten after GRAB_ENOMEM / GRAB_EHIP. */
grab_status grab_build_remote(grab_index *ix);

/* Range-constrained search (Algorithm 2) for nq queries: queries[nq][dim], closed ranges
 * lo[i] <= attribute <= hi[i], k results per query from a candidate queue of `beam` entries
 * (the paper's itopk).  out_ids[nq][k] external ids and out_dist[nq][k] distances, ascending
 * by (distance, slot); rows with fewer than k reachable valid objects are padded with
 * (0xFFFFFFFF, +inf); lo > hi or a range that meets no bucket gives a fully padded row.
 * Requires 1 <= k <= beam <= 512, n_seeds <= visited_cap, search_width * degree <= 512.
 * Allocates nothing once its per-batch work buffers have grown to nq.
 * Errors: GRAB_EINVAL, GRAB_ESTATE (no graph), GRAB_ENOMEM, GRAB_EHIP. */
grab_status grab_search_range(grab_index *ix, const float *queries, const int32_t *lo,
                              const int32_t *hi, int64_t nq, int32_t k, int32_t beam,
                              uint32_t *out_ids, float *out_dist);

/* grab_search_range for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same results, same counters
 * and timing read-backs as grab_search_range, but the per-batch work buffers (query plans, seed
 * slots, counters, launch order) live in one static device array of about 18 MiB that every GPU
 * the library runs on holds until the process ends; the call performs no hipMalloc, hipFree or
 * other allocating call.  Limits: every pointer must be a device pointer (staging a host buffer
 * would allocate); nq <= 16,384; nq * n_seeds <= 4,194,304 (n_seeds as grab_search_range
 * resolves it).  Beyond either limit, or with a host pointer: GRAB_EINVAL, nothing launched.
 * All calls on one GPU, from any handle, share that GPU's array: calls whose kernels could
 * overlap on one GPU (different streams, different threads) race and must be serialised by the
 * caller; the counters of a call stay readable until the next call on that GPU.
 * Other errors: GRAB_ESTATE (no graph), GRAB_EHIP. */
grab_status grab_search_range_noalloc(grab_index *ix, const float *queries, const int32_t *lo,
                                      const int32_t *hi, int64_t nq, int32_t k, int32_t beam,
                                      uint32_t *out_ids, float *out_dist);

/* Batched insertion (Section 4.4): appends m objects at the tails of their buckets without
 * moving any existing slot (bucket = the one whose attribute interval holds the new value, else
 * the first one above it; slot = stable order of arrival inside the bucket).  Decisions about
 * existing nodes use the index as it was before the batch.  Per new object: candidate neighbours
 * by a search restricted to its bucket (queue GRAB_P_APPEND_BEAM; the current GRAB_P_N_SEEDS,
 * GRAB_P_SEARCH_WIDTH, GRAB_P_VISITED_CAP and GRAB_P_MAX_ITER govern this search too, so a caller
 * who caps iterations for its queries caps them here as well); local forward edges by the
 * diversity rule (Eq. 2) with back-fill; the remote part and the reverse requests as
 * GRAB_P_REMOTE_MODE says:
 *   0: remote entry j = nearest among the j-th remote entries of the candidates (this departs from
 *      Section 4.4's candidate search, which also looks outside the target bucket: in a graph wired
 *      by target bucket the candidates' own remote entries already name the nodes to look at);
 *      a remote request overwrites the target's remote entry that lies in the new object's
 *      bucket iff the biased distance is smaller, else fills an empty entry.
 *   1: a second candidate search over every slot outside the target bucket (Section 4.4, Parallel
 *      Candidate Search: candidates from the target bucket and from the global scope), proximal and
 *      global picks as in grab_build_remote, a position without a pick taking the nearest local
 *      candidate not yet in the row; a remote request competes for the target's remote positions of
 *      its class (proximal or global relative to the target): it takes the first one that is empty
 *      or holds a node of the target's own bucket, else the one farthest from the target gives way
 *      iff the biased distance is smaller.
 * One reverse request per written edge that leaves no doubt about its kind, applied per target in
 * (kind, distance, source) order: a local request must pass Eq. 2 with the freshness-biased
 * distance (Eq. 3) and then fills an empty entry or overwrites, among the target's neighbours that
 * the new object points to itself, the one farthest from the target.  The bias acts as alpha^2 on
 * squared L2 distances; under GRAB_IP both sides of a biased comparison are first shifted to
 * max(0, 1 + d), half the squared Euclidean distance on unit vectors (scaling minus the inner
 * product itself would push similar newcomers away).  New external ids are n_prev .. n_prev+m-1 in
 * input order.
 * Capacity: a bucket holds count_b + floor((n_cap - n) / n_buckets) objects (see
 * grab_build_buckets), so up to n_buckets - 1 of the n_cap slots asked for do not exist;
 * grab_get_sizes reports the slots there are.  GRAB_EFULL if any bucket would overflow its slab,
 * and GRAB_EINVAL: nothing is written then.  After GRAB_ENOMEM / GRAB_EHIP, which can strike
 * between kernels, new rows may be written while the object count is not advanced: rebuild.
 * Needs k_local <= 64 and k_remote <= 64.
 * Errors: GRAB_EINVAL, GRAB_ESTATE (no graph), GRAB_EFULL, GRAB_ENOMEM, GRAB_EHIP. */
grab_status grab_append_batch(grab_index *ix, const float *vectors, const int32_t *attrs, int64_t m);

/* Sets a grab_param.  GRAB_EINVAL if `which` is unknown or `value` is out of range. */
grab_status grab_set_param(grab_index *ix, int32_t which, double value);

/* Sizes of the index: out[0] objects, out[1] slots, out[2] buckets, out[3] k_local,
 * out[4] k_remote, out[5] dim, out[6] metric, out[7] 1 if a graph is loaded. (host array) */
grab_status grab_get_sizes(const grab_index *ix, int64_t out[8]);

/* Copies out the layout of Section 4.2.4 (the maps M_B2I / M_I2B, here the bucket table and the
 * id <-> slot arrays): bucket_table[B][6] = {base, n_sorted, n_total, cap, min_attr,
 * max_attr}, id2slot[objects], slot2id[slots].  Any pointer may be NULL to skip it. */
grab_status grab_get_layout(grab_index *ix, int32_t *bucket_table, uint32_t *id2slot, uint32_t *slot2id);

/* Copies out the adjacency matrix of Section 4.2.3 (fixed degree, local entries first, then the
 * remote ones) in slot space: adj[slots][k_local + k_remote]. */
grab_status grab_get_graph(grab_index *ix, uint32_t *adj_slots);

/* Copies out the stored feature rows and attributes in slot space (either may be NULL). */
grab_status grab_get_rows(grab_index *ix, float *vectors_slots, int32_t *attr_slots);

/* Bucket selection and seeding alone (Algorithm 2, lines 1-2) for nq ranges, as the search
 * computes them: info[nq][6] int32 = {first bucket, last bucket (< first when none),
 * population size V, first valid sorted slot of the first bucket, end of valid sorted slots
 * of the last bucket, seed count}; seeds[nq][n_seeds] slots, 0xFFFFFFFF-padded.  `beam`
 * only fixes the default seed count.  seeds may be NULL. */
grab_status grab_select_range(grab_index *ix, const int32_t *lo, const int32_t *hi, int64_t nq,
                              int32_t beam, int32_t *info, uint32_t *seeds);

/* Per-query counters of the most recent grab_search_range, one per step of Algorithm 2 (iterations
 * of its loop, PopUnvisited, ComputeDistance, the seeds of line 2, the range pre-check of its
 * lines 8-10, the visited test): per_query[nq][8] uint32 =
 * {iterations, parents expanded, distance evaluations (seeds included), seed evaluations,
 *  neighbours rejected by the scalar pre-check, slots whose attribute had to be read
 *  (appended tails of the two edge buckets), visited-set size, stop reason
 *  (0 queue exhausted, 1 max_iter, 2 visited capacity, 3 empty range)}. */
grab_status grab_get_counters(grab_index *ix, uint32_t *per_query, int64_t nq);

/* Kernel durations of the most recent grab_search_range, measured with HIP events on the
 * index's stream (needs GRAB_P_PROFILE = 1 before that search): ms[0] bucket-select + seeding
 * kernel and, for batches of 2,048 queries and more, the three small kernels that fix the order
 * in which the queries run; ms[1] beam-search kernel; in milliseconds (host array).  Waits for the search to
 * finish.  GRAB_ESTATE if profiling was off. */
grab_status grab_get_timing(grab_index *ix, float ms[2]);

/* Work counters and phase durations of the most recent grab_append_batch (either may be NULL).
 * counts[12] (host) = {reverse requests made for local edges, for remote edges; (target, kind)
 * groups of requests for local parts, for remote parts; requests that rewrote an entry, local,
 * remote; candidates examined by the Eq. 2 scans of the forward selection; vector rows evaluated
 * for the remote parts of the new rows (reading by target bucket only); local requests that passed
 * the biased Eq. 2 test; distance evaluations, and expanded parents, of the candidate searches;
 * 0}.  ms[4] (host, needs GRAB_P_PROFILE = 1 before the call) = candidate search(es), forward
 * selection, new rows + request sorting, reverse rewiring, in milliseconds, from HIP events on
 * the index's stream.  GRAB_ESTATE if no insertion has run, or ms is asked for without profiling. */
grab_status grab_get_append_stats(grab_index *ix, uint64_t counts[12], float ms[4]);

/* ---- float attributes ------------------------------------------------------------------------
 * The filter of Section 3 is over a scalar attribute, and Section 5.1 draws it as a float in
 * [0,1].  These calls take fp32 attributes and bounds.  Internally every float is replaced by
 * its order-preserving int32 image (non-negative values: the IEEE-754 bit pattern; negative
 * values: the bit pattern with its 31 magnitude bits flipped; -0 is stored as +0), so that
 *     lo <= x <= hi   in float arithmetic   <=>   image(lo) <= image(x) <= image(hi),
 * and everything else is the integer path: same layout, same results, same counters.  Read-back
 * calls (grab_get_rows, the bucket table of grab_get_layout) report images; grab_attr_value turns
 * an image back into the float.  An index is either integer- or float-keyed: use one family of
 * calls throughout. */

/* image of one float / float of one image; pure host functions */
int32_t grab_attr_image(float x);
float grab_attr_value(int32_t image);

/* grab_build_buckets with attrs[n] fp32 (host or device).  GRAB_EINVAL if an attribute is NaN.
 * Otherwise as grab_build_buckets on the images. */
grab_status grab_build_buckets_f32(grab_index *ix, const float *vectors, const float *attrs, int64_t n,
                                   int32_t n_buckets, int64_t n_cap);

/* grab_search_range with closed ranges [lo[i], hi[i]] in fp32 (host or device).  A NaN bound makes
 * that query's range empty (every result is padding).  Infinite bounds are allowed. */
grab_status grab_search_range_f32(grab_index *ix, const float *queries, const float *lo, const float *hi, int64_t nq,
                                  int32_t k, int32_t beam, uint32_t *out_ids, float *out_dist);

/* grab_append_batch with attrs[m] fp32 (host or device).  GRAB_EINVAL, with nothing written, if an
 * attribute is NaN. */
grab_status grab_append_batch_f32(grab_index *ix, const float *vectors, const float *attrs, int64_t m);

/* Measurement aid (no passage of the paper: it prices the memory system, not the method).
 * `waves` wavefronts each read `batches` batches of whole vector rows of the index at
 * pseudo-random slots, eight lanes per row as the distance evaluation of Algorithm 2 reads them,
 * and do nothing else.  *ms (host) = duration of that launch measured with HIP events on the
 * index's stream, *bytes (host) = rows read x row size.  bytes / ms is the rate the device
 * sustains for random rows of this size over this index's footprint: the practical ceiling of
 * the gathered distance evaluation, to be read beside the HBM peak.  Waits for the launch.
 * Needs grab_build_buckets before it; invalidates grab_get_timing of an earlier search.
 * waves in 1..2^24, batches in 1..65536, else GRAB_EINVAL. */
grab_status grab_probe_gather(grab_index *ix, int64_t waves, int32_t batches, float *ms, double *bytes);

#ifdef __cplusplus
}
#endif
#endif /* GRAB_H */
