// Internal declarations shared by the translation units of libgrab.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "grab.h"

#define GRAB_EMPTY 0xFFFFFFFFu
#define GRAB_MAX_BUCKETS 1024
#define GRAB_MAX_BEAM 512
#define GRAB_MAX_CAND 512   // search_width * degree, and the seed chunk size
#define GRAB_WAVE 64
// counter block of the search's launch order: one 128-byte line per bin, one more for the tail
#define GRAB_BIN_STRIDE 32
#define GRAB_BIN_BLOCK_WORDS (GRAB_BIN_STRIDE * (GRAB_MAX_BUCKETS + 2))
#define GRAB_BIN_BLOCK_BYTES ((size_t)GRAB_BIN_BLOCK_WORDS * 4)
// Fence of a bucket: every GRAB_FENCE-th attribute of its sorted prefix, in one array for all
// buckets; bucket b's entries start at grab_fence_offset(base of the bucket's slab, b) and never
// reach the next bucket's (a slab of c slots holds at most c / GRAB_FENCE + 1 entries).
#define GRAB_FENCE 128
__host__ __device__ inline int64_t grab_fence_offset(int64_t slab_base, int32_t b) { return slab_base / GRAB_FENCE + b; }

// The vector lengths the kernels are built for, in 32-float (128-byte) units: every kernel that
// reads feature rows is instantiated once per entry, so that a whole row's loads can be issued
// before the first multiply.  grab_create refuses any other length.
#define GRAB_FOR_EACH_NCH(X) X(1) X(2) X(3) X(4) X(5) X(6) X(8) X(12) X(16) X(20) X(24) X(30) X(32) X(48) X(64)
#define GRAB_DIM_LIST "32, 64, 96, 128, 160, 192, 256, 384, 512, 640, 768, 960, 1024, 1536, 2048"
inline bool grab_dim_supported(int dim) {
    if (dim % 32) return false;
    switch (dim / 32) {
#define GRAB_DIM_CASE(N) case N:
        GRAB_FOR_EACH_NCH(GRAB_DIM_CASE)
#undef GRAB_DIM_CASE
        return true;
        default: return false;
    }
}

// bucket table columns (Section 4.2.4: the bucket<->index metadata)
enum { T_BASE = 0, T_NSORT = 1, T_NTOT = 2, T_CAP = 3, T_MIN = 4, T_MAX = 5, T_COLS = 6 };

// What the select kernel hands to the beam kernel for one query: the bucket run and the
// slot intervals that decide the scalar pre-check without reading an attribute.
struct QueryPlan {
    int32_t b0, b1;    // selected bucket run; b1 < b0: the range meets no bucket
    int32_t V;         // seed population size
    int32_t n_seeds;   // seeds written for this query
    int32_t s0, e0;    // valid sorted slots of bucket b0
    int32_t t0s, t0e;  // appended tail of b0: attribute must be read
    int32_t ms, e1;    // buckets after b0 up to the valid sorted end of b1: all valid
    int32_t t1s, t1e;  // appended tail of b1 (b1 > b0): attribute must be read
    int32_t first_valid, end_valid;
    int32_t pad0, pad1;
};

struct SearchParams {
    int32_t search_width = 1;
    int32_t max_iter = 0;      // 0: 2 * beam
    int32_t n_seeds = 0;       // 0: min(beam, 64)
    int32_t visited_cap = 2800;
    uint32_t seed_salt = 0;
    float alpha = 0.6f;
    int32_t append_beam = 64;
    int32_t remote_mode = 0;      // 0: remote entry j belongs to the j-th target bucket; 1: proximal / global split
    int32_t n_proximal = -1;      // mode 1: remote positions for proximal candidates; -1: ceil(k_remote / 2)
    double remote_window = 0.2;   // mode 1: proximal = attribute within this fraction of the attribute span
    int32_t append_remote_cands = 0;  // mode 0 insertion: candidates whose remote entries are looked at; 0: all
};

// the remote wiring in force for one construction or insertion call (Section 4.3, Remote Edge Construction)
struct RemoteRule {
    int32_t mode, n_proximal;
    int64_t window;
};
RemoteRule grab_remote_rule(const grab_index *ix, int32_t kr);

struct DevBuf {
    void *p = nullptr;
    size_t bytes = 0;
};

struct grab_index {
    int32_t dim = 0;
    int32_t metric = 0;
    hipStream_t stream = nullptr;
    std::string err;

    // layout (device)
    int64_t n = 0;        // objects
    int64_t n_slots = 0;  // physical rows
    int32_t B = 0;
    float *X = nullptr;          // [n_slots][dim]
    int32_t *attr = nullptr;     // [n_slots]
    int32_t *fence = nullptr;    // every GRAB_FENCE-th attribute of each bucket's sorted prefix (see k_fence)
    uint32_t *slot2id = nullptr; // [n_slots]
    uint32_t *id2slot = nullptr; // [n_slots] (ids grow up to the slot count)
    int32_t *table = nullptr;    // [B][6] device copy
    int32_t *h_table = nullptr;  // host copy (pinned), followed by B + 4 words that insertion reads results into

    // graph (device)
    int32_t kl = 0, kr = 0;
    uint32_t *A = nullptr;       // [n_slots][kl+kr]
    bool has_graph = false;

    SearchParams prm;

    // grow-only work buffers
    DevBuf plans, seeds, counters, stage_q, stage_lo, stage_hi, stage_ids, stage_dist, stage_misc, flags;
    // float attributes: staged floats, their int32 images, the NaN flag
    DevBuf stage_fa, stage_flo, stage_fhi, conv_a, conv_lo, conv_hi, attr_flag;
    // launch order of the queries of a search (grab_plan_order)
    DevBuf q_bin, q_rank, q_order, bin_count;
    int64_t last_nq = 0;
    bool order_dirty = true;     // the bin counters of the launch order may not be zero
    int order_block = 0;         // which of the two counter blocks the next counted launch order uses
    const uint32_t *last_counters = nullptr;   // where the most recent search wrote its counters
    std::vector<DevBuf> app;     // append's work arena
    DevBuf app_stats;            // work counters of the last insertion (12 x uint64)
    bool app_has_stats = false, app_timed = false;
    hipEvent_t app_ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    hipEvent_t sync_ev = nullptr;   // lets the host wait for one copy while later kernels are already queued

    bool profile = false;
    bool timed = false;          // the last search recorded events
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
};

// error plumbing ------------------------------------------------------------------------
grab_status grab_fail(grab_index *ix, grab_status st, const char *fmt, ...);
#define GRAB_HIP(ix, call)                                                                     \
    do {                                                                                       \
        hipError_t e__ = (call);                                                               \
        if (e__ != hipSuccess)                                                                 \
            return grab_fail((ix), e__ == hipErrorOutOfMemory ? GRAB_ENOMEM : GRAB_EHIP,       \
                             "%s failed: %s", #call, hipGetErrorString(e__));                  \
    } while (0)

bool grab_is_device_ptr(const void *p);
grab_status grab_reserve(grab_index *ix, DevBuf &b, size_t bytes);
// returns a device view of `src` (copying from host through `stage` when needed)
grab_status grab_to_device(grab_index *ix, const void *src, size_t bytes, DevBuf &stage, const void **out);

// kernels' host launchers -----------------------------------------------------------------
// layout
grab_status grab_launch_build(grab_index *ix, const float *d_vectors, const int32_t *d_attrs,
                              int64_t n, int32_t B, int64_t slack);
grab_status grab_launch_load_graph(grab_index *ix, const uint32_t *d_local, int32_t kl,
                                   const uint32_t *d_remote, int32_t kr, int32_t *d_err);
// search
struct SearchLaunch {
    const float *queries;   // device [nq][dim]
    const int32_t *lo, *hi; // device [nq]
    // device [nq] or nullptr: the scope of each query when it is not an attribute range (candidate
    // searches of insertion and construction): b >= 0 = the slots of bucket b's slab, -2 - b = every
    // slot outside it, INT32_MIN = nothing (a row without an object)
    const int32_t *only_bucket;
    const uint32_t *adj = nullptr;   // adjacency to walk instead of the index's own (construction's snapshot)
    int64_t nq;
    int32_t k, beam, width, max_iter, n_seeds, visited_cap;
    uint32_t salt;
    QueryPlan *plans;   // device [nq]
    uint32_t *seeds;    // device [nq][n_seeds]
    uint32_t *counters; // device [nq][8]
    uint32_t *out_ids;  // device [nq][k] (external ids, or slots when out_slots)
    float *out_dist;    // device [nq][k]
    bool out_slots;
    // launch order (all nullptr: query i runs in workgroup i): see grab_plan_order
    int32_t *q_bin = nullptr, *q_rank = nullptr;
    // counters of the bins: two blocks of GRAB_BIN_BLOCK_BYTES used in turn (order_block says which
    // is next; each k_order clears the block of the call before), or one block that is cleared
    // before every use (order_block null)
    int32_t *bin_count = nullptr;
    int *order_block = nullptr;
    uint32_t *order = nullptr;   // [order_len]: query of each workgroup, GRAB_EMPTY for none
    int64_t order_len = 0;
    bool *order_dirty = nullptr; // host flag: bin_count may not be zero (null: always clear it first)
    // device [nq] or nullptr: the queries already listed by bin (a batch sorted by the bucket it is
    // scoped to); the launch order is then read off this list and nothing is counted
    const uint32_t *sorted_queries = nullptr;
};
// Reserves the buffers that let the search run its queries grouped by first selected bucket, one
// contiguous run of that order per XCD (queries that read the same buckets then share L2 and the
// Infinity Cache); fills the order fields of `s`, or leaves them null for small batches.
grab_status grab_plan_order(grab_index *ix, SearchLaunch &s);
// entries of the launch-order array for a batch of nq queries (nq >= 2048)
int64_t grab_order_len(int64_t nq);
// fills the parameter fields of `s` from the index's tunables for (k, beam); validates them
grab_status grab_resolve_search(grab_index *ix, int32_t k, int32_t beam, SearchLaunch &s);
// device address, on the current device, of the static work array of grab_search_range_noalloc
grab_status grab_scratch_init(grab_index *ix, unsigned char **out);
grab_status grab_launch_select(grab_index *ix, const SearchLaunch &s);
grab_status grab_launch_beam(grab_index *ix, const SearchLaunch &s);
// measurement aid: `waves` wavefronts each read `batches` batches of random rows; *bytes = rows read x row size
grab_status grab_launch_gather_probe(grab_index *ix, int64_t waves, int32_t batches, float *sink, double *bytes);
// append: the whole insertion for m objects already on the device; `proto` carries the search
// parameters resolved for beam = append_beam
// construction: fills ix->A (already allocated for kl+kr entries per slot)
grab_status grab_build_graph_device(grab_index *ix, int32_t kl, int32_t kr, int32_t pool, const SearchLaunch &proto);
// pass 2 alone on the graph the index holds; `proto` as for append
grab_status grab_build_remote_device(grab_index *ix, const SearchLaunch &proto);
grab_status grab_append_device(grab_index *ix, const float *d_vecs, const int32_t *d_attrs, int64_t m,
                               const SearchLaunch &proto);
// construction's nearest-neighbour passes as a matrix-core filter with an exact re-rank (grab_knn.hip)
struct KnnFilter;
grab_status grab_knn_prepare(grab_index *ix, KnnFilter **out);
void grab_knn_release(KnnFilter *f);
grab_status grab_knn_pass(grab_index *ix, KnnFilter *f, const int32_t *d_tgt, uint32_t *out_s, float *out_d, int64_t out_stride,
                          int64_t out_off, int32_t P, int32_t exclude_self, bool *overflow);
