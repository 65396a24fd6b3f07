// grab_search_range_noalloc: the search entry point for callers that cannot allocate (code
// under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same kernels
// as grab_search_range; the per-batch work buffers those kernels need (query plans, seed slots,
// counters, the launch order) live in one file-scope device array instead of grow-only
// allocations.
//
// The array's name is a host-side stand-in, not a device address: host code asks the runtime
// for the device address once per device (hipGetSymbolAddress with that device current) and
// hands kernels that pointer, exactly as the allocating entry point hands them its buffers.
#include "grab_internal.h"

namespace {

constexpr int64_t NOALLOC_MAX_NQ = 16384;                 // queries per call
constexpr int64_t NOALLOC_MAX_SEED_WORDS = 4ll << 20;     // nq * n_seeds
constexpr int NOALLOC_MAX_DEVICES = 64;

// carve-up of the array, every part 256-byte aligned
constexpr size_t OFF_PLANS = 0;
constexpr size_t SZ_PLANS = (size_t)NOALLOC_MAX_NQ * sizeof(QueryPlan);
constexpr size_t OFF_COUNTERS = OFF_PLANS + SZ_PLANS;
constexpr size_t SZ_COUNTERS = (size_t)NOALLOC_MAX_NQ * 8 * 4;
constexpr size_t OFF_QBIN = OFF_COUNTERS + SZ_COUNTERS;
constexpr size_t SZ_Q32 = (size_t)NOALLOC_MAX_NQ * 4;
constexpr size_t OFF_QRANK = OFF_QBIN + SZ_Q32;
constexpr size_t OFF_ORDER = OFF_QRANK + SZ_Q32;
constexpr size_t SZ_ORDER = (size_t)(NOALLOC_MAX_NQ + 2048) * 4;   // nq rounded up to eight short runs
constexpr size_t OFF_BINS = OFF_ORDER + SZ_ORDER;
constexpr size_t SZ_BINS = (GRAB_BIN_BLOCK_BYTES + 255) / 256 * 256;   // the counter block of the launch order
constexpr size_t OFF_SEEDS = OFF_BINS + SZ_BINS;
constexpr size_t SZ_SEEDS = (size_t)NOALLOC_MAX_SEED_WORDS * 4;
constexpr size_t SCRATCH_BYTES = OFF_SEEDS + SZ_SEEDS;            // about 18 MiB per GPU
static_assert(OFF_COUNTERS % 256 == 0 && OFF_QBIN % 256 == 0 && OFF_QRANK % 256 == 0 && OFF_ORDER % 256 == 0 &&
              OFF_BINS % 256 == 0 && OFF_SEEDS % 256 == 0, "parts must stay 256-byte aligned");

static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

// device address of `scratch` on each device, filled on first use with that device current
unsigned char *g_scratch_ptr[NOALLOC_MAX_DEVICES];

}  // namespace

grab_status grab_scratch_init(grab_index *ix, unsigned char **out) {
    int dev = -1;
    GRAB_HIP(ix, hipGetDevice(&dev));
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return grab_fail(ix, GRAB_EHIP, "device ordinal %d out of range", dev);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        GRAB_HIP(ix, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return grab_fail(ix, GRAB_EHIP, "the runtime gave no address for the work array");
        g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    if (out) *out = g_scratch_ptr[dev];
    return GRAB_OK;
}

extern "C" grab_status grab_search_range_noalloc(grab_index *ix, const float *queries, const int32_t *lo, const int32_t *hi,
                                                 int64_t nq, int32_t k, int32_t beam, uint32_t *out_ids, float *out_dist) {
    if (!ix) return GRAB_EINVAL;
    if (!ix->has_graph) return grab_fail(ix, GRAB_ESTATE, "no graph loaded");
    if (nq < 0) return grab_fail(ix, GRAB_EINVAL, "bad query count");
    SearchLaunch s;
    grab_status st = grab_resolve_search(ix, k, beam, s);
    if (st != GRAB_OK) return st;
    if (nq > NOALLOC_MAX_NQ)
        return grab_fail(ix, GRAB_EINVAL, "%lld queries exceed the %lld this entry point has room for", (long long)nq,
                         (long long)NOALLOC_MAX_NQ);
    if (nq * (int64_t)s.n_seeds > NOALLOC_MAX_SEED_WORDS)
        return grab_fail(ix, GRAB_EINVAL, "%lld queries x %d seeds exceed the %lld seed slots this entry point has room for",
                         (long long)nq, s.n_seeds, (long long)NOALLOC_MAX_SEED_WORDS);
    if (nq == 0) { ix->last_nq = 0; return GRAB_OK; }
    if (!queries || !lo || !hi || !out_ids || !out_dist) return grab_fail(ix, GRAB_EINVAL, "null argument");
    if (!grab_is_device_ptr(queries) || !grab_is_device_ptr(lo) || !grab_is_device_ptr(hi) || !grab_is_device_ptr(out_ids) ||
        !grab_is_device_ptr(out_dist))
        return grab_fail(ix, GRAB_EINVAL, "this entry point takes device pointers only (staging host buffers would allocate)");
    unsigned char *base = nullptr;
    if ((st = grab_scratch_init(ix, &base)) != GRAB_OK) return st;
    s.nq = nq;
    s.queries = queries; s.lo = lo; s.hi = hi;
    s.plans = reinterpret_cast<QueryPlan *>(base + OFF_PLANS);
    s.seeds = reinterpret_cast<uint32_t *>(base + OFF_SEEDS);
    s.counters = reinterpret_cast<uint32_t *>(base + OFF_COUNTERS);
    s.out_ids = out_ids; s.out_dist = out_dist;
    if (nq >= 2048) {   // the launch order of grab_search_range, in the same parts of the array every time
        s.q_bin = reinterpret_cast<int32_t *>(base + OFF_QBIN);
        s.q_rank = reinterpret_cast<int32_t *>(base + OFF_QRANK);
        s.bin_count = reinterpret_cast<int32_t *>(base + OFF_BINS);
        s.order = reinterpret_cast<uint32_t *>(base + OFF_ORDER);
        s.order_len = grab_order_len(nq);
        s.order_dirty = nullptr;   // the array is shared by every handle on this GPU: one counter block,
        s.order_block = nullptr;   // cleared before each use
    }
    ix->timed = false;
    if (ix->profile) GRAB_HIP(ix, hipEventRecord(ix->ev[0], ix->stream));
    // the bin counters are cleared before use and every entry of the order is written; plans, seeds
    // and counters are written in full for queries 0..nq-1 and nothing beyond is read
    if ((st = grab_launch_select(ix, s)) != GRAB_OK) return st;
    if (ix->profile) GRAB_HIP(ix, hipEventRecord(ix->ev[1], ix->stream));
    if ((st = grab_launch_beam(ix, s)) != GRAB_OK) return st;
    if (ix->profile) { GRAB_HIP(ix, hipEventRecord(ix->ev[2], ix->stream)); ix->timed = true; }
    ix->last_nq = nq;
    ix->last_counters = s.counters;
    return GRAB_OK;
}
