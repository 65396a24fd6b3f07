// C ABI of libgrab.so: argument checking, device arenas, and the order of kernel launches.
// Every computation happens in the kernels of grab_layout.hip / grab_search.hip /
// grab_append.hip; this file only validates, allocates and enqueues.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>

#include "grab_internal.h"

grab_status grab_fail(grab_index *ix, grab_status st, const char *fmt, ...) {
    if (ix) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof(buf), fmt, ap);
        va_end(ap);
        ix->err = buf;
    }
    return st;
}

bool grab_is_device_ptr(const void *p) {
    hipPointerAttribute_t at;
    memset(&at, 0, sizeof(at));
    hipError_t e = hipPointerGetAttributes(&at, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();  // an ordinary host pointer is reported as an error on some runtimes
        return false;
    }
    return at.type == hipMemoryTypeDevice || at.type == hipMemoryTypeManaged;
}

grab_status grab_reserve(grab_index *ix, DevBuf &b, size_t bytes) {
    if (bytes <= b.bytes) return GRAB_OK;
    if (b.p) {
        GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
        GRAB_HIP(ix, hipFree(b.p));
        b.p = nullptr;
        b.bytes = 0;
    }
    size_t want = bytes + bytes / 4;
    GRAB_HIP(ix, hipMalloc(&b.p, want));
    b.bytes = want;
    return GRAB_OK;
}

grab_status grab_to_device(grab_index *ix, const void *src, size_t bytes, DevBuf &stage, const void **out) {
    if (grab_is_device_ptr(src)) {
        *out = src;
        return GRAB_OK;
    }
    grab_status st = grab_reserve(ix, stage, bytes);
    if (st != GRAB_OK) return st;
    GRAB_HIP(ix, hipMemcpyAsync(stage.p, src, bytes, hipMemcpyHostToDevice, ix->stream));
    *out = stage.p;
    return GRAB_OK;
}

static void free_buf(DevBuf &b) {
    if (b.p) (void)hipFree(b.p);
    b.p = nullptr;
    b.bytes = 0;
}

static void drop_layout(grab_index *ix) {
    (void)hipFree(ix->X); (void)hipFree(ix->attr); (void)hipFree(ix->slot2id); (void)hipFree(ix->id2slot);
    (void)hipFree(ix->table); (void)hipFree(ix->A); (void)hipFree(ix->fence);
    if (ix->h_table) (void)hipHostFree(ix->h_table);
    ix->fence = nullptr;
    ix->order_dirty = true;   // another bucket count: the launch order's counters are cleared before their next use
    ix->X = nullptr; ix->attr = nullptr; ix->slot2id = nullptr; ix->id2slot = nullptr; ix->table = nullptr;
    ix->A = nullptr; ix->h_table = nullptr;
    ix->n = ix->n_slots = 0; ix->B = 0; ix->kl = ix->kr = 0; ix->has_graph = false;
}

static grab_status check_remote_rule(grab_index *ix) {
    if (ix->prm.remote_mode == 1 && ix->prm.n_proximal > ix->kr)
        return grab_fail(ix, GRAB_EINVAL, "n_proximal %d exceeds k_remote %d", ix->prm.n_proximal, ix->kr);
    return GRAB_OK;
}

RemoteRule grab_remote_rule(const grab_index *ix, int32_t kr) {
    RemoteRule r;
    r.mode = ix->prm.remote_mode;
    r.n_proximal = ix->prm.n_proximal >= 0 ? ix->prm.n_proximal : (kr + 1) / 2;
    if (r.n_proximal > kr) r.n_proximal = kr;
    // attribute span of the index now, from the host copy of the bucket table
    const double span = ix->B > 0 ? (double)((int64_t)ix->h_table[T_COLS * (ix->B - 1) + T_MAX] - (int64_t)ix->h_table[T_MIN]) : 0.0;
    r.window = (int64_t)__builtin_floor(ix->prm.remote_window * span);
    return r;
}

grab_status grab_resolve_search(grab_index *ix, int32_t k, int32_t beam, SearchLaunch &s) {
    const SearchParams &p = ix->prm;
    if (k < 1 || beam < k || beam > GRAB_MAX_BEAM) return grab_fail(ix, GRAB_EINVAL, "need 1 <= k <= beam <= %d", GRAB_MAX_BEAM);
    s.k = k; s.beam = beam;
    s.width = p.search_width;
    s.max_iter = p.max_iter > 0 ? p.max_iter : 2 * beam;
    s.n_seeds = p.n_seeds > 0 ? p.n_seeds : (beam < 64 ? beam : 64);
    s.visited_cap = p.visited_cap;
    s.salt = p.seed_salt;
    if (s.n_seeds > s.visited_cap) return grab_fail(ix, GRAB_EINVAL, "n_seeds %d exceeds visited_cap %d", s.n_seeds, s.visited_cap);
    if (s.width * (ix->kl + ix->kr) > GRAB_MAX_CAND) return grab_fail(ix, GRAB_EINVAL, "search_width * degree exceeds %d", GRAB_MAX_CAND);
    s.only_bucket = nullptr;
    s.out_slots = false;
    return GRAB_OK;
}

extern "C" {

grab_status grab_create(grab_index **out, int32_t dim, int32_t metric, void *hip_stream) {
    if (!out) return GRAB_EINVAL;
    *out = nullptr;
    if (!grab_dim_supported(dim)) return GRAB_EINVAL;   // one of GRAB_DIM_LIST
    if (metric != GRAB_L2SQ && metric != GRAB_IP) return GRAB_EINVAL;
    grab_index *ix = new (std::nothrow) grab_index();
    if (!ix) return GRAB_ENOMEM;
    ix->dim = dim;
    ix->metric = metric;
    ix->stream = (hipStream_t)hip_stream;
    // with a device present: look up, once per device, where grab_search_range_noalloc's static
    // work array lives on it (a host without a GPU can still create and destroy handles)
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess) { (void)hipGetLastError(); n_dev = 0; }
    if (n_dev > 0 && grab_scratch_init(ix, nullptr) != GRAB_OK) {
        delete ix;
        return GRAB_EHIP;
    }
    *out = ix;
    return GRAB_OK;
}

void grab_destroy(grab_index *ix) {
    if (!ix) return;
    (void)hipStreamSynchronize(ix->stream);
    drop_layout(ix);
    DevBuf *bufs[] = {&ix->plans, &ix->seeds, &ix->counters, &ix->stage_q, &ix->stage_lo, &ix->stage_hi,
                      &ix->stage_ids, &ix->stage_dist, &ix->stage_misc, &ix->flags, &ix->stage_fa, &ix->stage_flo,
                      &ix->stage_fhi, &ix->conv_a, &ix->conv_lo, &ix->conv_hi, &ix->attr_flag, &ix->q_bin, &ix->q_rank,
                      &ix->q_order, &ix->bin_count, &ix->app_stats};
    for (DevBuf *b : bufs) free_buf(*b);
    for (DevBuf &b : ix->app) free_buf(b);
    for (hipEvent_t e : ix->ev)
        if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : ix->app_ev)
        if (e) (void)hipEventDestroy(e);
    if (ix->sync_ev) (void)hipEventDestroy(ix->sync_ev);
    delete ix;
}

const char *grab_last_error(const grab_index *ix) { return ix ? ix->err.c_str() : "null index"; }

grab_status grab_set_param(grab_index *ix, int32_t which, double value) {
    if (!ix) return GRAB_EINVAL;
    SearchParams &p = ix->prm;
    switch (which) {
        case GRAB_P_SEARCH_WIDTH:
            if (value < 1 || value > 8) return grab_fail(ix, GRAB_EINVAL, "search_width must be 1..8");
            p.search_width = (int32_t)value; return GRAB_OK;
        case GRAB_P_MAX_ITER:
            if (value < 0 || value > 1e6) return grab_fail(ix, GRAB_EINVAL, "max_iter must be 0..1e6");
            p.max_iter = (int32_t)value; return GRAB_OK;
        case GRAB_P_N_SEEDS:
            if (value < 0 || value > 24000) return grab_fail(ix, GRAB_EINVAL, "n_seeds must be 0..24000");
            p.n_seeds = (int32_t)value; return GRAB_OK;
        case GRAB_P_VISITED_CAP:
            if (value < 1 || value > 24000) return grab_fail(ix, GRAB_EINVAL, "visited_cap must be 1..24000");
            p.visited_cap = (int32_t)value; return GRAB_OK;
        case GRAB_P_SEED_SALT:
            if (value < 0 || value > 4294967295.0) return grab_fail(ix, GRAB_EINVAL, "seed_salt must fit 32 bits");
            p.seed_salt = (uint32_t)value; return GRAB_OK;
        case GRAB_P_ALPHA:
            if (!(value > 0.0 && value <= 1.0)) return grab_fail(ix, GRAB_EINVAL, "alpha must be in (0, 1]");
            p.alpha = (float)value; return GRAB_OK;
        case GRAB_P_APPEND_BEAM:
            if (value < 1 || value > GRAB_MAX_BEAM) return grab_fail(ix, GRAB_EINVAL, "append_beam must be 1..512");
            p.append_beam = (int32_t)value; return GRAB_OK;
        case GRAB_P_PROFILE:
            if (value != 0.0 && value != 1.0) return grab_fail(ix, GRAB_EINVAL, "profile must be 0 or 1");
            if (value == 1.0) {
                for (hipEvent_t &e : ix->ev)
                    if (!e) GRAB_HIP(ix, hipEventCreate(&e));
                for (hipEvent_t &e : ix->app_ev)
                    if (!e) GRAB_HIP(ix, hipEventCreate(&e));
            }
            ix->profile = value == 1.0; return GRAB_OK;
        case GRAB_P_REMOTE_MODE:
            if (value != 0.0 && value != 1.0) return grab_fail(ix, GRAB_EINVAL, "remote_mode must be 0 or 1");
            p.remote_mode = (int32_t)value; return GRAB_OK;
        case GRAB_P_N_PROXIMAL:
            if (value < -1 || value > 64 || value != (double)(int32_t)value) return grab_fail(ix, GRAB_EINVAL, "n_proximal must be -1..64");
            p.n_proximal = (int32_t)value; return GRAB_OK;
        case GRAB_P_APPEND_REMOTE_CANDS:
            if (value < 0 || value > GRAB_MAX_BEAM || value != (double)(int32_t)value) return grab_fail(ix, GRAB_EINVAL, "append_remote_cands must be 0..512");
            p.append_remote_cands = (int32_t)value; return GRAB_OK;
        case GRAB_P_REMOTE_WINDOW:
            if (!(value >= 0.0 && value <= 1.0)) return grab_fail(ix, GRAB_EINVAL, "remote_window must be in [0, 1]");
            p.remote_window = value; return GRAB_OK;
        default:
            return grab_fail(ix, GRAB_EINVAL, "unknown parameter %d", which);
    }
}

grab_status grab_build_buckets(grab_index *ix, const float *vectors, const int32_t *attrs, int64_t n,
                               int32_t n_buckets, int64_t n_cap) {
    if (!ix) return GRAB_EINVAL;
    if (!vectors || !attrs) return grab_fail(ix, GRAB_EINVAL, "null input");
    if (n_buckets < 1 || n_buckets > GRAB_MAX_BUCKETS) return grab_fail(ix, GRAB_EINVAL, "n_buckets must be 1..%d", GRAB_MAX_BUCKETS);
    if (n < n_buckets || n_cap < n || n_cap >= (1ll << 31)) return grab_fail(ix, GRAB_EINVAL, "need n_buckets <= n <= n_cap < 2^31");
    if (n_cap * (int64_t)(ix->dim / 4) > (1ll << 38)) return grab_fail(ix, GRAB_EINVAL, "n_cap * dim exceeds 2^40 elements");
    GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    drop_layout(ix);
    const int64_t slack = (n_cap - n) / n_buckets;
    const int64_t n_slots = n + slack * n_buckets;
    const size_t row = (size_t)ix->dim * sizeof(float);
    auto fail = [&](grab_status st) { drop_layout(ix); return st; };
#define B_HIP(call)                                                                                         \
    do {                                                                                                    \
        hipError_t e__ = (call);                                                                            \
        if (e__ != hipSuccess)                                                                              \
            return fail(grab_fail(ix, e__ == hipErrorOutOfMemory ? GRAB_ENOMEM : GRAB_EHIP, "%s failed: %s", \
                                  #call, hipGetErrorString(e__)));                                          \
    } while (0)
    B_HIP(hipMalloc((void **)&ix->X, n_slots * row));
    B_HIP(hipMalloc((void **)&ix->attr, n_slots * 4));
    B_HIP(hipMalloc((void **)&ix->slot2id, n_slots * 4));
    B_HIP(hipMalloc((void **)&ix->id2slot, n_slots * 4));
    B_HIP(hipMalloc((void **)&ix->table, sizeof(int32_t) * T_COLS * n_buckets));
    B_HIP(hipMalloc((void **)&ix->fence, sizeof(int32_t) * (size_t)(n_slots / GRAB_FENCE + n_buckets + 1)));
    B_HIP(hipHostMalloc((void **)&ix->h_table, sizeof(int32_t) * ((size_t)T_COLS * n_buckets + n_buckets + 4), hipHostMallocDefault));
    B_HIP(hipMemsetAsync(ix->X, 0, n_slots * row, ix->stream));
    B_HIP(hipMemsetAsync(ix->attr, 0, n_slots * 4, ix->stream));
    B_HIP(hipMemsetAsync(ix->slot2id, 0xFF, n_slots * 4, ix->stream));
    B_HIP(hipMemsetAsync(ix->id2slot, 0xFF, n_slots * 4, ix->stream));
#undef B_HIP
    ix->n = n; ix->n_slots = n_slots; ix->B = n_buckets;
    DevBuf tmp_v, tmp_a;
    const void *dv = nullptr, *da = nullptr;
    grab_status st = grab_to_device(ix, vectors, n * row, tmp_v, &dv);
    if (st == GRAB_OK) st = grab_to_device(ix, attrs, n * 4, tmp_a, &da);
    if (st == GRAB_OK) st = grab_launch_build(ix, (const float *)dv, (const int32_t *)da, n, n_buckets, slack);
    (void)hipStreamSynchronize(ix->stream);
    free_buf(tmp_v);
    free_buf(tmp_a);
    if (st != GRAB_OK) return fail(st);
    return GRAB_OK;
}

grab_status grab_load_graph(grab_index *ix, const uint32_t *local_adj, int32_t k_local, const uint32_t *remote_adj,
                            int32_t k_remote) {
    if (!ix) return GRAB_EINVAL;
    if (!ix->X) return grab_fail(ix, GRAB_ESTATE, "build_buckets first");
    if (k_local < 0 || k_remote < 0 || k_local + k_remote < 1 || k_local + k_remote > 128)
        return grab_fail(ix, GRAB_EINVAL, "k_local + k_remote must be 1..128");
    if ((k_local > 0 && !local_adj) || (k_remote > 0 && !remote_adj)) return grab_fail(ix, GRAB_EINVAL, "null adjacency");
    GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    ix->has_graph = false;
    (void)hipFree(ix->A);
    ix->A = nullptr;
    const int32_t K = k_local + k_remote;
    GRAB_HIP(ix, hipMalloc((void **)&ix->A, (size_t)ix->n_slots * K * 4));
    GRAB_HIP(ix, hipMemsetAsync(ix->A, 0xFF, (size_t)ix->n_slots * K * 4, ix->stream));
    DevBuf tmp_l, tmp_r;
    const void *dl = nullptr, *dr = nullptr;
    grab_status st = GRAB_OK;
    if (k_local > 0) st = grab_to_device(ix, local_adj, (size_t)ix->n * k_local * 4, tmp_l, &dl);
    if (st == GRAB_OK && k_remote > 0) st = grab_to_device(ix, remote_adj, (size_t)ix->n * k_remote * 4, tmp_r, &dr);
    int32_t h_err[3] = {0, 0, 0};
    if (st == GRAB_OK) st = grab_reserve(ix, ix->flags, 64);
    if (st == GRAB_OK) {
        hipError_t e = hipMemsetAsync(ix->flags.p, 0, 64, ix->stream);
        if (e != hipSuccess) st = grab_fail(ix, GRAB_EHIP, "memset failed: %s", hipGetErrorString(e));
    }
    if (st == GRAB_OK)
        st = grab_launch_load_graph(ix, (const uint32_t *)dl, k_local, (const uint32_t *)dr, k_remote, (int32_t *)ix->flags.p);
    if (st == GRAB_OK) {
        hipError_t e = hipMemcpyAsync(h_err, ix->flags.p, sizeof(h_err), hipMemcpyDeviceToHost, ix->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ix->stream);
        if (e != hipSuccess) st = grab_fail(ix, GRAB_EHIP, "load_graph failed: %s", hipGetErrorString(e));
    }
    (void)hipStreamSynchronize(ix->stream);
    free_buf(tmp_l);
    free_buf(tmp_r);
    if (ix->prm.remote_mode == 1) h_err[2] = 0;   // that reading keeps redundant local edges in the remote part
    if (st == GRAB_OK && (h_err[0] || h_err[1] || h_err[2]))
        st = grab_fail(ix, GRAB_EINVAL, "malformed graph: %d ids out of range, %d local edges leave their bucket, %d remote edges stay in it",
                       h_err[0], h_err[1], h_err[2]);
    if (st != GRAB_OK) {
        (void)hipFree(ix->A);
        ix->A = nullptr;
        return st;
    }
    ix->kl = k_local; ix->kr = k_remote; ix->has_graph = true;
    return GRAB_OK;
}

grab_status grab_build_graph(grab_index *ix, int32_t k_local, int32_t k_remote, int32_t pool) {
    if (!ix) return GRAB_EINVAL;
    if (!ix->X) return grab_fail(ix, GRAB_ESTATE, "build_buckets first");
    if (k_local < 1 || k_local > 64 || k_remote < 0 || k_remote > 64) return grab_fail(ix, GRAB_EINVAL, "need 1 <= k_local <= 64 and 0 <= k_remote <= 64");
    if (pool == 0) pool = 4 * k_local < 128 ? 4 * k_local : 128;
    if (pool < k_local || pool > 128) return grab_fail(ix, GRAB_EINVAL, "pool must be k_local..128");
    GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    ix->has_graph = false;
    (void)hipFree(ix->A);
    ix->A = nullptr;
    GRAB_HIP(ix, hipMalloc((void **)&ix->A, (size_t)ix->n_slots * (k_local + k_remote) * 4));
    ix->kl = k_local; ix->kr = k_remote;
    SearchLaunch proto;
    grab_status st = check_remote_rule(ix);
    if (st == GRAB_OK) st = grab_resolve_search(ix, ix->prm.append_beam, ix->prm.append_beam, proto);
    if (st == GRAB_OK) st = grab_build_graph_device(ix, k_local, k_remote, pool, proto);
    if (st != GRAB_OK) {
        (void)hipFree(ix->A);
        ix->A = nullptr;
        ix->kl = ix->kr = 0;
        return st;
    }
    ix->has_graph = true;
    return GRAB_OK;
}

grab_status grab_build_remote(grab_index *ix) {
    if (!ix) return GRAB_EINVAL;
    if (!ix->has_graph) return grab_fail(ix, GRAB_ESTATE, "no graph loaded");
    SearchLaunch proto;
    grab_status st = check_remote_rule(ix);
    if (st == GRAB_OK) st = grab_resolve_search(ix, ix->prm.append_beam, ix->prm.append_beam, proto);
    if (st != GRAB_OK) return st;
    GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    ix->timed = false;
    return grab_build_remote_device(ix, proto);
}

grab_status grab_search_range(grab_index *ix, const float *queries, const int32_t *lo, const int32_t *hi, int64_t nq,
                              int32_t k, int32_t beam, uint32_t *out_ids, float *out_dist) {
    if (!ix) return GRAB_EINVAL;
    if (!ix->has_graph) return grab_fail(ix, GRAB_ESTATE, "no graph loaded");
    if (nq < 0 || nq > (1ll << 30)) return grab_fail(ix, GRAB_EINVAL, "bad query count");
    SearchLaunch s;
    grab_status st = grab_resolve_search(ix, k, beam, s);
    if (st != GRAB_OK) return st;
    if (nq == 0) { ix->last_nq = 0; return GRAB_OK; }
    if (!queries || !lo || !hi || !out_ids || !out_dist) return grab_fail(ix, GRAB_EINVAL, "null argument");
    s.nq = nq;
    if ((st = grab_reserve(ix, ix->plans, nq * sizeof(QueryPlan))) != GRAB_OK) return st;
    if ((st = grab_reserve(ix, ix->seeds, (size_t)nq * s.n_seeds * 4)) != GRAB_OK) return st;
    if ((st = grab_reserve(ix, ix->counters, (size_t)nq * 8 * 4)) != GRAB_OK) return st;
    const void *dq, *dlo, *dhi;
    if ((st = grab_to_device(ix, queries, (size_t)nq * ix->dim * 4, ix->stage_q, &dq)) != GRAB_OK) return st;
    if ((st = grab_to_device(ix, lo, (size_t)nq * 4, ix->stage_lo, &dlo)) != GRAB_OK) return st;
    if ((st = grab_to_device(ix, hi, (size_t)nq * 4, ix->stage_hi, &dhi)) != GRAB_OK) return st;
    const bool ids_dev = grab_is_device_ptr(out_ids), dist_dev = grab_is_device_ptr(out_dist);
    if (!ids_dev && (st = grab_reserve(ix, ix->stage_ids, (size_t)nq * k * 4)) != GRAB_OK) return st;
    if (!dist_dev && (st = grab_reserve(ix, ix->stage_dist, (size_t)nq * k * 4)) != GRAB_OK) return st;
    s.queries = (const float *)dq; s.lo = (const int32_t *)dlo; s.hi = (const int32_t *)dhi;
    s.plans = (QueryPlan *)ix->plans.p; s.seeds = (uint32_t *)ix->seeds.p; s.counters = (uint32_t *)ix->counters.p;
    s.out_ids = ids_dev ? out_ids : (uint32_t *)ix->stage_ids.p;
    s.out_dist = dist_dev ? out_dist : (float *)ix->stage_dist.p;
    if ((st = grab_plan_order(ix, s)) != GRAB_OK) return st;
    ix->timed = false;
    if (ix->profile) GRAB_HIP(ix, hipEventRecord(ix->ev[0], ix->stream));
    if ((st = grab_launch_select(ix, s)) != GRAB_OK) return st;
    if (ix->profile) GRAB_HIP(ix, hipEventRecord(ix->ev[1], ix->stream));
    if ((st = grab_launch_beam(ix, s)) != GRAB_OK) return st;
    if (ix->profile) { GRAB_HIP(ix, hipEventRecord(ix->ev[2], ix->stream)); ix->timed = true; }
    ix->last_nq = nq;
    ix->last_counters = s.counters;
    if (!ids_dev) GRAB_HIP(ix, hipMemcpyAsync(out_ids, s.out_ids, (size_t)nq * k * 4, hipMemcpyDeviceToHost, ix->stream));
    if (!dist_dev) GRAB_HIP(ix, hipMemcpyAsync(out_dist, s.out_dist, (size_t)nq * k * 4, hipMemcpyDeviceToHost, ix->stream));
    if (!ids_dev || !dist_dev || dq != (const void *)queries || dlo != (const void *)lo || dhi != (const void *)hi)
        GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    return GRAB_OK;
}

grab_status grab_select_range(grab_index *ix, const int32_t *lo, const int32_t *hi, int64_t nq, int32_t beam,
                              int32_t *info, uint32_t *seeds) {
    if (!ix) return GRAB_EINVAL;
    if (!ix->X) return grab_fail(ix, GRAB_ESTATE, "build_buckets first");
    if (nq < 0) return grab_fail(ix, GRAB_EINVAL, "bad query count");
    SearchLaunch s;
    grab_status st = grab_resolve_search(ix, 1, beam, s);
    if (st != GRAB_OK) return st;
    if (nq == 0) return GRAB_OK;
    if (!lo || !hi || !info) return grab_fail(ix, GRAB_EINVAL, "null argument");
    s.nq = nq;
    if ((st = grab_reserve(ix, ix->plans, nq * sizeof(QueryPlan))) != GRAB_OK) return st;
    if ((st = grab_reserve(ix, ix->seeds, (size_t)nq * s.n_seeds * 4)) != GRAB_OK) return st;
    const void *dlo, *dhi;
    if ((st = grab_to_device(ix, lo, (size_t)nq * 4, ix->stage_lo, &dlo)) != GRAB_OK) return st;
    if ((st = grab_to_device(ix, hi, (size_t)nq * 4, ix->stage_hi, &dhi)) != GRAB_OK) return st;
    s.lo = (const int32_t *)dlo; s.hi = (const int32_t *)dhi;
    s.plans = (QueryPlan *)ix->plans.p; s.seeds = (uint32_t *)ix->seeds.p;
    if ((st = grab_launch_select(ix, s)) != GRAB_OK) return st;
    // gather the six reported fields on the host side of the boundary
    QueryPlan *hp = new (std::nothrow) QueryPlan[nq];
    if (!hp) return grab_fail(ix, GRAB_ENOMEM, "host allocation failed");
    hipError_t e = hipMemcpyAsync(hp, s.plans, nq * sizeof(QueryPlan), hipMemcpyDeviceToHost, ix->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ix->stream);
    if (e != hipSuccess) { delete[] hp; return grab_fail(ix, GRAB_EHIP, "copy failed: %s", hipGetErrorString(e)); }
    int32_t *hinfo = new (std::nothrow) int32_t[nq * 6];
    if (!hinfo) { delete[] hp; return grab_fail(ix, GRAB_ENOMEM, "host allocation failed"); }
    for (int64_t i = 0; i < nq; ++i) {
        hinfo[6 * i + 0] = hp[i].b0; hinfo[6 * i + 1] = hp[i].b1; hinfo[6 * i + 2] = hp[i].V;
        hinfo[6 * i + 3] = hp[i].first_valid; hinfo[6 * i + 4] = hp[i].end_valid; hinfo[6 * i + 5] = hp[i].n_seeds;
    }
    e = hipMemcpy(info, hinfo, nq * 6 * 4, grab_is_device_ptr(info) ? hipMemcpyHostToDevice : hipMemcpyHostToHost);
    delete[] hp;
    delete[] hinfo;
    if (e != hipSuccess) return grab_fail(ix, GRAB_EHIP, "copy failed: %s", hipGetErrorString(e));
    if (seeds) GRAB_HIP(ix, hipMemcpy(seeds, s.seeds, (size_t)nq * s.n_seeds * 4, hipMemcpyDefault));
    return GRAB_OK;
}

grab_status grab_get_sizes(const grab_index *ix, int64_t out[8]) {
    if (!ix || !out) return GRAB_EINVAL;
    out[0] = ix->n; out[1] = ix->n_slots; out[2] = ix->B; out[3] = ix->kl; out[4] = ix->kr;
    out[5] = ix->dim; out[6] = ix->metric; out[7] = ix->has_graph ? 1 : 0;
    return GRAB_OK;
}

grab_status grab_get_layout(grab_index *ix, int32_t *bucket_table, uint32_t *id2slot, uint32_t *slot2id) {
    if (!ix) return GRAB_EINVAL;
    if (!ix->X) return grab_fail(ix, GRAB_ESTATE, "build_buckets first");
    GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    if (bucket_table) GRAB_HIP(ix, hipMemcpy(bucket_table, ix->table, sizeof(int32_t) * T_COLS * ix->B, hipMemcpyDefault));
    if (id2slot) GRAB_HIP(ix, hipMemcpy(id2slot, ix->id2slot, (size_t)ix->n * 4, hipMemcpyDefault));
    if (slot2id) GRAB_HIP(ix, hipMemcpy(slot2id, ix->slot2id, (size_t)ix->n_slots * 4, hipMemcpyDefault));
    return GRAB_OK;
}

grab_status grab_get_graph(grab_index *ix, uint32_t *adj_slots) {
    if (!ix) return GRAB_EINVAL;
    if (!ix->has_graph) return grab_fail(ix, GRAB_ESTATE, "no graph loaded");
    if (!adj_slots) return grab_fail(ix, GRAB_EINVAL, "null argument");
    GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    GRAB_HIP(ix, hipMemcpy(adj_slots, ix->A, (size_t)ix->n_slots * (ix->kl + ix->kr) * 4, hipMemcpyDefault));
    return GRAB_OK;
}

grab_status grab_get_rows(grab_index *ix, float *vectors_slots, int32_t *attr_slots) {
    if (!ix) return GRAB_EINVAL;
    if (!ix->X) return grab_fail(ix, GRAB_ESTATE, "build_buckets first");
    GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    if (vectors_slots) GRAB_HIP(ix, hipMemcpy(vectors_slots, ix->X, (size_t)ix->n_slots * ix->dim * 4, hipMemcpyDefault));
    if (attr_slots) GRAB_HIP(ix, hipMemcpy(attr_slots, ix->attr, (size_t)ix->n_slots * 4, hipMemcpyDefault));
    return GRAB_OK;
}

grab_status grab_get_counters(grab_index *ix, uint32_t *per_query, int64_t nq) {
    if (!ix) return GRAB_EINVAL;
    if (!per_query || nq < 0) return grab_fail(ix, GRAB_EINVAL, "bad argument");
    if (nq > ix->last_nq) return grab_fail(ix, GRAB_EINVAL, "last search had %lld queries", (long long)ix->last_nq);
    if (nq == 0) return GRAB_OK;
    GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    GRAB_HIP(ix, hipMemcpy(per_query, ix->last_counters, (size_t)nq * 8 * 4, hipMemcpyDefault));
    return GRAB_OK;
}

grab_status grab_get_timing(grab_index *ix, float ms[2]) {
    if (!ix) return GRAB_EINVAL;
    if (!ms) return grab_fail(ix, GRAB_EINVAL, "null argument");
    if (!ix->timed) return grab_fail(ix, GRAB_ESTATE, "the last search was not profiled");
    GRAB_HIP(ix, hipEventSynchronize(ix->ev[2]));
    GRAB_HIP(ix, hipEventElapsedTime(&ms[0], ix->ev[0], ix->ev[1]));
    GRAB_HIP(ix, hipEventElapsedTime(&ms[1], ix->ev[1], ix->ev[2]));
    return GRAB_OK;
}

grab_status grab_get_append_stats(grab_index *ix, uint64_t counts[12], float ms[4]) {
    if (!ix) return GRAB_EINVAL;
    if (!ix->app_has_stats) return grab_fail(ix, GRAB_ESTATE, "no insertion has run on this index");
    GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    if (counts) GRAB_HIP(ix, hipMemcpy(counts, ix->app_stats.p, 12 * sizeof(uint64_t), hipMemcpyDefault));
    if (ms) {
        if (!ix->app_timed) return grab_fail(ix, GRAB_ESTATE, "the last insertion was not profiled");
        for (int i = 0; i < 4; ++i) GRAB_HIP(ix, hipEventElapsedTime(&ms[i], ix->app_ev[i], ix->app_ev[i + 1]));
    }
    return GRAB_OK;
}

grab_status grab_probe_gather(grab_index *ix, int64_t waves, int32_t batches, float *ms, double *bytes) {
    if (!ix) return GRAB_EINVAL;
    if (!ms || !bytes) return grab_fail(ix, GRAB_EINVAL, "null argument");
    if (!ix->X || ix->n_slots <= 0) return grab_fail(ix, GRAB_ESTATE, "no vectors loaded");
    if (waves < 1 || waves > (1 << 24) || batches < 1 || batches > (1 << 16))
        return grab_fail(ix, GRAB_EINVAL, "waves must lie in 1..2^24 and batches in 1..2^16");
    grab_status st = grab_reserve(ix, ix->flags, 256);
    if (st != GRAB_OK) return st;
    for (int i = 0; i < 2; ++i)
        if (!ix->ev[i]) GRAB_HIP(ix, hipEventCreate(&ix->ev[i]));
    double b = 0;
    if ((st = grab_launch_gather_probe(ix, waves, 1, reinterpret_cast<float *>(ix->flags.p), &b)) != GRAB_OK) return st;   // warm-up
    GRAB_HIP(ix, hipEventRecord(ix->ev[0], ix->stream));
    if ((st = grab_launch_gather_probe(ix, waves, batches, reinterpret_cast<float *>(ix->flags.p), &b)) != GRAB_OK) return st;
    GRAB_HIP(ix, hipEventRecord(ix->ev[1], ix->stream));
    GRAB_HIP(ix, hipEventSynchronize(ix->ev[1]));
    GRAB_HIP(ix, hipEventElapsedTime(ms, ix->ev[0], ix->ev[1]));
    ix->timed = false;   // the search events were reused
    *bytes = b;
    return GRAB_OK;
}

grab_status grab_append_batch(grab_index *ix, const float *vectors, const int32_t *attrs, int64_t m) {
    if (!ix) return GRAB_EINVAL;
    if (!ix->has_graph) return grab_fail(ix, GRAB_ESTATE, "no graph loaded");
    if (m < 0) return grab_fail(ix, GRAB_EINVAL, "bad batch size");
    if (m == 0) return GRAB_OK;
    if (!vectors || !attrs) return grab_fail(ix, GRAB_EINVAL, "null argument");
    if (ix->kl > 64 || ix->kr > 64) return grab_fail(ix, GRAB_EINVAL, "append needs k_local <= 64 and k_remote <= 64");
    if (ix->n + m > ix->n_slots)
        return grab_fail(ix, GRAB_EFULL, "%lld objects + %lld new exceed the %lld slots of the index", (long long)ix->n,
                         (long long)m, (long long)ix->n_slots);
    SearchLaunch proto;
    grab_status st = check_remote_rule(ix);
    if (st == GRAB_OK) st = grab_resolve_search(ix, ix->prm.append_beam, ix->prm.append_beam, proto);
    if (st != GRAB_OK) return st;
    const void *dv, *da;
    if ((st = grab_to_device(ix, vectors, (size_t)m * ix->dim * 4, ix->stage_q, &dv)) != GRAB_OK) return st;
    if ((st = grab_to_device(ix, attrs, (size_t)m * 4, ix->stage_lo, &da)) != GRAB_OK) return st;
    ix->timed = false;
    return grab_append_device(ix, (const float *)dv, (const int32_t *)da, m, proto);
}

}  // extern "C"
