// Bucket-major layout kernels: predicate-based partitioning (Section 4.2.1) into the unified
// device layout (Section 4.2.4), and installation of the fixed-degree hybrid adjacency
// (Sections 4.2.2-4.2.3).  gfx950 only.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include "grab_internal.h"

namespace {

constexpr int TPB = 256;

__global__ void k_make_keys(const int32_t *__restrict__ attrs, uint32_t *__restrict__ keys,
                            uint32_t *__restrict__ ids, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < n) {
        keys[i] = (uint32_t)attrs[i] ^ 0x80000000u;  // signed order -> unsigned order
        ids[i] = (uint32_t)i;
    }
}

// bucket of sorted rank r under equal-count cuts floor(b*n/B): the largest b with cut(b) <= r
__device__ __forceinline__ int32_t bucket_of_rank(int64_t r, int64_t n, int32_t B) {
    return (int32_t)(((r + 1) * (int64_t)B - 1) / n);
}

// one thread per sorted rank: slot = rank + bucket * slack (every slab = its count + slack)
__global__ void k_place(const uint32_t *__restrict__ sorted_keys, const uint32_t *__restrict__ sorted_ids,
                        int64_t n, int32_t B, int64_t slack, int32_t *__restrict__ attr_s,
                        uint32_t *__restrict__ slot2id, uint32_t *__restrict__ id2slot) {
    int64_t r = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (r >= n) return;
    int32_t b = bucket_of_rank(r, n, B);
    int64_t slot = r + (int64_t)b * slack;
    uint32_t id = sorted_ids[r];
    attr_s[slot] = (int32_t)(sorted_keys[r] ^ 0x80000000u);
    slot2id[slot] = id;
    id2slot[id] = (uint32_t)slot;
}

// one thread per 16-byte piece of a row: gathered read of the caller's row, coalesced write
__global__ void k_permute_rows(const float4 *__restrict__ src, const uint32_t *__restrict__ sorted_ids,
                               int64_t n, int32_t B, int64_t slack, int32_t row_f4, float4 *__restrict__ dst) {
    int64_t t = (int64_t)blockIdx.x * TPB + threadIdx.x;
    int64_t r = t / row_f4;
    if (r >= n) return;
    int32_t c = (int32_t)(t - r * row_f4);
    int32_t b = bucket_of_rank(r, n, B);
    int64_t slot = r + (int64_t)b * slack;
    dst[slot * row_f4 + c] = src[(int64_t)sorted_ids[r] * row_f4 + c];
}

__global__ void k_table(const uint32_t *__restrict__ sorted_keys, int64_t n, int32_t B, int64_t slack,
                        int32_t *__restrict__ table) {
    int32_t b = blockIdx.x * TPB + threadIdx.x;
    if (b >= B) return;
    int64_t s = ((int64_t)b * n) / B, e = ((int64_t)(b + 1) * n) / B;
    int32_t *t = table + T_COLS * b;
    t[T_BASE] = (int32_t)(s + (int64_t)b * slack);
    t[T_NSORT] = (int32_t)(e - s);
    t[T_NTOT] = (int32_t)(e - s);
    t[T_CAP] = (int32_t)(e - s + slack);
    t[T_MIN] = (int32_t)(sorted_keys[s] ^ 0x80000000u);
    t[T_MAX] = (int32_t)(sorted_keys[e - 1] ^ 0x80000000u);
}

__device__ __forceinline__ int32_t bucket_of_slot(const int32_t *__restrict__ table, int32_t B, uint32_t slot) {
    int32_t l = 0, r = B;  // last bucket whose base <= slot
    while (r - l > 1) {
        int32_t m = (l + r) >> 1;
        if ((uint32_t)table[T_COLS * m + T_BASE] <= slot) l = m; else r = m;
    }
    return l;
}

// one thread per adjacency entry: id -> slot, row = [local | remote]; counts rule violations
__global__ void k_load_graph(const uint32_t *__restrict__ local, int32_t kl, const uint32_t *__restrict__ remote,
                             int32_t kr, int64_t n, const uint32_t *__restrict__ id2slot,
                             const int32_t *__restrict__ table, int32_t B, uint32_t *__restrict__ A,
                             int32_t *__restrict__ err) {
    const int32_t K = kl + kr;
    int64_t t = (int64_t)blockIdx.x * TPB + threadIdx.x;
    int64_t i = t / K;
    if (i >= n) return;
    int32_t j = (int32_t)(t - i * K);
    uint32_t v = j < kl ? local[i * kl + j] : remote[i * kr + (j - kl)];
    uint32_t self = id2slot[i];
    uint32_t out = GRAB_EMPTY;
    if (v != GRAB_EMPTY) {
        if ((int64_t)v >= n) {
            atomicAdd(err + 0, 1);
        } else {
            out = id2slot[v];
            bool same = bucket_of_slot(table, B, out) == bucket_of_slot(table, B, self);
            if (j < kl && !same) atomicAdd(err + 1, 1);
            if (j >= kl && same) atomicAdd(err + 2, 1);
        }
    }
    A[(int64_t)self * K + j] = out;
}

// Fence of every bucket: entry i of bucket b = the attribute at position i * GRAB_FENCE of the
// bucket's sorted prefix.  Range selection searches the few cache lines of a fence first and then
// the GRAB_FENCE - 1 attributes between two of its entries (Algorithm 2, line 1: the valid part of
// an edge bucket).  The sorted prefix of a bucket never changes after the layout is built
// (insertion appends to the tail), so neither does the fence.  blockIdx.y = bucket.
__global__ void k_fence(const int32_t *__restrict__ table, const int32_t *__restrict__ attr, int32_t *__restrict__ fence) {
    const int b = blockIdx.y;
    const int32_t *t = table + T_COLS * b;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i * GRAB_FENCE < t[T_NSORT]) fence[grab_fence_offset(t[T_BASE], b) + i] = attr[(int64_t)t[T_BASE] + i * GRAB_FENCE];
}

inline unsigned blocks_for(int64_t work) { return (unsigned)((work + TPB - 1) / TPB); }

}  // namespace

grab_status grab_launch_build(grab_index *ix, const float *d_vectors, const int32_t *d_attrs, int64_t n,
                              int32_t B, int64_t slack) {
    hipStream_t st = ix->stream;
    uint32_t *keys = nullptr, *ids = nullptr, *keys_s = nullptr, *ids_s = nullptr;
    void *tmp = nullptr;
    size_t tmp_bytes = 0;
    auto cleanup = [&]() {
        (void)hipFree(keys); (void)hipFree(ids); (void)hipFree(keys_s); (void)hipFree(ids_s); (void)hipFree(tmp);
    };
#define BUILD_HIP(call)                                                                          \
    do {                                                                                         \
        hipError_t e__ = (call);                                                                 \
        if (e__ != hipSuccess) {                                                                 \
            cleanup();                                                                           \
            return grab_fail(ix, e__ == hipErrorOutOfMemory ? GRAB_ENOMEM : GRAB_EHIP,           \
                             "%s failed: %s", #call, hipGetErrorString(e__));                    \
        }                                                                                        \
    } while (0)
    BUILD_HIP(hipMalloc(&keys, n * 4));
    BUILD_HIP(hipMalloc(&ids, n * 4));
    BUILD_HIP(hipMalloc(&keys_s, n * 4));
    BUILD_HIP(hipMalloc(&ids_s, n * 4));
    k_make_keys<<<blocks_for(n), TPB, 0, st>>>(d_attrs, keys, ids, n);
    // stable LSD radix sort on the attribute; ids start ascending, so ties end up ordered by id
    BUILD_HIP(rocprim::radix_sort_pairs(nullptr, tmp_bytes, keys, keys_s, ids, ids_s, (size_t)n, 0, 32, st));
    BUILD_HIP(hipMalloc(&tmp, tmp_bytes ? tmp_bytes : 4));
    BUILD_HIP(rocprim::radix_sort_pairs(tmp, tmp_bytes, keys, keys_s, ids, ids_s, (size_t)n, 0, 32, st));
    k_place<<<blocks_for(n), TPB, 0, st>>>(keys_s, ids_s, n, B, slack, ix->attr, ix->slot2id, ix->id2slot);
    const int32_t row_f4 = ix->dim / 4;
    k_permute_rows<<<blocks_for(n * row_f4), TPB, 0, st>>>((const float4 *)d_vectors, ids_s, n, B, slack, row_f4,
                                                           (float4 *)ix->X);
    k_table<<<blocks_for(B), TPB, 0, st>>>(keys_s, n, B, slack, ix->table);
    // a bucket's sorted prefix holds at most ceil(n / B) objects
    k_fence<<<dim3(blocks_for(((n + B - 1) / B + GRAB_FENCE - 1) / GRAB_FENCE), (unsigned)B), TPB, 0, st>>>(ix->table, ix->attr,
                                                                                                             ix->fence);
    BUILD_HIP(hipGetLastError());
    BUILD_HIP(hipMemcpyAsync(ix->h_table, ix->table, sizeof(int32_t) * T_COLS * B, hipMemcpyDeviceToHost, st));
    BUILD_HIP(hipStreamSynchronize(st));
#undef BUILD_HIP
    cleanup();
    return GRAB_OK;
}

grab_status grab_launch_load_graph(grab_index *ix, const uint32_t *d_local, int32_t kl, const uint32_t *d_remote,
                                   int32_t kr, int32_t *d_err) {
    k_load_graph<<<blocks_for(ix->n * (kl + kr)), TPB, 0, ix->stream>>>(d_local, kl, d_remote, kr, ix->n, ix->id2slot,
                                                                       ix->table, ix->B, ix->A, d_err);
    GRAB_HIP(ix, hipGetLastError());
    return GRAB_OK;
}
