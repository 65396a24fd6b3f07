// Float scalar attributes (Section 3 states the filter over a scalar attribute; the experiments
// of Section 5.1 draw it uniformly from [0,1]): every float is replaced by an int32 that orders
// the same way and the integer path does the rest.  For IEEE-754 binary32 the bit pattern of a
// non-negative value already orders like the value; for a negative value the magnitude bits order
// the other way round, so those 31 bits are flipped.  -0 is stored as +0 (they compare equal).
#include "grab_internal.h"

namespace {

__host__ __device__ inline int32_t attr_image(float x) {
    if (x == 0.0f) return 0;
    union { float f; int32_t i; } u;
    u.f = x;
    return u.i >= 0 ? u.i : (int32_t)(u.i ^ 0x7FFFFFFF);
}

__host__ __device__ inline float attr_value(int32_t s) {
    union { float f; int32_t i; } u;
    u.i = s >= 0 ? s : (int32_t)(s ^ 0x7FFFFFFF);
    return u.f;
}

__global__ void k_attr_image(const float *__restrict__ in, int32_t *__restrict__ out, int64_t n, int32_t *nan_seen) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float x = in[i];
    if (x != x) atomicOr(nan_seen, 1);
    out[i] = attr_image(x);
}

// closed ranges; a NaN bound compares false with everything, so such a range selects nothing
__global__ void k_range_image(const float *__restrict__ lo, const float *__restrict__ hi, int32_t *__restrict__ lo_i,
                              int32_t *__restrict__ hi_i, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float a = lo[i], b = hi[i];
    const bool empty = a != a || b != b;
    lo_i[i] = empty ? 1 : attr_image(a);
    hi_i[i] = empty ? 0 : attr_image(b);
}

__global__ void k_clear_word(int32_t *w) { *w = 0; }

// attrs[n] (host or device floats) -> device int32 images in `conv`.  GRAB_EINVAL if one is NaN
// (no range could ever select it).  Waits for the conversion.
grab_status convert_attrs(grab_index *ix, const float *attrs, int64_t n, DevBuf &stage, DevBuf &conv) {
    const void *da;
    grab_status st = grab_to_device(ix, attrs, (size_t)n * 4, stage, &da);
    if (st != GRAB_OK) return st;
    if ((st = grab_reserve(ix, conv, (size_t)n * 4)) != GRAB_OK) return st;
    if ((st = grab_reserve(ix, ix->attr_flag, 64)) != GRAB_OK) return st;
    int32_t *flag = reinterpret_cast<int32_t *>(ix->attr_flag.p);
    k_clear_word<<<1, 1, 0, ix->stream>>>(flag);
    GRAB_HIP(ix, hipGetLastError());
    k_attr_image<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ix->stream>>>((const float *)da, (int32_t *)conv.p, n, flag);
    GRAB_HIP(ix, hipGetLastError());
    int32_t seen = 0;
    GRAB_HIP(ix, hipMemcpyAsync(&seen, flag, 4, hipMemcpyDeviceToHost, ix->stream));
    GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    if (seen) return grab_fail(ix, GRAB_EINVAL, "an attribute is NaN");
    return GRAB_OK;
}

}  // namespace

extern "C" {

int32_t grab_attr_image(float x) { return attr_image(x); }
float grab_attr_value(int32_t image) { return attr_value(image); }

grab_status grab_build_buckets_f32(grab_index *ix, const float *vectors, const float *attrs, int64_t n,
                                   int32_t n_buckets, int64_t n_cap) {
    if (!ix) return GRAB_EINVAL;
    if (!vectors || !attrs) return grab_fail(ix, GRAB_EINVAL, "null input");
    if (n < 1 || n >= (1ll << 31)) return grab_fail(ix, GRAB_EINVAL, "need 1 <= n < 2^31");
    grab_status st = convert_attrs(ix, attrs, n, ix->stage_fa, ix->conv_a);
    if (st != GRAB_OK) return st;
    return grab_build_buckets(ix, vectors, (const int32_t *)ix->conv_a.p, n, n_buckets, n_cap);
}

grab_status grab_append_batch_f32(grab_index *ix, const float *vectors, const float *attrs, int64_t m) {
    if (!ix) return GRAB_EINVAL;
    if (m < 0 || m >= (1ll << 31)) return grab_fail(ix, GRAB_EINVAL, "bad batch size");
    if (m == 0) return grab_append_batch(ix, vectors, nullptr, 0);
    if (!vectors || !attrs) return grab_fail(ix, GRAB_EINVAL, "null argument");
    grab_status st = convert_attrs(ix, attrs, m, ix->stage_fa, ix->conv_a);
    if (st != GRAB_OK) return st;
    return grab_append_batch(ix, vectors, (const int32_t *)ix->conv_a.p, m);
}

grab_status grab_search_range_f32(grab_index *ix, const float *queries, const float *lo, const float *hi, int64_t nq,
                                  int32_t k, int32_t beam, uint32_t *out_ids, float *out_dist) {
    if (!ix) return GRAB_EINVAL;
    if (nq < 0 || nq > (1ll << 30)) return grab_fail(ix, GRAB_EINVAL, "bad query count");
    if (nq == 0) return grab_search_range(ix, queries, nullptr, nullptr, 0, k, beam, out_ids, out_dist);
    if (!lo || !hi) return grab_fail(ix, GRAB_EINVAL, "null argument");
    const void *dlo, *dhi;
    grab_status st = grab_to_device(ix, lo, (size_t)nq * 4, ix->stage_flo, &dlo);
    if (st == GRAB_OK) st = grab_to_device(ix, hi, (size_t)nq * 4, ix->stage_fhi, &dhi);
    if (st == GRAB_OK) st = grab_reserve(ix, ix->conv_lo, (size_t)nq * 4);
    if (st == GRAB_OK) st = grab_reserve(ix, ix->conv_hi, (size_t)nq * 4);
    if (st != GRAB_OK) return st;
    k_range_image<<<dim3((unsigned)((nq + 255) / 256)), dim3(256), 0, ix->stream>>>(
        (const float *)dlo, (const float *)dhi, (int32_t *)ix->conv_lo.p, (int32_t *)ix->conv_hi.p, nq);
    GRAB_HIP(ix, hipGetLastError());
    st = grab_search_range(ix, queries, (const int32_t *)ix->conv_lo.p, (const int32_t *)ix->conv_hi.p, nq, k, beam,
                           out_ids, out_dist);
    // host bounds were copied from the caller's arrays: do not return before that copy has run
    if (st == GRAB_OK && (dlo != (const void *)lo || dhi != (const void *)hi)) GRAB_HIP(ix, hipStreamSynchronize(ix->stream));
    return st;
}

}  // extern "C"
