// Range (min / max / NaN) bookkeeping shared by the histogram sweeps and by the producer of u that fuses the range
// into its own pass: order-preserving integer keys, the per-workgroup partial record and its workgroup reduction.
#ifndef COREY_RANGE_H
#define COREY_RANGE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "corey.h"

namespace corey_range {

constexpr int kThreads = 256;      // lanes per workgroup of every kernel that uses reduce_range_keys

__device__ __forceinline__ uint32_t order_key(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float key_value(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

struct RangePart {        // what one workgroup of a range sweep saw (lo_key 0xffffffff / hi_key 0: nothing)
    uint32_t lo_key, hi_key, saw_nan, pad;
};

struct RangeSlot {        // the range of one histogram, in a caller's workspace
    uint32_t lo_key;      // order-preserving image of the minimum (0xffffffff: nothing seen)
    uint32_t hi_key;      // order-preserving image of the maximum (0: nothing seen)
    uint32_t saw_nan;
    uint32_t pad;
};

constexpr int kParts = 16;         // partial histograms per histogram in a workspace (spreads the merging atomics)

// What the producer of a tensor hands to the statistic of that tensor (COREY_HANDOFF_BYTES): the partial ranges it saw
// and, cleared by it, the partial histograms the count sweep adds into, so that the statistic needs no clearing launch.
struct Handoff {
    RangePart parts[COREY_RANGE_PARTS];
    uint32_t counts[kParts * COREY_MAX_BINS];
};
static_assert(sizeof(Handoff) == COREY_HANDOFF_BYTES, "the header's size of the hand-over buffer");

// Clear the hand-over buffer's partial histograms, spread over the workgroups of the kernel that calls it.
__device__ __forceinline__ void clear_handoff_counts(Handoff* h)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < kParts * COREY_MAX_BINS; i += gridDim.x * blockDim.x) h->counts[i] = 0u;
}

// Workgroup reduction of (lo, hi, nan flag) as order-preserving keys over NT lanes; the result is valid in thread 0.
template <int NT = kThreads>
__device__ __forceinline__ void reduce_range_keys(uint32_t& klo, uint32_t& khi, uint32_t& knan)
{
    for (int off = 32; off > 0; off >>= 1) {
        klo = min(klo, (uint32_t)__shfl_xor((int)klo, off));
        khi = max(khi, (uint32_t)__shfl_xor((int)khi, off));
        knan |= (uint32_t)__shfl_xor((int)knan, off);
    }
    __shared__ uint32_t s_lo[NT / 64], s_hi[NT / 64], s_nan[NT / 64];
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { s_lo[wave] = klo; s_hi[wave] = khi; s_nan[wave] = knan; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < NT / 64; ++w) {
            klo = min(klo, s_lo[w]);
            khi = max(khi, s_hi[w]);
            knan |= s_nan[w];
        }
    }
}

// min/max that ignore a NaN operand (hardware behaviour of v_min3/v_max3 in IEEE mode), two values per
// instruction; written as instructions so that no canonicalising v_max(x, x) is added per operand.
__device__ __forceinline__ void minmax3(float& lo, float& hi, float a, float b)
{
    asm("v_min3_f32 %0, %0, %1, %2" : "+v"(lo) : "v"(a), "v"(b));
    asm("v_max3_f32 %0, %0, %1, %2" : "+v"(hi) : "v"(a), "v"(b));
}

typedef uint32_t word4 __attribute__((ext_vector_type(4)));

// Fold one 16-byte word of stored values into a running range.  `mag` tracks the largest magnitude bit pattern seen
// (per 16-bit half for bf16), from which NaN (pattern above infinity's) is read off at the end.
template <typename T> struct RangeFold;
template <> struct RangeFold<uint16_t> {                  // bfloat16 bit patterns
    typedef uint16_t half2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void fold(const word4& q, float& lo, float& hi, uint32_t& mag)
    {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            minmax3(lo, hi, __uint_as_float(w[k] << 16), __uint_as_float(w[k] & 0xffff0000u));
            half2 m, c;
            const uint32_t a = w[k] & 0x7fff7fffu;
            __builtin_memcpy(&m, &mag, 4);
            __builtin_memcpy(&c, &a, 4);
            m = __builtin_elementwise_max(m, c);
            __builtin_memcpy(&mag, &m, 4);
        }
    }
    static __device__ __forceinline__ bool saw_nan(uint32_t mag) { return (mag & 0xffffu) > 0x7f80u || (mag >> 16) > 0x7f80u; }
};
template <> struct RangeFold<_Float16> {
    static __device__ __forceinline__ void fold(const word4& q, float& lo, float& hi, uint32_t& mag)
    {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            h2 h;
            __builtin_memcpy(&h, &w[k], 4);
            const float a = (float)h.x, b = (float)h.y;
            minmax3(lo, hi, a, b);
            mag = max(mag, max(__float_as_uint(a) & 0x7fffffffu, __float_as_uint(b) & 0x7fffffffu));
        }
    }
    static __device__ __forceinline__ bool saw_nan(uint32_t mag) { return mag > 0x7f800000u; }
};
template <> struct RangeFold<float> {
    static __device__ __forceinline__ void fold(const word4& q, float& lo, float& hi, uint32_t& mag)
    {
        minmax3(lo, hi, __uint_as_float(q.x), __uint_as_float(q.y));
        minmax3(lo, hi, __uint_as_float(q.z), __uint_as_float(q.w));
        mag = max(max(mag, q.x & 0x7fffffffu), max(q.y & 0x7fffffffu, max(q.z & 0x7fffffffu, q.w & 0x7fffffffu)));
    }
    static __device__ __forceinline__ bool saw_nan(uint32_t mag) { return mag > 0x7f800000u; }
};

// A usable range: something was seen, no NaN, both ends finite.
__device__ __forceinline__ bool usable_range(const RangeSlot& s, float* lo, float* hi)
{
    if (s.saw_nan || s.lo_key == 0xffffffffu || s.hi_key == 0u) return false;
    *lo = key_value(s.lo_key);
    *hi = key_value(s.hi_key);
    return isfinite(*lo) && isfinite(*hi);
}

}  // namespace corey_range
#endif
