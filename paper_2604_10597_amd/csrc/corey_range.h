// Range (min / max / NaN) bookkeeping shared by the histogram sweeps and by the producer of u that fuses the range
// into its own pass: order-preserving integer keys, the per-workgroup partial record and its workgroup reduction.
#ifndef COREY_RANGE_H
#define COREY_RANGE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

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

// Workgroup reduction of (lo, hi, nan flag) as order-preserving keys; the result is valid in thread 0.
__device__ __forceinline__ void reduce_range_keys(uint32_t& klo, uint32_t& khi, uint32_t& knan)
{
    for (int off = 32; off > 0; off >>= 1) {
        klo = min(klo, (uint32_t)__shfl_xor((int)klo, off));
        khi = max(khi, (uint32_t)__shfl_xor((int)khi, off));
        knan |= (uint32_t)__shfl_xor((int)knan, off);
    }
    __shared__ uint32_t s_lo[kThreads / 64], s_hi[kThreads / 64], s_nan[kThreads / 64];
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { s_lo[wave] = klo; s_hi[wave] = khi; s_nan[wave] = knan; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) {
            klo = min(klo, s_lo[w]);
            khi = max(khi, s_hi[w]);
            knan |= s_nan[w];
        }
    }
}

}  // namespace corey_range
#endif
