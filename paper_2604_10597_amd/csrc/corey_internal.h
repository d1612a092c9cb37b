// Internal helpers shared by the translation units of libcorey (host side only, plus two device
// conversions).  Nothing here is part of the ABI.
#ifndef COREY_INTERNAL_H
#define COREY_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "corey.h"

namespace corey {

// Record a message for corey_last_error() and hand back `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline int hip_fail(hipError_t e, const char* what)
{
    return fail(COREY_EHIP, "%s: %s", what, hipGetErrorString(e));
}

inline bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

// bfloat16 storage <-> binary32 (bit patterns; widening is exact, narrowing rounds to nearest even).
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t w = __float_as_uint(f);
    if ((w & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((w >> 16) | 0x40u);   // quiet NaN
    w += 0x7fffu + ((w >> 16) & 1u);
    return (uint16_t)(w >> 16);
}

// Launch the O(K) reduction of corey_entropy_hist for ONE histogram whose kParts partial histograms of K bins sit in
// `parts` and whose range sits in `slot` (a corey_range::RangeSlot): sums the partials into counts, H, r, optionally the
// range and, with a policy, the chunk for sequence length L; leaves the partial histograms cleared.  Defined in
// corey_entropy.hip.
int launch_entropy_finalise(const uint32_t* parts, uint32_t* counts, int32_t K, double eps, const void* slot, double* H_out,
                            double* r_out, float* range_out, const corey_policy* pol, int32_t* chunks_out, int64_t L,
                            hipStream_t stream);

// The checks corey_select_chunk_device makes on a policy before the GPU applies it (corey_entropy.hip).
int check_device_policy(const char* who, const corey_policy* p, int64_t L);

}  // namespace corey
#endif
