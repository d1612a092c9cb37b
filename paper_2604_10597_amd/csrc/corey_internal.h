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

}  // namespace corey
#endif
