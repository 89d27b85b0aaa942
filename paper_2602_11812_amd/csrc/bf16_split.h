// An fp32 value as the exact sum of three bf16 values: its top 8 significant bits (truncated, not
// rounded), the top 8 of what is left, and the rest (at most 8 more bits, since fp32 has 24).  bf16 has
// fp32's exponent range, so every piece is representable; products of two pieces are exact in fp32, which
// is what lets the bf16 matrix cores accumulate fp32-grade dot products.  Device-side header.
#pragma once
#include <hip/hip_runtime.h>

namespace egtp {
namespace {

// the three pieces as fp32 bit patterns with the low 16 bits clear (bf16 = the high half)
__device__ __forceinline__ void split3_bits(float f, unsigned &hi, unsigned &mid, unsigned &lo)
{
    hi = __float_as_uint(f) & 0xffff0000u;
    const float r1 = f - __uint_as_float(hi);
    mid = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(mid);
    lo = __float_as_uint(r2) & 0xffff0000u;
}

}  // namespace
}  // namespace egtp
