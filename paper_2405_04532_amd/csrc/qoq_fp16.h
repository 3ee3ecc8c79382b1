// Exact FP64 -> FP16 rounding on the device (internal to the library).
#pragma once
#include <cstdint>
#include <hip/hip_runtime.h>

namespace qoq {

__device__ __forceinline__ uint16_t double_to_half_rne(double d)   // finite d; exact round-to-nearest-even, integer arithmetic only
{
    const uint64_t bits = (uint64_t)__double_as_longlong(d);
    const uint16_t sign = (uint16_t)((bits >> 48) & 0x8000u);
    const int e = (int)((bits >> 52) & 0x7FF) - 1023;    // d = 1.m * 2^e (FP64 subnormals are far below FP16's range)
    if (e < -25) return sign;                            // below half of the smallest FP16 subnormal (or zero)
    if (e > 15) return sign | 0x7C00u;
    const uint64_t mant = (bits & 0xFFFFFFFFFFFFFull) | (1ull << 52);   // 53 significant bits
    // FP16 keeps 10 fraction bits for e >= -14, fewer below: drop `shift` low bits with round-half-to-even
    const int shift = e >= -14 ? 42 : 42 + (-14 - e);    // 42 .. 53
    const uint64_t kept = mant >> shift, rest = mant & ((1ull << shift) - 1), half = 1ull << (shift - 1);
    const uint64_t rounded = kept + ((rest > half || (rest == half && (kept & 1))) ? 1 : 0);
    // e >= -14: rounded in [1024, 2048]; the biased exponent is added on top of the hidden bit, so a carry to
    // 2048 bumps the exponent by itself (and 65520 and above become infinity).  e < -14: rounded is the
    // subnormal pattern (1024 = smallest normal).
    const uint32_t h = e >= -14 ? (uint32_t)((e + 14) << 10) + (uint32_t)rounded : (uint32_t)rounded;
    return sign | (uint16_t)(h > 0x7C00u ? 0x7C00u : h);
}


}  // namespace qoq
