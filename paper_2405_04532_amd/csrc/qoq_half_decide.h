// Deciding the FP16 rounding of an FP64-defined value from FP32 arithmetic (internal to the library).
//
// The fused producers (normalisation and activation function with the quantizer inside, Section 5.1) define their
// FP16 output as the FP64 evaluation rounded once.  The routines here reach the same bits from FP32 values with
// known error bounds, and say when they cannot.  They are templates over a policy P that supplies the machine
// operations, so that the kernels instantiate them with device intrinsics and a host test with portable ones:
//   P::bits(float) -> uint32_t, P::from_bits(uint32_t) -> float        bit casts
//   P::half_bits(float) -> uint32_t                                     FP32 -> FP16, round to nearest even
//   P::keep(float) -> float                                             identity the compiler cannot see through
#pragma once
#include <cstdint>
#include "qoq_layout.h"

namespace qoq {

// FP16 bits of two producer outputs from FP32 evaluations p0, p1 of them and factors below < 1 < above such that the
// FP64 value that defines each result lies between fl32(p below) and fl32(p above).  Rounding to FP16 is monotonic,
// so where the two bounds round to the same FP16 number, every value between them does, the FP64 one included:
// subnormal and overflowing results need no case of their own.  word = the two results (element 0 in the low
// half); the return value is zero if both are decided and has a bit set in the half of an element that is not (a
// rounding midpoint lies between the two bounds: about 1 element in 1000 for factors 1 -+ 4 * 2^-23), which the
// caller evaluates more precisely.  Five instructions per element and no branch: a wave alone on its SIMD pays
// every instruction and every taken branch in full, and a test with comparisons per case cost more than the rest
// of the kernel.  keep() stops the compiler from merging a product with the conversion after it into one
// mixed-precision multiply-add with a zero addend, which turns a product of -0 into +0.
template <class P>
QOQ_HD uint32_t half2_bits_from_bounds(float p0, float p1, float below, float above, uint32_t& word)
{
    const uint32_t lo = P::half_bits(P::keep(p0 * below)) | (P::half_bits(P::keep(p1 * below)) << 16);
    const uint32_t hi = P::half_bits(P::keep(p0 * above)) | (P::half_bits(P::keep(p1 * above)) << 16);
    word = lo;
    return lo ^ hi;
}

// The same decision from a value known much more precisely: hi + lo with |lo| of the order of an FP32 unit in the
// last place of hi and hi + lo within 2^-40 (relative) of the FP64 value.  All values between two neighbouring FP16
// numbers round down below their midpoint and up above it, so only the side of the midpoint matters:
// (|hi| - midpoint) is exact, adding lo keeps its sign unless the value sits within 2^-36 of the midpoint itself,
// and any FP32 number strictly on that side of the midpoint then rounds (in hardware) to the right neighbour,
// infinity above 65520 included.  Below 2^-13 the FP16 numbers are the multiples k 2^-24, whose bit pattern is k.
// Returns false for the one element in about 10^8 that stays undecided (and for infinities and NaN): the caller
// evaluates it in FP64.  Straight-line code: it runs, for all lanes of the wave, wherever one lane needs it.
template <class P>
QOQ_HD bool half_bits_from_pair(float hi, float lo, uint32_t& bits)
{
    const uint32_t u = P::bits(hi), a = u & 0x7FFFFFFFu, sign = u & 0x80000000u;
    const float ah = P::from_bits(a), alo = sign ? -lo : lo;   // magnitude = ah + alo
    // 2^-13 and above: 13 dropped mantissa bits, midpoint 0x1000
    const uint32_t mid = (a & ~0x1FFFu) | 0x1000u;
    const float side_n = (ah - P::from_bits(mid)) + alo;
    const uint32_t mag = side_n > 0.f ? mid + 1u : mid - 1u;
    const uint32_t bits_n = P::half_bits(P::keep(P::from_bits(mag | sign)));
    // below 2^-13
    const float t = ah * 0x1p24f, fl = __builtin_floorf(t);
    const float side_t = ((t - fl) - 0.5f) + alo * 0x1p24f;
    const uint32_t bits_t = (sign >> 16) | ((uint32_t)fl + (side_t > 0.f ? 1u : 0u));
    const bool tiny = a < 0x39000000u;
    bits = tiny ? bits_t : bits_n;
    const float side = tiny ? side_t : side_n, ref = tiny ? t : ah;
    return (__builtin_fabsf(side) > ref * 0x1p-36f) & (a < 0x7F800000u);
}

// x * r * g for FP16 x, g and an FP64 factor r = r_hi + r_lo (r_hi = fl32(r)), as an FP32 pair hi + lo that carries
// the rounding errors of both products along (fused multiply-adds): within 2^-40 of the FP64 product.
template <class P>
QOQ_HD void scaled_product_pair(float x, float r_hi, float r_lo, float g, float& hi, float& lo)
{
    const float p1 = x * r_hi, e1 = __builtin_fmaf(x, r_hi, -p1) + x * r_lo;
    hi = p1 * g;
    lo = __builtin_fmaf(p1, g, -hi) + e1 * g;
}

}  // namespace qoq
