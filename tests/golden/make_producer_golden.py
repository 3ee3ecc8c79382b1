#!/usr/bin/env python3
"""Writes tests/golden/silu_mul_decimal.txt and tests/golden/rmsnorm_decimal.txt: expected FP16 bit patterns of
the two memory-bound producers the activation quantization is fused into (Section 5.1 of arXiv 2405.04532),
computed here from their textbook formulas in 60-digit decimal arithmetic and rounded once to FP16
(round to nearest, ties to even, subnormals and overflow to infinity handled on exact rationals).

    SiLU(gate) * up :  y = g / (1 + exp(-g)) * u
    RMSNorm         :  y[k] = x[k] * gamma[k] / sqrt(mean_k x[k]^2 + eps)

This script imports nothing from the oracle or from the library: the numbers it writes pin the oracle to
arithmetic other than its own.  Inputs are FP16 bit patterns drawn from a small linear congruential generator, so
the files can be regenerated bit for bit:  python tests/golden/make_producer_golden.py
"""
import os
import struct
from decimal import Decimal, getcontext
from fractions import Fraction

getcontext().prec = 60
HERE = os.path.dirname(os.path.abspath(__file__))


def half_to_fraction(bits):
    return Fraction(struct.unpack("<e", struct.pack("<H", bits))[0])


def fraction_to_half_bits(v):
    """Exact round-to-nearest-even of a rational to an FP16 bit pattern."""
    sign = 0x8000 if v < 0 else 0
    a = -v if v < 0 else v
    if a == 0:
        return sign
    e = 0                                  # a = f * 2^e with 1 <= f < 2
    while a >= Fraction(2) ** (e + 1):
        e += 1
    while a < Fraction(2) ** e:
        e -= 1
    e = max(e, -14)                        # subnormal range: fixed exponent
    ulp = Fraction(2) ** (e - 10)
    q, r = divmod(a, ulp)                  # q = integer number of ulps
    q = int(q)
    if r * 2 > ulp or (r * 2 == ulp and (q & 1)):
        q += 1
    # q in [0, 2048]: q == 2048 carries into the next exponent; encoding by addition handles it
    bits = ((e + 14) << 10) + q if e > -14 or q >= 1024 else q
    if e == -14 and q >= 1024:
        bits = (1 << 10) + (q - 1024)
    elif e > -14:
        bits = ((e + 15) << 10) + (q - 1024)
    if bits >= 0x7C00:
        bits = 0x7C00                      # overflow -> infinity
    return sign | bits


def lcg(seed):
    s = seed
    while True:
        s = (s * 6364136223846793005 + 1442695040888963407) & ((1 << 64) - 1)
        yield s >> 33


def finite_half(rng, max_exp_field):
    """A finite FP16 bit pattern with exponent field <= max_exp_field (random sign and mantissa)."""
    while True:
        b = next(rng) & 0xFFFF
        if ((b >> 10) & 0x1F) <= max_exp_field:
            return b


def dec(fr):
    return Decimal(fr.numerator) / Decimal(fr.denominator)


def main():
    rng = lcg(20240507)
    lines = ["# g_bits u_bits y_bits  (hex FP16 patterns; y = RNE_fp16(g / (1 + exp(-g)) * u) in 60-digit decimal)"]
    pairs = [(0x0000, 0x4200), (0x3C00, 0x4000), (0xBC00, 0x4000), (0x4800, 0x3C00), (0xC800, 0x3C00), (0x3800, 0xC400),
             (0x4B00, 0x4B00), (0xCB00, 0x4B00), (0x0001, 0x3C00), (0x8001, 0x7BFF), (0x7BFF, 0x0400), (0xFBFF, 0x7BFF),
             (0x4D00, 0x7000), (0xCC00, 0x7BFF), (0x5640, 0x5640)]
    while len(pairs) < 400:
        pairs.append((finite_half(rng, 0x16), finite_half(rng, 0x18)))      # |g| < 256, |u| < 1024
    for gb, ub in pairs:
        g, u = half_to_fraction(gb), half_to_fraction(ub)
        y = dec(g) / (Decimal(1) + (-dec(g)).exp()) * dec(u)
        lines.append("%04x %04x %04x" % (gb, ub, fraction_to_half_bits(Fraction(y))))
    with open(os.path.join(HERE, "silu_mul_decimal.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")

    lines = ["# rows of 32 elements: eps (float hex), then x_bits, gamma_bits, y_bits per element;",
             "# y = RNE_fp16(x * gamma / sqrt(mean(x^2) + eps)) in 60-digit decimal"]
    for row in range(8):
        K = 32
        xs = [finite_half(rng, 0x13) for _ in range(K)]                    # |x| < 32
        gs = [finite_half(rng, 0x10) & 0x7FFF for _ in range(K)]           # 0 <= gamma < 4
        eps = [0.0, 1e-5, 1e-6, 1e-3, 1e-5, 1e-5, 0.5, 1e-5][row]
        if row == 5:
            xs = [0x0000] * K                                              # an all-zero token: y = 0, no division by zero
        if row == 0:
            xs[0] |= 0x0400                                                # eps = 0 needs a non-zero row
        ms = sum(half_to_fraction(b) ** 2 for b in xs) / K + Fraction(eps)
        root = dec(ms).sqrt()
        lines.append("row %d eps %s" % (row, float(eps).hex()))
        for xb, gb in zip(xs, gs):
            y = dec(half_to_fraction(xb)) * dec(half_to_fraction(gb)) / root
            lines.append("%04x %04x %04x" % (xb, gb, fraction_to_half_bits(Fraction(y))))
    with open(os.path.join(HERE, "rmsnorm_decimal.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
