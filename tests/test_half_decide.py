"""Host check of the FP32 routines with which the fused producers (normalisation / activation function with the
quantizer inside, Section 5.1) decide the FP16 rounding of their FP64-defined output.

The routines (csrc/qoq_half_decide.h) are templates over the machine operations; here they are compiled for the CPU
and fed millions of (x, r, gamma) triples: every result they call decided must be the FP16 rounding of the FP64
product x * r * gamma as numpy computes it, the undecided ones must be rare, and the compensated path must hold when
it is forced on every element (on the GPU it only sees the elements next to a rounding midpoint)."""
import os
import shutil
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = shutil.which("clang++", path="/opt/rocm/llvm/bin") or shutil.which("clang++")

SRC = r'''
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <vector>
#include "qoq_half_decide.h"
struct HostF32 {
    static uint32_t bits(float x) { uint32_t u; memcpy(&u, &x, 4); return u; }
    static float from_bits(uint32_t u) { float x; memcpy(&x, &u, 4); return x; }
    static uint32_t half_bits(float x) { _Float16 h = (_Float16)x; uint16_t b; memcpy(&b, &h, 2); return b; }
    static float keep(float x) { return x; }
};
static float half_value(uint16_t b) { _Float16 h; memcpy(&h, &b, 2); return (float)h; }
int main(int argc, char** argv)
{
    // input: n records of (uint16 x, uint16 gamma, double r); output: n uint32, the FP16 bits or 0xFFFFFFFF = undecided
    const bool force_pair = atoi(argv[3]) != 0;
    FILE* fi = fopen(argv[1], "rb"); FILE* fo = fopen(argv[2], "wb");
    if (!fi || !fo) return 2;
    long n; if (fread(&n, 8, 1, fi) != 1) return 2;
    std::vector<uint16_t> xs(n), gs(n); std::vector<double> rs(n); std::vector<uint32_t> out(n);
    if (fread(xs.data(), 2, n, fi) != (size_t)n || fread(gs.data(), 2, n, fi) != (size_t)n || fread(rs.data(), 8, n, fi) != (size_t)n) return 2;
    for (long i = 0; i < n; i += 2) {
        const float r_hi = (float)rs[i], r_lo = (float)(rs[i] - (double)r_hi);   // one factor per pair of elements
        const float x0 = half_value(xs[i]), x1 = half_value(xs[i + 1]), g0 = half_value(gs[i]), g1 = half_value(gs[i + 1]);
        uint32_t word;
        uint32_t diff = qoq::half2_bits_from_bounds<HostF32>(x0 * r_hi * g0, x1 * r_hi * g1, 1.0f - 4 * 0x1p-23f, 1.0f + 4 * 0x1p-23f, word);
        if (force_pair) diff = 0xFFFFFFFFu;
        for (int j = 0; j < 2; ++j) {
            uint32_t b = (word >> (16 * j)) & 0xFFFFu;
            if ((diff >> (16 * j)) & 0xFFFFu) {
                float hi, lo;
                qoq::scaled_product_pair<HostF32>(j ? x1 : x0, r_hi, r_lo, j ? g1 : g0, hi, lo);
                if (!qoq::half_bits_from_pair<HostF32>(hi, lo, b)) b = 0xFFFFFFFFu;
            }
            out[i + j] = b;
        }
    }
    fwrite(out.data(), 4, n, fo);
    fclose(fo);
    return 0;
}
'''


def _triples(seed, n):
    """FP16 x and gamma with every exponent, FP64 factors over twelve decades; zeros of both signs included."""
    rng = np.random.default_rng(seed)
    def halves():
        b = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
        b[(b & 0x7C00) == 0x7C00] &= 0x83FF                       # no infinities or NaN: subnormals instead
        return b
    x, g = halves(), halves()
    x[:1000:2] = 0x8000                                           # -0
    x[1:1000:2] = 0x0000
    r = np.exp(rng.uniform(-14.0, 14.0, size=n // 2)).repeat(2)   # shared by the two elements of a word
    return x, g, r


@pytest.mark.skipif(CLANG is None, reason="needs a clang++ (for _Float16 on the host)")
@pytest.mark.parametrize("force_pair", [0, 1])
def test_fp32_decisions_match_fp64_rounding(tmp_path, force_pair):
    exe = tmp_path / "decide"
    src = tmp_path / "decide.cpp"
    src.write_text(SRC)
    subprocess.check_call([CLANG, "-std=c++17", "-O1", "-I", os.path.join(ROOT, "paper_2405_04532_amd", "csrc"),
                           str(src), "-o", str(exe)])
    n = 4_000_000
    x, g, r = _triples(20 + force_pair, n)
    fin, fout = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(fin, "wb") as f:
        f.write(np.int64(n).tobytes()); f.write(x.tobytes()); f.write(g.tobytes()); f.write(r.tobytes())
    subprocess.check_call([str(exe), str(fin), str(fout), str(force_pair)])
    got = np.fromfile(fout, dtype=np.uint32)
    with np.errstate(over="ignore"):
        want = (x.view(np.float16).astype(np.float64) * r * g.view(np.float16).astype(np.float64)).astype(np.float16)
    want = want.view(np.uint16).astype(np.uint32)
    decided = got != 0xFFFFFFFF
    assert (got[decided] == want[decided]).all(), np.argwhere(decided & (got != want))[:5]
    assert (~decided).sum() <= 8                                  # within 2^-36 of a midpoint: a handful in millions
    # the sample does exercise what it is meant to: subnormal, zero, ordinary and overflowing results
    assert ((want & 0x7FFF) == 0x7C00).sum() > 1000 and ((want & 0x7C00) == 0).sum() > 1000 and (want == 0x8000).sum() >= 400
