"""Pins for the CPU oracle's quantizers: what the paper prints, exhaustive integer
sweeps, half-step bounds, exact-rational recomputation and closed forms (CPU only)."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import qoq_quant as qq

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split()
            out[k] = int(v)
    return out


# ------------------------------------------------------------------ level 2, printed example
def test_paper_overflow_example():
    """Section 4.1: [-113, 120] -> scale 16, zero 7, 120 -> code 15 -> 128 (overflow)."""
    g = _golden("protective_range_example.txt")
    s1, z = qq.level2_group_params(g["group_min"], g["group_max"])
    assert int(s1) == g["scale"] and int(z) == g["zero"]
    code = qq.level2_encode(g["value"], s1, z)
    assert int(code) == g["code"]                      # the tie 14.5 goes up
    assert int((code - z) * s1) == g["dequantized"]    # beyond INT8 max 127
    assert g["dequantized"] > 127


def test_paper_scale_bound_and_protective_max():
    """Section 4.1: s_u8 <= (127-(-128))/15 = 17 over the full INT8 span; inside the
    protective range the span is at most 238, so s1 <= 16 and 119 + 16/2 = 127 still fits."""
    g = _golden("protective_range_example.txt")
    s1, _ = qq.level2_group_params(-128, 127)
    assert int(s1) == g["scale_bound"]
    assert qq.PROTECT == g["protective_max"]
    s1, _ = qq.level2_group_params(-qq.PROTECT, qq.PROTECT)
    assert int(s1) == 16 and qq.PROTECT + int(s1) // 2 == 127


# ------------------------------------------------------------------ level 2, exhaustive sweep
def _all_groups(limit):
    lo, hi = np.meshgrid(np.arange(-limit, 1), np.arange(0, limit + 1), indexing="ij")
    return lo.ravel(), hi.ravel()


def test_level2_exhaustive_inside_protective_range():
    """Every (lo, hi, q) with lo <= q <= hi inside [-119, 119]: half-step round trip, no
    INT8 overflow, parameter ranges, and the byte-product bounds the packed dequantizer of
    Section 5.2.3 relies on (code*s1 and z*s1 fit one unsigned byte)."""
    lo, hi = _all_groups(119)
    s1, z = qq.level2_group_params(lo, hi)
    assert s1.min() >= 1 and s1.max() <= 16
    assert z.min() >= 0 and z.max() <= 15
    assert (z * s1).max() <= 240
    worst = 0
    for q in range(-119, 120):
        m = (lo <= q) & (q <= hi)
        code = qq.level2_encode(q, s1[m], z[m])
        assert code.min() >= 0 and code.max() <= 15
        w_hat = (code - z[m]) * s1[m]
        assert (2 * np.abs(w_hat - q) <= s1[m]).all(), q          # |q_hat - q| <= s1/2
        assert w_hat.min() >= -127 and w_hat.max() <= 127
        assert (code * s1[m]).max() <= 240
        assert (w_hat + 128).min() >= 1 and (w_hat + 128).max() <= 255
        worst = max(worst, int(np.abs(w_hat).max()))
    assert worst > 119      # dequantized values do leave [-119,119]; the margin is used


def test_level2_overflows_without_protection():
    """Without the protective range (full INT8 span) some group does overflow INT8: the
    paper's reason for shrinking level 1 to [-119, 119]."""
    lo, hi = _all_groups(127)
    s1, z = qq.level2_group_params(lo, hi)
    w_top = (qq.level2_encode(hi, s1, z) - z) * s1
    assert w_top.max() > 127


def test_level2_literal_nearest_scale_breaks_half_step():
    """Why the scale is rounded up: the encoder run with the scale rounded to NEAREST (span 112 -> 7, which covers
    only 105) saturates the top code and breaks the half-step bound the protective range is derived from; with
    the oracle's own scale (8) the same values round-trip within half a step."""
    lo, hi = 0, 112
    q = np.arange(lo, hi + 1)
    s_near = np.int64((2 * (hi - lo) + 15) // 30)                    # round-half-up of span / 15
    z_near = np.int64((2 * (-lo) + s_near) // (2 * s_near))
    assert int(s_near) == 7 and int(z_near) == 0
    back = (qq.level2_encode(q, s_near, z_near) - z_near) * s_near    # the oracle's encoder, literal nearest scale
    assert int(back.max()) == 105                                     # 112 saturates at code 15
    assert (2 * np.abs(back - q) > s_near).any()                      # half-step bound violated (112 - 105 = 7 > 3.5)
    s1, z = qq.level2_group_params(lo, hi)
    assert int(s1) == 8 and int(z) == 0
    back = (qq.level2_encode(q, s1, z) - z) * s1
    assert (2 * np.abs(back - q) <= s1).all() and int(back.max()) == 112


def test_level2_group_layout_and_roundtrip():
    rng = np.random.default_rng(1)
    q0 = rng.integers(-119, 120, size=(6, 384))
    q0[0, :128] = 5            # constant positive group: range widened to include 0
    q0[1, 128:256] = 0         # all-zero group
    q0[2, :] = -119
    code, s1, z = qq.level2_quant(q0)
    assert s1.shape == (6, 3) and z.shape == (6, 3)
    w_hat = qq.level2_dequant(code, s1, z)
    assert (2 * np.abs(w_hat - q0) <= np.repeat(s1, 128, axis=1)).all()
    assert (w_hat[0, :128] == 5).all() and int(s1[0, 0]) == 1 and int(z[0, 0]) == 0
    assert (w_hat[1, 128:256] == 0).all() and int(s1[1, 1]) == 1
    # groups are consecutive k: changing one element only changes its own group
    q1 = q0.copy()
    q1[3, 130] = 119
    c1, s1b, zb = qq.level2_quant(q1)
    assert (c1[3, :128] == code[3, :128]).all() and (c1[3, 256:] == code[3, 256:]).all()
    assert (s1b[3, [0, 2]] == s1[3, [0, 2]]).all()


# ------------------------------------------------------------------ level 1
def _exact_half_away(fr):
    n = abs(fr)
    r = (2 * n.numerator + n.denominator) // (2 * n.denominator)
    return r if fr >= 0 else -r


def test_level1_half_step_and_range():
    rng = np.random.default_rng(2)
    w = (rng.standard_normal((64, 512)) * 0.02).astype(np.float16)
    w[3] *= 10
    w[5] = 0                     # zero channel
    q0, s0 = qq.level1_quant(w)
    assert s0.dtype == np.float16 and q0.min() >= -119 and q0.max() <= 119
    assert s0[5] == 1.0 and (q0[5] == 0).all()
    err = np.abs(w.astype(np.float64) - q0 * s0.astype(np.float64)[:, None])
    assert (err <= s0.astype(np.float64)[:, None] / 2).all()
    assert (np.abs(q0).max(axis=1)[[0, 1, 2, 3, 4]] == 119).all()   # the max element maps to +-119


def test_level1_exact_rational():
    """Recompute scale and codes with exact fractions (independent of float64 division)."""
    rng = np.random.default_rng(3)
    w = (rng.standard_normal((8, 128)) * 0.05).astype(np.float16)
    w[0, :5] = np.float16(0.5) * np.array([1, 3, 5, 7, 119], dtype=np.float16) / 119  # near ties
    q0, s0 = qq.level1_quant(w)
    for n in range(w.shape[0]):
        amax = max(abs(Fraction(float(v))) for v in w[n])
        s_exact = amax / 119
        # FP16 RNE of the exact scale: nearest of the two neighbouring halves
        s_f = np.float16(float(s_exact))
        cands = [np.nextafter(s_f, np.float16(0)), s_f, np.nextafter(s_f, np.float16(np.inf))]
        best = min(cands, key=lambda c: (abs(Fraction(float(c)) - s_exact), int(c.view(np.uint16)) & 1))
        assert s0[n] == best
        sf = Fraction(float(s0[n]))
        for k in range(w.shape[1]):
            q = _exact_half_away(Fraction(float(w[n, k])) / sf)
            assert q0[n, k] == max(-119, min(119, q))


def test_level1_closed_form_exact_roundtrip():
    """A row made of integer multiples of a power-of-two step whose max is 119 steps
    round-trips exactly."""
    step = 2.0 ** -10
    ints = np.arange(-119, 120)
    w = (ints * step).astype(np.float16)[None, :]
    q0, s0 = qq.level1_quant(np.tile(w, (1, 1)))
    assert float(s0[0]) == step and (q0[0] == ints).all()


def test_half_away_ties():
    assert list(qq._half_away(np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 14.5, 0.49, -0.49]))) == \
        [1, 2, 3, -1, -2, -3, 15, 0, 0]


# ------------------------------------------------------------------ activations
def test_act_quant_bounds_and_sums():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((9, 256)).astype(np.float16)
    x[:, 7] *= 20
    x[4] = 0
    qx, sx, rowsum, tx = qq.act_quant(x)
    assert qx.min() >= -127 and qx.max() <= 127 and sx.dtype == np.float16
    assert sx[4] == 1.0 and (qx[4] == 0).all() and rowsum[4] == 0
    xs = x.astype(np.float64)
    assert (np.abs(xs - qx * sx.astype(np.float64)[:, None]) <= sx.astype(np.float64)[:, None] / 2).all()
    assert (np.abs(qx).max(axis=1)[[0, 1, 2, 3]] == 127).all()
    assert (rowsum == [int(sum(int(v) for v in r)) for r in qx]).all()
    assert np.allclose(tx, [sum(float(v) for v in r) for r in x], rtol=0, atol=1e-9)


def test_act_quant_closed_form():
    ints = np.arange(-127, 128)
    x = (ints * 2.0 ** -6).astype(np.float16)[None, :]
    qx, sx, rowsum, tx = qq.act_quant(x)
    assert float(sx[0]) == 2.0 ** -6 and (qx[0] == ints).all() and rowsum[0] == 0 and tx[0] == 0.0


def test_act_quant_exact_rational():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((4, 64)).astype(np.float16)
    qx, sx, _, _ = qq.act_quant(x)
    for m in range(4):
        sf = Fraction(float(sx[m]))
        for k in range(64):
            assert qx[m, k] == max(-127, min(127, _exact_half_away(Fraction(float(x[m, k])) / sf)))


# ------------------------------------------------------------------ per-channel variant
def test_per_channel_quant_bounds():
    rng = np.random.default_rng(6)
    w = (rng.standard_normal((32, 256)) * 0.02).astype(np.float16)
    w[1] = np.abs(w[1])          # all-positive channel: zero point 0
    w[2] = 0
    code, z, sw = qq.per_channel_quant(w)
    assert code.min() >= 0 and code.max() <= 15 and z.min() >= 0 and z.max() <= 15
    assert z[1] == 0 and sw[2] == 1.0 and (code[2] == z[2]).all()
    s = sw.astype(np.float64)[:, None]
    w_hat = (code - z[:, None]) * s
    inner = (code > 0) & (code < 15)
    assert (np.abs(w.astype(np.float64) - w_hat)[inner] <= (s / 2 + 0 * w_hat)[inner]).all()
    # saturated ends can only be off by the FP16 rounding of the scale: below one full step
    assert (np.abs(w.astype(np.float64) - w_hat) <= s).all()


def test_per_channel_closed_form():
    codes = np.arange(16)
    w = ((codes - 5) * 2.0 ** -7).astype(np.float16)[None, :]
    code, z, sw = qq.per_channel_quant(w)
    assert float(sw[0]) == 2.0 ** -7 and int(z[0]) == 5 and (code[0] == codes).all()


def test_per_channel_exact_rational():
    rng = np.random.default_rng(7)
    w = (rng.standard_normal((4, 64)) * 0.02).astype(np.float16)
    code, z, sw = qq.per_channel_quant(w)
    for n in range(4):
        sf = Fraction(float(sw[n]))
        lo = min(Fraction(0), min(Fraction(float(v)) for v in w[n]))
        assert z[n] == max(0, min(15, _exact_half_away(-lo / sf)))
        for k in range(64):
            assert code[n, k] == max(0, min(15, _exact_half_away(Fraction(float(w[n, k])) / sf + int(z[n]))))


# ------------------------------------------------------------------ FP16 output rounding
def test_output_fp16_is_rne():
    acc = np.array([[2049, 2051, 1]], dtype=np.int64)          # 2049 and 2051 are FP16 ties
    out = qq.output_fp16(acc, np.array([1.0], np.float16), np.array([1.0, 1.0, 1.0], np.float16))
    assert list(out[0][:2]) == [2048.0, 2052.0]                 # ties to even
    out = qq.output_fp16(np.array([[3]]), np.array([0.5], np.float16), np.array([0.25], np.float16))
    assert float(out[0, 0]) == 0.375


@pytest.mark.parametrize("bad", ["no_zero", "trunc", "nearest_scale"])
def test_pins_catch_planted_mistakes(bad, monkeypatch):
    """Plant a plausible mistake in the oracle and check that a pin above fails."""
    if bad == "no_zero":
        monkeypatch.setattr(qq, "level2_encode", lambda q, s1, z: np.clip(np.floor_divide(2 * np.asarray(q) + s1, 2 * s1), 0, 15))
        with pytest.raises(AssertionError):
            test_paper_overflow_example()
    elif bad == "trunc":
        monkeypatch.setattr(qq, "_half_away", lambda x: np.trunc(np.asarray(x, dtype=np.float64)).astype(np.int64))
        with pytest.raises(AssertionError):
            test_level1_exact_rational()
    else:
        def near(lo, hi):
            lo = np.minimum(np.asarray(lo, dtype=np.int64), 0)
            hi = np.maximum(np.asarray(hi, dtype=np.int64), 0)
            s1 = np.maximum(1, (2 * (hi - lo) + 15) // 30)
            return s1, np.clip((2 * (-lo) + s1) // (2 * s1), 0, 15)
        monkeypatch.setattr(qq, "level2_group_params", near)
        with pytest.raises(AssertionError):
            test_level2_exhaustive_inside_protective_range()


# ------------------------------------------------------------------ producers of the fused quantization
def test_rmsnorm_closed_forms():
    import math
    # constant row c: mean square c^2, y = gamma * c / sqrt(c^2 + eps)
    x = np.full((1, 64), 0.5, dtype=np.float16)
    g = np.linspace(0.5, 2.0, 64).astype(np.float16)
    y = qq.rmsnorm_fp16(x, g, 1e-5)
    expect = (g.astype(np.float64) * 0.5 / math.sqrt(0.25 + 1e-5)).astype(np.float16)
    assert np.array_equal(y[0].view(np.uint16), expect.view(np.uint16))
    # eps = 0: scale invariance, and unit mean square before gamma
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 128)).astype(np.float16)
    ones = np.ones(128, dtype=np.float16)
    y1 = qq.rmsnorm_fp16(x, ones, 0.0).astype(np.float64)
    y2 = qq.rmsnorm_fp16((x.astype(np.float64) * 4).astype(np.float16), ones, 0.0).astype(np.float64)   # exact scaling by 4
    assert np.array_equal(y1, y2)
    assert np.allclose((y1 * y1).mean(axis=1), 1.0, atol=2e-3)


def test_rmsnorm_against_per_element_fractions():
    from fractions import Fraction
    import math
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 16)).astype(np.float16)
    g = (rng.random(16) + 0.5).astype(np.float16)
    eps = 1e-6
    y = qq.rmsnorm_fp16(x, g, eps)
    for m in range(2):
        ms = sum(Fraction(float(v)) ** 2 for v in x[m]) / 16 + Fraction(eps)
        inv = 1.0 / math.sqrt(float(ms))
        for k in range(16):
            want = np.float16(float(x[m, k]) * inv * float(g[k]))
            assert abs(float(y[m, k]) - float(want)) <= abs(float(want)) * 2 ** -10   # at most one FP16 ulp apart


def _golden_lines(name):
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
    return [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]


def _silu_mul_against_decimal():
    """400 (gate, up) pairs whose expected FP16 bits were computed from g / (1 + exp(-g)) * u in 60-digit decimal
    arithmetic by tests/golden/make_producer_golden.py (which imports nothing of the oracle)."""
    rows = _golden_lines("silu_mul_decimal.txt")
    assert len(rows) == 400
    g = np.array([int(r[0], 16) for r in rows], dtype=np.uint16).view(np.float16)
    u = np.array([int(r[1], 16) for r in rows], dtype=np.uint16).view(np.float16)
    want = np.array([int(r[2], 16) for r in rows], dtype=np.uint16)
    with np.errstate(over="ignore"):
        got = qq.silu_mul_fp16(np.concatenate([g, u])[None, :])[0].view(np.uint16)
    # +0 and -0 are the same number: the decimal computation has no signed zero
    same = (got == want) | (((got | want) & 0x7FFF) == 0)
    assert same.all(), "first mismatch at pair %d" % int(np.argmin(same))
    assert int(((want & 0x7FFF) != 0).sum()) > 300                 # most pairs have a non-zero result


def test_silu_mul_literal_values():
    _silu_mul_against_decimal()
    # a few values one can check by hand: silu(0) = 0; silu(1) * 2 = 2 / (1 + 1/e) = 1.46211715...; silu(-1) * 2 = -0.53788...
    y = qq.silu_mul_fp16(np.array([[0.0, 1.0, -1.0, 3.0, 2.0, 2.0]], dtype=np.float16))[0].astype(np.float64)
    assert y[0] == 0.0 and abs(y[1] - 1.4621171572600098) < 2 ** -10 and abs(y[2] + 0.5378828427399902) < 2 ** -11
    # orientation: gate is the FIRST half
    z = qq.silu_mul_fp16(np.array([[0.0, 5.0]], dtype=np.float16))
    assert float(z[0, 0]) == 0.0


@pytest.mark.parametrize("bad", ["exponent_sign", "halves_swapped", "sigmoid_only"])
def test_silu_mul_pins_catch_planted_mistakes(bad, monkeypatch):
    def wrong(gate_up_fp16):
        a = np.asarray(gate_up_fp16, dtype=np.float16).astype(np.float64)
        k = a.shape[1] // 2
        gate, up = (a[:, k:], a[:, :k]) if bad == "halves_swapped" else (a[:, :k], a[:, k:])
        with np.errstate(over="ignore"):
            if bad == "exponent_sign":
                return (gate / (1.0 + np.exp(gate)) * up).astype(np.float16)
            if bad == "sigmoid_only":
                return (1.0 / (1.0 + np.exp(-gate)) * up).astype(np.float16)
            return (gate / (1.0 + np.exp(-gate)) * up).astype(np.float16)
    monkeypatch.setattr(qq, "silu_mul_fp16", wrong)
    with pytest.raises(AssertionError):
        _silu_mul_against_decimal()


def _rmsnorm_against_decimal():
    """Eight token rows (eps = 0, the usual 1e-5/1e-6, large eps, an all-zero token) whose expected FP16 bits come
    from x * gamma / sqrt(mean(x^2) + eps) in 60-digit decimal arithmetic (tests/golden/make_producer_golden.py)."""
    rows = _golden_lines("rmsnorm_decimal.txt")
    i = 0
    seen = 0
    while i < len(rows):
        assert rows[i][0] == "row" and rows[i][2] == "eps"
        eps = float.fromhex(rows[i][3])
        body = rows[i + 1:i + 33]
        x = np.array([int(r[0], 16) for r in body], dtype=np.uint16).view(np.float16)
        g = np.array([int(r[1], 16) for r in body], dtype=np.uint16).view(np.float16)
        want = np.array([int(r[2], 16) for r in body], dtype=np.uint16)
        got = qq.rmsnorm_fp16(x[None, :], g, eps)[0].view(np.uint16)
        same = (got == want) | (((got | want) & 0x7FFF) == 0)
        assert same.all(), "row %d element %d" % (seen, int(np.argmin(same)))
        i += 33
        seen += 1
    assert seen == 8


def test_rmsnorm_literal_values():
    _rmsnorm_against_decimal()


@pytest.mark.parametrize("bad", ["sum_not_mean", "eps_outside_root", "no_gamma", "no_root"])
def test_rmsnorm_pins_catch_planted_mistakes(bad, monkeypatch):
    def wrong(x_fp16, gamma_fp16, eps):
        x = np.asarray(x_fp16, dtype=np.float16).astype(np.float64)
        g = np.asarray(gamma_fp16, dtype=np.float16).astype(np.float64)
        ms = (x * x).sum(axis=1) / (1 if bad == "sum_not_mean" else x.shape[1])
        with np.errstate(divide="ignore", invalid="ignore"):
            if bad == "eps_outside_root":
                r = 1.0 / (np.sqrt(ms) + float(eps))
            elif bad == "no_root":
                r = 1.0 / (ms + float(eps))
            else:
                r = 1.0 / np.sqrt(ms + float(eps))
            y = x * r[:, None] * (1.0 if bad == "no_gamma" else g[None, :])
        return np.nan_to_num(y).astype(np.float16)
    monkeypatch.setattr(qq, "rmsnorm_fp16", wrong)
    with pytest.raises(AssertionError):
        _rmsnorm_against_decimal()


def test_rmsnorm_evaluation_order_is_pinned():
    """The order of the FP64 operations is part of the definition: y = fp16((x * r) * gamma) with r = 1 / sqrt(mean(x^2) + eps)
    formed once per token.  The other natural order, (x / sqrt(...)) * gamma, agrees except when the exact value
    lies within about 1e-16 (relative) of an FP16 rounding midpoint.  Such inputs are constructed here by steering
    eps (any non-negative double is a valid input) so that one element's exact value falls next to a midpoint; in
    every case below the two orders round to different FP16 numbers, and the oracle must give the first order's.
    Which of the two is the correctly rounded exact value varies from case to case (checked in exact rationals):
    neither order is "the" right one, so the choice is a convention, and this test is what fixes it."""
    import math
    from fractions import Fraction
    K = 128
    x = np.array([(((k * 37) % 129) - 64) / 64.0 for k in range(K)], dtype=np.float16)
    ms = sum(Fraction(float(v)) ** 2 for v in x) / K
    cases = [(1, 15039, "0x1.4482d7f405400p-12"), (1, 14558, "0x1.e2b71aa2c8000p-14"), (2, 14521, "0x1.0c3642b521200p-11"),
             (2, 14632, "0x1.fb0326ebc4400p-12"), (1, 15409, "0x1.8986b51166800p-12"), (1, 15816, "0x1.03f1748838600p-11")]
    chosen_is_exact = []
    for k0, gbits, eps_hex in cases:
        eps = float.fromhex(eps_hex)
        g = np.ones(K, dtype=np.float16)
        g[k0] = np.array([gbits], dtype=np.uint16).view(np.float16)[0]
        x0, g0 = float(x[k0]), float(g[k0])
        t = float(ms) + eps
        assert Fraction(t) == ms + Fraction(eps)                           # the sum under the root is exact here
        root = math.sqrt(t)
        first = np.float16((x0 * (1.0 / root)) * g0)                       # reciprocal root once per token, multiplied in
        other = np.float16((x0 / root) * g0)
        assert first != other                                              # a genuine straddle
        y = qq.rmsnorm_fp16(x[None, :], g, eps)[0]
        assert y[k0] == first, (k0, gbits)
        # the exact value: |x0 g0| / sqrt(t) compared with the midpoint between the two candidates, on squares
        mid = (Fraction(float(first)) + Fraction(float(other))) / 2
        above = (Fraction(x0) * Fraction(g0)) ** 2 > mid ** 2 * Fraction(t)
        exact = max(first, other, key=lambda v: abs(float(v))) if above else min(first, other, key=lambda v: abs(float(v)))
        chosen_is_exact.append(bool(exact == first))
    assert any(chosen_is_exact) and not all(chosen_is_exact)
