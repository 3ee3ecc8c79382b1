"""CPU oracle for the QoQ W4A8 quantizers and epilogue (TEST INFRASTRUCTURE ONLY).

This file is the slow, plain definition of what the W4A8 hot path computes, written
from the paper (arXiv 2405.04532).  It is test infrastructure: only tests, the smoke
check and the benchmark's cpu_baseline leg may import it.  It shares no code with the
HIP path and must never be imported by the product package.

All floating-point math is float64, all integer math is int64.  FP16 tensors are
numpy float16 arrays whose values are read exactly; the only roundings to FP16 are the
stored scales and the final output (IEEE round-to-nearest-even, numpy's conversion).

Rounding: the paper's round-to-nearest symbol is read as "round half away from zero"
(the one tie the paper prints, 14.5 -> 15 in the protective-range example of Section
4.1, goes up).  On the non-negative level-2 operands this is round-half-up and is done
in exact integer arithmetic.

Pins (tests/test_oracle_*.py): the printed protective-range example, an exhaustive
sweep of every level-2 group range inside [-119, 119], half-step round-trip bounds at
both levels, exact-fraction re-computation on small inputs, and brute-force
dequantize-then-FP64-matmul on tiny shapes.  The two producers (rmsnorm_fp16,
silu_mul_fp16) are pinned by FP16 bit patterns computed in 60-digit decimal arithmetic
(tests/golden/make_producer_golden.py, which imports nothing from here) and, for the
order of the FP64 operations of rmsnorm_fp16, by inputs constructed next to FP16
rounding midpoints on which the other natural order rounds differently.
"""
import numpy as np

GROUP = 128          # level-2 group size g along k (Section 4.1, Eq. 4)
PROTECT = 119        # protective level-1 range [-119, 119] (Section 4.1)


def _half_away(x):
    """Round float64 array to nearest integer, ties away from zero."""
    x = np.asarray(x, dtype=np.float64)
    return (np.sign(x) * np.floor(np.abs(x) + 0.5)).astype(np.int64)


def _fp16_scale(v):
    """Round float64 scale(s) to FP16 (RNE); a zero scale becomes 1.0 (degenerate row)."""
    s = np.asarray(v, dtype=np.float64).astype(np.float16)
    s = np.where(s == 0, np.float16(1.0), s).astype(np.float16)
    return s


def level1_quant(w_fp16, qmax=PROTECT):
    """Per-output-channel symmetric INT8 with the protective range (Section 4.1, Eq. 3).

    w_fp16: [N, K] float16, one row per output channel.
    Returns (q0 int64 [N, K] in [-qmax, qmax], s0 float16 [N]).
    The FP16-rounded stored scale is the divisor, because it is what dequantizes.
    """
    w = np.asarray(w_fp16, dtype=np.float16).astype(np.float64)
    absmax = np.max(np.abs(w), axis=1)
    s0 = _fp16_scale(absmax / float(qmax))
    q0 = _half_away(w / s0.astype(np.float64)[:, None])
    q0 = np.clip(q0, -qmax, qmax)
    return q0, s0


def level2_group_params(lo, hi):
    """Level-2 scale and zero of one group from its integer min/max (Section 4.1, Eq. 4
    with Eq. 1 for n = 4 bits).

    The range is widened to contain 0 so the zero point is a valid UINT4.  The scale is
    the range over 15 rounded UP: with round-to-nearest the top code can saturate and
    the half-step bound q_hat <= q + s/2 that the protective range is derived from no
    longer holds; the paper's printed example (233/15 -> 16) is the same either way.
    z = round_half_up(-lo / s1) in exact integer arithmetic.
    """
    lo = np.minimum(np.asarray(lo, dtype=np.int64), 0)
    hi = np.maximum(np.asarray(hi, dtype=np.int64), 0)
    span = hi - lo
    s1 = np.maximum(1, -((-span) // 15))                 # ceil(span / 15), at least 1
    z = (2 * (-lo) + s1) // (2 * s1)                     # floor(-lo/s1 + 1/2)
    z = np.clip(z, 0, 15)
    return s1, z


def level2_encode(q, s1, z):
    """UINT4 code of integer q under (s1, z): clamp(round_half_up(q/s1 + z), 0, 15)."""
    q = np.asarray(q, dtype=np.int64)
    num = 2 * q + (2 * z + 1) * s1                       # 2*s1*(q/s1 + z + 1/2)
    code = np.floor_divide(num, 2 * s1)                  # mathematical floor
    return np.clip(code, 0, 15)


def level2_quant(q0, group=GROUP):
    """Per-group asymmetric UINT4 on the INT8 intermediates (Section 4.1, Eq. 4).

    q0: int64 [N, K], K a multiple of `group`; groups are `group` consecutive k.
    Returns (Q int64 [N, K] in [0, 15], s1 int64 [N, K/group], z int64 [N, K/group]).
    """
    q0 = np.asarray(q0, dtype=np.int64)
    n, k = q0.shape
    assert k % group == 0
    g = q0.reshape(n, k // group, group)
    s1, z = level2_group_params(g.min(axis=2), g.max(axis=2))
    code = level2_encode(g, s1[:, :, None], z[:, :, None])
    return code.reshape(n, k), s1, z


def level2_dequant(code, s1, z, group=GROUP):
    """INT8 intermediate reconstructed from the 4-bit codes: (Q - z) * s1 (Eq. 4)."""
    code = np.asarray(code, dtype=np.int64)
    n, k = code.shape
    g = code.reshape(n, k // group, group)
    w = (g - z[:, :, None]) * s1[:, :, None]
    return w.reshape(n, k)


def progressive_quant(w_fp16, group=GROUP):
    """Both levels of progressive group quantization (Section 4.1).

    Returns dict with Q, s1, z, s0 and w_hat (the INT8 operand the GEMM multiplies).
    """
    q0, s0 = level1_quant(w_fp16)
    code, s1, z = level2_quant(q0, group)
    w_hat = level2_dequant(code, s1, z, group)
    return dict(q0=q0, s0=s0, Q=code, s1=s1, z=z, w_hat=w_hat)


def per_channel_quant(w_fp16):
    """Per-channel W4 variant: unsigned 4-bit codes with a zero point and one FP16
    scale per output channel, no second level (Section 5.2.2, Eq. 1 with n = 4).

    Returns (Q int64 [N, K] in [0, 15], z int64 [N], sw float16 [N]).
    The range is widened to contain 0; the FP16-rounded scale is the divisor.
    """
    w = np.asarray(w_fp16, dtype=np.float16).astype(np.float64)
    lo = np.minimum(w.min(axis=1), 0.0)
    hi = np.maximum(w.max(axis=1), 0.0)
    sw = _fp16_scale((hi - lo) / 15.0)
    s = sw.astype(np.float64)
    z = np.clip(_half_away(-lo / s), 0, 15)
    code = np.clip(_half_away(w / s[:, None] + z[:, None].astype(np.float64)), 0, 15)
    return code, z, sw


def act_quant(x_fp16):
    """Per-token symmetric INT8 activation quantization (Section 6.1; Eq. 1 symmetric,
    n = 8, so the codes span [-127, 127]).

    x_fp16: [M, K] float16.  Returns (qx int64 [M, K], sx float16 [M],
    rowsum int64 [M] = sum_k qx, tx float64 [M] = sum_k x  (t_X of Eq. 7)).
    """
    x = np.asarray(x_fp16, dtype=np.float16).astype(np.float64)
    absmax = np.max(np.abs(x), axis=1)
    sx = _fp16_scale(absmax / 127.0)
    qx = np.clip(_half_away(x / sx.astype(np.float64)[:, None]), -127, 127)
    return qx, sx, qx.sum(axis=1), x.sum(axis=1)


def gemm_i64_numpy(qx, w_hat):
    """acc[m, n] = sum_k qx[m, k] * w_hat[n, k] in int64 (the INT8 GEMM of Section 4.1).
    Slow library matmul on int64; oracle/gemm_i64.c is the same loop in plain C."""
    qx = np.asarray(qx, dtype=np.int64)
    w_hat = np.asarray(w_hat, dtype=np.int64)
    return qx @ w_hat.T


def per_channel_acc(raw, z, rowsum):
    """Zero-point fold of the per-channel variant in exact integers (Eq. 6):
    sum_k qx*(Q - z) = raw - z[n] * sum_k qx[m, k]."""
    return np.asarray(raw, dtype=np.int64) - np.asarray(rowsum, dtype=np.int64)[:, None] * np.asarray(z, dtype=np.int64)[None, :]


def output_fp64(acc, sx, sw):
    """Epilogue in float64, before the FP16 rounding: acc * sx[m] * sw[n]
    (outer-product scaling of Section 5.2.2; sw is s0 in group mode)."""
    return (np.asarray(acc, dtype=np.float64)
            * np.asarray(sx, dtype=np.float16).astype(np.float64)[:, None]
            * np.asarray(sw, dtype=np.float16).astype(np.float64)[None, :])


def output_fp16(acc, sx, sw):
    """FP16 GEMM output (Section 5.1: every GEMM produces FP16): one RNE rounding."""
    return output_fp64(acc, sx, sw).astype(np.float16)


def output_fp64_token_sum(raw, sx, sw, z, tx):
    """Per-channel epilogue in the subtraction-after-multiplication form the paper fuses into the
    GEMM (Section 5.2.2, Eq. 6 with the quantized activations of its second term replaced by the
    unquantized ones, Eq. 7):

        out[m, n] = raw[m, n] * sx[m] * sw[n]  -  tx[m] * (z[n] * sw[n]),

    raw = sum_k qx * Q (unsigned codes, no zero point), tx[m] = sum_k X[m, k] over the UNQUANTIZED
    activations.  It differs from the exact fold (per_channel_acc + output_fp64) by
    z[n] * sw[n] * sum_k (X - qx * sx)[m, k], the quantization error of the token summed over k.
    """
    s = np.asarray(sw, dtype=np.float16).astype(np.float64)
    first = (np.asarray(raw, dtype=np.float64)
             * np.asarray(sx, dtype=np.float16).astype(np.float64)[:, None] * s[None, :])
    second = np.asarray(tx, dtype=np.float64)[:, None] * (np.asarray(z, dtype=np.float64) * s)[None, :]
    return first - second


# --- memory-bound producers the activation quantization is fused into (Section 5.1) -------------
# The paper quantizes the activations inside the kernel that produces them: the normalisation in front
# of the QKV and first FFN projections, the activation function in front of the second FFN projection.
# The Llama-family models it evaluates use RMSNorm and SiLU(gate) * up.  Both producers emit FP16
# (every tensor between kernels is FP16, Section 5.1), so the fused result is defined as
# act_quant(fp16(producer(x))): one FP64 evaluation, one RNE rounding to FP16, then the quantizer.

def rmsnorm_fp16(x_fp16, gamma_fp16, eps):
    """y[m, k] = fp16( x[m, k] * r[m] * gamma[k] ), r[m] = 1 / sqrt(mean_k x[m, :]^2 + eps): the reciprocal root is
    formed once per token and multiplied in (the usual statement of RMSNorm), all in float64."""
    x = np.asarray(x_fp16, dtype=np.float16).astype(np.float64)
    g = np.asarray(gamma_fp16, dtype=np.float16).astype(np.float64)
    ms = (x * x).sum(axis=1) / x.shape[1]
    r = 1.0 / np.sqrt(ms + float(eps))
    return (x * r[:, None] * g[None, :]).astype(np.float16)


def silu_mul_fp16(gate_up_fp16):
    """gate_up [M, 2K]: gate = first K columns, up = last K.  y = fp16( gate / (1 + exp(-gate)) * up )."""
    a = np.asarray(gate_up_fp16, dtype=np.float16).astype(np.float64)
    k = a.shape[1] // 2
    gate, up = a[:, :k], a[:, k:]
    return (gate / (1.0 + np.exp(-gate)) * up).astype(np.float16)
