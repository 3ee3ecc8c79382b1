"""CPU oracle for the KV4 cache quantizer and decode attention (TEST INFRASTRUCTURE ONLY).

Plain definition, written from the paper (arXiv 2405.04532), of
  * per-head, dynamic, asymmetric 4-bit quantization of key/value vectors (Section 5.1 "KV Cache
    Management" and Section 6.1: per-head asymmetric INT4; Eq. 1-2 with q_min = 0, q_max = 15), with the
    FP16 scale and zero point the cache stores per head and token;
  * attention of one new query token per sequence over the dequantized cache (Section 3.1, the attention
    equation: o_h = softmax(q_h K^T / sqrt(D)) V with h_KV = floor(h / r)).
Only tests, the smoke check and the benchmark's cpu_baseline leg may import this file.  It shares no code
with the HIP path.

All arithmetic is float64; FP16 inputs are read exactly; the only rounding to FP16 is the stored scale.
Readings (the paper gives Eq. 1 and says "per-head", "dynamic", "FP16 scaling factors and zero points"):
  * one (scale, zero) pair per token and KV head, from that head's D values of that token;
  * the range is widened to contain 0, as for the weights, so the zero point is an integer in [0, 15]
    (exactly representable in FP16) and a vector of one sign keeps its zero representable;
  * s = fp16((max - min) / 15); an all-zero vector gets s = 1; the stored s is the divisor;
  * rounding is half up (floor(t + 1/2)): every rounded quantity here is non-negative, where this equals
    the round-half-away reading used for the weights;
  * codes are clamped to [0, 15] (the FP16 rounding of s can push the top code to 16);
  * an empty sequence (length 0) gives a zero output row.
"""
import numpy as np

QMAX = 15


def kv4_quantize(x_fp16):
    """Eq. 1 per vector along the last axis.

    x_fp16: [..., D] float16.  Returns (codes uint8 [..., D] in [0, 15], s float16 [...], z float16 [...]).
    """
    x = np.asarray(x_fp16, dtype=np.float16).astype(np.float64)
    lo = np.minimum(x.min(axis=-1), 0.0)
    hi = np.maximum(x.max(axis=-1), 0.0)
    s = ((hi - lo) / float(QMAX)).astype(np.float16)
    s = np.where(s == 0, np.float16(1.0), s).astype(np.float16)
    s64 = s.astype(np.float64)
    z = np.clip(np.floor(-lo / s64 + 0.5), 0, QMAX)
    t = x / s64[..., None] + z[..., None]
    codes = np.clip(np.floor(t + 0.5), 0, QMAX).astype(np.uint8)
    return codes, s, z.astype(np.float16)


def kv4_dequantize(codes, s, z):
    """Eq. 2: (Q - z) * s, exact in float64."""
    return (codes.astype(np.float64) - z.astype(np.float64)[..., None]) * s.astype(np.float64)[..., None]


def attention_decode(q_fp16, k_codes, k_s, k_z, v_codes, v_s, v_z, seq_lens):
    """One query token per sequence against its quantized cache (Section 3.1).

    q_fp16 [B, H, D]; k_codes, v_codes [B, Hkv, S, D] uint8; k_s, k_z, v_s, v_z [B, Hkv, S] float16;
    seq_lens [B] (tokens of the cache that count).  Returns float64 [B, H, D].
    """
    q = np.asarray(q_fp16, dtype=np.float16).astype(np.float64)
    B, H, D = q.shape
    Hkv = k_codes.shape[1]
    assert H % Hkv == 0
    r = H // Hkv
    out = np.zeros((B, H, D), dtype=np.float64)
    for b in range(B):
        L = int(seq_lens[b])
        if L == 0:
            continue
        for h in range(H):
            hk = h // r
            k_hat = kv4_dequantize(k_codes[b, hk, :L], k_s[b, hk, :L], k_z[b, hk, :L])
            v_hat = kv4_dequantize(v_codes[b, hk, :L], v_s[b, hk, :L], v_z[b, hk, :L])
            score = k_hat @ q[b, h] / np.sqrt(float(D))
            p = np.exp(score - score.max())
            p = p / p.sum()
            out[b, h] = p @ v_hat
    return out
