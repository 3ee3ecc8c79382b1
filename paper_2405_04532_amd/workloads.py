"""Seeded synthetic inputs and layer shapes for the W4A8 GEMM workloads.

This module holds no quantization or GEMM arithmetic: it only names the layer shapes
of the benchmark configurations and draws FP16 weights and activations from a
counter-based generator, so the CPU oracle and the HIP path can be fed the very same
tensors.  It imports neither of them.

The tensors stand in for LLM checkpoints and real activations, which are not available:
Gaussian bulk plus a small fixed set of outlier channels roughly 10x (weights) or 20x
(activations) larger, the structure Sections 4.2-4.3 of arXiv 2405.04532 describe
for Key/activation channels.

Generator: value(i) is a pure function of (seed, stream, flat index i): a SplitMix64
finalizer gives 64 uniform bits per counter, two counters feed one Box-Muller normal in
float64.  It runs on any torch device; a run draws each tensor once and hands the same
tensor to both sides, so results need not be bit-identical across devices.
"""
import math

import torch

_M64 = (1 << 64) - 1


def _s64(v):
    """Python int -> value representable in torch.int64 with the same low 64 bits."""
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)


def _lsr(x, s):
    """Logical right shift of int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x):
    """SplitMix64 finalizer on an int64 tensor (wrapping arithmetic)."""
    x = (x ^ _lsr(x, 30)) * _C1
    x = (x ^ _lsr(x, 27)) * _C2
    return x ^ _lsr(x, 31)


def _key(seed, stream):
    k = (seed * 0x9E3779B97F4A7C15 + (stream + 1) * 0xD1B54A32D192ED03) & _M64
    # one scalar mixing round in Python
    k ^= k >> 30
    k = (k * 0xBF58476D1CE4E5B9) & _M64
    k ^= k >> 27
    k = (k * 0x94D049BB133111EB) & _M64
    k ^= k >> 31
    return _s64(k)


def uniform_bits(seed, stream, start, count, device):
    """64 random bits for counters start .. start+count-1, as int64 tensor."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix(idx * _GOLDEN + _key(seed, stream))


def _unit(bits):
    """(0, 1] float64 from the top 53 bits."""
    return (_lsr(bits, 11).to(torch.float64) + 1.0) * (1.0 / 9007199254740992.0)


def normal(seed, stream, count, device, start=0):
    """`count` standard normals (float64) for counters start.. of (seed, stream)."""
    u1 = _unit(uniform_bits(seed, 2 * stream, start, count, device))
    u2 = _unit(uniform_bits(seed, 2 * stream + 1, start, count, device))
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def pick_channels(seed, stream, total, count, device="cpu"):
    """`count` distinct channel indices out of `total`: smallest hashes win."""
    if count <= 0:
        return torch.empty(0, dtype=torch.int64, device=device)
    h = uniform_bits(seed, stream, 0, total, "cpu")
    return torch.argsort(h, stable=True)[:count].sort().values.to(device)


def _rows_normal(seed, stream, rows, cols, device, chunk_rows=None):
    """[rows, cols] standard normals, drawn in row chunks to bound peak memory."""
    out = torch.empty((rows, cols), dtype=torch.float64, device=device)
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 24) // max(cols, 1))
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        out[r0:r1] = normal(seed, stream, (r1 - r0) * cols, device, start=r0 * cols).view(r1 - r0, cols)
    return out


def make_weights(N, K, seed, device="cpu", sigma=0.02, outlier_rate=0.01, outlier_count=None,
                 outlier_kind="x10"):
    """FP16 weights [N, K] (one row per output channel).

    Bulk ~ N(0, sigma).  A seeded set of round(outlier_rate*N) output channels (or exactly
    `outlier_count`) is either scaled x10 ("x10") or redrawn as sigma * Student-t(nu=3)
    ("t3": heavy tails inside the channel).
    """
    w = _rows_normal(seed, 0, N, K, device) * sigma
    cnt = outlier_count if outlier_count is not None else int(round(outlier_rate * N))
    rows = pick_channels(seed, 101, N, cnt, device)
    if cnt > 0:
        if outlier_kind == "x10":
            w[rows] = w[rows] * 10.0
        elif outlier_kind == "t3":
            z0 = normal(seed, 10, cnt * K, device).view(cnt, K)
            d = sum(normal(seed, 11 + j, cnt * K, device).view(cnt, K) ** 2 for j in range(3))
            w[rows] = sigma * z0 / torch.sqrt(d / 3.0)
        else:
            raise ValueError(outlier_kind)
    return w.to(torch.float16)


def make_activations(M, K, seed, device="cpu", outlier_rate=0.01, outlier_count=None, gain=20.0):
    """FP16 activations [M, K] ~ N(0, 1) with a seeded set of input channels x`gain`."""
    x = _rows_normal(seed, 1, M, K, device)
    cnt = outlier_count if outlier_count is not None else int(round(outlier_rate * K))
    cols = pick_channels(seed, 102, K, cnt, device)
    if cnt > 0:
        x[:, cols] = x[:, cols] * gain
    return x.to(torch.float16)


# ---------------------------------------------------------------------------------------
# Layer shapes (K = input channels, N = output channels) of the benchmark configurations.
# ---------------------------------------------------------------------------------------
LLAMA2_7B = {"qkv": (4096, 12288), "o": (4096, 4096), "gate_up": (4096, 22016), "down": (11008, 4096)}
LLAMA3_70B = {"qkv": (8192, 10240), "o": (8192, 8192), "gate_up": (8192, 57344), "down": (28672, 8192)}
LLAMA3_8B = {"qkv": (4096, 6144), "gate_up": (4096, 28672), "down": (14336, 4096)}

M_SWEEP = (1, 8, 32, 128, 256, 512, 1024, 2048, 4096)


def _layer_seed(base, layer):
    return base * 1000 + sum(ord(c) * (i + 1) for i, c in enumerate(layer))


def config0(device="cpu"):
    """Tiny case: M=16, K=256, N=256, seed 0; 2 outlier output channels x10, 4 outlier
    input channels x20."""
    w = make_weights(256, 256, 0, device, outlier_count=2)
    x = make_activations(16, 256, 0, device, outlier_count=4)
    return w, x


def layer_weights(family, layer, base_seed, device="cpu"):
    """Weights of one named layer. family: 'llama2_7b' | 'llama3_70b' | 'llama3_8b'."""
    shapes = {"llama2_7b": LLAMA2_7B, "llama3_70b": LLAMA3_70B, "llama3_8b": LLAMA3_8B}[family]
    K, N = shapes[layer]
    seed = _layer_seed(base_seed, layer)
    if family == "llama3_70b":
        return make_weights(N, K, seed, device, sigma=0.01, outlier_kind="t3")
    return make_weights(N, K, seed, device)


def layer_activations(family, layer, M, base_seed, device="cpu"):
    shapes = {"llama2_7b": LLAMA2_7B, "llama3_70b": LLAMA3_70B, "llama3_8b": LLAMA3_8B}[family]
    K, _ = shapes[layer]
    return make_activations(M, K, _layer_seed(base_seed, layer) + 7919 * M, device)


# ---------------------------------------------------------------------------------------
# Decode attention over a 4-bit KV cache: synthetic keys, values and queries.
# ---------------------------------------------------------------------------------------
KV4_DECODE = {"llama2_7b": dict(H=32, Hkv=32, D=128), "llama3_8b": dict(H=32, Hkv=8, D=128),
              "llama3_70b": dict(H=64, Hkv=8, D=128)}


def make_kv(B, Hkv, S, D, seed, device="cpu", key_outliers=2, gain=8.0):
    """FP16 keys and values [B, Hkv, S, D] ~ N(0, 1).  In every KV head `key_outliers` seeded channels of
    the keys are scaled by `gain` for all tokens (keys have a few fixed large channels, values do not)."""
    k = _rows_normal(seed, 3, B * Hkv * S, D, device).view(B, Hkv, S, D)
    v = _rows_normal(seed, 4, B * Hkv * S, D, device).view(B, Hkv, S, D)
    for h in range(Hkv):
        cols = pick_channels(seed, 200 + h, D, key_outliers, device)
        if key_outliers > 0:
            k[:, h, :, cols] = k[:, h, :, cols] * gain
    return k.to(torch.float16), v.to(torch.float16)


def make_queries(B, H, D, seed, device="cpu"):
    """FP16 queries [B, H, D] ~ N(0, 1), one new token per sequence."""
    return _rows_normal(seed, 5, B * H, D, device).view(B, H, D).to(torch.float16)
