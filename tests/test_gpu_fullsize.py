"""Parity at the full layer shapes, in the launch configuration the library picks by itself
(the one bench.py times): sampled output channels are recomputed one by one by the CPU oracle.

For each (family, layer, M) the GPU path runs on the whole layer: pack -> per-token activation
quantization -> GEMM (raw INT32 accumulators and FP16 output).  The oracle quantizes every
token row (cheap) and only the sampled weight rows, and must agree
  * bit for bit on qx, sx and rowsum of every token,
  * bit for bit on the unpacked codes / level-2 scales / zeros / channel scales of the sampled rows,
  * bit for bit on the INT32 accumulators of (all tokens) x (sampled channels),
  * within 1e-3 relative (+2^-24 absolute, the FP16 subnormal step) on the FP16 outputs.
Sampled channels always include the first and last channel, both sides of a 256-channel tile
boundary, and seeded picks elsewhere, so every corner of the tiling is touched.
"""
import numpy as np
import pytest
import torch

from paper_2405_04532_amd import api, workloads as wl

pytestmark = pytest.mark.gpu

REL_TOL = 1e-3           # stated FP16 tolerance of the W4A8 GEMM output
ABS_TOL = 2.0 ** -24     # one FP16 subnormal step

FAMILIES = {"llama2_7b": wl.LLAMA2_7B, "llama3_70b": wl.LLAMA3_70B, "llama3_8b": wl.LLAMA3_8B}


def _sample_channels(N, count, seed):
    fixed = {0, 1, N - 1, N - 2, 255, 256, N // 2 - 1, N // 2, 63, 64}
    rng = np.random.default_rng(seed)
    extra = rng.choice(N, size=count, replace=False)
    picks = sorted(set(int(v) for v in fixed if 0 <= v < N) | set(int(v) for v in extra))
    return np.array(picks, dtype=np.int64)


def _check_layer(family, layer, Ms, mode, base_seed, samples=48):
    from oracle import gemm as ogemm
    from oracle import qoq_quant as qq

    dev = "cuda:0"
    K, N = FAMILIES[family][layer]
    w = wl.layer_weights(family, layer, base_seed, dev)
    blob = api.pack_weights(w, mode)
    idx = _sample_channels(N, samples, base_seed * 1000 + N % 997)
    w_rows = w[torch.from_numpy(idx).to(dev)].cpu().numpy()
    del w
    torch.cuda.empty_cache()

    # ---- packed weights of the sampled rows
    q, s1, z, s = api.unpack_weights(blob, N, K, mode)
    tidx = torch.from_numpy(idx).to(dev)
    q_rows = q[tidx].cpu().numpy()
    s_rows = s[tidx].cpu().numpy()
    z_rows = z[tidx].cpu().numpy()
    s1_rows = s1[tidx].cpu().numpy() if s1 is not None else None
    del q, s1, z, s
    torch.cuda.empty_cache()
    if mode == api.QOQ_GROUP128:
        wq = qq.progressive_quant(w_rows)
        assert np.array_equal(q_rows, wq["Q"]), "codes"
        assert np.array_equal(s1_rows, wq["s1"]), "s1"
        assert np.array_equal(z_rows, wq["z"]), "z"
        assert np.array_equal(s_rows.view(np.uint16), wq["s0"].astype(np.float16).view(np.uint16)), "s0"
        operand, zc, sw = wq["w_hat"], None, wq["s0"]
    else:
        code, zc, sw = qq.per_channel_quant(w_rows)
        assert np.array_equal(q_rows, code), "codes"
        assert np.array_equal(z_rows, zc), "z"
        assert np.array_equal(s_rows.view(np.uint16), sw.astype(np.float16).view(np.uint16)), "sw"
        operand = code

    for M in Ms:
        print(f"[fullsize] {family}/{layer} K={K} N={N} M={M} mode={mode}", flush=True)
        x = wl.layer_activations(family, layer, M, base_seed, dev)
        qx, sx, rowsum, _ = api.quant_act_per_token(x)
        oqx, osx, orowsum, _ = qq.act_quant(x.cpu().numpy())
        assert np.array_equal(qx.cpu().numpy(), oqx), "qx"
        assert np.array_equal(sx.cpu().numpy().view(np.uint16), osx.astype(np.float16).view(np.uint16)), "sx"
        assert np.array_equal(rowsum.cpu().numpy(), orowsum), "rowsum"

        acc = api.w4a8_gemm_i32(qx, blob, N, mode, rowsum=rowsum if mode else None)
        out = api.w4a8_gemm(qx, sx, blob, N, mode, rowsum=rowsum if mode else None)
        torch.cuda.synchronize()
        acc_s = acc[:, tidx].cpu().numpy()
        out_s = out[:, tidx].cpu().numpy().astype(np.float64)
        del acc, out, x

        ref = ogemm.gemm_i64(oqx, operand)
        if mode == api.QOQ_PER_CHANNEL:
            ref = qq.per_channel_acc(ref, zc, orowsum)
        assert np.abs(ref).max(initial=0) < 2 ** 31
        assert np.array_equal(acc_s.astype(np.int64), ref), "INT32 accumulators"
        ref64 = qq.output_fp64(ref, osx, sw)
        err = np.abs(out_s - ref64)
        assert np.all(err <= REL_TOL * np.abs(ref64) + ABS_TOL), f"fp16 out, worst {err.max()}"
        del qx, sx, rowsum
        torch.cuda.empty_cache()
    del blob
    torch.cuda.empty_cache()


# C1: the benchmark workload itself, every layer at M = 64 (and the neighbouring tile sizes).
@pytest.mark.parametrize("layer", list(wl.LLAMA2_7B))
def test_llama2_7b_decode(layer):
    _check_layer("llama2_7b", layer, (64, 16, 1), api.QOQ_GROUP128, 1)


# C2: the M sweep on the same layers (weights shared across M).
@pytest.mark.parametrize("layer", list(wl.LLAMA2_7B))
def test_llama2_7b_m_sweep(layer):
    _check_layer("llama2_7b", layer, (8, 32, 128, 256, 512, 1024, 2048, 4096), api.QOQ_GROUP128, 2, samples=32)


# C3: Llama-3-70B-shaped layers with heavy-tailed outlier channels (plus the decode and few-hundred-token sizes at
# which the widest layers run blocks in lockstep).
@pytest.mark.parametrize("layer", list(wl.LLAMA3_70B))
def test_llama3_70b(layer):
    _check_layer("llama3_70b", layer, (64, 192, 512, 2048), api.QOQ_GROUP128, 3, samples=32)


# C4: per-channel variant on Llama-3-8B-shaped layers.
@pytest.mark.parametrize("layer", list(wl.LLAMA3_8B))
def test_llama3_8b_per_channel(layer):
    _check_layer("llama3_8b", layer, (64, 256, 1024), api.QOQ_PER_CHANNEL, 4, samples=32)
