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
boundary, seeded picks elsewhere and, derived from the launch configuration the library reports for the shape,
a channel of every block that two workgroups share, of the first and last block (pair, quad, fragment) of every
workgroup, and the first and last channel of every tile of the compute-bound kernel.

The decode configurations themselves (every Llama-2-7B layer and every per-channel Llama-3-8B layer at M = 64) are
also compared as WHOLE tensors: every packed code, scale and zero, every INT32 accumulator, every FP16 output.
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


def _partition_channels(M, N, K, mode, rng):
    """Channels that sit where the launch configuration of this shape cuts the work: see the module docstring."""
    tile, split = api.query_gemm_config(M, N, K, mode)
    G = K // 128
    picks = set()

    def block(b, width=64):                      # two channels of the `width`-channel set b
        lo = min(b * width, N - width)
        picks.update(int(v) for v in lo + rng.choice(width, size=2, replace=False))

    if tile in (16, 32, 64):                     # units = (64-channel block, group), dealt in runs of upw
        units = (N // 64) * G
        upw = -(-units // split)
        for k in range(split + 1):
            for u in (k * upw - 1, k * upw):
                if 0 <= u < units:
                    block(u // G)
    elif tile in (65, 66, 67, 68):               # whole pairs / quads of blocks per workgroup
        width = 256 if tile == 66 else 128
        sets = N // width
        per = -(-sets // split)
        for k in range(split + 1):
            for sset in (k * per - 1, k * per):
                if 0 <= sset < sets:
                    block(sset, width)
    elif tile in (69, 70, 71):                   # 16-channel fragments in runs of unequal length
        frags = N // 16
        base, rem = divmod(frags, split)
        f = 0
        for k in range(split):
            n = base + (1 if k < rem else 0)
            for frag in (f, f + n - 1):
                if 0 <= frag < frags and n > 0:
                    picks.add((frag >> 2) * 64 + 16 * int(rng.integers(4)) + 4 * (frag & 3) + int(rng.integers(4)))
            f += n
    else:                                        # compute-bound kernel: first and last channel of every tile
        tn = {128: 256, 129: 256, 130: 128, 131: 192, 132: 256}[tile]
        for n0 in range(0, N, tn):
            picks.update((n0, min(N, n0 + tn) - 1))
    return picks


def _check_whole_layer(family, layer, M, mode, base_seed, launches=1):
    """Every element of one layer at M tokens against the oracle; `launches` > 1 repeats the GEMM and demands
    identical accumulators every time (the partial tiles of shared blocks cross workgroups without fences)."""
    from oracle import gemm as ogemm
    from oracle import qoq_quant as qq

    dev = "cuda:0"
    K, N = FAMILIES[family][layer]
    print(f"[whole tensor] {family}/{layer} K={K} N={N} M={M} mode={mode} cfg={api.query_gemm_config(M, N, K, mode)}", flush=True)
    w = wl.layer_weights(family, layer, base_seed, dev)
    blob = api.pack_weights(w, mode)
    q, s1, z, s = api.unpack_weights(blob, N, K, mode)
    q, z, s = q.cpu().numpy(), z.cpu().numpy(), s.cpu().numpy()
    s1 = s1.cpu().numpy() if s1 is not None else None
    w_np = w.cpu().numpy()
    del w
    operand = np.empty((N, K), dtype=np.int8)
    scale = np.empty(N, dtype=np.float16)
    zc = np.empty(N, dtype=np.int64)
    for r0 in range(0, N, 1024):                 # the oracle's quantizers, 1024 channels at a time
        r1 = min(N, r0 + 1024)
        if mode == api.QOQ_GROUP128:
            wq = qq.progressive_quant(w_np[r0:r1])
            assert np.array_equal(q[r0:r1], wq["Q"]) and np.array_equal(s1[r0:r1], wq["s1"]) and np.array_equal(z[r0:r1], wq["z"])
            operand[r0:r1], scale[r0:r1] = wq["w_hat"], wq["s0"]
        else:
            code, zz, sw = qq.per_channel_quant(w_np[r0:r1])
            assert np.array_equal(q[r0:r1], code) and np.array_equal(z[r0:r1], zz)
            operand[r0:r1], scale[r0:r1], zc[r0:r1] = code, sw, zz
    assert np.array_equal(s.view(np.uint16), scale.view(np.uint16))
    del q, s1, z, s, w_np

    x = wl.layer_activations(family, layer, M, base_seed, dev)
    qx, sx, rowsum, _ = api.quant_act_per_token(x)
    oqx, osx, orowsum, _ = qq.act_quant(x.cpu().numpy())
    assert np.array_equal(qx.cpu().numpy(), oqx) and np.array_equal(rowsum.cpu().numpy(), orowsum)
    ref = ogemm.gemm_i64(oqx, operand)
    if mode == api.QOQ_PER_CHANNEL:
        ref = qq.per_channel_acc(ref, zc, orowsum)
    assert np.abs(ref).max(initial=0) < 2 ** 31
    ws = api.new_workspace(api.gemm_workspace_bytes(M, N, K, mode), dev)
    for it in range(launches):
        acc = api.w4a8_gemm_i32(qx, blob, N, mode, rowsum=rowsum if mode else None, workspace=ws)
        bad = (acc.cpu().numpy().astype(np.int64) != ref)
        assert not bad.any(), f"launch {it}: {int(bad.sum())} INT32 accumulators differ, first at {np.argwhere(bad)[0]}"
    out = api.w4a8_gemm(qx, sx, blob, N, mode, rowsum=rowsum if mode else None, workspace=ws)
    ref64 = qq.output_fp64(ref, osx, scale)
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref64)
    assert np.all(err <= REL_TOL * np.abs(ref64) + ABS_TOL), f"fp16 out, worst {err.max()}"


def _check_layer(family, layer, Ms, mode, base_seed, samples=48):
    from oracle import gemm as ogemm
    from oracle import qoq_quant as qq

    dev = "cuda:0"
    K, N = FAMILIES[family][layer]
    w = wl.layer_weights(family, layer, base_seed, dev)
    blob = api.pack_weights(w, mode)
    idx = _sample_channels(N, samples, base_seed * 1000 + N % 997)
    rng = np.random.default_rng(base_seed * 7919 + N)
    cut = set()
    for M in Ms:                                   # where each of these launches cuts the layer
        cut |= _partition_channels(M, N, K, mode, rng)
    idx = np.array(sorted(set(int(v) for v in idx) | cut), dtype=np.int64)
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


# C1 and C4 at M = 64, whole tensors; the layers whose blocks are shared between workgroups (down, and O at one
# token) are launched 50 times over.
@pytest.mark.parametrize("layer", list(wl.LLAMA2_7B))
def test_llama2_7b_decode_whole_tensor(layer):
    _check_whole_layer("llama2_7b", layer, 64, api.QOQ_GROUP128, 1, launches=50 if layer in ("down", "o") else 2)


@pytest.mark.parametrize("layer", list(wl.LLAMA3_8B))
def test_llama3_8b_per_channel_decode_whole_tensor(layer):
    _check_whole_layer("llama3_8b", layer, 64, api.QOQ_PER_CHANNEL, 4, launches=50 if layer == "down" else 2)


def test_llama2_7b_down_one_token_whole_tensor_repeated():
    _check_whole_layer("llama2_7b", "down", 1, api.QOQ_GROUP128, 1, launches=50)


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
