"""GPU parity of the KV4 cache quantizer and the decode attention kernel against the CPU oracle, through the C ABI.

Codes, scales and zero points must be bit-exact.  The attention output is floating point: the integer codes enter the
products exactly, the softmax weight of a token (times its value scale) is rounded to FP16 before the second
product, sums and the softmax run in FP32 and the result is rounded once to FP16, so
    |gpu - ref| <= 1e-3 * |ref| + 1e-3 * max|V^|
The first term is the final rounding (4.9e-4 relative) with margin.  The second bounds the effect of the FP16
weights: each weight carries an independent relative error of at most 2^-11 = 4.9e-4, so the weighted average moves
by at most 4.9e-4 * sum_t p_t |v_t| <= 4.9e-4 * max|V^|, again with margin (FP32 accumulation and the hardware
exp2 are two orders of magnitude below)."""
import numpy as np
import pytest
import torch

from oracle import kv4
from paper_2405_04532_amd import api, workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _special_vectors(x):
    """Overwrite a few vectors with the degenerate cases of the quantizer."""
    x = x.clone()
    flat = x.view(-1, x.shape[-1])
    flat[0] = flat[0].abs()                       # one sign
    flat[1] = -flat[1].abs()
    flat[2] = 0.3                                 # constant
    flat[3] = 0                                   # zero
    flat[4] = flat[4] * 1e-4                      # tiny
    flat[5] = 0; flat[5, 7] = 3.5                 # one-hot
    flat[6] = torch.arange(flat.shape[1], dtype=torch.float16) * 0.5 - 3    # many exact ties
    return x


def _check_cache(cache, B, Hkv, S_max, k_ref, v_ref, written):
    """k_ref, v_ref: [B, Hkv, S_max, D] FP16 (CPU numpy) of what was appended; written: bool [B, S_max]."""
    kc, ks, kz, vc, vs, vz = [t.cpu().numpy() for t in api.kv4_unpack(cache, B, Hkv, S_max)]
    okc, oks, okz = kv4.kv4_quantize(k_ref)
    ovc, ovs, ovz = kv4.kv4_quantize(v_ref)
    w = np.broadcast_to(written[:, None, :], (B, Hkv, S_max))
    assert np.array_equal(kc[w], okc[w]) and np.array_equal(vc[w], ovc[w]), "codes"
    assert np.array_equal(ks.view(np.uint16)[w], oks.view(np.uint16)[w]) and np.array_equal(vs.view(np.uint16)[w], ovs.view(np.uint16)[w]), "scales"
    assert np.array_equal(kz.view(np.uint16)[w], okz.view(np.uint16)[w]) and np.array_equal(vz.view(np.uint16)[w], ovz.view(np.uint16)[w]), "zeros"
    return (okc, oks, okz, ovc, ovs, ovz)


def test_append_prefill_then_decode_steps_bit_exact():
    B, Hkv, S_max, D = 3, 4, 150, 128
    k, v = wl.make_kv(B, Hkv, S_max, D, 31, DEV)
    k, v = _special_vectors(k), _special_vectors(v)
    cache = api.kv4_new_cache(B, Hkv, S_max, DEV)
    lens = [100, 1, 64]
    T = 100
    # prefill: T tokens per sequence at position 0 (sequences shorter than T simply overwrite later)
    kt = k[:, :, :T].permute(0, 2, 1, 3).contiguous()          # [B, T, Hkv, D]
    vt = v[:, :, :T].permute(0, 2, 1, 3).contiguous()
    api.kv4_append(cache, kt, vt, torch.zeros(B, dtype=torch.int32, device=DEV), S_max)
    written = np.zeros((B, S_max), dtype=bool)
    written[:, :T] = True
    # three decode steps: one token per sequence at its own position
    pos = torch.tensor(lens, dtype=torch.int32, device=DEV)
    k_ref, v_ref = k.cpu().numpy().copy(), v.cpu().numpy().copy()
    for step in range(3):
        src = 120 + step                                       # take fresh vectors from the tail of the tensors
        kn = k[:, :, src].unsqueeze(1).contiguous()            # [B, 1, Hkv, D]
        vn = v[:, :, src].unsqueeze(1).contiguous()
        api.kv4_append(cache, kn, vn, pos, S_max)
        for b in range(B):
            p = int(pos[b])
            k_ref[b, :, p] = k_ref[b, :, src]; v_ref[b, :, p] = v_ref[b, :, src]
            written[b, p] = True
        pos = pos + 1
    torch.cuda.synchronize()
    _check_cache(cache, B, Hkv, S_max, k_ref, v_ref, written)


def test_append_outside_the_cache_is_dropped():
    B, Hkv, S_max, D = 2, 2, 70, 128
    k, v = wl.make_kv(B, Hkv, 8, D, 32, DEV)
    cache = api.kv4_new_cache(B, Hkv, S_max, DEV)
    before = cache.clone()
    kt, vt = k.permute(0, 2, 1, 3).contiguous(), v.permute(0, 2, 1, 3).contiguous()
    api.kv4_append(cache, kt, vt, torch.tensor([66, -3], dtype=torch.int32, device=DEV), S_max)
    torch.cuda.synchronize()
    kc, ks, kz, vc, vs, vz = [t.cpu().numpy() for t in api.kv4_unpack(cache, B, Hkv, S_max)]
    okc, oks, okz = kv4.kv4_quantize(k.cpu().numpy())
    # sequence 0: tokens 0..3 land at 66..69, 4..7 are dropped; sequence 1: tokens 3..7 land at 0..4
    assert np.array_equal(kc[0, :, 66:70], okc[0, :, 0:4]) and np.array_equal(kc[1, :, 0:5], okc[1, :, 3:8])
    assert np.array_equal(ks.view(np.uint16)[1, :, 0:5], oks.view(np.uint16)[1, :, 3:8])
    assert not kc[0, :, :66].any() and not kc[1, :, 5:].any()
    assert cache.numel() == before.numel()


def _attention_case(B, H, Hkv, S_max, lens, seed, split=False):
    D = 128
    k, v = wl.make_kv(B, Hkv, S_max, D, seed, DEV)
    q = wl.make_queries(B, H, D, seed, DEV)
    cache = api.kv4_new_cache(B, Hkv, S_max, DEV)
    api.kv4_append(cache, k.permute(0, 2, 1, 3).contiguous(), v.permute(0, 2, 1, 3).contiguous(),
                   torch.zeros(B, dtype=torch.int32, device=DEV), S_max)
    seq = torch.tensor(lens, dtype=torch.int32, device=DEV)
    ws = None
    if split:
        nbytes = api.kv4_attention_workspace_bytes(B, H, Hkv, S_max)
        assert nbytes > 0, "this shape was meant to exercise the split variant"
        ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=DEV)     # contents on entry are irrelevant (NaN here)
    out = api.kv4_attention_decode(q, cache, seq, Hkv, S_max, workspace=ws)
    torch.cuda.synchronize()
    o = _check_cache(cache, B, Hkv, S_max, k.cpu().numpy(), v.cpu().numpy(), np.ones((B, S_max), dtype=bool))
    ref = kv4.attention_decode(q.cpu().numpy(), *o, np.array(lens))
    got = out.cpu().numpy().astype(np.float64)
    v_hat = kv4.kv4_dequantize(o[3], o[4], o[5])
    vmax = np.abs(v_hat).max(axis=(2, 3))                       # [B, Hkv]
    tol = 1e-3 * np.abs(ref) + 1e-3 * np.repeat(vmax, H // Hkv, axis=1)[:, :, None]
    assert np.isfinite(got).all()
    bad = np.abs(got - ref) > tol
    assert not bad.any(), (int(bad.sum()), float(np.abs(got - ref).max()))
    # the bound above is a worst case; the roundings are independent, so the typical error is far smaller
    live = np.array(lens) > 0
    rms = np.sqrt(np.mean((got[live] - ref[live]) ** 2))
    assert rms <= 2e-4 * vmax[live].mean(), float(rms)
    return got, ref


@pytest.mark.parametrize("H,Hkv", [(4, 4), (4, 2), (8, 2), (8, 1), (6, 2), (16, 1)])
def test_attention_ragged_lengths(H, Hkv):
    """Lengths around chunk and page boundaries, one token, none; every ratio of query to KV heads."""
    lens = [0, 1, 3, 15, 16, 17, 63, 64, 65, 130, 200]
    got, ref = _attention_case(len(lens), H, Hkv, 200, lens, 40 + H + Hkv)
    assert not got[0].any()                                     # empty sequence: zero rows


@pytest.mark.parametrize("H,Hkv", [(4, 1), (8, 2), (6, 6)])
def test_attention_split_over_workgroups(H, Hkv):
    """Few (sequence, KV head) pairs and long caches: the sequence is cut into ranges; lengths that leave ranges
    empty, partly filled, and exactly filled."""
    lens = [0, 1, 31, 32, 33, 127, 128, 129, 500, 1000, 1023, 1024]
    _attention_case(len(lens), H, Hkv, 1024, lens, 70 + H)
    got, ref = _attention_case(len(lens), H, Hkv, 1024, lens, 70 + H, split=True)
    assert not got[0].any()
    # the two variants compute the same sums in a different order
    k, v = wl.make_kv(2, Hkv, 2000, 128, 71, DEV)
    q = wl.make_queries(2, H, 128, 71, DEV)
    cache = api.kv4_new_cache(2, Hkv, 2000, DEV)
    api.kv4_append(cache, k.permute(0, 2, 1, 3).contiguous(), v.permute(0, 2, 1, 3).contiguous(),
                   torch.zeros(2, dtype=torch.int32, device=DEV), 2000)
    seq = torch.tensor([2000, 777], dtype=torch.int32, device=DEV)
    ws = torch.zeros(api.kv4_attention_workspace_bytes(2, H, Hkv, 2000), dtype=torch.uint8, device=DEV)
    a = api.kv4_attention_decode(q, cache, seq, Hkv, 2000).float()
    b = api.kv4_attention_decode(q, cache, seq, Hkv, 2000, workspace=ws).float()
    assert torch.allclose(a, b, rtol=2e-3, atol=2e-3)
    # a workspace that is too small is refused
    L = api.lib()
    out = torch.empty_like(q)
    assert L.qoq_kv4_attention_decode_split(q.data_ptr(), cache.data_ptr(), seq.data_ptr(), 2, H, Hkv, 128, 2000, out.data_ptr(),
                                            ws.data_ptr(), 16, None) == api.QOQ_ERR_WORKSPACE


def test_attention_long_sequence_many_pages():
    _attention_case(2, 2, 2, 2500, [2500, 1999], 50)


def test_attention_ignores_tokens_past_the_length():
    B, H, Hkv, S_max, D = 1, 2, 2, 128, 128
    k, v = wl.make_kv(B, Hkv, S_max, D, 51, DEV)
    q = wl.make_queries(B, H, D, 51, DEV)
    seq = torch.tensor([70], dtype=torch.int32, device=DEV)
    outs = []
    for fill in (0x00, 0xFF):                                   # all-ones bytes: codes 15, NaN scales and zeros
        cache = torch.full((api.kv4_cache_bytes(B, Hkv, S_max),), fill, dtype=torch.uint8, device=DEV)
        api.kv4_append(cache, k[:, :, :70].permute(0, 2, 1, 3).contiguous(), v[:, :, :70].permute(0, 2, 1, 3).contiguous(),
                       torch.zeros(B, dtype=torch.int32, device=DEV), S_max)
        outs.append(api.kv4_attention_decode(q, cache, seq, Hkv, S_max).cpu().numpy())
    assert np.isfinite(outs[1].astype(np.float64)).all() and np.array_equal(outs[0].view(np.uint16), outs[1].view(np.uint16))


def test_attention_full_size_sampled():
    """The configuration bench.py --attention times (64 sequences x 1024 tokens, 32 heads), sampled (b, h)."""
    B, H, Hkv, S, D = 64, 32, 32, 1024, 128
    k, v = wl.make_kv(B, Hkv, S, D, 52, DEV)
    q = wl.make_queries(B, H, D, 52, DEV)
    cache = api.kv4_new_cache(B, Hkv, S, DEV)
    api.kv4_append(cache, k.permute(0, 2, 1, 3).contiguous(), v.permute(0, 2, 1, 3).contiguous(),
                   torch.zeros(B, dtype=torch.int32, device=DEV), S)
    lens = np.full(B, S); lens[5] = 1000; lens[63] = 517
    out = api.kv4_attention_decode(q, cache, torch.tensor(lens, dtype=torch.int32, device=DEV), Hkv, S)
    torch.cuda.synchronize()
    rng = np.random.default_rng(9)
    picks = [(0, 0), (63, 31), (5, 17), (63, 0)] + [(int(rng.integers(B)), int(rng.integers(H))) for _ in range(8)]
    for b, h in picks:
        kb, vb = k[b:b + 1, h:h + 1].cpu().numpy(), v[b:b + 1, h:h + 1].cpu().numpy()
        kc, ks, kz = kv4.kv4_quantize(kb)
        vc, vs, vz = kv4.kv4_quantize(vb)
        ref = kv4.attention_decode(q[b:b + 1, h:h + 1].cpu().numpy(), kc, ks, kz, vc, vs, vz, lens[b:b + 1])[0, 0]
        got = out[b, h].cpu().numpy().astype(np.float64)
        tol = 1e-3 * np.abs(ref) + 1e-3 * np.abs(kv4.kv4_dequantize(vc, vs, vz)).max()
        assert np.all(np.abs(got - ref) <= tol), (b, h, float(np.abs(got - ref).max()))


def test_kv4_argument_validation():
    q = torch.zeros((1, 4, 128), dtype=torch.float16, device=DEV)
    cache = api.kv4_new_cache(1, 4, 64, DEV)
    seq = torch.zeros(1, dtype=torch.int32, device=DEV)
    out = torch.empty_like(q)
    L = api.lib()
    args = lambda H, Hkv, D: (q.data_ptr(), cache.data_ptr(), seq.data_ptr(), 1, H, Hkv, D, 64, out.data_ptr(), None)
    assert L.qoq_kv4_attention_decode(*args(4, 4, 64)) == 2          # head dimension
    assert L.qoq_kv4_attention_decode(*args(4, 3, 128)) == 2         # H not a multiple of Hkv
    assert L.qoq_kv4_attention_decode(*args(68, 4, 128)) == 2        # ratio 17: more than one matrix tile of heads
    assert L.qoq_kv4_attention_decode(None, cache.data_ptr(), seq.data_ptr(), 1, 4, 4, 128, 64, out.data_ptr(), None) == 1
    assert L.qoq_kv4_attention_decode(q.data_ptr() + 2, cache.data_ptr(), seq.data_ptr(), 1, 4, 4, 128, 64, out.data_ptr(), None) == 3
    assert api.kv4_cache_bytes(1, 4, 64, 64) == 0
    assert api.kv4_cache_bytes(2, 4, 65) == 2 * 4 * 2 * 8704


def test_append_many_vectors_bit_exact():
    """Sixteen million elements (131072 key and value vectors), all codes, scales and zeros compared; half of the
    vectors are scaled to magnitudes between 1e-3 and 1e3 so that many exponents of x / s occur."""
    B, Hkv, S, D = 8, 8, 1024, 128
    k, v = wl.make_kv(B, Hkv, S, D, 53, DEV)
    gain = torch.pow(10.0, torch.linspace(-3, 3, S, device=DEV)).to(torch.float16)
    v = (v.float() * gain[None, None, :, None].float()).to(torch.float16)
    k[:, :, ::2] = (k[:, :, ::2].float() * gain[None, None, ::2, None].float()).to(torch.float16)
    cache = api.kv4_new_cache(B, Hkv, S, DEV)
    api.kv4_append(cache, k.permute(0, 2, 1, 3).contiguous(), v.permute(0, 2, 1, 3).contiguous(),
                   torch.zeros(B, dtype=torch.int32, device=DEV), S)
    torch.cuda.synchronize()
    _check_cache(cache, B, Hkv, S, k.cpu().numpy(), v.cpu().numpy(), np.ones((B, S), dtype=bool))
