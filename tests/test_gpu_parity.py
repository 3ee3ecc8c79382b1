"""GPU parity: every entry point of the C-ABI library against the CPU oracle, element by
element, on the same seeded inputs.  Integer results (codes, scales' bit patterns, INT8
activations, INT32 accumulators) must be bit-exact; the FP16 output must satisfy
|gpu - ref64| <= 1e-3*|ref64| + 2^-24 against the oracle's FP64 epilogue."""
import numpy as np
import pytest
import torch

from oracle import gemm as ogemm
from oracle import qoq_quant as qq
from paper_2405_04532_amd import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def api():
    from paper_2405_04532_amd import api as a
    a.lib()
    a.set_gemm_config(0, 0)
    yield a
    a.set_gemm_config(0, 0)


def _np(t):
    return t.detach().cpu().numpy()


def check_fp16(out_gpu, ref64):
    got = _np(out_gpu).astype(np.float64)
    tol = 1e-3 * np.abs(ref64) + 2.0 ** -24
    bad = np.abs(got - ref64) > tol
    assert not bad.any(), f"{int(bad.sum())} outputs outside tolerance, worst {np.abs(got - ref64).max()}"


def rand_inputs(M, N, K, seed, zero_row=True):
    w = wl.make_weights(N, K, seed, DEV, outlier_count=max(1, N // 100))
    x = wl.make_activations(M, K, seed, DEV, outlier_count=max(1, K // 100)) if M else \
        torch.empty((0, K), dtype=torch.float16, device=DEV)
    if zero_row and N >= 128:
        w[5] = 0                      # all-zero channel
        w[7, :128] = 0.03125          # constant group
    if zero_row and M >= 4:
        x[2] = 0                      # all-zero token
    return w, x


# ---------------------------------------------------------------------------- weight path
@pytest.mark.parametrize("N,K", [(256, 256), (64, 128), (320, 1152)])
def test_pack_group_matches_oracle(api, N, K):
    w, _ = rand_inputs(0, N, K, seed=N + K)
    blob = api.pack_weights(w, api.QOQ_GROUP128)
    q, s1, z, s0 = api.unpack_weights(blob, N, K, api.QOQ_GROUP128)
    ref = qq.progressive_quant(_np(w))
    assert (_np(s0).view(np.uint16) == ref["s0"].view(np.uint16)).all()
    assert (_np(s1).astype(np.int64) == ref["s1"]).all()
    assert (_np(z).astype(np.int64) == ref["z"]).all()
    assert (_np(q).astype(np.int64) == ref["Q"]).all()


@pytest.mark.parametrize("N,K", [(256, 256), (192, 640)])
def test_pack_per_channel_matches_oracle(api, N, K):
    w, _ = rand_inputs(0, N, K, seed=N + K + 1)
    w[3] = w[3].abs()
    blob = api.pack_weights(w, api.QOQ_PER_CHANNEL)
    q, _, z, sw = api.unpack_weights(blob, N, K, api.QOQ_PER_CHANNEL)
    code, zr, swr = qq.per_channel_quant(_np(w))
    assert (_np(sw).view(np.uint16) == swr.view(np.uint16)).all()
    assert (_np(z).astype(np.int64) == zr).all()
    assert (_np(q).astype(np.int64) == code).all()


def test_pack_quantized_roundtrip(api):
    rng = np.random.default_rng(3)
    N, K = 128, 384
    q0 = rng.integers(-119, 120, size=(N, K))
    code, s1, z = qq.level2_quant(q0)
    s0 = (rng.random(N) * 0.01 + 0.001).astype(np.float16)
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a.astype(dt))).to(DEV)
    blob = api.pack_quantized(t(code, np.uint8), t(s1, np.uint8), t(z, np.uint8), t(s0, np.float16))
    q, s1g, zg, s0g = api.unpack_weights(blob, N, K)
    assert (_np(q) == code).all() and (_np(s1g) == s1).all() and (_np(zg) == z).all()
    assert (_np(s0g).view(np.uint16) == s0.view(np.uint16)).all()


def test_unpack_refuses_a_blob_of_another_layer(api):
    """The blob describes itself (shape, mode, section offsets); the debug unpack reads that header back and
    refuses arguments that do not match it, instead of reading the sections at the wrong places."""
    w = wl.make_weights(256, 512, 11, DEV)
    blob = api.pack_weights(w, api.QOQ_GROUP128)
    api.unpack_weights(blob, 256, 512, api.QOQ_GROUP128)                       # the right description passes
    for N, K, mode in ((512, 256, api.QOQ_GROUP128), (256, 256, api.QOQ_GROUP128), (128, 512, api.QOQ_GROUP128),
                       (256, 512, api.QOQ_PER_CHANNEL)):
        with pytest.raises(api.QoqError) as e:
            api.unpack_weights(blob, N, K, mode)
        assert e.value.status == api.QOQ_ERR_BLOB, (N, K, mode)
    junk = torch.zeros_like(blob)                                               # no magic at all
    with pytest.raises(api.QoqError) as e:
        api.unpack_weights(junk, 256, 512, api.QOQ_GROUP128)
    assert e.value.status == api.QOQ_ERR_BLOB
    blob_c = api.pack_weights(w, api.QOQ_PER_CHANNEL)
    with pytest.raises(api.QoqError) as e:
        api.unpack_weights(blob_c, 256, 512, api.QOQ_GROUP128)
    assert e.value.status == api.QOQ_ERR_BLOB


# ---------------------------------------------------------------------------- activations
@pytest.mark.parametrize("M,K", [(16, 256), (1, 128), (37, 4096), (5, 11008), (3, 28672), (2, 32768), (3, 40960),
                                 (2048, 4096), (2100, 1024), (2048, 4224)])   # last three: many rows (256 threads per row where a row is short)
def test_act_quant_matches_oracle(api, M, K):
    _, x = rand_inputs(M, 64, K, seed=M * 7 + K)
    qx, sx, rowsum, tx = api.quant_act_per_token(x, want_rowsum=True, want_tx=True)
    rqx, rsx, rrow, rtx = qq.act_quant(_np(x))
    assert (_np(sx).view(np.uint16) == rsx.view(np.uint16)).all()
    assert (_np(qx).astype(np.int64) == rqx).all()
    assert (_np(rowsum).astype(np.int64) == rrow).all()
    assert np.allclose(_np(tx), rtx, rtol=1e-4, atol=1e-2)


def test_act_quant_ties_round_away(api):
    """Rows made of exact half-integer multiples of the scale: every tie rounds away from 0."""
    vals = np.concatenate([np.arange(-127, 128) + 0.5, [127.0, -127.0]])[:256] * 2.0 ** -6
    vals[vals > 127 * 2.0 ** -6] = 127 * 2.0 ** -6
    x = torch.from_numpy(vals.astype(np.float16)[None, :]).to(DEV)
    qx, sx, _, _ = api.quant_act_per_token(x)
    rqx, rsx, _, _ = qq.act_quant(_np(x))
    assert (_np(sx).view(np.uint16) == rsx.view(np.uint16)).all() and (_np(qx) == rqx).all()


@pytest.mark.parametrize("K", [1024, 11008, 40960])
def test_act_quant_midpoint_neighbours(api, K):
    """Rows whose elements are the FP16 values next to (and on) every rounding midpoint (k + 1/2) * s of their own
    scale, for 96 scales over the FP16 range (normal, subnormal, few and many significant bits): the codes must be
    the oracle's for every one of them, and so must the scale."""
    rng = np.random.default_rng(K)
    allh = np.arange(1, 0x7C00, dtype=np.uint16).view(np.float16)
    scales = np.concatenate([allh[rng.choice(len(allh), 64, replace=False)], allh[:8], allh[0x0400:0x0408],
                             np.array([2.0 ** -6, 3 * 2.0 ** -10, 1.0, 5.5, 96.0, 257.0, 384.0, 500.0], dtype=np.float16),
                             allh[-8:]])
    rows = []
    for s16 in scales:
        s = float(s16)
        top = np.float16(min(127.0 * s, 65504.0))                      # the row maximum fixes the row's scale near s
        mids = (np.arange(0, 127) + 0.5) * s
        mids = mids[mids <= 65504.0].astype(np.float16)
        with np.errstate(over="ignore"):
            cand = np.concatenate([mids, np.nextafter(mids, np.float16(np.inf)), np.nextafter(mids, np.float16(-np.inf))])
        cand = cand[np.isfinite(cand) & (np.abs(cand.astype(np.float64)) <= float(top))]
        row = np.zeros(K, dtype=np.float16)
        vals = np.concatenate([[top], cand, -cand])[:K]
        row[:len(vals)] = vals
        rows.append(rng.permutation(row))
    x = torch.from_numpy(np.stack(rows)).to(DEV)
    qx, sx, rowsum, _ = api.quant_act_per_token(x, want_rowsum=True)
    rqx, rsx, rrow, _ = qq.act_quant(_np(x))
    assert (_np(sx).view(np.uint16) == rsx.view(np.uint16)).all()
    assert (_np(qx).astype(np.int64) == rqx).all()
    assert (_np(rowsum).astype(np.int64) == rrow).all()


# ---------------------------------------------------------------------------- GEMM
def run_group_case(api, M, N, K, seed, tile_m=0, split_k=0):
    w, x = rand_inputs(M, N, K, seed)
    ref = ogemm.forward_group(_np(w), _np(x))
    blob = api.pack_weights(w, api.QOQ_GROUP128)
    qx, sx, _, _ = api.quant_act_per_token(x)
    api.set_gemm_config(tile_m, split_k)
    try:
        acc = api.w4a8_gemm_i32(qx, blob, N)
        out = api.w4a8_gemm(qx, sx, blob, N)
        torch.cuda.synchronize()
    finally:
        api.set_gemm_config(0, 0)
    assert (_np(qx).astype(np.int64) == ref["qx"]).all()
    assert (_np(acc).astype(np.int64) == ref["acc"]).all(), f"INT32 mismatch M={M} N={N} K={K} tile={tile_m} split={split_k}"
    check_fp16(out, ref["out64"])


def test_config0_tiny(api):
    """M=16, K=256, N=256, seed 0 with 2 outlier output channels and 4 outlier input channels."""
    w, x = wl.config0(DEV)
    ref = ogemm.forward_group(_np(w), _np(x))
    blob = api.pack_weights(w)
    qx, sx, _, _ = api.quant_act_per_token(x)
    acc = api.w4a8_gemm_i32(qx, blob, 256)
    out = api.w4a8_gemm(qx, sx, blob, 256)
    assert (_np(acc).astype(np.int64) == ref["acc"]).all()
    check_fp16(out, ref["out64"])
    # stricter: at most one FP16 ulp from the oracle's own FP16 rounding
    a = _np(out).view(np.int16).astype(np.int64)
    b = ref["out"].view(np.int16).astype(np.int64)
    assert np.abs(a - b).max() <= 1


@pytest.mark.parametrize("M", [1, 8, 17, 63, 64, 100, 130, 257])
def test_group_ragged_m(api, M):
    run_group_case(api, M, 320, 640, seed=100 + M)


@pytest.mark.parametrize("tile_m,split_k", [(16, 1), (32, 1), (64, 1), (128, 1), (16, 3), (64, 5), (128, 2), (32, 9),
                                            (64, 2), (128, 9), (129, 1), (130, 1), (129, 3), (130, 2), (129, 9), (130, 4),
                                            (131, 1), (131, 2), (131, 5), (132, 1), (132, 2), (132, 9)])
def test_group_forced_variants(api, tile_m, split_k):
    run_group_case(api, 150, 576, 1152, seed=7, tile_m=tile_m, split_k=split_k)


@pytest.mark.parametrize("M,N,K,tile_m", [(1, 256, 128, 0), (40, 64, 128, 0), (64, 256, 128, 0), (150, 256, 128, 0), (64, 320, 256, 0),
                                          (40, 256, 128, 16), (40, 256, 128, 32), (40, 256, 128, 64), (200, 256, 128, 129),
                                          (64, 4096, 512, 0), (48, 1024, 640, 0), (100, 512, 384, 0)])
def test_group_one_or_few_groups(api, M, N, K, tile_m):
    """K of one to five groups (runs of a single unit, odd group counts) and the token-tile splitting the library
    chooses for layers of few blocks."""
    run_group_case(api, M, N, K, seed=3 + M + K, tile_m=tile_m)


@pytest.mark.parametrize("M,N,K,split_k", [(64, 640, 1152, 0), (1, 640, 1152, 1), (17, 640, 1152, 3), (100, 640, 1152, 5),
                                           (150, 384, 128, 0), (64, 384, 384, 2), (63, 1280, 2048, 0), (64, 128, 256, 0),
                                           (64, 576, 1152, 0)])
def test_group_pair_streaming_kernel(api, M, N, K, split_k):
    """The kernel that streams two adjacent blocks in lockstep (whole pairs per workgroup): several pairs per
    workgroup, one group and an odd number of groups per pair, ragged and several token tiles, a single pair; the
    last case has an odd number of blocks, for which the library falls back to the single-block kernel."""
    run_group_case(api, M, N, K, seed=41 + M, tile_m=65, split_k=split_k)


@pytest.mark.parametrize("tile_m", [67, 68])
@pytest.mark.parametrize("M,N,K,split_k,mode", [(32, 640, 1152, 0, 0), (1, 640, 1152, 1, 1), (17, 640, 1152, 3, 0), (50, 384, 128, 0, 1),
                                                (16, 384, 384, 2, 0), (31, 1280, 2048, 0, 1), (100, 128, 256, 0, 0), (32, 576, 1152, 0, 0)])
def test_pair_streaming_kernel_small_token_tiles(api, tile_m, M, N, K, split_k, mode):
    """Block pairs in lockstep with 32- and 16-token tiles (codes 67, 68), both modes; the last case has an odd
    number of blocks and falls back to the single-block kernel of that tile."""
    w, x = rand_inputs(M, N, K, seed=5 + M + N)
    ref = (ogemm.forward_per_channel if mode else ogemm.forward_group)(_np(w), _np(x))
    blob = api.pack_weights(w, mode)
    qx, sx, rowsum, _ = api.quant_act_per_token(x)
    api.set_gemm_config(tile_m, split_k)
    try:
        acc = api.w4a8_gemm_i32(qx, blob, N, mode, rowsum=rowsum)
        out = api.w4a8_gemm(qx, sx, blob, N, mode, rowsum=rowsum)
        torch.cuda.synchronize()
    finally:
        api.set_gemm_config(0, 0)
    assert (_np(acc).astype(np.int64) == ref["acc"]).all()
    check_fp16(out, ref["out64"])


@pytest.mark.parametrize("M,N,K,split_k,mode", [(64, 1280, 1152, 0, 0), (1, 768, 1152, 1, 0), (17, 1280, 1152, 3, 1), (100, 768, 640, 2, 0),
                                                (150, 512, 128, 0, 1), (64, 512, 384, 2, 0), (63, 2560, 2048, 0, 1), (64, 256, 256, 0, 0),
                                                (64, 640, 1152, 0, 0)])
def test_quad_streaming_kernel(api, M, N, K, split_k, mode):
    """The kernel that streams four adjacent blocks in lockstep, in both modes: several quads per workgroup, one
    group and an odd number of groups, ragged and several token tiles, a single quad; the last case is not a
    multiple of 256 channels, for which the library falls back to block pairs."""
    w, x = rand_inputs(M, N, K, seed=77 + M + N)
    ref = (ogemm.forward_per_channel if mode else ogemm.forward_group)(_np(w), _np(x))
    blob = api.pack_weights(w, mode)
    qx, sx, rowsum, _ = api.quant_act_per_token(x)
    api.set_gemm_config(66, split_k)
    try:
        acc = api.w4a8_gemm_i32(qx, blob, N, mode, rowsum=rowsum)
        out = api.w4a8_gemm(qx, sx, blob, N, mode, rowsum=rowsum)
        torch.cuda.synchronize()
    finally:
        api.set_gemm_config(0, 0)
    assert (_np(acc).astype(np.int64) == ref["acc"]).all()
    check_fp16(out, ref["out64"])


@pytest.mark.parametrize("tile_m", [69, 70, 71])
@pytest.mark.parametrize("M,N,K,split_k,mode", [
    (64, 640, 1152, 0, 0),      # nine groups: slots past the slice in most waves
    (1, 640, 1152, 1, 1),       # one workgroup walks all forty fragments
    (17, 320, 640, 3, 0),       # ragged tokens, fragment runs of unequal length
    (50, 384, 128, 0, 1),       # a single group
    (64, 256, 4096, 0, 0),      # thirty-two groups: every register slot of a 64-token tile in use
    (63, 1280, 2048, 7, 1),
    (100, 128, 256, 0, 0),      # several token tiles side by side
    (33, 192, 5120, 0, 0),      # forty groups: two k-slices for 64-token tiles, one for the smaller ones
    (64, 256, 11008, 5, 1),     # eighty-six groups: k-slices meet in the workspace (3 / 2 / 1 slices), ragged last slice
    (130, 320, 8192, 0, 0),     # k-slices and several token tiles
])
def test_activation_stationary_kernels(api, tile_m, M, N, K, split_k, mode):
    """The kernels that keep the activations in registers and stream nothing but weights (codes 69, 70, 71 = 16, 32
    and 64 tokens per tile), both modes, with and without k-slices."""
    w, x = rand_inputs(M, N, K, seed=11 + M + N)
    ref = (ogemm.forward_per_channel if mode else ogemm.forward_group)(_np(w), _np(x))
    blob = api.pack_weights(w, mode)
    qx, sx, rowsum, _ = api.quant_act_per_token(x)
    api.set_gemm_config(tile_m, split_k)
    try:
        assert api.query_gemm_config(M, N, K, mode)[0] == tile_m
        acc = api.w4a8_gemm_i32(qx, blob, N, mode, rowsum=rowsum)
        out = api.w4a8_gemm(qx, sx, blob, N, mode, rowsum=rowsum)
        acc2 = api.w4a8_gemm_i32(qx, blob, N, mode, rowsum=rowsum)      # again over the same workspace contract
        torch.cuda.synchronize()
    finally:
        api.set_gemm_config(0, 0)
    assert (_np(acc).astype(np.int64) == ref["acc"]).all()
    assert (_np(acc2).astype(np.int64) == ref["acc"]).all()
    check_fp16(out, ref["out64"])


@pytest.mark.parametrize("M,tile_m,split_k", [(256, 64, 0), (256, 64, 8), (200, 32, 6), (320, 64, 12)])
def test_group_streaming_kernel_many_token_tiles(api, M, tile_m, split_k):
    """The M <= 64 kernel forced onto several token tiles, with runs that end exactly at a block end and
    blocks shared between workgroups (cross-workgroup reduction per token tile)."""
    run_group_case(api, M, 256, 1024, seed=23, tile_m=tile_m, split_k=split_k)


def test_group_several_tiles_all_axes(api):
    run_group_case(api, 300, 1088, 2048, seed=11)


@pytest.mark.parametrize("tile_m,split_k", [(128, 1), (129, 1), (130, 1), (129, 2), (130, 3), (131, 1), (131, 2), (132, 1), (132, 3)])
def test_group_compute_kernel_shapes_ragged(api, tile_m, split_k):
    """Every tile shape of the compute-bound kernel on a problem ragged in tokens and channels (M % 128 != 0,
    N % 128 != 0) with several tiles on both axes and, with a split, odd slice lengths (17 groups)."""
    run_group_case(api, 389, 1472, 2176, seed=13, tile_m=tile_m, split_k=split_k)


def _pack_logical(api, code, s1, z, s0):
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a.astype(dt))).to(DEV)
    return api.pack_quantized(t(code, np.uint8), t(s1, np.uint8), t(z, np.uint8), t(s0, np.float16))


def test_one_hot_operands_pin_fragment_maps(api):
    """One-hot activations select single weights: checks the (n, k) <-> lane/byte maps of the
    packed layout and the MFMA operand order independently of any averaging."""
    N, K, M = 128, 256, 48
    rng = np.random.default_rng(5)
    q0 = rng.integers(-119, 120, size=(N, K))
    code, s1, z = qq.level2_quant(q0)
    w_hat = qq.level2_dequant(code, s1, z)
    blob = _pack_logical(api, code, s1, z, np.ones(N, np.float16))
    qx = np.zeros((M, K), dtype=np.int8)
    ks = rng.permutation(K)[:M]
    qx[np.arange(M), ks] = 1
    # in every kernel family: each has its own staging, swizzle and operand order
    for cfg in [(0, 0), (16, 0), (32, 2), (64, 0), (65, 0), (67, 0), (69, 0), (70, 0), (71, 0), (71, 1), (128, 1), (129, 1), (131, 1), (132, 1)]:
        api.set_gemm_config(*cfg)
        try:
            acc = api.w4a8_gemm_i32(torch.from_numpy(qx).to(DEV), blob, N)
        finally:
            api.set_gemm_config(0, 0)
        assert (_np(acc).astype(np.int64) == w_hat[:, ks].T).all(), cfg


def test_extreme_magnitudes_fit_int32(api):
    """All activations 127 against the largest representable weights, K = 28672."""
    N, K, M = 64, 28672, 16
    code = np.full((N, K), 15)
    code[1::2] = 0
    s1 = np.full((N, K // 128), 16)
    z = np.full((N, K // 128), 8)          # w_hat = (15-8)*16 = 112 or (0-8)*16 = -128
    blob = _pack_logical(api, code, s1, z, np.ones(N, np.float16))
    qx = torch.full((M, K), 127, dtype=torch.int8, device=DEV)
    qx[1::2] = -127
    ref = ogemm.gemm_i64(_np(qx), qq.level2_dequant(code, s1, z))
    assert np.abs(ref).max() == 127 * 128 * K
    for cfg in [(0, 0), (64, 0), (69, 0), (71, 0), (129, 1), (132, 1)]:
        api.set_gemm_config(*cfg)
        try:
            acc = _np(api.w4a8_gemm_i32(qx, blob, N)).astype(np.int64)
        finally:
            api.set_gemm_config(0, 0)
        assert (acc == ref).all(), cfg


@pytest.mark.parametrize("M,N,K", [(16, 256, 256), (70, 192, 640), (200, 448, 1152), (64, 640, 1152), (50, 384, 384)])
def test_per_channel_gemm(api, M, N, K):
    w, x = rand_inputs(M, N, K, seed=M + N)
    ref = ogemm.forward_per_channel(_np(w), _np(x))
    blob = api.pack_weights(w, api.QOQ_PER_CHANNEL)
    qx, sx, rowsum, _ = api.quant_act_per_token(x)
    for tile_m, split_k in [(0, 0), (32, 3), (65, 0), (65, 1), (128, 1), (129, 1), (130, 1), (131, 1), (129, 2), (128, 3), (131, 3)]:
        api.set_gemm_config(tile_m, split_k)
        try:
            acc = api.w4a8_gemm_i32(qx, blob, N, api.QOQ_PER_CHANNEL, rowsum=rowsum)
            out = api.w4a8_gemm(qx, sx, blob, N, api.QOQ_PER_CHANNEL, rowsum=rowsum)
        finally:
            api.set_gemm_config(0, 0)
        assert (_np(acc).astype(np.int64) == ref["acc"]).all()
        check_fp16(out, ref["out64"])


def test_random_shapes_in_the_configuration_the_library_picks(api):
    """Thirty seeded shapes (tokens, channels, depth, mode) in whatever kernel, tile and partition the library
    chooses for them: INT32 accumulators bit for bit, FP16 output within tolerance."""
    rng = np.random.default_rng(2405)
    seen = set()
    for it in range(30):
        N = int(rng.integers(1, 17)) * 64
        K = int(rng.integers(1, 17)) * 128
        M = int(rng.choice([1, 3, 16, 17, 31, 32, 33, 48, 63, 64, 65, 96, 100, 128, 130, 200, 257, 300]))
        mode = int(rng.integers(0, 2))
        if it >= 26:      # wide ones: activations resident, block pairs in lockstep, two compute-bound tile shapes
            M, N, K = [(64, 22016, 256), (48, 24576, 4224), (520, 12288, 384), (1030, 12288, 128)][it - 26]
        w, x = rand_inputs(M, N, K, seed=1000 + it)
        ref = (ogemm.forward_per_channel if mode else ogemm.forward_group)(_np(w), _np(x))
        blob = api.pack_weights(w, mode)
        qx, sx, rowsum, _ = api.quant_act_per_token(x)
        seen.add(api.query_gemm_config(M, N, K, mode)[0])
        acc = api.w4a8_gemm_i32(qx, blob, N, mode, rowsum=rowsum)
        out = api.w4a8_gemm(qx, sx, blob, N, mode, rowsum=rowsum)
        assert (_np(acc).astype(np.int64) == ref["acc"]).all(), (M, N, K, mode)
        check_fp16(out, ref["out64"])
    assert {16, 64, 65, 71, 128, 129} <= seen, seen    # the draw reaches the kernel families


def test_repeated_launches_are_identical(api):
    """Double-buffer hazards would show as run-to-run differences."""
    w, x = rand_inputs(96, 512, 2048, seed=21)
    blob = api.pack_weights(w)
    qx, sx, _, _ = api.quant_act_per_token(x)
    first = api.w4a8_gemm_i32(qx, blob, 512).clone()
    for _ in range(5):
        assert torch.equal(api.w4a8_gemm_i32(qx, blob, 512), first)


def test_empty_batch(api):
    w, _ = rand_inputs(0, 64, 128, seed=1, zero_row=False)
    blob = api.pack_weights(w)
    x = torch.empty((0, 128), dtype=torch.float16, device=DEV)
    qx, sx, _, _ = api.quant_act_per_token(x)
    out = api.w4a8_gemm(qx, sx, blob, 64)
    assert out.shape == (0, 64)


def test_runtime_errors_leave_outputs_untouched(api):
    w, x = rand_inputs(16, 256, 4096, seed=2)
    blob = api.pack_weights(w)
    qx, sx, _, _ = api.quant_act_per_token(x)
    out = torch.full((16, 256), 7.0, dtype=torch.float16, device=DEV)
    assert api.gemm_workspace_bytes(16, 256, 4096) > 16
    tiny = torch.empty(16, dtype=torch.uint8, device=DEV)
    with pytest.raises(api.QoqError) as e:
        api.w4a8_gemm(qx, sx, blob, 256, out=out, workspace=tiny)
    assert e.value.status == api.QOQ_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


# ---------------------------------------------------------------------------- quantization + GEMM in one call
@pytest.mark.parametrize("M,N,K,mode", [(64, 256, 1024, 0), (1, 128, 256, 0), (17, 320, 640, 0), (48, 4096, 4096, 0),
                                        (64, 256, 1024, 1), (33, 4096, 11008, 1), (100, 256, 1024, 0),
                                        (300, 512, 1024, 1)])
def test_linear_equals_quant_then_gemm(api, M, N, K, mode):
    """qoq_w4a8_linear == qoq_quant_act_per_token followed by qoq_w4a8_gemm, bit for bit, and matches the
    oracle; called three times on the same buffers with different inputs (the second and third call must
    not see anything of the previous one: counters re-armed, no stale activations)."""
    w, _ = rand_inputs(M, N, K, seed=5 + M + K + mode)
    blob = api.pack_weights(w, mode)
    dev = w.device
    out = torch.empty((M, N), dtype=torch.float16, device=dev)
    qx = torch.empty((M, K), dtype=torch.int8, device=dev)
    sx = torch.empty(M, dtype=torch.float16, device=dev)
    rowsum = torch.empty(M, dtype=torch.int32, device=dev)
    ws = api.new_workspace(max(16, api.gemm_workspace_bytes(M, N, K, mode)), dev)
    for rep in range(3):
        x = wl.make_activations(M, K, 1000 * rep + M + K, DEV, outlier_count=max(1, K // 100))
        if rep == 1 and M >= 4:
            x[1] = 0
        api.w4a8_linear(x, blob, N, mode, out=out, qx=qx, sx=sx, rowsum=rowsum, workspace=ws)
        qx2, sx2, rowsum2, _ = api.quant_act_per_token(x)
        out2 = api.w4a8_gemm(qx2, sx2, blob, N, mode, rowsum=rowsum2 if mode else None)
        assert torch.equal(qx, qx2) and torch.equal(sx.view(torch.int16), sx2.view(torch.int16))
        assert torch.equal(rowsum, rowsum2)
        assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
        ref = (ogemm.forward_per_channel if mode else ogemm.forward_group)(_np(w), _np(x))
        check_fp16(out, ref["out64"])
        assert (_np(qx).astype(np.int64) == ref["qx"]).all()


# ---------------------------------------------------------------------------- token-sum form of the per-channel epilogue
@pytest.mark.parametrize("M,N,K,cfg", [(16, 256, 256, (0, 0)), (64, 512, 4096, (0, 0)), (70, 192, 640, (32, 3)),
                                       (200, 448, 1152, (128, 1)), (200, 448, 1152, (129, 2)), (300, 320, 2048, (130, 1)),
                                       (300, 320, 2048, (131, 1)), (200, 448, 1152, (131, 2)), (257, 256, 640, (131, 1)),
                                       (64, 640, 1152, (65, 0)), (100, 384, 384, (65, 2)), (64, 512, 1024, (66, 0)),
                                       (16, 3072, 512, (69, 0)), (40, 320, 1152, (70, 0)), (64, 256, 4096, (71, 0)),
                                       (64, 256, 11008, (71, 5)), (130, 320, 2048, (71, 0)), (300, 512, 1024, (132, 1))])
def test_per_channel_token_sum_epilogue(api, M, N, K, cfg):
    """out = acc * sx * sw - t_X * (z * sw) with t_X summed over the unquantized activations (Section 5.2.2),
    against the oracle's FP64 form.  Tolerance: the stated 1e-3 relative on the result plus the FP32 rounding
    of the two products, which nearly cancel (2^-21 of their magnitudes)."""
    w, x = rand_inputs(M, N, K, seed=3 * M + N)
    blob = api.pack_weights(w, api.QOQ_PER_CHANNEL)
    qx, sx, rowsum, tx = api.quant_act_per_token(x, want_rowsum=True, want_tx=True)
    api.set_gemm_config(*cfg)
    try:
        out = api.w4a8_gemm_token_sum(qx, sx, tx, blob, N)
        exact = api.w4a8_gemm(qx, sx, blob, N, api.QOQ_PER_CHANNEL, rowsum=rowsum)
        torch.cuda.synchronize()
    finally:
        api.set_gemm_config(0, 0)
    code, z, sw = qq.per_channel_quant(_np(w))
    oqx, osx, orow, otx = qq.act_quant(_np(x))
    raw = ogemm.gemm_i64(oqx, code)
    s = sw.astype(np.float64)
    first = raw.astype(np.float64) * osx.astype(np.float64)[:, None] * s[None, :]
    second = otx[:, None] * (z.astype(np.float64) * s)[None, :]
    ref = qq.output_fp64_token_sum(raw, osx, sw, z, otx)
    # the kernel takes t_X from the activation kernel, which sums the row in FP32: 2^-18 of sum |x| covers it
    tx_err = 2.0 ** -18 * np.abs(_np(x).astype(np.float64)).sum(axis=1)
    tol = 1e-3 * np.abs(ref) + 2.0 ** -24 + 2.0 ** -21 * (np.abs(first) + np.abs(second)) + \
        tx_err[:, None] * (z.astype(np.float64) * s)[None, :]
    got = _np(out).astype(np.float64)
    assert np.all(np.abs(got - ref) <= tol), f"worst {np.max(np.abs(got - ref) - tol)}"
    # and it is an approximation of the exact fold, not the same thing: bounded by z*sw*K*sx/2
    bound = (K * osx.astype(np.float64) / 2)[:, None] * (z.astype(np.float64) * s)[None, :]
    assert np.all(np.abs(got - _np(exact).astype(np.float64)) <= bound + 2e-3 * (np.abs(ref) + 1e-3))


# ---------------------------------------------------------------------------- quantization fused into the producer
def _producer_inputs(M, K, seed):
    x = wl.make_activations(M, K, seed, DEV, outlier_count=max(1, K // 100))
    gamma = (wl.normal(seed + 1, 7, K, DEV) * 0.1 + 1.0).to(torch.float16)
    return x, gamma


@pytest.mark.parametrize("M,K", [(16, 256), (1, 128), (37, 4096), (5, 11008), (3, 28672), (2, 32768),
                                 (2048, 4096), (2100, 1024), (2048, 4224)])   # last three: many rows (256 threads per row where a row is short)
def test_rmsnorm_quant_matches_oracle(api, M, K):
    x, gamma = _producer_inputs(M, K, seed=11 * M + K)
    if M >= 4:
        x[2] = 0                                   # all-zero token: y = 0, scale 1.0
    eps = 1e-5
    y, qx, sx, rowsum, tx = api.rmsnorm_quant(x, gamma, eps, want_y=True, want_rowsum=True, want_tx=True)
    ry = qq.rmsnorm_fp16(_np(x), _np(gamma), eps)
    assert (_np(y).view(np.uint16) == ry.view(np.uint16)).all()
    rqx, rsx, rrow, rtx = qq.act_quant(ry)
    assert (_np(sx).view(np.uint16) == rsx.view(np.uint16)).all()
    assert (_np(qx).astype(np.int64) == rqx).all()
    assert (_np(rowsum).astype(np.int64) == rrow).all()
    assert np.allclose(_np(tx), rtx, rtol=1e-4, atol=1e-2)
    # without the FP16 activations written, and equal to the unfused path on the same y
    _, qx2, sx2, _, _ = api.rmsnorm_quant(x, gamma, eps, want_y=False, want_rowsum=False)
    qx3, sx3, _, _ = api.quant_act_per_token(y)
    assert torch.equal(qx, qx2) and torch.equal(qx, qx3)
    assert torch.equal(sx.view(torch.int16), sx2.view(torch.int16)) and torch.equal(sx.view(torch.int16), sx3.view(torch.int16))


@pytest.mark.parametrize("M,K", [(16, 256), (1, 128), (37, 11008), (4, 14336), (2, 28672), (2048, 4096), (2100, 896)])
def test_silu_mul_quant_matches_oracle(api, M, K):
    gu = wl.make_activations(M, 2 * K, 5 * M + K, DEV, outlier_count=max(1, K // 50), gain=6.0)
    y, qx, sx, rowsum, tx = api.silu_mul_quant(gu, want_y=True, want_rowsum=True, want_tx=True)
    ry = qq.silu_mul_fp16(_np(gu))
    assert (_np(y).view(np.uint16) == ry.view(np.uint16)).all()
    rqx, rsx, rrow, rtx = qq.act_quant(ry)
    assert (_np(sx).view(np.uint16) == rsx.view(np.uint16)).all()
    assert (_np(qx).astype(np.int64) == rqx).all()
    assert (_np(rowsum).astype(np.int64) == rrow).all()
    assert np.allclose(_np(tx), rtx, rtol=1e-4, atol=1e-2)


def test_fused_producers_many_elements_bit_exact(api):
    """Two million elements each, with small, ordinary and large magnitudes: the producers round their FP32
    evaluation where that is provably the FP64 result and evaluate in FP64 otherwise; every FP16 output bit must be
    the oracle's (a wrong margin would show up among the thousands of elements that fall near a rounding midpoint)."""
    M, K = 256, 8192
    rng = np.random.default_rng(99)
    scale = np.exp(rng.uniform(-9.0, 3.0, size=(M, 1)))              # per-token magnitude from 1e-4 to 20
    x = torch.from_numpy((rng.standard_normal((M, K)) * scale).astype(np.float16)).to(DEV)
    gamma = torch.from_numpy((1.0 + 0.5 * rng.standard_normal(K)).astype(np.float16)).to(DEV)
    y, _, _, _, _ = api.rmsnorm_quant(x, gamma, 1e-5, want_y=True, want_rowsum=False)
    ry = qq.rmsnorm_fp16(_np(x), _np(gamma), 1e-5)
    assert (_np(y).view(np.uint16) == ry.view(np.uint16)).all()
    gu = torch.from_numpy((rng.standard_normal((M, 2 * K)) * scale * 0.5).astype(np.float16)).to(DEV)
    y, _, _, _, _ = api.silu_mul_quant(gu, want_y=True, want_rowsum=False)
    ry = qq.silu_mul_fp16(_np(gu))
    assert (_np(y).view(np.uint16) == ry.view(np.uint16)).all()


def test_fused_producers_reject_long_rows(api):
    x = torch.zeros((1, 40960), dtype=torch.float16, device=DEV)
    g = torch.ones(40960, dtype=torch.float16, device=DEV)
    with pytest.raises(api.QoqError) as e:
        api.rmsnorm_quant(x, g, 1e-5)
    assert e.value.status == 2


def test_act_quant_without_token_sums(api):
    """Group mode asks for neither row sums nor token sums: codes and scales are the same as with them."""
    x = wl.make_activations(37, 4096, 77, DEV)
    qx0, sx0, _, _ = api.quant_act_per_token(x, want_rowsum=True, want_tx=True)
    qx1, sx1, rs1, tx1 = api.quant_act_per_token(x, want_rowsum=False, want_tx=False)
    assert rs1 is None and tx1 is None
    assert torch.equal(qx0, qx1) and torch.equal(sx0, sx1)
