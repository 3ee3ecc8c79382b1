"""qoq_w4a8_gemm_noalloc (the entry point for callers that cannot allocate: its split-k scratch is an array inside
the library) against qoq_w4a8_gemm with a caller's workspace: same kernels, same configuration, so the FP16
outputs must be identical bit for bit -- on two calls in a row, the second with a smaller input, and on shapes of
every kernel family that exchanges partial tiles through the scratch."""
import ctypes

import numpy as np
import pytest
import torch

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


def _problem(api, M, N, K, mode, seed):
    w = wl.make_weights(N, K, seed, DEV, outlier_count=max(1, N // 100))
    x = wl.make_activations(M, K, seed, DEV, outlier_count=max(1, K // 100))
    blob = api.pack_weights(w, mode)
    qx, sx, rowsum, _ = api.quant_act_per_token(x)
    return blob, qx, sx, rowsum


def _both(api, M, N, K, mode, seed):
    blob, qx, sx, rowsum = _problem(api, M, N, K, mode, seed)
    want = api.w4a8_gemm(qx, sx, blob, N, mode, rowsum=rowsum)
    got = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    api.w4a8_gemm_noalloc(qx, sx, blob, N, got, mode, rowsum=rowsum)
    torch.cuda.synchronize()
    return got, want


def _same_bits(a, b):
    return bool((a.view(torch.int16) == b.view(torch.int16)).all())


def test_two_calls_in_a_row_second_one_smaller(api):
    # both problems exchange partial tiles through the scratch (their workspace size is not zero)
    big, small = (64, 4096, 11008, 0), (16, 256, 4096, 0)
    assert api.gemm_workspace_bytes(*big[:3]) > 0 and api.gemm_workspace_bytes(*small[:3]) > 0
    got, want = _both(api, *big, seed=21)
    assert _same_bits(got, want)
    got, want = _both(api, *small, seed=22)
    assert _same_bits(got, want)
    got, want = _both(api, *big, seed=23)          # and the large one again, over the small one's leftovers
    assert _same_bits(got, want)


@pytest.mark.parametrize("M,N,K,mode,cfg", [(17, 640, 1152, 0, (16, 3)), (64, 320, 1152, 0, (64, 5)), (40, 256, 4096, 1, (32, 9)),
                                            (300, 512, 3072, 0, (128, 2)), (200, 256, 4096, 1, (130, 3)), (64, 640, 1152, 0, (65, 0)),
                                            (1, 4096, 4096, 0, (0, 0)), (64, 12288, 4096, 0, (0, 0)), (64, 256, 11008, 1, (71, 5)),
                                            (33, 192, 5120, 0, (71, 0)), (16, 4096, 11008, 0, (0, 0)), (128, 12288, 4096, 0, (0, 0))])
def test_every_kernel_family(api, M, N, K, mode, cfg):
    api.set_gemm_config(*cfg)
    try:
        got, want = _both(api, M, N, K, mode, seed=30 + M)
    finally:
        api.set_gemm_config(0, 0)
    assert _same_bits(got, want)


def test_scratch_limit_is_an_error_not_an_allocation(api):
    """A configuration whose partial tiles exceed the 16 MiB of the library's array is refused; the output is untouched."""
    M, N, K = 2048, 4096, 8192
    api.set_gemm_config(128, 8)                     # 128 tiles x 8 slices x 256 KiB = 256 MiB of partial tiles
    try:
        assert api.gemm_workspace_bytes(M, N, K) > (16 << 20)
        qx = torch.zeros((M, K), dtype=torch.int8, device=DEV)
        sx = torch.ones(M, dtype=torch.float16, device=DEV)
        blob = torch.zeros(api.packed_bytes(N, K), dtype=torch.uint8, device=DEV)
        out = torch.full((M, N), 7.0, dtype=torch.float16, device=DEV)
        with pytest.raises(api.QoqError) as e:
            api.w4a8_gemm_noalloc(qx, sx, blob, N, out)
        assert e.value.status == api.QOQ_ERR_WORKSPACE
        torch.cuda.synchronize()
        assert bool((out == 7.0).all())
    finally:
        api.set_gemm_config(0, 0)


def test_no_allocation_during_the_call(api):
    """The calls leave the device's free memory and the memory torch has reserved from it unchanged."""
    blob, qx, sx, rowsum = _problem(api, 64, 4096, 11008, 0, 41)
    out = torch.empty((64, 4096), dtype=torch.float16, device=DEV)
    api.w4a8_gemm_noalloc(qx, sx, blob, 4096, out)   # first call on the device: the address lookup happens here
    torch.cuda.synchronize()
    before = (torch.cuda.memory_reserved(), torch.cuda.mem_get_info()[0])
    for _ in range(3):
        api.w4a8_gemm_noalloc(qx, sx, blob, 4096, out)
    torch.cuda.synchronize()
    after = (torch.cuda.memory_reserved(), torch.cuda.mem_get_info()[0])
    assert before == after
