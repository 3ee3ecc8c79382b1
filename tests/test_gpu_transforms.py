"""GPU parity of the data-free offline transforms (channel salience, order, gather, reordered activation
quantizer, Hadamard rotation) against the CPU oracle, through the C ABI.  Everything here is exact: indices,
FP16 bit patterns, INT8 codes, INT32 accumulators."""
import numpy as np
import pytest
import torch

from oracle import gemm as ogemm
from oracle import qoq_quant as qq
from oracle import transforms as tr
from paper_2405_04532_amd import api, workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bits(a):
    return np.asarray(a).view(np.uint16)


@pytest.mark.parametrize("M,K", [(100, 1024), (1, 128), (257, 4096)])
def test_salience_and_order(M, K):
    x = wl.make_activations(M, K, 60 + M, DEV)
    x[:, 7] = x[:, 3]                                            # exact ties in salience
    sal = api.channel_absmax(x)
    ref = tr.channel_salience(x.cpu().numpy())
    assert np.array_equal(sal.cpu().numpy(), ref)
    perm = api.channel_order(sal)
    assert np.array_equal(perm.cpu().numpy(), tr.channel_order(ref))
    assert not api.channel_absmax(x[:0]).any()                   # no tokens: zeros


def test_gather_and_reordered_quantizer_bit_exact():
    M, K, N = 70, 2048, 192
    x = wl.make_activations(M, K, 61, DEV)
    w = wl.make_weights(N, K, 61, DEV)
    perm = api.channel_order(api.channel_absmax(x))
    p = perm.cpu().numpy()
    wr = api.gather_channels(w, perm)
    assert np.array_equal(_bits(wr.cpu().numpy()), _bits(tr.reorder_channels(w.cpu().numpy(), p)))
    qx, sx, rowsum, tx = api.quant_act_per_token_reordered(x, perm, want_tx=True)
    oqx, osx, ors, otx = qq.act_quant(tr.reorder_channels(x.cpu().numpy(), p))
    assert np.array_equal(qx.cpu().numpy(), oqx) and np.array_equal(_bits(sx.cpu().numpy()), _bits(osx))
    assert np.array_equal(rowsum.cpu().numpy(), ors)
    # the fused gather equals gather-then-quantize on the GPU as well
    qx2, sx2, _, _ = api.quant_act_per_token(api.gather_channels(x, perm))
    assert torch.equal(qx, qx2) and torch.equal(sx, sx2)
    # whole reordered layer: INT32 accumulators bit-exact, FP16 output within the GEMM tolerance
    blob = api.pack_weights(wr)
    acc = api.w4a8_gemm_i32(qx, blob, N).cpu().numpy().astype(np.int64)
    out = api.w4a8_gemm(qx, sx, blob, N).cpu().numpy().astype(np.float64)
    ref = ogemm.forward_group(tr.reorder_channels(w.cpu().numpy(), p), tr.reorder_channels(x.cpu().numpy(), p))
    assert np.array_equal(acc, ref["acc"])
    assert np.all(np.abs(out - ref["out64"]) <= 1e-3 * np.abs(ref["out64"]) + 2.0 ** -24)


def test_reordering_clamps_bad_indices():
    x = wl.make_activations(4, 256, 62, DEV)
    perm = torch.arange(256, dtype=torch.int32, device=DEV)
    perm[5], perm[9] = -7, 100000
    g = api.gather_channels(x, perm).cpu().numpy()
    xc = x.cpu().numpy()
    assert np.array_equal(_bits(g[:, 5]), _bits(xc[:, 0])) and np.array_equal(_bits(g[:, 9]), _bits(xc[:, 255]))
    assert np.array_equal(_bits(g[:, 10:]), _bits(xc[:, 10:]))


@pytest.mark.parametrize("rows,K,block", [(5, 64, 2), (3, 256, 64), (70, 4096, 4096), (2, 8192, 8192), (9, 11008, 256),
                                          (4, 512, 1)])
def test_hadamard_rotation_bit_exact(rows, K, block):
    x = wl.make_activations(rows, K, 63 + block % 97, DEV)
    got = api.hadamard_rotate(x, block)
    ref = tr.rotate_fp16(x.cpu().numpy(), block)
    assert np.array_equal(_bits(got.cpu().numpy()), _bits(ref))
    y = x.clone()
    api.hadamard_rotate(y, block, out=y)                         # in place
    assert torch.equal(y, got)


def test_rotated_layer_matches_the_oracle_and_the_unrotated_product():
    M, K, N = 33, 1024, 128
    x = wl.make_activations(M, K, 64, DEV)
    w = wl.make_weights(N, K, 64, DEV)
    xr, wr = api.hadamard_rotate(x), api.hadamard_rotate(w)      # default block: the whole row (1024)
    blob = api.pack_weights(wr)
    qx, sx, _, _ = api.quant_act_per_token(xr)
    acc = api.w4a8_gemm_i32(qx, blob, N).cpu().numpy().astype(np.int64)
    ref = ogemm.forward_group(tr.rotate_fp16(w.cpu().numpy(), K), tr.rotate_fp16(x.cpu().numpy(), K))
    assert np.array_equal(acc, ref["acc"])
    exact = x.cpu().numpy().astype(np.float64) @ w.cpu().numpy().astype(np.float64).T
    plain = ogemm.forward_group(w.cpu().numpy(), x.cpu().numpy())["out64"]
    err_rot = np.sqrt(np.mean((ref["out64"] - exact) ** 2))
    err_plain = np.sqrt(np.mean((plain - exact) ** 2))
    assert err_rot < err_plain                                   # what the rotation is for, on outlier activations


def test_transform_argument_validation():
    L = api.lib()
    x = torch.zeros((4, 256), dtype=torch.float16, device=DEV)
    out = torch.empty_like(x)
    perm = torch.arange(256, dtype=torch.int32, device=DEV)
    assert L.qoq_hadamard_rotate(x.data_ptr(), 4, 256, 48, out.data_ptr(), None) == 2        # not a power of two
    assert L.qoq_hadamard_rotate(x.data_ptr(), 4, 256, 512, out.data_ptr(), None) == 2       # does not divide K
    assert L.qoq_hadamard_rotate(x.data_ptr(), 4, 1 << 15, 1 << 14, out.data_ptr(), None) == 2   # block too large
    assert L.qoq_hadamard_rotate(None, 4, 256, 256, out.data_ptr(), None) == 1
    assert L.qoq_gather_channels(x.data_ptr(), perm.data_ptr(), 4, 256, x.data_ptr(), None) == 2  # in place
    assert L.qoq_gather_channels(x.data_ptr(), perm.data_ptr(), 4, 252, out.data_ptr(), None) == 2
    assert L.qoq_quant_act_per_token_reordered(x.data_ptr(), None, 4, 256, out.data_ptr(), out.data_ptr(), None, None, None) == 1
    assert L.qoq_channel_order_host(None, 16, None) == 1
