"""Whole-tensor parity at prefill sizes: the INT32 accumulators of entire layers, computed by the HIP path in the launch
configuration the library picks, digested block by block and compared with digests the CPU oracle wrote beforehand
(tests/golden/gemm_acc_digests.txt, written by tests/golden/make_gemm_digests.py, which runs only the oracle).

Integer sums have exactly one correct value, so equal digests mean every one of the M x N accumulators is right; the
FP16 output of the same launch configuration is then checked over the whole tensor against the FP64 product of those
accumulators with the token and channel scales (tolerance of the W4A8 output: 1e-3 relative + 2^-24).
"""
import hashlib
import os

import numpy as np
import pytest
import torch

from paper_2405_04532_amd import api, workloads as wl

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))
FAMILIES = {"llama2_7b": wl.LLAMA2_7B, "llama3_70b": wl.LLAMA3_70B, "llama3_8b": wl.LLAMA3_8B}
ROWS = 64


def _golden():
    cases = {}
    with open(os.path.join(HERE, "golden", "gemm_acc_digests.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            family, layer, M, mode, seed, block, digest = line.split()
            cases.setdefault((family, layer, int(M), int(mode), int(seed)), {})[int(block)] = digest
    return cases


GOLDEN = _golden()


def test_digest_file_covers_the_prefill_rows():
    keys = set(k[:4] for k in GOLDEN)
    assert ("llama2_7b", "gate_up", 1024, 0) in keys and ("llama3_8b", "down", 1024, 1) in keys
    assert ("llama3_70b", "down", 512, 0) in keys
    # the compute-bound leg of the benchmark and the largest Llama-2-7B rows
    assert all(("llama3_70b", n, 2048, 0) in keys for n in ("qkv", "o", "gate_up", "down"))
    assert all(("llama2_7b", n, 4096, 0) in keys for n in ("qkv", "o", "gate_up", "down"))
    for (family, layer, M, mode, seed), blocks in GOLDEN.items():
        assert sorted(blocks) == list(range(-(-M // ROWS))), (family, layer)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("case", sorted(GOLDEN), ids=lambda c: "%s-%s-M%d-mode%d" % c[:4])
def test_whole_layer_accumulators_match_the_oracle_digests(case):
    family, layer, M, mode, seed = case
    K, N = FAMILIES[family][layer]
    dev = "cuda:0"
    api.lib()
    api.set_gemm_config(0, 0)
    w = wl.layer_weights(family, layer, seed, dev)
    blob = api.pack_weights(w, mode)
    del w
    x = wl.layer_activations(family, layer, M, seed, dev)
    qx, sx, rowsum, _ = api.quant_act_per_token(x)
    del x
    acc = api.w4a8_gemm_i32(qx, blob, N, mode, rowsum=rowsum)
    out = api.w4a8_gemm(qx, sx, blob, N, mode, rowsum=rowsum)
    torch.cuda.synchronize()
    a = np.ascontiguousarray(acc.cpu().numpy().astype("<i4"))
    bad = [i for i in range(-(-M // ROWS))
           if hashlib.blake2b(a[i * ROWS:(i + 1) * ROWS].tobytes(), digest_size=8).hexdigest() != GOLDEN[case][i]]
    assert not bad, "token-row blocks whose accumulators differ from the oracle: %s (config %s)" % (
        bad[:8], api.query_gemm_config(M, N, K, mode))
    # epilogue over the whole tensor: FP64 product of the (now verified) accumulators with the stored scales
    scales = api.unpack_weights(blob, N, K, mode)[-1].cpu().numpy().astype(np.float64)       # s0 / sw [N]
    ref = a.astype(np.float64) * sx.cpu().numpy().astype(np.float64)[:, None] * scales[None, :]
    got = out.cpu().numpy().astype(np.float64)
    assert (np.abs(got - ref) <= 1e-3 * np.abs(ref) + 2.0 ** -24).all()
