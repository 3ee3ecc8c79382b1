"""Writes tests/golden/gemm_acc_digests.txt: digests of the INT32 accumulators of whole layers at large token counts,
computed by the CPU oracle alone (nothing here imports or runs the HIP path).

Usage, from the repository root:  python tests/golden/make_gemm_digests.py            (about a quarter of an hour on 8 cores, 30 GB of memory for the largest layer)

For every (family, layer, M, mode) of CASES the seeded inputs of the workload module are generated on the CPU, the oracle
runs the whole W4A8 path (Section 4.1 quantizers, integer GEMM, Eq. 5 / Eq. 6), and the accumulators acc[M, N] are
digested as little-endian INT32: one BLAKE2b-64 per block of 64 token rows.  The accumulators have exactly one correct
value (integer sums), so the GPU test recomputes the same digests from qoq_w4a8_gemm_i32 and compares strings.
"""
import hashlib
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import gemm as ogemm                                  # noqa: E402
from paper_2405_04532_amd import workloads as wl                  # noqa: E402  (seeded inputs only)

# (family, layer, M, mode, base seed): the prefill-size rows of the benchmark configurations -- Llama-2-7B layers at
# 1024 and 4096 tokens, per-channel Llama-3-8B layers at 1024 tokens, Llama-3-70B layers at 512 and at 2048 tokens (the
# compute-bound leg of the benchmark)
CASES = [("llama2_7b", name, 1024, 0, 2) for name in ("qkv", "o", "gate_up", "down")] + \
        [("llama3_8b", name, 1024, 1, 4) for name in ("qkv", "gate_up", "down")] + \
        [("llama3_70b", name, 512, 0, 3) for name in ("qkv", "o", "gate_up", "down")] + \
        [("llama2_7b", name, 4096, 0, 2) for name in ("qkv", "o", "gate_up", "down")] + \
        [("llama3_70b", name, 2048, 0, 3) for name in ("qkv", "o", "gate_up", "down")]
ROWS = 64
OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "gemm_acc_digests.txt")


def digests(acc):
    """acc [M, N] integer -> list of hex digests, one per block of ROWS token rows."""
    a = np.ascontiguousarray(acc.astype("<i4"))
    return [hashlib.blake2b(a[r:r + ROWS].tobytes(), digest_size=8).hexdigest() for r in range(0, a.shape[0], ROWS)]


def main():
    ogemm.build()
    lines = ["# family layer M mode base_seed row_block digest   (BLAKE2b-64 of acc[64*row_block : 64*row_block+64, :] as little-endian INT32;",
             "# written by tests/golden/make_gemm_digests.py from the CPU oracle)"]
    for family, layer, M, mode, seed in CASES:
        t0 = time.time()
        w = wl.layer_weights(family, layer, seed, "cpu").numpy()
        x = wl.layer_activations(family, layer, M, seed, "cpu").numpy()
        ref = (ogemm.forward_per_channel if mode else ogemm.forward_group)(w, x)
        for i, d in enumerate(digests(ref["acc"])):
            lines.append("%s %s %d %d %d %d %s" % (family, layer, M, mode, seed, i, d))
        print("%s %s M=%d mode=%d: %.0f s" % (family, layer, M, mode, time.time() - t0), flush=True)
        del w, x, ref
    with open(OUT, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", OUT)


if __name__ == "__main__":
    main()
