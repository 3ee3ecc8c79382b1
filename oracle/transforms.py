"""CPU oracle for the data-free offline transforms of QoQ (TEST INFRASTRUCTURE ONLY).

Written from the paper (arXiv 2405.04532):
  * activation-aware channel reordering (Section 4.3, "Activation-Aware Channel Reordering"): the salience of
    an input channel is max|X| over the calibration tokens; input channels are reordered so that channels of
    similar salience share a quantization group; weights and activations are permuted alike, which leaves
    X W^T unchanged;
  * block input module rotation (Section 4.3, "Block Input Module Rotation"): activations and the weights of
    the input modules are multiplied by the same scaled Hadamard matrix, which leaves X W^T unchanged and
    spreads outlier channels over all channels.
Only tests, the smoke check and the benchmark's cpu_baseline leg may import this file.  It shares no code with
the HIP path.  All arithmetic is float64; the only rounding is the final one to FP16.

Readings (the paper gives no formulas here):
  * order = channels sorted by decreasing salience, ties by increasing channel index (a sort is the simplest
    map that puts similar salience into the same group of 128 consecutive channels);
  * rotation matrix = H_n / sqrt(n) with H_n the Sylvester Hadamard matrix (H_1 = [1], H_2n = [[H, H], [H, -H]]);
    for a channel count that is not a power of two, the block-diagonal matrix of H_b / sqrt(b) blocks with b a
    power of two that divides it;
  * a rotated FP16 tensor is the exact product rounded once to FP16 (sums of FP16 numbers are exact in FP64 for
    the sizes used here, so the result does not depend on the order of summation).
"""
import numpy as np


def channel_salience(x_fp16):
    """max over tokens of |X| per input channel: [M, K] -> [K] (float32 holding FP16-exact values)."""
    x = np.asarray(x_fp16, dtype=np.float16).astype(np.float64)
    return np.abs(x).max(axis=0).astype(np.float32)


def channel_order(salience):
    """Permutation p: new channel j is old channel p[j]; most salient first, ties by channel index."""
    s = np.asarray(salience, dtype=np.float64)
    return np.argsort(-s, kind="stable").astype(np.int32)


def reorder_channels(a, perm):
    """Columns (input channels) of a [rows, K] tensor in the new order."""
    return np.asarray(a)[:, np.asarray(perm, dtype=np.int64)]


def hadamard(n):
    """Sylvester Hadamard matrix of order n (a power of two), entries +-1, float64."""
    assert n >= 1 and (n & (n - 1)) == 0
    h = np.ones((1, 1))
    while h.shape[0] < n:
        h = np.block([[h, h], [h, -h]])
    return h


def rotate_fp16(a_fp16, block):
    """a (I (x) H_block / sqrt(block)) rounded once to FP16: [rows, K] -> [rows, K], K % block == 0."""
    a = np.asarray(a_fp16, dtype=np.float16).astype(np.float64)
    rows, K = a.shape
    assert K % block == 0
    h = hadamard(block)
    out = (a.reshape(rows, K // block, block) @ h) * (1.0 / np.sqrt(float(block)))
    return out.reshape(rows, K).astype(np.float16)
