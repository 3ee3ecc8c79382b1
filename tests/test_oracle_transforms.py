"""Pins for the oracle of the data-free offline transforms (CPU only): permutation and rotation invariance of
X W^T, textbook properties of the Hadamard matrix, a library Hadamard matrix, what the transforms are for
(similar salience per group, suppressed outlier channels, smaller quantization error), planted mistakes."""
import numpy as np
import scipy.linalg

from oracle import qoq_quant as qq
from oracle import transforms as tr
from paper_2405_04532_amd import workloads as wl


def test_salience_and_order():
    x = np.array([[1.0, -3.0, 0.5, 3.0], [-2.0, 1.0, 0.25, -1.0]], dtype=np.float16)
    s = tr.channel_salience(x)
    assert s.tolist() == [2.0, 3.0, 0.5, 3.0]
    assert tr.channel_order(s).tolist() == [1, 3, 0, 2]             # ties keep the channel order
    x = wl.make_activations(32, 512, 3).numpy()
    p = tr.channel_order(tr.channel_salience(x))
    assert sorted(p.tolist()) == list(range(512))
    sal = tr.channel_salience(x)[p]
    assert np.all(sal[:-1] >= sal[1:])
    # brute force
    for j in (0, 100, 511):
        assert sal[j] == max(abs(float(v)) for v in x[:, p[j]])


def test_reordering_leaves_the_product_unchanged_and_groups_similar_salience():
    x = wl.make_activations(16, 512, 4).numpy()
    w = wl.make_weights(64, 512, 4).numpy()
    p = tr.channel_order(tr.channel_salience(x))
    xr, wr = tr.reorder_channels(x, p), tr.reorder_channels(w, p)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.allclose(xr.astype(np.float64) @ wr.astype(np.float64).T, ref, rtol=1e-12, atol=1e-12)
    # per-token quantization does not depend on the channel order
    qx, sx, rs, _ = qq.act_quant(x)
    qxr, sxr, rsr, _ = qq.act_quant(xr)
    assert np.array_equal(qxr, qx[:, p]) and np.array_equal(sxr.view(np.uint16), sx.view(np.uint16)) and np.array_equal(rs, rsr)
    # the 1% outlier channels (5 of 512) all land in the first group
    sal = tr.channel_salience(x)
    top = set(np.argsort(-sal.astype(np.float64), kind="stable")[:5].tolist())
    assert top <= set(p[:128].tolist())
    ratio = lambda s: s.reshape(-1, 128).max(axis=1) / s.reshape(-1, 128).min(axis=1)
    assert ratio(sal[p])[1:].max() < ratio(sal).max()               # groups are more homogeneous after sorting


def test_hadamard_matrix_properties():
    for n in (1, 2, 8, 64, 256):
        h = tr.hadamard(n)
        assert np.array_equal(h @ h.T, n * np.eye(n)) and np.array_equal(h, h.T)
        assert np.array_equal(h, scipy.linalg.hadamard(n).astype(np.float64))
        i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
        pop = np.array([[bin(a & b).count("1") for b in range(n)] for a in range(n)])
        assert np.array_equal(h, (-1.0) ** pop)                     # entry (i, j) = (-1)^popcount(i & j)


def test_rotation_leaves_the_product_unchanged_and_spreads_outliers():
    x = wl.make_activations(16, 256, 5).numpy()
    w = wl.make_weights(32, 256, 5).numpy()
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    for block in (256, 64):
        r = np.kron(np.eye(256 // block), tr.hadamard(block) / np.sqrt(block))
        assert np.allclose(r @ r.T, np.eye(256), atol=1e-12)
        exact = (x.astype(np.float64) @ r) @ (w.astype(np.float64) @ r).T
        assert np.allclose(exact, ref, rtol=1e-10, atol=1e-10)
        xr, wr = tr.rotate_fp16(x, block), tr.rotate_fp16(w, block)
        assert np.array_equal(xr.astype(np.float64), (x.astype(np.float64) @ r).astype(np.float16).astype(np.float64))
        got = xr.astype(np.float64) @ wr.astype(np.float64).T        # only the two FP16 roundings differ
        assert np.abs(got - ref).max() <= 4 * 2.0 ** -11 * np.abs(x.astype(np.float64)).max() * np.abs(w.astype(np.float64)).sum(axis=1).max()
    # energy is preserved, the outlier channels (x20) are spread out
    xr = tr.rotate_fp16(x, 256).astype(np.float64)
    assert np.allclose((xr ** 2).sum(axis=1), (x.astype(np.float64) ** 2).sum(axis=1), rtol=2e-3)
    assert np.abs(xr).max() < 0.5 * np.abs(x.astype(np.float64)).max()
    # one-hot row -> a row of the scaled matrix; constant row -> all energy in channel 0
    e = np.zeros((1, 64), dtype=np.float16); e[0, 5] = 8.0
    assert np.array_equal(tr.rotate_fp16(e, 64)[0].astype(np.float64), tr.hadamard(64)[5])
    c = np.full((1, 64), 0.5, dtype=np.float16)
    out = tr.rotate_fp16(c, 64)[0].astype(np.float64)
    assert out[0] == 4.0 and not out[1:].any()
    # applying it twice gives the input back (H / sqrt(n) is symmetric and orthogonal) when nothing rounds
    g = (np.random.default_rng(0).integers(-8, 9, size=(3, 64))).astype(np.float16)
    assert np.array_equal(tr.rotate_fp16(tr.rotate_fp16(g, 64), 64), g)


def test_rotation_lowers_the_activation_quantization_error_on_outlier_data():
    """What the rotation is for: per-token INT8 activations lose less once the outlier channels are spread out."""
    x = wl.make_activations(32, 1024, 6).numpy()
    w = wl.make_weights(64, 1024, 6).numpy()
    ref = x.astype(np.float64) @ w.astype(np.float64).T

    def act_error(xa, wa):
        qx, sx, _, _ = qq.act_quant(xa)
        return np.sqrt(np.mean(((qx * sx.astype(np.float64)[:, None]) @ wa.astype(np.float64).T - ref) ** 2))

    assert act_error(tr.rotate_fp16(x, 1024), tr.rotate_fp16(w, 1024)) < 0.5 * act_error(x, w)


def test_planted_mistakes():
    x = wl.make_activations(8, 128, 7).numpy()
    w = wl.make_weights(16, 128, 7).numpy()
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    p = tr.channel_order(tr.channel_salience(x))
    inv = np.argsort(p)
    bad = tr.reorder_channels(x, p).astype(np.float64) @ tr.reorder_channels(w, inv).astype(np.float64).T
    assert not np.allclose(bad, ref, atol=1e-3)                      # weights permuted with the inverse map
    unscaled = (x.astype(np.float64) @ tr.hadamard(128)) @ (w.astype(np.float64) @ tr.hadamard(128)).T
    assert not np.allclose(unscaled, ref, atol=1e-3)                 # forgot the 1 / sqrt(n)
    assert tr.channel_order(np.array([1.0, 3.0, 2.0])).tolist() != np.argsort(np.array([1.0, 3.0, 2.0])).tolist()   # ascending
