"""Pins for the oracle's integer GEMM, zero-point fold and end-to-end forward:
brute force on tiny shapes, textbook special cases, the Eq. 5 == Eq. 6 identity,
dequantize-then-FP64-matmul, and planted-mistake checks (CPU only)."""
import numpy as np
import pytest

from oracle import gemm, qoq_quant as qq


def _brute(qx, w):
    m, k = qx.shape
    n = w.shape[0]
    out = [[0] * n for _ in range(m)]
    for i in range(m):
        for j in range(n):
            out[i][j] = sum(int(qx[i, t]) * int(w[j, t]) for t in range(k))
    return np.array(out, dtype=np.int64)


def test_c_gemm_vs_brute_force_and_numpy():
    rng = np.random.default_rng(10)
    qx = rng.integers(-127, 128, size=(5, 37))
    w = rng.integers(-128, 128, size=(7, 37))
    ref = _brute(qx, w)
    assert (gemm.gemm_i64(qx, w) == ref).all()
    assert (qq.gemm_i64_numpy(qx, w) == ref).all()
    qx = rng.integers(-127, 128, size=(33, 640))
    w = rng.integers(-127, 128, size=(129, 640))
    assert (gemm.gemm_i64(qx, w) == qq.gemm_i64_numpy(qx, w)).all()


def test_c_gemm_orientation_one_hot():
    """One-hot operands: acc[m, n] picks w[n, k] -- catches a transposed operand."""
    qx = np.zeros((3, 8), dtype=np.int64)
    qx[1, 5] = 2
    w = np.arange(4 * 8).reshape(4, 8) - 10
    acc = gemm.gemm_i64(qx, w)
    assert (acc[0] == 0).all() and (acc[2] == 0).all()
    assert (acc[1] == 2 * w[:, 5]).all()


def test_c_gemm_worst_case_magnitude_fits_int32():
    """Largest K of the workloads (28672) with extreme operands stays below 2^31."""
    k = 28672
    qx = np.full((1, k), 127)
    w = np.full((2, k), 127)
    w[1] = -127
    acc = gemm.gemm_i64(qx, w)
    assert acc[0, 0] == 127 * 127 * k and acc[0, 1] == -127 * 127 * k and abs(acc).max() < 2 ** 31


def test_unit_scale_reduces_to_int8_gemm():
    """With s1 = 1 and z = 0 the level-2 codes are the INT8 operand itself: the path is the
    textbook W8A8 GEMM (Section 4.1: 'as if it was W8A8 per-channel')."""
    rng = np.random.default_rng(11)
    code = rng.integers(0, 16, size=(6, 256))
    s1 = np.ones((6, 2), dtype=np.int64)
    z = np.zeros((6, 2), dtype=np.int64)
    assert (qq.level2_dequant(code, s1, z) == code).all()
    qx = rng.integers(-127, 128, size=(4, 256))
    assert (gemm.gemm_i64(qx, qq.level2_dequant(code, s1, z)) == _brute(qx, code)).all()


def test_group_forward_vs_dequantized_fp64_matmul():
    """Tiny shape: dequantize every operand to FP64 and multiply; equals acc*sx*s0."""
    rng = np.random.default_rng(12)
    w = (rng.standard_normal((24, 256)) * 0.02).astype(np.float16)
    w[3] *= 10
    x = rng.standard_normal((5, 256)).astype(np.float16)
    x[:, 9] *= 20
    r = gemm.forward_group(w, x)
    wq = r["wq"]
    assert wq["q0"].min() >= -119 and wq["q0"].max() <= 119
    assert wq["w_hat"].min() >= -127 and wq["w_hat"].max() <= 127
    w_deq = wq["w_hat"].astype(np.float64) * wq["s0"].astype(np.float64)[:, None]
    x_deq = r["qx"].astype(np.float64) * r["sx"].astype(np.float64)[:, None]
    ref = x_deq @ w_deq.T
    assert np.allclose(r["out64"], ref, rtol=1e-12, atol=1e-12)
    assert (r["out"] == ref.astype(np.float16)).mean() > 0.999      # same up to FP64 rounding at ties
    # the quantized product tracks the unquantized one (sanity of scales' orientation)
    full = x.astype(np.float64) @ w.astype(np.float64).T
    rel = np.linalg.norm(r["out64"] - full) / np.linalg.norm(full)
    assert rel < 0.15


def test_per_channel_identity_eq5_eq6():
    """Eq. 5 (dequantize, then multiply) == Eq. 6 with the exact integer zero fold."""
    rng = np.random.default_rng(13)
    w = (rng.standard_normal((20, 128)) * 0.02).astype(np.float16)
    x = rng.standard_normal((6, 128)).astype(np.float16)
    r = gemm.forward_per_channel(w, x)
    sw = r["sw"].astype(np.float64)
    sx = r["sx"].astype(np.float64)
    w_deq = (r["Q"] - r["z"][:, None]).astype(np.float64) * sw[:, None]
    x_deq = r["qx"].astype(np.float64) * sx[:, None]
    eq5 = x_deq @ w_deq.T
    assert np.allclose(r["out64"], eq5, rtol=1e-12, atol=1e-12)
    # Eq. 6 literally: first term minus (Qx.Sx) ZS_W
    eq6 = (r["raw"].astype(np.float64) * sx[:, None] * sw[None, :]
           - (x_deq.sum(axis=1))[:, None] * (r["z"] * sw)[None, :])
    assert np.allclose(eq6, eq5, rtol=1e-11, atol=1e-11)
    assert (r["acc"] == _brute(r["qx"], r["Q"] - r["z"][:, None])).all()


def test_group_equals_k_matches_single_group():
    """group = K: one (s1, z) per channel; the forward still equals its own dequantized
    FP64 product (the grouping index is the only thing that changes)."""
    rng = np.random.default_rng(14)
    w = (rng.standard_normal((8, 128)) * 0.02).astype(np.float16)
    x = rng.standard_normal((3, 128)).astype(np.float16)
    r = gemm.forward_group(w, x, group=128)
    assert r["wq"]["s1"].shape == (8, 1)
    r2 = gemm.forward_group(np.concatenate([w, w], axis=1), np.concatenate([x, x], axis=1))
    # duplicated K: each half is its own group with the same parameters -> acc doubles
    assert (r2["wq"]["s1"][:, 0] == r2["wq"]["s1"][:, 1]).all()
    assert (r2["acc"] == 2 * r["acc"]).all()


@pytest.mark.parametrize("bad", ["reversed_k", "dropped_zero", "wrong_scale_axis"])
def test_gemm_pins_catch_planted_mistakes(bad, monkeypatch):
    if bad == "reversed_k":
        monkeypatch.setattr(gemm, "gemm_i64", lambda a, b: qq.gemm_i64_numpy(a, np.asarray(b)[:, ::-1]))
        with pytest.raises(AssertionError):
            test_group_forward_vs_dequantized_fp64_matmul()
    elif bad == "dropped_zero":
        monkeypatch.setattr(qq, "per_channel_acc", lambda raw, z, rowsum: np.asarray(raw, dtype=np.int64))
        with pytest.raises(AssertionError):
            test_per_channel_identity_eq5_eq6()
    else:
        orig = qq.output_fp64
        monkeypatch.setattr(qq, "output_fp64", lambda acc, sx, sw: orig(acc, sx, np.roll(np.asarray(sw), 1)))
        with pytest.raises(AssertionError):
            test_group_forward_vs_dequantized_fp64_matmul()


# ------------------------------------------------------------------ token-sum form of the per-channel epilogue
def _per_channel_case(seed, M=6, N=5, K=64):
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
    x = rng.standard_normal((M, K)).astype(np.float16)
    code, z, sw = qq.per_channel_quant(w)
    qx, sx, rowsum, tx = qq.act_quant(x)
    raw = qq.gemm_i64_numpy(qx, code)
    return w, x, code, z, sw, qx, sx, rowsum, tx, raw


def test_token_sum_form_matches_matrix_form():
    """Eq. 7 written out with matrices: X_hat (W_hat + ZS) - X ZS, all operands dequantized to FP64."""
    w, x, code, z, sw, qx, sx, rowsum, tx, raw = _per_channel_case(3)
    s = sw.astype(np.float64)
    x_hat = qx.astype(np.float64) * sx.astype(np.float64)[:, None]
    qs = code.astype(np.float64) * s[:, None]                   # Q_W (.) S_W, [N, K]
    zs = np.repeat((z.astype(np.float64) * s)[:, None], x.shape[1], axis=1)   # ZS_W, [N, K]
    expect = x_hat @ qs.T - x.astype(np.float64) @ zs.T
    got = qq.output_fp64_token_sum(raw, sx, sw, z, tx)
    assert np.allclose(got, expect, rtol=1e-12, atol=1e-12)


def test_token_sum_form_equals_exact_fold_when_activations_are_on_the_grid():
    """If every activation is an exact multiple of its token scale, X_hat == X and both forms coincide."""
    rng = np.random.default_rng(5)
    qx0 = rng.integers(-127, 128, size=(4, 64))
    qx0[:, 0] = 127                                              # pins absmax so that sx is the chosen scale
    sx0 = np.array([0.5, 0.25, 1.0, 0.125])
    x = (qx0 * sx0[:, None]).astype(np.float16)
    assert np.array_equal(x.astype(np.float64), qx0 * sx0[:, None])
    w = (rng.standard_normal((7, 64)) * 0.05).astype(np.float16)
    code, z, sw = qq.per_channel_quant(w)
    qx, sx, rowsum, tx = qq.act_quant(x)
    assert np.array_equal(qx, qx0)
    raw = qq.gemm_i64_numpy(qx, code)
    exact = qq.output_fp64(qq.per_channel_acc(raw, z, rowsum), sx, sw)
    assert np.allclose(qq.output_fp64_token_sum(raw, sx, sw, z, tx), exact, rtol=1e-13, atol=1e-13)


def test_token_sum_form_differs_by_the_summed_quantization_error():
    w, x, code, z, sw, qx, sx, rowsum, tx, raw = _per_channel_case(9, M=8, N=6, K=128)
    exact = qq.output_fp64(qq.per_channel_acc(raw, z, rowsum), sx, sw)
    approx = qq.output_fp64_token_sum(raw, sx, sw, z, tx)
    err_sum = (x.astype(np.float64) - qx * sx.astype(np.float64)[:, None]).sum(axis=1)       # [M]
    zs = z.astype(np.float64) * sw.astype(np.float64)
    assert np.allclose(exact - approx, err_sum[:, None] * zs[None, :], rtol=1e-10, atol=1e-12)
    # and the bound that follows from |X - qx*sx| <= sx/2 per element
    bound = (x.shape[1] * sx.astype(np.float64) / 2)[:, None] * zs[None, :]
    assert np.all(np.abs(exact - approx) <= bound + 1e-12)


@pytest.mark.parametrize("bad", ["plus", "rowsum", "no_scale"])
def test_token_sum_pins_catch_planted_mistakes(bad, monkeypatch):
    def wrong(raw, sx, sw, z, tx):
        s = np.asarray(sw, dtype=np.float16).astype(np.float64)
        first = np.asarray(raw, dtype=np.float64) * np.asarray(sx, dtype=np.float16).astype(np.float64)[:, None] * s[None, :]
        if bad == "plus":
            return first + np.asarray(tx)[:, None] * (np.asarray(z, dtype=np.float64) * s)[None, :]
        if bad == "no_scale":
            return first - np.asarray(tx)[:, None] * np.asarray(z, dtype=np.float64)[None, :]
        return first - np.asarray(tx)[:, None] * (np.asarray(z, dtype=np.float64) * s)[None, :] * 1.01
    monkeypatch.setattr(qq, "output_fp64_token_sum", wrong)
    with pytest.raises(AssertionError):
        test_token_sum_form_matches_matrix_form()
