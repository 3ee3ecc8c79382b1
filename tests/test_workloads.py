"""Seeded input generator: determinism, distribution and outlier structure (CPU only)."""
import numpy as np
import torch

from paper_2405_04532_amd import workloads as wl


def test_deterministic_and_chunk_invariant():
    a = wl.normal(3, 0, 1000, "cpu")
    b = torch.cat([wl.normal(3, 0, 400, "cpu"), wl.normal(3, 0, 600, "cpu", start=400)])
    assert torch.equal(a, b)
    assert not torch.equal(a, wl.normal(4, 0, 1000, "cpu"))
    assert not torch.equal(a, wl.normal(3, 1, 1000, "cpu"))


def test_normal_moments():
    z = wl.normal(7, 0, 400000, "cpu").numpy()
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01
    assert abs((z ** 4).mean() - 3) < 0.1 and np.isfinite(z).all()


def test_config0_shapes_and_outliers():
    w, x = wl.config0()
    assert w.shape == (256, 256) and x.shape == (16, 256) and w.dtype == torch.float16
    row_rms = w.double().pow(2).mean(dim=1).sqrt()
    assert int((row_rms > 0.1).sum()) == 2 and abs(float(row_rms.median()) - 0.02) < 0.003
    col_rms = x.double().pow(2).mean(dim=0).sqrt()
    assert int((col_rms > 8).sum()) == 4
    w2, x2 = wl.config0()
    assert torch.equal(w, w2) and torch.equal(x, x2)


def test_layer_tables():
    assert wl.LLAMA2_7B["gate_up"] == (4096, 22016) and wl.LLAMA2_7B["down"] == (11008, 4096)
    assert wl.LLAMA3_70B["qkv"] == (8192, 10240) and wl.LLAMA3_70B["down"] == (28672, 8192)
    assert wl.LLAMA3_8B["gate_up"] == (4096, 28672)
    for fam in (wl.LLAMA2_7B, wl.LLAMA3_70B, wl.LLAMA3_8B):
        for k, n in fam.values():
            assert k % 128 == 0 and n % 256 == 0


def test_t3_outlier_rows_are_heavy_tailed():
    w = wl.make_weights(400, 512, 5, sigma=0.01, outlier_kind="t3")
    kurt = ((w.double() / 0.01) ** 4).mean(dim=1)
    assert int((kurt > 6).sum()) >= 2 and int((kurt > 6).sum()) <= 8   # about 1% = 4 rows
