"""The seeded input recipe: shapes, determinism and the stated structure.  CPU only."""
import numpy as np

from paper_2605_20315_amd import workloads as wl


def test_config_table_shapes():
    c = wl.configs()
    assert [x.M for x in c[:4]] == [256, 2048, 8192, 16384]
    assert c[4].M == 108351 and c[4].M % 16 == 15
    assert [(l.K, l.N) for l in c[2].layers] == [(4096, 6144), (4096, 4096), (4096, 28672), (14336, 4096)]
    assert [(l.K, l.N) for l in c[3].layers] == [(5120, 7168), (5120, 5120), (5120, 51200), (25600, 5120)]
    assert [(l.K, l.N) for l in c[4].layers] == [(4096, 28672), (14336, 4096)]
    assert sum(wl.layer_flops(c[2].M, l) for l in c[2].layers) == 2.0 * 8192 * (
        4096 * 6144 + 4096 * 4096 + 4096 * 28672 + 14336 * 4096)
    assert wl.ragged_lengths().tolist()[:4] == [7045, 5404, 4438, 2584]


def test_outlier_columns_and_distributions():
    c = wl.configs()
    assert len(wl.outlier_columns(c[0], 0)) == 4
    assert len(wl.outlier_columns(c[2], 0)) == 4 and len(wl.outlier_columns(c[2], 3)) == 14
    assert len(wl.outlier_columns(c[3], 0)) == 5 and len(wl.outlier_columns(c[3], 3)) == 26
    x = wl.bf16_bits_to_f32(wl.activation(c[0], 0))
    cols = wl.outlier_columns(c[0], 0)
    rest = np.setdiff1d(np.arange(1024), cols)
    assert 0.9 < x[:, rest].std() < 1.1 and 15 < x[:, cols].std() < 25
    w = wl.bf16_bits_to_f32(wl.weight(c[0], 0))
    assert w.shape == (1024, 1024) and 0.019 < w.std() < 0.021


def test_generation_is_deterministic_and_chunked(monkeypatch):
    c = wl.configs()[1]
    a = wl.activation(c, 1)
    monkeypatch.setattr(wl, "_workers", lambda: 1)
    b = wl.activation(c, 1)
    assert a.dtype == np.uint16 and a.shape == (2048, 4096) and np.array_equal(a, b)
    assert not np.array_equal(a[:1024], a[1024:])
    assert not np.array_equal(wl.activation(c, 1, seed=1)[:8], a[:8])


def test_bf16_helpers_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], dtype=np.float32)
    bits = wl.f32_to_bf16_bits(x)
    assert bits.tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC020, 0x0000]
    assert np.array_equal(wl.bf16_bits_to_f32(bits), np.array([1.0, 1.0, 1.015625, -2.5, 0.0], dtype=np.float32))
