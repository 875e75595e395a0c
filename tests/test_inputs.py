"""The seeded generator: reproducible, windowable, right shape of distribution."""
import numpy as np

from paper_2401_01728_amd.inputs import gen


def test_windows_and_streams():
    a = gen.normal_f32(7, 3, 1000)
    b = gen.normal_f32(7, 3, 100, offset=400)
    assert np.array_equal(a[400:500], b)
    assert not np.array_equal(a, gen.normal_f32(7, 4, 1000))
    assert not np.array_equal(a, gen.normal_f32(8, 3, 1000))
    idx = np.array([5, 999, 2**33 + 1], dtype=np.uint64)
    assert np.array_equal(gen.normal_f32_at(7, 3, idx)[:2], a[[5, 999]])


def test_moments():
    z = gen.normal_f32(1, 0, 400000).astype(np.float64)
    assert abs(z.mean()) < 5e-3 and abs(z.std() - 1) < 5e-3 and np.abs(z).max() < 4.9
    assert abs((z ** 4).mean() - 2.85) < 0.05          # Irwin-Hall n=8: kurtosis 3 - 0.15
    v = gen.normal_f32(1, 0, 1000, mean=1.0, std=0.02)
    assert abs(v.mean() - 1) < 3e-3
    u = gen.uniform_f32(1, 5, 100000, lo=-0.5, hi=0.5)
    assert u.min() >= -0.5 and u.max() < 0.5 and abs(u.mean()) < 5e-3


def test_bf16_rounding_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], dtype=np.float32)
    r = gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(x))
    assert np.array_equal(r, np.array([1.0, 1.0, 1.015625, -2.5, 0.0], dtype=np.float32))
