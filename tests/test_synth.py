"""The seeded generators: published SplitMix64 outputs, ranges, moments, bf16 rounding."""
import numpy as np

import synth


def test_splitmix64_published_vectors():
    # first three outputs of SplitMix64 started from state 0 (reference implementation)
    g = np.uint64(0x9E3779B97F4A7C15)
    with np.errstate(over="ignore"):
        got = [int(synth.splitmix64(np.uint64(i) * g)) for i in range(3)]
    assert got == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_uniform_range_and_moments():
    u = synth.uniform_pm1(0, 0, (200000,))
    assert u.dtype == np.float32 and u.min() >= -1.0 and u.max() < 1.0
    assert abs(u.mean()) < 0.01 and abs((u.astype(np.float64) ** 2).mean() - 1 / 3) < 0.01
    assert np.array_equal(u[:100], synth.uniform_pm1(0, 0, (100,)))        # counter based
    assert not np.array_equal(u[:100], synth.uniform_pm1(0, 1, (100,)))    # streams differ
    assert not np.array_equal(u[:100], synth.uniform_pm1(1, 0, (100,)))    # seeds differ


def test_normal_moments():
    z = synth.normal(3, 0, (200001,), sigma=0.5).astype(np.float64)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 0.5) < 0.01
    assert abs((z ** 4).mean() / z.var() ** 2 - 3.0) < 0.1


def test_small_ints():
    v = synth.small_ints(4, 0, (50000,))
    assert set(np.unique(v)) == {-3.0, -2.0, -1.0, 0.0, 1.0, 2.0, 3.0}


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5],
                 np.float32)
    bits = synth.to_bf16_bits(x)
    assert [int(b) for b in bits] == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xC020]
    assert np.array_equal(synth.bf16_bits_to_f32(bits),
                          np.array([1.0, 1.0, 1.015625, 1.0078125, -2.5], np.float32))
