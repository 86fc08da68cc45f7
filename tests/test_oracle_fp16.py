"""Pins for the oracle's own binary16 conversions: numpy's float16 is the independent library routine."""
import numpy as np


def test_f16_to_f32_all_patterns(ref):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([ref.f16_bits_to_f32(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_f32_to_f16_random_and_ties(ref):
    rng = np.random.default_rng(7)
    xs = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-8, 5, 20000).astype(np.float32),
        # exact midpoints between neighbouring binary16 values (ties -> even), normal and subnormal
        np.array([(2 * k + 1) * 2.0 ** -25 for k in range(0, 40)], dtype=np.float32),
        np.array([1.0 + (2 * k + 1) * 2.0 ** -11 for k in range(0, 40)], dtype=np.float32),
        np.array([65504.0, 65519.9, 65520.0, 70000.0, 0.0, -0.0, 6.1e-5, 5.96e-8, 2.98e-8, 2.99e-8], dtype=np.float32),
    ])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([ref.f32_to_f16_bits(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_f64_to_f16_single_rounding(ref):
    # 1 + 2^-11 + 2^-30 lies just above a tie: a direct rounding goes up, rounding through binary32
    # first (which drops the 2^-30) would hit the tie and go down to even.
    x = 1.0 + 2.0 ** -11 + 2.0 ** -30
    assert ref.f64_to_f16_bits(x) == 0x3C01
    assert np.float32(x).astype(np.float16).view(np.uint16) == 0x3C00
    rng = np.random.default_rng(3)
    xs = rng.standard_normal(5000) * 10.0 ** rng.integers(-7, 4, 5000)
    want = xs.astype(np.float16).view(np.uint16)          # numpy rounds float64 -> float16 directly
    got = np.array([ref.f64_to_f16_bits(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)
