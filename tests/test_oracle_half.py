"""Pins for the oracle's binary16 conversions: numpy's float16 (an independent
implementation of IEEE 754 binary16) over the whole code space and on
hand-picked rounding cases."""
import numpy as np

import oracle


def test_half_decode_all_65536_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_half_decode_known_values():
    # values fixed by the format: 1.0, -2.0, largest finite, smallest normal, smallest subnormal
    assert oracle.half_to_double(0x3C00) == 1.0
    assert oracle.half_to_double(0xC000) == -2.0
    assert oracle.half_to_double(0x7BFF) == 65504.0
    assert oracle.half_to_double(0x0400) == 2.0 ** -14
    assert oracle.half_to_double(0x0001) == 2.0 ** -24
    assert oracle.half_to_double(0x7C00) == float("inf")


def test_half_encode_roundtrip_every_finite_half():
    bits = np.arange(65536, dtype=np.uint16)
    vals = bits.view(np.float16)
    fin = np.isfinite(vals)
    for b in bits[fin][::7]:
        f = float(np.uint16(b).view(np.float16))
        assert oracle.float_to_half(f) == int(b)


def test_half_encode_matches_numpy_rne_on_random_floats():
    rng = np.random.default_rng(1)
    xs = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(1e-4),   # many subnormal halves
        rng.standard_normal(20000).astype(np.float32),
        rng.standard_normal(5000).astype(np.float32) * np.float32(3e4),     # some overflow to inf
        np.asarray([0.0, -0.0, 65504.0, 65519.996, 65520.0, 1e9, -1e9, 2.0 ** -25, 2.0 ** -24,
                    1.5 * 2.0 ** -24, 2.5 * 2.0 ** -24, 2.0 ** -14, np.inf, -np.inf], dtype=np.float32),
    ])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_half_encode_ties_go_to_even():
    # 1 + 2^-11 lies exactly between 1 (even mantissa) and 1 + 2^-10 (odd): goes down to 1
    assert oracle.float_to_half(1.0 + 2.0 ** -11) == 0x3C00
    # 1 + 3*2^-11 lies between 1+2^-10 (odd) and 1+2^-9 (even): goes up
    assert oracle.float_to_half(1.0 + 3 * 2.0 ** -11) == 0x3C02
    # half of the smallest subnormal ties to zero; just above it rounds up
    assert oracle.float_to_half(2.0 ** -25) == 0x0000
    assert oracle.float_to_half(float(np.nextafter(np.float32(2.0 ** -25), np.float32(1)))) == 0x0001
    assert oracle.float_to_half(float("nan")) & 0x7C00 == 0x7C00
    assert oracle.float_to_half(float("nan")) & 0x03FF != 0
