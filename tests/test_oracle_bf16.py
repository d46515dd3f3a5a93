"""Pins for the oracle's bfloat16 conversions and for bfloat16 gradient storage.

bfloat16 is fixed by its format (1 sign, 8 exponent, 7 fraction bits: the upper
half of an IEEE binary32).  Decoding is pinned over the whole code space against
that definition evaluated with numpy bit operations; encoding (round to nearest,
ties to even) against torch's CPU conversion, an independent library routine, and
against hand-worked ties."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as W


def test_bf16_decode_all_65536_patterns_are_the_upper_half_of_a_binary32():
    bits = np.arange(65536, dtype=np.uint16)
    with np.errstate(invalid="ignore"):
        want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    got = np.array([oracle.bf16_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_bf16_decode_known_values():
    assert oracle.bf16_to_double(0x3F80) == 1.0
    assert oracle.bf16_to_double(0xC000) == -2.0
    assert oracle.bf16_to_double(0x3FC0) == 1.5
    assert oracle.bf16_to_double(0x7F7F) == (2.0 - 2.0 ** -7) * 2.0 ** 127      # largest finite
    assert oracle.bf16_to_double(0x0080) == 2.0 ** -126                          # smallest normal
    assert oracle.bf16_to_double(0x0001) == 2.0 ** -133                          # smallest subnormal
    assert oracle.bf16_to_double(0x7F80) == float("inf")
    assert math.isnan(oracle.bf16_to_double(0x7FC0))


def test_bf16_encode_roundtrips_every_finite_code():
    for b in range(0, 65536, 3):
        x = oracle.bf16_to_double(b)
        if math.isfinite(x):
            assert oracle.float_to_bf16(x) == b


def test_bf16_encode_matches_torch_cpu_rne_on_random_floats():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    with np.errstate(over="ignore"):
        big = rng.standard_normal(5000).astype(np.float32) * np.float32(2e38)    # some round up to inf
    xs = np.concatenate([
        rng.standard_normal(20000).astype(np.float32),
        rng.standard_normal(10000).astype(np.float32) * np.float32(1e-3),
        (rng.standard_normal(5000) * 1e-39).astype(np.float32),                 # binary32 subnormals -> bf16 subnormals
        big,
        np.asarray([0.0, -0.0, np.inf, -np.inf, 3.3895314e38, 3.4e38, 2.0 ** -133, 2.0 ** -134, 1.5 * 2.0 ** -133],
                   dtype=np.float32),
    ])
    want = torch.from_numpy(xs).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.float_to_bf16(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)
    assert (got == 0x7F80).sum() > 10 and ((got & 0x7F80) == 0).sum() > 1000     # both regimes were exercised


def test_bf16_encode_ties_go_to_even():
    # 1 + 2^-8 lies exactly between 1 (even) and 1 + 2^-7 (odd): goes down to 1
    assert oracle.float_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    # 1 + 3*2^-8 lies between 1 + 2^-7 (odd) and 1 + 2^-6 (even): goes up
    assert oracle.float_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    # just above a tie rounds up
    assert oracle.float_to_bf16(float(np.nextafter(np.float32(1.0 + 2.0 ** -8), np.float32(2)))) == 0x3F81
    # half of the smallest subnormal ties to zero
    assert oracle.float_to_bf16(2.0 ** -134) == 0x0000


def test_norm_of_bf16_gradients_vs_exact_rational_sum():
    numels = [700, 33, 1200]
    lay = W.layout_flat_split(numels, 500)
    bits = W.normal_bf16_tensors(numels, 4, 1e-2, threads=1)
    got = oracle.bucket_norms(lay, oracle.Bf16(bits))
    vals = [W.bf16_bits_to_float32(b) for b in bits]
    for b in range(lay.n_buckets):
        s = Fraction(0)
        for t, beg, ln in lay.segments_of(b):
            s += sum(Fraction(float(x)) ** 2 for x in vals[t][beg:beg + ln])
        assert got[b] == pytest.approx(math.sqrt(s), rel=1e-14)
    # the same numbers stored as fp32 give the same norms
    assert np.array_equal(got, oracle.bucket_norms(lay, vals))


def test_scale_bf16_rounds_the_fp32_product_to_nearest_even():
    torch = pytest.importorskip("torch")
    numels = [4096]
    lay = W.layout_one_tensor_per_bucket(numels)
    bits = W.normal_bf16_tensors(numels, 5, 1.0, threads=1)
    g = oracle.Bf16([bits[0].copy()])
    coef = np.asarray([0.3137], np.float32)
    oracle.bucket_scale(lay, g, coef)
    prod = (W.bf16_bits_to_float32(bits[0]).astype(np.float64) * np.float64(coef[0])).astype(np.float32)
    want = torch.from_numpy(prod).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(g[0], want)
    assert not np.array_equal(g[0], bits[0])


def test_fused_step_on_bf16_gradients_equals_the_same_values_stored_as_fp32():
    numels = [900, 50, 2000]
    lay = W.layout_flat_split(numels, 800)
    bits = W.normal_bf16_tensors(numels, 6, 1e-2, threads=1)
    vals = [W.bf16_bits_to_float32(b) for b in bits]
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-6, weight_decay=0.01)
    thr = np.full(lay.n_buckets, 0.1, np.float32)

    def state():
        return ([x.astype(np.float64) for x in W.normal_tensors(numels, 6, "p", 0.02)],
                [np.zeros(n) for n in numels], [np.zeros(n) for n in numels])
    pa, ma, va = state()
    pb, mb, vb = state()
    na, ca, _ = oracle.bucket_clip_adam(lay, oracle.Bf16([b.copy() for b in bits]), pa, ma, va, thr, step=1, **hp)
    nb, cb, _ = oracle.bucket_clip_adam(lay, [v.copy() for v in vals], pb, mb, vb, thr, step=1, **hp)
    assert (ca < 1).any()
    assert np.array_equal(na, nb) and np.array_equal(ca, cb)
    for a, b in zip(pa + ma + va, pb + mb + vb):
        assert np.array_equal(a, b)
