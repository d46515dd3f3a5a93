"""Pins for the oracle's per-bucket norm, clip coefficient and in-place scale.

Each test fixes the oracle against something other than itself: closed forms,
exact rational arithmetic on small inputs (math.fsum / fractions), invariants
that follow from the clipping-by-norm definition (Sec. 2.3) and from the
per-bucket rule of Alg. 1 (App. B)."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as W


def lay1(n):
    return W.layout_one_tensor_per_bucket([n])


# ------------------------------------------------------------------ norm


@pytest.mark.parametrize("c0,n", [(0.5, 1), (0.25, 1000), (-3.0, 4096), (1e-3, 12345), (2.0, 1 << 20)])
def test_norm_constant_bucket_closed_form(c0, n):
    # a bucket of n copies of c0 has norm |c0| * sqrt(n)
    g = [np.full(n, c0, np.float32)]
    got = oracle.bucket_norms(lay1(n), g)[0]
    want = abs(float(np.float32(c0))) * math.sqrt(n)
    assert got == pytest.approx(want, rel=1e-13)


def test_norm_pythagorean_and_unit_vectors():
    g = np.zeros(50, np.float32)
    g[7], g[31] = 3.0, -4.0
    assert oracle.bucket_norms(lay1(50), [g])[0] == 5.0
    for i in (0, 17, 49):
        e = np.zeros(50, np.float32)
        e[i] = 1.0
        assert oracle.bucket_norms(lay1(50), [e])[0] == 1.0
    assert oracle.bucket_norms(lay1(50), [np.zeros(50, np.float32)])[0] == 0.0


def test_norm_is_l2_not_l1_or_max():
    g = np.asarray([1, 1, 1, 1], np.float32)
    assert oracle.bucket_norms(lay1(4), [g])[0] == 2.0      # L1 would give 4, max-norm 1


def test_norm_homogeneous_under_power_of_two_scaling():
    rng = np.random.default_rng(3)
    g = rng.standard_normal(3000).astype(np.float32)
    n1 = oracle.bucket_norms(lay1(3000), [g])[0]
    n2 = oracle.bucket_norms(lay1(3000), [g * np.float32(-4.0)])[0]
    assert n2 == 4.0 * n1                                   # exact: scaling by 4 is exact in every step


def _exact_norm(vals):
    s = sum(Fraction(float(x)) ** 2 for x in vals)
    return math.sqrt(s)                                     # Fraction -> correctly rounded double, then sqrt


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_norm_vs_exact_rational_sum_multi_tensor_split_layout(dtype):
    # 5 tensors cut into buckets of 37 elements in reverse order: segments start
    # in the middle of tensors, buckets hold pieces of several tensors.
    numels = [50, 3, 120, 1, 64]
    lay = W.layout_flat_split(numels, 37)
    assert lay.tensors_split() >= 3
    rng = np.random.default_rng(11)
    g = [(rng.standard_normal(n) * 0.3).astype(dtype) for n in numels]
    got = oracle.bucket_norms(lay, g)
    for b in range(lay.n_buckets):
        vals = []
        for t, beg, ln in lay.segments_of(b):
            vals += list(g[t][beg:beg + ln])
        assert got[b] == pytest.approx(_exact_norm(vals), rel=1e-14), b
    # the squares of the bucket norms add up to the square of the whole-gradient norm
    whole = _exact_norm(np.concatenate(g))
    assert math.sqrt(float(np.sum(got ** 2))) == pytest.approx(whole, rel=1e-13)


def test_norm_fp16_subnormal_inputs_are_not_flushed():
    # all-subnormal fp16 bucket: 2^-24 * k
    ks = np.arange(1, 200, dtype=np.uint16)
    g = ks.view(np.float16).copy()
    got = oracle.bucket_norms(lay1(len(ks)), [g])[0]
    want = 2.0 ** -24 * math.sqrt(sum(int(k) ** 2 for k in ks))
    assert got == pytest.approx(want, rel=1e-14) and got > 0


def test_norm_independent_of_how_a_tensor_is_segmented():
    rng = np.random.default_rng(5)
    g = [rng.standard_normal(1000).astype(np.float32)]
    whole = oracle.bucket_norms(lay1(1000), g)[0]
    pieces = W.Layout(np.asarray([1000], np.uint64), np.asarray([0, 3], np.uint64),
                      np.asarray([0, 0, 0], np.uint32), np.asarray([0, 333, 334], np.uint64),
                      np.asarray([333, 1, 666], np.uint64))
    assert oracle.bucket_norms(pieces, g)[0] == pytest.approx(whole, rel=1e-14)


def test_norm_tiny_config_matches_sigma_sqrt_n():
    w = W.config_tiny()
    norms = oracle.bucket_norms(w.layout, w.grads())
    for nb, n in zip(norms, (1000, 4096, 12345)):
        # chi distribution: mean ~ sigma*sqrt(n), sd ~ sigma/sqrt(2); allow 5 sd
        assert abs(nb - 1e-2 * math.sqrt(n)) < 5 * 1e-2 / math.sqrt(2)


# ------------------------------------------------------------------ coefficient


def test_coef_definition_cases():
    norms = np.asarray([0.0, 0.5, 1.0, 2.0, 8.0, 1e-30])
    thr = np.asarray([1.0, 1.0, 1.0, 1.0, 0.5, 1e-3], np.float32)
    coefs, st = oracle.clip_coefs(norms, thr)
    assert st == 0
    # below threshold -> 1; at threshold -> c/n = 1; above -> c/n
    assert list(coefs) == [1.0, 1.0, 1.0, 0.5, 0.0625, 1.0]


def test_coef_in_unit_interval_and_one_iff_below_threshold():
    rng = np.random.default_rng(9)
    norms = np.abs(rng.standard_normal(5000)) * 3
    thr = (np.abs(rng.standard_normal(5000)) + 1e-3).astype(np.float32)
    coefs, st = oracle.clip_coefs(norms, thr)
    assert st == 0
    assert np.all(coefs > 0) and np.all(coefs <= 1)
    below = norms < thr.astype(np.float64)
    assert np.all(coefs[below] == 1.0)
    clipped = norms >= thr.astype(np.float64) * (1 + 1e-6)
    assert np.all(coefs[clipped] < 1.0)
    assert np.allclose(coefs[clipped].astype(np.float64) * norms[clipped], thr[clipped], rtol=1e-7)


def test_coef_bad_threshold_and_nonfinite_norm_flags():
    coefs, st = oracle.clip_coefs(np.asarray([2.0, 2.0, 2.0]), np.asarray([0.0, -1.0, np.nan], np.float32))
    assert st == oracle.STATUS_BAD_THRESHOLD and list(coefs) == [1.0, 1.0, 1.0]
    _, st = oracle.clip_coefs(np.asarray([np.inf]), np.asarray([1.0], np.float32))
    assert st & oracle.STATUS_NONFINITE
    _, st = oracle.clip_coefs(np.asarray([np.nan]), np.asarray([1.0], np.float32))
    assert st & oracle.STATUS_NONFINITE
    # an infinite threshold is valid and never clips a finite bucket
    coefs, st = oracle.clip_coefs(np.asarray([1e30]), np.asarray([np.inf], np.float32))
    assert st == 0 and coefs[0] == 1.0


# ------------------------------------------------------------------ scale in place


def _clip(lay, g, thr):
    norms = oracle.bucket_norms(lay, g)
    coefs, st = oracle.clip_coefs(norms, thr)
    oracle.bucket_scale(lay, g, coefs)
    return norms, coefs


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_scale_leaves_unclipped_buckets_bit_identical_and_clips_the_rest_to_c(dtype):
    numels = [300, 500, 700, 900]
    lay = W.layout_one_tensor_per_bucket(numels)
    rng = np.random.default_rng(2)
    g = [(rng.standard_normal(n) * 0.05).astype(dtype) for n in numels]
    before = [x.copy() for x in g]
    n0 = oracle.bucket_norms(lay, g)
    thr = np.asarray([n0[0] * 2, n0[1] * 0.5, n0[2] * 1.0001, n0[3] * 0.01], np.float32)
    _clip(lay, g, thr)
    assert np.array_equal(g[0].view(np.uint8), before[0].view(np.uint8))
    assert np.array_equal(g[2].view(np.uint8), before[2].view(np.uint8))
    n1 = oracle.bucket_norms(lay, g)
    tol = 1e-6 if dtype == np.float32 else 2e-3            # fp16 storage rounds every element
    assert n1[1] == pytest.approx(float(thr[1]), rel=tol)
    assert n1[3] == pytest.approx(float(thr[3]), rel=tol)
    # direction preserved: every element scaled by the same factor c/norm
    k = float(thr[1]) / n0[1]
    assert np.allclose(g[1].astype(np.float64), before[1].astype(np.float64) * k,
                       rtol=2e-7 if dtype == np.float32 else 1e-3, atol=0 if dtype == np.float32 else 6e-8)


def test_scale_fp32_is_the_correctly_rounded_product():
    rng = np.random.default_rng(4)
    g = [rng.standard_normal(2000).astype(np.float32)]
    before = g[0].copy()
    lay = lay1(2000)
    _, coefs = _clip(lay, g, np.asarray([1.0], np.float32))
    want = (before.astype(np.float64) * float(coefs[0])).astype(np.float32)   # exact product, one rounding
    assert np.array_equal(g[0], want)
    assert np.array_equal(g[0], before * coefs[0])                              # = IEEE fp32 multiply


def test_scale_fp16_rounds_the_fp32_product_to_nearest_even():
    rng = np.random.default_rng(6)
    g = [(rng.standard_t(3, 5000) * 1e-4).astype(np.float16)]
    before = g[0].copy()
    _, coefs = _clip(lay1(5000), g, np.asarray([1e-3], np.float32))
    assert coefs[0] < 1
    want = (before.astype(np.float32) * coefs[0]).astype(np.float16)
    assert np.array_equal(g[0].view(np.uint16), want.view(np.uint16))


def test_alg1_threshold_bounds_the_whole_gradient_norm():
    # Alg. 1 compares every bucket with c/sqrt(B): afterwards sum_b ||G_b||^2 <= c^2,
    # with equality when every bucket was clipped.
    numels = W.scaled_bert_numels(32, 2, 64, vocab=200, max_pos=16)
    lay = W.layout_flat_split(numels, 1000)
    B = lay.n_buckets
    c = 1.0
    assert oracle.alg1_threshold(c, B) == pytest.approx(c / math.sqrt(B), rel=1e-15)
    assert oracle.alg1_threshold(3.0, 16) == 0.75
    thr = np.full(B, oracle.alg1_threshold(c, B), np.float32)
    g = W.normal_tensors(numels, 0, "g", 1.0)               # big gradients: every bucket clips
    _clip(lay, g, thr)
    after = oracle.bucket_norms(lay, g)
    assert math.sqrt(float(np.sum(after ** 2))) == pytest.approx(c, rel=1e-6)
    g = W.normal_tensors(numels, 1, "g", 1.0)
    W.scale_buckets_inplace(lay, g, range(0, B, 2), 1e-4)   # every other bucket tiny: not clipped
    norms, coefs = _clip(lay, g, thr)
    assert np.all(coefs[0::2] == 1.0) and np.all(coefs[1::2] < 1.0)
    after = oracle.bucket_norms(lay, g)
    assert math.sqrt(float(np.sum(after ** 2))) < c


def test_buckets_are_clipped_independently():
    # Sec. 4.2: clipping is applied to each bucket on its own.  Changing bucket 1's
    # gradients must not change a single bit of buckets 0 and 2.
    numels = [400, 400, 400]
    lay = W.layout_one_tensor_per_bucket(numels)
    thr = np.asarray([0.5, 0.5, 0.5], np.float32)
    ga = W.normal_tensors(numels, 0, "g", 0.1)
    gb = [x.copy() for x in ga]
    gb[1] *= np.float32(1000.0)
    na, ca = _clip(lay, ga, thr)
    nb, cb = _clip(lay, gb, thr)
    assert ca[0] == cb[0] and ca[2] == cb[2] and ca[1] != cb[1]
    assert np.array_equal(ga[0], gb[0]) and np.array_equal(ga[2], gb[2])
