"""Pins of the acceptance rule itself (oracle.compare_f32, CPU only).

Every p / m / v parity assertion of the GPU tests goes through this one function,
so it is held to hand-made arrays on both sides of each clause of the rule
(BASELINE tolerances: relative error <= 1e-5, or absolute error <= 1e-7 where
|oracle| < 1e-2).  All inputs are chosen so that the errors are exact binary
fractions or lie far from the bound: the expected verdicts follow from the rule
as stated, not from re-evaluating the function's own expression."""
import numpy as np
import pytest

import oracle

F = np.float32


def verdict(got, want, **kw):
    return oracle.compare_f32(np.array(got, F), np.array(want, np.float64), **kw)


# ---- relative clause, |oracle| >= small ---------------------------------------------

def test_relative_error_just_inside_and_just_outside():
    # 1 + 2^-17 and 1 + 2^-16 are binary32 numbers: relative errors 7.6e-6 and 1.5e-5 against 1.0
    assert verdict([1 + 2.0 ** -17], [1.0])["n_bad"] == 0
    assert verdict([1 + 2.0 ** -16], [1.0])["n_bad"] == 1
    assert verdict([1 - 2.0 ** -17], [1.0])["n_bad"] == 0
    assert verdict([1 - 2.0 ** -16], [1.0])["n_bad"] == 1
    # sign and scale do not matter
    assert verdict([-4096 * (1 + 2.0 ** -17)], [-4096.0])["n_bad"] == 0
    assert verdict([-4096 * (1 + 2.0 ** -16)], [-4096.0])["n_bad"] == 1
    # a wrong sign is an error of 200 %
    assert verdict([-1.0], [1.0])["n_bad"] == 1


def test_relative_bound_is_inclusive():
    # error exactly equal to the tolerance passes (the rule says "<=")
    r = verdict([1 + 2.0 ** -17], [1.0], rel_tol=2.0 ** -17)
    assert r["n_bad"] == 0 and r["max_rel_big"] == 2.0 ** -17
    assert verdict([1 + 2.0 ** -17], [1.0], rel_tol=2.0 ** -17 * (1 - 1e-12))["n_bad"] == 1


def test_relative_error_is_measured_against_the_oracle_value():
    # got = 2, want = 1: 100 % (against got it would be 50 %)
    r = verdict([2.0], [1.0], rel_tol=0.75)
    assert r["n_bad"] == 1 and r["max_rel_big"] == 1.0
    # got = 1, want = 2: 50 %
    r = verdict([1.0], [2.0], rel_tol=0.75)
    assert r["n_bad"] == 0 and r["max_rel_big"] == 0.5


# ---- absolute clause, |oracle| < small ----------------------------------------------

def test_absolute_error_just_inside_and_just_outside_below_small():
    w = 2.0 ** -10                                   # 9.8e-4 < 1e-2
    inside, outside = w + 2.0 ** -24, w + 2.0 ** -23  # errors 6.0e-8 and 1.2e-7, relative 6e-5 and 1.2e-4
    assert verdict([inside], [w])["n_bad"] == 0
    assert verdict([outside], [w])["n_bad"] == 1
    assert verdict([-inside], [-w])["n_bad"] == 0
    assert verdict([-outside], [-w])["n_bad"] == 1
    r = verdict([inside], [w])
    assert r["max_abs_small"] == 2.0 ** -24 and r["max_rel_big"] == 0.0


def test_absolute_bound_is_inclusive():
    w = 2.0 ** -10
    assert verdict([w + 2.0 ** -24], [w], abs_tol=2.0 ** -24)["n_bad"] == 0
    assert verdict([w + 2.0 ** -24], [w], abs_tol=2.0 ** -24 * (1 - 1e-12))["n_bad"] == 1


def test_absolute_clause_needs_both_conditions():
    # small error in absolute terms but |oracle| >= small: the absolute clause must not apply
    kw = dict(rel_tol=1e-5, abs_tol=2.0 ** -8, small=1.0)
    assert verdict([1 + 2.0 ** -10], [1.0], **kw)["n_bad"] == 1           # |w| == small: not "below"
    assert verdict([4 + 2.0 ** -10], [4.0], **kw)["n_bad"] == 1           # |w| > small
    assert verdict([0.5 + 2.0 ** -10], [0.5], **kw)["n_bad"] == 0         # |w| < small, error <= abs_tol
    # |oracle| below small but the error above the absolute bound
    assert verdict([0.5 + 2.0 ** -7], [0.5], **kw)["n_bad"] == 1


def test_zero_oracle_value():
    assert verdict([0.0], [0.0])["n_bad"] == 0
    assert verdict([2.0 ** -24], [0.0])["n_bad"] == 0          # 6e-8 <= 1e-7
    assert verdict([2.0 ** -23], [0.0])["n_bad"] == 1          # 1.2e-7
    assert verdict([-0.0], [0.0])["n_bad"] == 0
    # with no absolute allowance, any difference from an exact zero fails
    assert verdict([1e-30], [0.0], abs_tol=0.0)["n_bad"] == 1
    assert verdict([0.0], [0.0], abs_tol=0.0)["n_bad"] == 0


# ---- non-finite values --------------------------------------------------------------

def test_nan_and_inf():
    nan, inf = float("nan"), float("inf")
    assert verdict([nan], [nan])["n_bad"] == 0
    assert verdict([nan], [1.0])["n_bad"] == 1
    assert verdict([1.0], [nan])["n_bad"] == 1
    assert verdict([nan], [0.0])["n_bad"] == 1
    assert verdict([inf], [inf])["n_bad"] == 0
    assert verdict([-inf], [-inf])["n_bad"] == 0
    assert verdict([inf], [-inf])["n_bad"] == 1
    assert verdict([inf], [3.0e38])["n_bad"] == 1
    assert verdict([3.0e38], [inf])["n_bad"] == 1
    assert verdict([inf], [nan])["n_bad"] == 1
    assert verdict([nan], [inf])["n_bad"] == 1


# ---- counting, worst element, summary figures -----------------------------------------

def test_every_failing_element_is_counted_and_the_worst_is_named():
    want = np.array([1.0, 2.0, 2.0 ** -10, 8.0, 0.0, 16.0], np.float64)
    got = want.astype(F).copy()
    assert verdict(got, want) == {"n_bad": 0, "max_rel_big": 0.0, "max_abs_small": 0.0, "max_rel_all": 0.0,
                                  "worst_index": -1}
    got[1] = 2.5        # error 0.5
    got[3] = 6.0        # error 2.0: the worst
    got[4] = 1.0        # error 1.0
    r = verdict(got, want)
    assert r["n_bad"] == 3 and r["worst_index"] == 3
    assert r["max_rel_big"] == 0.25 and r["max_abs_small"] == 1.0
    # order of the elements does not decide which one is worst
    r = verdict(got[::-1].copy(), want[::-1].copy())
    assert r["n_bad"] == 3 and r["worst_index"] == 2
    # a NaN where a number is expected is counted and named when nothing else fails
    got = want.astype(F).copy()
    got[5] = np.nan
    r = verdict(got, want)
    assert r["n_bad"] == 1 and r["worst_index"] == 5


def test_max_rel_all_sees_small_values_that_pass_by_the_absolute_clause():
    # v-like values: 1e-9 with a 1 % error passes the stated rule (absolute 1e-11) but must show up in max_rel_all,
    # which is what the tests' additional "relative error on every v" requirement reads
    w = 2.0 ** -30
    r = verdict([w * (1 + 2.0 ** -7)], [w])
    assert r["n_bad"] == 0
    assert r["max_rel_all"] == 2.0 ** -7
    assert r["max_rel_big"] == 0.0
    # values at or below `tiny` are left out of it; above it they count
    r = verdict([2.0 ** -120], [2.0 ** -121], tiny=2.0 ** -121)
    assert r["n_bad"] == 0 and r["max_rel_all"] == 0.0
    r = verdict([2.0 ** -120], [2.0 ** -121], tiny=2.0 ** -122)
    assert r["max_rel_all"] == 1.0
    # large values count as well
    assert verdict([1 + 2.0 ** -17], [1.0])["max_rel_all"] == 2.0 ** -17


def test_empty_array():
    r = oracle.compare_f32(np.zeros(0, F), np.zeros(0, np.float64))
    assert r["n_bad"] == 0 and r["worst_index"] == -1


@pytest.mark.parametrize("seed", [0, 1])
def test_count_on_random_arrays_with_planted_errors(seed):
    """Errors of known size planted at known places: the count is the number planted beyond the bound."""
    rng = np.random.default_rng(seed)
    n = 20000
    want = np.where(rng.random(n) < 0.5, rng.normal(0, 1.0, n), rng.normal(0, 1e-4, n)).astype(F).astype(np.float64)
    want[np.abs(want) < 1e-12] = 1e-3
    got = want.astype(F)                                     # exact
    idx = rng.choice(n, 300, replace=False)
    big = np.abs(want[idx]) >= 1e-2
    fail = rng.random(300) < 0.5
    # beyond the bound: 3e-5 relative on large values, 3e-7 absolute (and far more than 1e-5 relative) on small ones;
    # within it: 3e-6 relative, 3e-8 absolute
    delta = np.where(big, np.abs(want[idx]) * np.where(fail, 3e-5, 3e-6), np.where(fail, 3e-7, 3e-8))
    got64 = want.copy()
    got64[idx] += delta * rng.choice([-1.0, 1.0], 300)
    got = got64.astype(F)
    # binary32 rounding of `got` adds at most 6e-8 relative: nowhere near moving a planted error across its bound
    r = oracle.compare_f32(got, want)
    assert r["n_bad"] == int(fail.sum())
    assert r["worst_index"] in set(idx[fail].tolist())
