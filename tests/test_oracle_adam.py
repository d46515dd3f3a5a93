"""Pins for the oracle's Adam update and for the fused clip + Adam step.

Adam is taken as published by Kingma & Ba (bias-corrected moments, eps added
to the square root of the corrected second moment) with decoupled weight
decay; the paper only names it (Alg. 1, last line) and lists its tuned
hyper-parameters (App. A, Table 4).  Pins: an independent high-precision
recurrence (fractions + decimal), closed forms, and torch.optim.AdamW on the
CPU in fp64 as a library routine for the no-clipping special case."""
import math
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as W

HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-6, weight_decay=0.01)


def one_elem_lay():
    return W.layout_one_tensor_per_bucket([1])


def run_adam(gs, p0, m0=0.0, v0=0.0, first_step=1, **hp):
    h = dict(HP, **hp)
    p, m, v = [np.asarray([p0], np.float64)], [np.asarray([m0], np.float64)], [np.asarray([v0], np.float64)]
    out = []
    for k, g in enumerate(gs):
        oracle.adam_step(np.asarray([1], np.uint64), [np.asarray([g], np.float32)], p, m, v, step=first_step + k, **h)
        out.append((p[0][0], m[0][0], v[0][0]))
    return out


def brute_force(gs, p0, lr, beta1, beta2, eps, weight_decay, first_step=1):
    """Independent evaluation: moments as exact rationals from their closed-form
    sums, the parameter recurrence in 60-digit decimal arithmetic."""
    getcontext().prec = 60
    b1, b2 = Fraction(beta1), Fraction(beta2)
    gq = [Fraction(float(np.float32(g))) for g in gs]
    p = Decimal(p0)
    out = []
    for k in range(len(gs)):
        t = first_step + k
        m = sum((1 - b1) * b1 ** (k - j) * gq[j] for j in range(k + 1))
        v = sum((1 - b2) * b2 ** (k - j) * gq[j] ** 2 for j in range(k + 1))
        mhat = m / (1 - b1 ** t)
        vhat = v / (1 - b2 ** t)
        dm = Decimal(mhat.numerator) / Decimal(mhat.denominator)
        dv = Decimal(vhat.numerator) / Decimal(vhat.denominator)
        p = p - Decimal(lr) * (dm / (dv.sqrt() + Decimal(eps)) + Decimal(weight_decay) * p)
        out.append((float(p), float(m), float(v)))
    return out


def test_adam_single_element_recurrence_vs_high_precision_brute_force():
    rng = np.random.default_rng(0)
    gs = (rng.standard_normal(25) * 1e-3).astype(np.float32)
    got = run_adam(gs, 0.0173)
    want = brute_force(gs, 0.0173, **HP)
    for (gp, gm, gv), (wp, wm, wv) in zip(got, want):
        assert gp == pytest.approx(wp, rel=1e-12)
        assert gm == pytest.approx(wm, rel=1e-11, abs=1e-18)
        assert gv == pytest.approx(wv, rel=1e-12)


def test_adam_recurrence_other_hyperparameters_from_the_tuned_ranges():
    # fine-stage ranges of Table 4: beta1 0.7-0.8, beta2 0.85-0.999, wd 1e-2..1e-1, eps 1e-11
    hp = dict(lr=1e-3, beta1=0.75, beta2=0.85, eps=1e-11, weight_decay=0.1)
    gs = np.asarray([2e-3, -1e-3, 5e-4, 0.0, -3e-3, 1e-6], np.float32)
    got = run_adam(gs, -0.4, **hp)
    want = brute_force(gs, -0.4, **hp)
    for a, b in zip(got, want):
        assert a[0] == pytest.approx(b[0], rel=1e-12)
        assert a[1] == pytest.approx(b[1], rel=1e-11, abs=1e-20)
        assert a[2] == pytest.approx(b[2], rel=1e-12)


def test_adam_first_step_closed_form():
    # from m = v = 0 at t = 1: mhat = g, vhat = g^2, so
    # p' = p - lr * ( g / (|g| + eps) + wd * p ),  m' = (1-b1) g,  v' = (1-b2) g^2
    for g32, p0 in [(np.float32(3e-3), 0.02), (np.float32(-7e-4), -0.01), (np.float32(1e-8), 0.5)]:
        g = float(g32)
        (p1, m1, v1), = run_adam([g32], p0)
        assert m1 == pytest.approx((1 - HP["beta1"]) * g, rel=1e-14)
        assert v1 == pytest.approx((1 - HP["beta2"]) * g * g, rel=1e-13)
        want = p0 - HP["lr"] * (g / (abs(g) + HP["eps"]) + HP["weight_decay"] * p0)
        assert p1 == pytest.approx(want, rel=1e-13)
    # sign: a positive gradient moves the parameter down
    assert run_adam([np.float32(1e-3)], 0.0, weight_decay=0.0)[0][0] < 0
    assert run_adam([np.float32(-1e-3)], 0.0, weight_decay=0.0)[0][0] > 0


def test_adam_constant_gradient_bias_correction_is_exact():
    # constant g from m = v = 0: mhat = g and vhat = g^2 at every t
    g32 = np.float32(2.5e-3)
    g = float(g32)
    res = run_adam([g32] * 12, 0.03)
    p = 0.03
    for t, (pt, mt, vt) in enumerate(res, start=1):
        assert mt / (1 - HP["beta1"] ** t) == pytest.approx(g, rel=1e-13)
        assert vt / (1 - HP["beta2"] ** t) == pytest.approx(g * g, rel=1e-12)
        p = p - HP["lr"] * (g / (abs(g) + HP["eps"]) + HP["weight_decay"] * p)
        assert pt == pytest.approx(p, rel=1e-12)


def test_adam_zero_gradient_only_decays():
    res = run_adam([np.float32(0)] * 5, 0.2, m0=1e-3, v0=1e-6, first_step=7)
    m, v, p = 1e-3, 1e-6, 0.2
    for k, (pt, mt, vt) in enumerate(res):
        t = 7 + k
        m *= HP["beta1"]
        v *= HP["beta2"]
        assert mt == pytest.approx(m, rel=1e-14) and vt == pytest.approx(v, rel=1e-14)
        mhat, vhat = m / (1 - HP["beta1"] ** t), v / (1 - HP["beta2"] ** t)
        p = p - HP["lr"] * (mhat / (math.sqrt(vhat) + HP["eps"]) + HP["weight_decay"] * p)
        assert pt == pytest.approx(p, rel=1e-13)
    # with no state at all the parameter just shrinks by (1 - lr*wd) per step
    res = run_adam([np.float32(0)] * 3, 0.2)
    assert res[2][0] == pytest.approx(0.2 * (1 - HP["lr"] * HP["weight_decay"]) ** 3, rel=1e-14)


def test_adam_lr_zero_keeps_parameter_but_updates_moments():
    (p1, m1, v1), = run_adam([np.float32(1e-2)], 0.3, lr=0.0)
    assert p1 == 0.3 and m1 > 0 and v1 > 0


def test_adam_eps_is_outside_the_square_root_and_after_bias_correction():
    # with a huge eps the update is mhat/eps (if eps sat inside the root it would be mhat/sqrt(eps))
    g32 = np.float32(1e-3)
    (p1, _, _), = run_adam([g32], 0.0, eps=10.0, weight_decay=0.0)
    assert p1 == pytest.approx(-1e-3 * float(g32) / (float(g32) + 10.0), rel=1e-12)
    # eps is added to sqrt(vhat), not to sqrt(v): at t=1 vhat = g^2 whereas v = (1-b2) g^2
    (p1, _, _), = run_adam([g32], 0.0, eps=float(g32), weight_decay=0.0)
    assert p1 == pytest.approx(-1e-3 * 0.5, rel=1e-9)


def test_adam_matches_torch_adamw_fp64_on_tiny_config_without_clipping():
    torch = pytest.importorskip("torch")
    w = W.config_tiny()
    lay = w.layout
    p32 = w.params()
    steps = 4
    gs = [W.normal_tensors(lay.tensor_numel, 100 + k, "g", 1e-2) for k in range(steps)]
    # oracle: fused step with thresholds so large that nothing clips
    p = [x.astype(np.float64) for x in p32]
    m = [np.zeros_like(x) for x in p]
    v = [np.zeros_like(x) for x in p]
    thr = np.full(lay.n_buckets, np.inf, np.float32)
    for k in range(steps):
        _, coefs, st = oracle.bucket_clip_adam(lay, [x.copy() for x in gs[k]], p, m, v, thr, step=k + 1, **HP)
        assert st == 0 and np.all(coefs == 1.0)
    # library routine
    tp = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in p32]
    opt = torch.optim.AdamW(tp, lr=HP["lr"], betas=(HP["beta1"], HP["beta2"]), eps=HP["eps"],
                            weight_decay=HP["weight_decay"])
    for k in range(steps):
        for t, x in zip(tp, gs[k]):
            t.grad = torch.tensor(x, dtype=torch.float64)
        opt.step()
    for t in range(lay.n_tensors):
        assert np.allclose(p[t], tp[t].detach().numpy(), rtol=1e-12, atol=1e-15)
        st_ = opt.state[tp[t]]
        assert np.allclose(m[t], st_["exp_avg"].numpy(), rtol=1e-12, atol=1e-18)
        assert np.allclose(v[t], st_["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-24)


# ------------------------------------------------------------------ fused step


def _state(w):
    p = [x.astype(np.float64) for x in w.params()]
    m = [x.astype(np.float64) for x in w.exp_avg()]
    v = [x.astype(np.float64) for x in w.exp_avg_sq()]
    return p, m, v


def small_bert_workload(dtype="f32", cap=1500):
    numels = W.scaled_bert_numels(32, 2, 64, vocab=200, max_pos=16)
    lay = W.layout_flat_split(numels, cap)
    thr = np.full(lay.n_buckets, 0.02, np.float32)
    return W.Workload("small", lay, dtype, thr, W.Hyper(), first_step=10, seed=3,
                      sigma_g=1e-3 if dtype == "f32" else 1e-3, warm=True)


def test_fused_equals_norm_coef_then_adam_on_scaled_gradient_elementwise():
    # definition check of the fused call, written out with numpy in fp64
    w = small_bert_workload()
    lay, g = w.layout, w.grads()
    p, m, v = _state(w)
    p0, m0, v0 = [x.copy() for x in p], [x.copy() for x in m], [x.copy() for x in v]
    norms, coefs, st = oracle.bucket_clip_adam(lay, g, p, m, v, w.thresholds, step=10, **HP)
    assert st == 0 and (coefs < 1).any()
    b1, b2 = HP["beta1"], HP["beta2"]
    for b in range(lay.n_buckets):
        sq = 0.0
        for t, beg, ln in lay.segments_of(b):
            sq += float(np.sum(g[t][beg:beg + ln].astype(np.float64) ** 2))
        assert norms[b] == pytest.approx(math.sqrt(sq), rel=1e-12)
        c = float(w.thresholds[b])
        want_coef = np.float32(c / norms[b]) if norms[b] >= c else np.float32(1)
        assert coefs[b] == want_coef
        for t, beg, ln in lay.segments_of(b):
            sl = slice(beg, beg + ln)
            gh = float(coefs[b]) * g[t][sl].astype(np.float64)
            mm = b1 * m0[t][sl] + (1 - b1) * gh
            vv = b2 * v0[t][sl] + (1 - b2) * gh * gh
            up = (mm / (1 - b1 ** 10)) / (np.sqrt(vv / (1 - b2 ** 10)) + HP["eps"])
            pp = p0[t][sl] - HP["lr"] * (up + HP["weight_decay"] * p0[t][sl])
            assert np.allclose(m[t][sl], mm, rtol=1e-12, atol=1e-19)
            assert np.allclose(v[t][sl], vv, rtol=1e-13, atol=0)
            assert np.allclose(p[t][sl], pp, rtol=1e-13, atol=0)


def test_fused_equals_unfused_chain_up_to_storage_rounding_over_20_steps():
    w = small_bert_workload()
    lay = w.layout
    pf, mf, vf = _state(w)
    pu, mu, vu = _state(w)
    for k in range(20):
        g = W.normal_tensors(lay.tensor_numel, 500 + k, "g", 1e-3)
        gf, gu = [x.copy() for x in g], [x.copy() for x in g]
        nf, cf, _ = oracle.bucket_clip_adam(lay, gf, pf, mf, vf, w.thresholds, step=k + 1, **HP)
        nu = oracle.bucket_norms(lay, gu)
        cu, _ = oracle.clip_coefs(nu, w.thresholds)
        oracle.bucket_scale(lay, gu, cu)
        oracle.adam_step(lay, gu, pu, mu, vu, step=k + 1, **HP)
        assert np.array_equal(nf, nu) and np.array_equal(cf, cu)
        assert all(np.array_equal(a, b) for a, b in zip(gf, g))          # no write-back: g untouched
    for t in range(lay.n_tensors):
        # the unfused chain rounds coef*g to fp32 (6e-8 relative) before Adam
        assert np.allclose(pf[t], pu[t], rtol=1e-6, atol=1e-9)
        assert np.allclose(vf[t], vu[t], rtol=1e-6, atol=0)
        assert np.allclose(mf[t], mu[t], rtol=1e-5, atol=1e-11)


def test_fused_equals_unfused_bitwise_when_the_coefficient_is_a_power_of_two():
    # bucket (3,4,0,...) has norm 5; threshold 2.5 gives coef exactly 0.5, so scaling is exact
    lay = W.layout_one_tensor_per_bucket([64, 64])
    g = [np.zeros(64, np.float32), np.zeros(64, np.float32)]
    g[0][3], g[0][9] = 3.0, 4.0
    g[1][:] = 0.001
    thr = np.asarray([2.5, 100.0], np.float32)
    rng = np.random.default_rng(8)
    mk = lambda: [rng.standard_normal(64) * 0.02 for _ in range(2)]
    p = mk()
    m = [x * 0.01 for x in mk()]
    v = [np.abs(x) * 1e-4 for x in mk()]
    p2, m2, v2 = [x.copy() for x in p], [x.copy() for x in m], [x.copy() for x in v]
    gu = [x.copy() for x in g]
    _, coefs, _ = oracle.bucket_clip_adam(lay, g, p, m, v, thr, step=3, **HP)
    assert list(coefs) == [0.5, 1.0]
    oracle.bucket_scale(lay, gu, coefs)
    oracle.adam_step(lay, gu, p2, m2, v2, step=3, **HP)
    for a, b in zip(p + m + v, p2 + m2 + v2):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_fused_write_back_stores_the_scaled_gradient_and_leaves_adam_unchanged(dtype):
    w = small_bert_workload(dtype)
    lay = w.layout
    g0 = w.grads()
    pa, ma, va = _state(w)
    pb, mb, vb = _state(w)
    ga, gb = [x.copy() for x in g0], [x.copy() for x in g0]
    _, coefs, _ = oracle.bucket_clip_adam(lay, ga, pa, ma, va, w.thresholds, step=10, write_back=False, **HP)
    oracle.bucket_clip_adam(lay, gb, pb, mb, vb, w.thresholds, step=10, write_back=True, **HP)
    assert (coefs < 1).any()
    for a, b in zip(pa + ma + va, pb + mb + vb):
        assert np.array_equal(a, b)
    gs = [x.copy() for x in g0]
    oracle.bucket_scale(lay, gs, coefs)
    for a, b, c in zip(gb, gs, ga):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8))
    assert all(np.array_equal(a.view(np.uint8), b.view(np.uint8)) for a, b in zip(ga, g0))


def test_fp16_fused_uses_the_unrounded_product_unfused_the_stored_one():
    w = small_bert_workload("f16")
    lay = w.layout
    g = w.grads()
    pf, mf, vf = _state(w)
    pu, mu, vu = _state(w)
    _, coefs, _ = oracle.bucket_clip_adam(lay, [x.copy() for x in g], pf, mf, vf, w.thresholds, step=10, **HP)
    gu = [x.copy() for x in g]
    oracle.bucket_scale(lay, gu, coefs)
    oracle.adam_step(lay, gu, pu, mu, vu, step=10, **HP)
    # fused: m' - b1*m0 = (1-b1) * coef * g exactly (to fp64 rounding)
    m0 = [x.astype(np.float64) for x in w.exp_avg()]
    clipped_any = False
    for b in range(lay.n_buckets):
        for t, beg, ln in lay.segments_of(b):
            sl = slice(beg, beg + ln)
            want = HP["beta1"] * m0[t][sl] + (1 - HP["beta1"]) * float(coefs[b]) * g[t][sl].astype(np.float64)
            assert np.allclose(mf[t][sl], want, rtol=1e-12, atol=1e-19)
            want_u = HP["beta1"] * m0[t][sl] + (1 - HP["beta1"]) * gu[t][sl].astype(np.float64)
            assert np.allclose(mu[t][sl], want_u, rtol=1e-12, atol=1e-19)
            clipped_any |= bool(coefs[b] < 1)
    assert clipped_any
    assert any(not np.array_equal(a, b) for a, b in zip(mf, mu))          # the two modes really differ


def test_nonfinite_gradient_sets_flag_and_skip_mode_is_a_bit_exact_noop():
    w = small_bert_workload()
    lay = w.layout
    g = w.grads()
    g[5][0] = np.inf
    p, m, v = _state(w)
    ref = [x.copy() for x in p + m + v]
    g_before = [x.copy() for x in g]
    _, _, st = oracle.bucket_clip_adam(lay, g, p, m, v, w.thresholds, step=10, write_back=True,
                                       skip_on_nonfinite=True, **HP)
    assert st & oracle.STATUS_NONFINITE
    assert all(np.array_equal(a, b) for a, b in zip(p + m + v, ref))
    assert all(np.array_equal(a.view(np.uint32), b.view(np.uint32)) for a, b in zip(g, g_before))
    # without the skip flag the step is taken (other buckets move) and the flag is still raised
    _, _, st = oracle.bucket_clip_adam(lay, g, p, m, v, w.thresholds, step=10, **HP)
    assert st & oracle.STATUS_NONFINITE
    assert any(not np.array_equal(a, b) for a, b in zip(p, ref[:len(p)]))


def test_values_that_propagate_from_inf_and_nan_gradients_are_what_ieee_arithmetic_gives():
    """The formulas applied as they stand (no special case beyond the status bit).  An infinite gradient makes its
    bucket's norm infinite and the coefficient c / inf = 0: every finite gradient of that bucket becomes 0, so its
    elements only decay (m' = b1 m, v' = b2 v, and p' follows from those: the zero-gradient closed form), while the
    infinite element itself is 0 * inf = NaN in m, v and p.  A NaN gradient makes the norm NaN, the comparison
    norm >= c false and the coefficient 1: the bucket is not scaled, the NaN stays in its own element and the other
    elements take an ordinary Adam step (held to the independent high-precision recurrence).  Buckets are
    independent: a third, clean bucket is clipped and updated as if the others were not there."""
    lay = W.layout_one_tensor_per_bucket([4, 3, 2])
    g = [np.asarray([np.inf, 3.0, -4.0, 0.0], np.float32), np.asarray([np.nan, 2.0, -0.5], np.float32),
         np.asarray([3.0, 4.0], np.float32)]
    p0 = [np.asarray([0.5, -0.25, 0.125, 1.0]), np.asarray([0.3, 0.2, -0.1]), np.asarray([1.0, -1.0])]
    m0 = [np.asarray([0.01, -0.02, 0.03, 0.0]), np.asarray([0.0, 0.0, 0.0]), np.asarray([0.0, 0.0])]
    v0 = [np.asarray([1e-4, 4e-4, 9e-4, 0.0]), np.asarray([0.0, 0.0, 0.0]), np.asarray([0.0, 0.0])]
    p, m, v = [x.copy() for x in p0], [x.copy() for x in m0], [x.copy() for x in v0]
    thr = np.asarray([1.0, 1.0, 2.5], np.float32)
    t = 3
    norms, coefs, st = oracle.bucket_clip_adam(lay, g, p, m, v, thr, step=t, **HP)
    assert st == oracle.STATUS_NONFINITE
    assert np.isposinf(norms[0]) and coefs[0] == 0.0
    assert np.isnan(norms[1]) and coefs[1] == 1.0
    assert norms[2] == 5.0 and coefs[2] == np.float32(0.5)
    b1, b2, lr, eps, wd = HP["beta1"], HP["beta2"], HP["lr"], HP["eps"], HP["weight_decay"]
    # bucket 0: element 0 is NaN everywhere; elements 1..3 see a zero gradient
    assert np.isnan(p[0][0]) and np.isnan(m[0][0]) and np.isnan(v[0][0])
    for i in (1, 2, 3):
        em, ev = b1 * m0[0][i], b2 * v0[0][i]
        ep = p0[0][i] - lr * ((em / (1 - b1 ** t)) / (math.sqrt(ev / (1 - b2 ** t)) + eps) + wd * p0[0][i])
        assert m[0][i] == pytest.approx(em, rel=1e-15, abs=0) and v[0][i] == pytest.approx(ev, rel=1e-15, abs=0)
        assert p[0][i] == pytest.approx(ep, rel=1e-14)
    # bucket 1: element 0 NaN, the others an ordinary first-moment-from-zero step at t = 3 with their own gradient
    assert np.isnan(p[1][0]) and np.isnan(m[1][0]) and np.isnan(v[1][0])
    for i, gi in ((1, 2.0), (2, -0.5)):
        em, ev = (1 - b1) * gi, (1 - b2) * gi * gi
        ep = p0[1][i] - lr * ((em / (1 - b1 ** t)) / (math.sqrt(ev / (1 - b2 ** t)) + eps) + wd * p0[1][i])
        assert m[1][i] == pytest.approx(em, rel=1e-15) and v[1][i] == pytest.approx(ev, rel=1e-15)
        assert p[1][i] == pytest.approx(ep, rel=1e-14)
    # bucket 2: clipped to half, as if alone
    for i, gi in ((0, 1.5), (1, 2.0)):
        assert m[2][i] == pytest.approx((1 - b1) * gi, rel=1e-15) and v[2][i] == pytest.approx((1 - b2) * gi * gi, rel=1e-15)
    # the unfused chain stores the scaled gradients: 0 * inf = NaN, 0 * finite = 0 (signed), the NaN bucket untouched
    g2 = [x.copy() for x in g]
    oracle.bucket_scale(lay, g2, coefs)
    assert np.isnan(g2[0][0]) and np.all(g2[0][1:] == 0.0) and np.signbit(g2[0][2]) and not np.signbit(g2[0][1])
    assert np.isnan(g2[1][0]) and np.array_equal(g2[1][1:], g[1][1:]) and np.array_equal(g2[2], np.asarray([1.5, 2.0], np.float32))
    # negative infinity and an overflowing sum of finite squares behave the same way
    for bad in (-np.inf, np.float32(3e38)):
        gg = [np.asarray([bad, 3e38 if bad > 0 else 1.0], np.float32)]
        pp, mm, vv = [np.asarray([1.0, 1.0])], [np.zeros(2)], [np.zeros(2)]
        n, c, s2 = oracle.bucket_clip_adam(W.layout_one_tensor_per_bucket([2]), gg, pp, mm, vv, np.asarray([1.0], np.float32), step=1, **HP)
        if np.isinf(bad):
            assert np.isposinf(n[0]) and c[0] == 0.0 and s2 == oracle.STATUS_NONFINITE and np.isnan(mm[0][0]) and mm[0][1] == 0.0
        else:       # 3e38^2 is finite in fp64: the oracle's norm is finite (the GPU's fp32 squares would overflow; see R14)
            assert np.isfinite(n[0]) and s2 == 0


def test_adam_and_lamb_steps_do_not_depend_on_the_gradient_scale_when_eps_is_zero():
    # Adam's direction mhat / sqrt(vhat) is homogeneous of degree 0 in the gradient history; scaling every
    # gradient by a power of two scales m by it and v by its square exactly, so p must come out bit-identical.
    numels = [257, 64]
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=0.0, weight_decay=0.01)
    outs = {}
    for scale in (1.0, 2.0 ** 7, 2.0 ** -9):
        for name, fn in (("adam", oracle.adam_step), ("lamb", oracle.lamb_step)):
            p = [x.astype(np.float64) for x in W.normal_tensors(numels, 1, "p", 0.02)]
            m = [np.zeros(n) for n in numels]
            v = [np.zeros(n) for n in numels]
            for step in (1, 2, 3):
                g = [x * np.float32(scale) for x in W.normal_tensors(numels, 30 + step, "g", 1e-2)]
                fn(np.asarray(numels, np.uint64), g, p, m, v, step=step, **hp)
            outs[(name, scale)] = (p, m, v)
    for name in ("adam", "lamb"):
        ref = outs[(name, 1.0)]
        for scale in (2.0 ** 7, 2.0 ** -9):
            got = outs[(name, scale)]
            assert all(np.array_equal(a, b) for a, b in zip(ref[0], got[0])), (name, scale)
            assert all(np.array_equal(a * scale, b) for a, b in zip(ref[1], got[1]))
            assert all(np.array_equal(a * scale * scale, b) for a, b in zip(ref[2], got[2]))


def test_clipping_twice_with_the_same_threshold_changes_nothing_more():
    numels = [3000, 500]
    lay = W.layout_flat_split(numels, 1200)
    g = [x.astype(np.float32) for x in W.normal_tensors(numels, 5, "g", 1e-2)]
    thr = np.full(lay.n_buckets, 0.05, np.float32)
    coefs1, _ = oracle.clip_coefs(oracle.bucket_norms(lay, g), thr)
    assert (coefs1 < 1).all()
    oracle.bucket_scale(lay, g, coefs1)
    n2 = oracle.bucket_norms(lay, g)
    assert np.allclose(n2, 0.05, rtol=1e-6)
    coefs2, _ = oracle.clip_coefs(n2, thr)
    assert np.all(coefs2 > 1 - 1e-6) and np.all(coefs2 <= 1)
