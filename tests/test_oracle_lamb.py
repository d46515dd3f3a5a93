"""Pins for the oracle's LAMB step and per-tensor weight-decay mask.

The paper compares Adam with LAMB (Sec. 2.2, Sec. 5, App. A) without restating
either.  LAMB is taken as published by You et al. (2020, Alg. 2): Adam's
bias-corrected direction plus weight decay, rescaled per tensor by the trust ratio
||p|| / ||update||.  Pins: an independent high-precision evaluation (fractions +
decimal), closed forms at step 1, the invariant ||delta p|| = lr ||p|| that holds
for every tensor and step, the reduction to Adam when the ratio is 1, and the
definition written out with numpy for the clip + LAMB composition.  The decay mask
is pinned against torch.optim.AdamW with two parameter groups."""
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as W

HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-6, weight_decay=0.01)


def dec(fr: Fraction) -> Decimal:
    return Decimal(fr.numerator) / Decimal(fr.denominator)


def lamb_brute_force(gs, p0, lr, beta1, beta2, eps, weight_decay, first_step=1):
    """gs: list over steps of fp32 gradient vectors of one tensor.  Moments as exact
    rationals from their closed-form sums; everything else in 60-digit decimals."""
    getcontext().prec = 60
    b1, b2 = Fraction(beta1), Fraction(beta2)
    n = len(p0)
    p = [Decimal(float(x)) for x in p0]
    out = []
    for k in range(len(gs)):
        t = first_step + k
        u = []
        for i in range(n):
            gq = [Fraction(float(np.float32(gs[j][i]))) for j in range(k + 1)]
            m = sum((1 - b1) * b1 ** (k - j) * gq[j] for j in range(k + 1))
            v = sum((1 - b2) * b2 ** (k - j) * gq[j] ** 2 for j in range(k + 1))
            mhat, vhat = dec(m / (1 - b1 ** t)), dec(v / (1 - b2 ** t))
            u.append(mhat / (vhat.sqrt() + Decimal(eps)) + Decimal(weight_decay) * p[i])
        pn = sum(x * x for x in p).sqrt()
        un = sum(x * x for x in u).sqrt()
        trust = pn / un if (pn > 0 and un > 0) else Decimal(1)
        p = [p[i] - Decimal(lr) * trust * u[i] for i in range(n)]
        out.append(([float(x) for x in p], float(trust)))
    return out


def run_lamb(gs, p0, first_step=1, decay=None, **hp):
    h = dict(HP, **hp)
    n = len(p0)
    numel = np.asarray([n], np.uint64)
    p, m, v = [np.asarray(p0, np.float64).copy()], [np.zeros(n)], [np.zeros(n)]
    out = []
    for k, g in enumerate(gs):
        tr = oracle.lamb_step(numel, [np.asarray(g, np.float32)], p, m, v, step=first_step + k, decay=decay, **h)
        out.append((p[0].copy(), float(tr[0])))
    return out


def test_lamb_recurrence_vs_high_precision_brute_force():
    rng = np.random.default_rng(0)
    n, steps = 7, 12
    gs = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(steps)]
    p0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    got = run_lamb(gs, p0)
    want = lamb_brute_force(gs, p0, **HP)
    for (gp, gt), (wp, wt) in zip(got, want):
        assert gt == pytest.approx(wt, rel=1e-12)
        assert np.allclose(gp, wp, rtol=1e-11, atol=0)


def test_lamb_recurrence_other_hyperparameters():
    hp = dict(lr=2e-3, beta1=0.75, beta2=0.85, eps=1e-11, weight_decay=0.1)
    gs = [np.asarray([2e-3, -1e-3, 5e-4], np.float32), np.asarray([0.0, 1e-6, -3e-3], np.float32),
          np.asarray([1e-3, 1e-3, 1e-3], np.float32)]
    p0 = np.asarray([-0.4, 0.01, 0.2], np.float32)
    got = run_lamb(gs, p0, **hp)
    want = lamb_brute_force(gs, p0, **hp)
    for (gp, gt), (wp, wt) in zip(got, want):
        assert gt == pytest.approx(wt, rel=1e-12)
        assert np.allclose(gp, wp, rtol=1e-11, atol=0)


def test_lamb_first_step_closed_form_without_eps_and_decay():
    # From m = v = 0 the corrected moments are g and g^2, so the direction is sign(g):
    # ||u|| = sqrt(n), trust = ||p|| / sqrt(n), p_i <- p_i - lr ||p|| sign(g_i) / sqrt(n).
    p0 = np.asarray([3.0, -4.0, 0.0, 12.0], np.float64)           # ||p|| = 13
    g = np.asarray([1e-3, -2e-2, 5e-5, -7.0], np.float32)
    (p1, trust), = run_lamb([g], p0, lr=0.01, eps=0.0, weight_decay=0.0)
    assert trust == pytest.approx(13.0 / 2.0, rel=1e-14)
    assert np.allclose(p1, p0 - 0.01 * 6.5 * np.sign(g), rtol=1e-13)


def test_lamb_update_length_is_lr_times_parameter_norm_for_every_tensor_and_step():
    numels = W.scaled_bert_numels(16, 2, 32, vocab=50, max_pos=8)
    p = [x.astype(np.float64) for x in W.normal_tensors(numels, 1, "p", 0.02)]
    m = [np.zeros(n) for n in numels]
    v = [np.zeros(n) for n in numels]
    for step in range(1, 6):
        g = W.normal_tensors(numels, 10 + step, "g", 1e-3)
        before = [x.copy() for x in p]
        trust = oracle.lamb_step(np.asarray(numels, np.uint64), g, p, m, v, step=step, **HP)
        for t in range(len(numels)):
            delta = np.linalg.norm(p[t] - before[t])
            assert delta == pytest.approx(HP["lr"] * np.linalg.norm(before[t]), rel=1e-12)
            assert trust[t] > 0


def test_lamb_zero_norm_cases_fall_back_to_ratio_one():
    # p = 0: the ratio has no meaning, it is taken as 1 and the step is Adam's
    n = 5
    g = np.asarray([1e-3, -2e-3, 3e-3, 0.0, 1e-4], np.float32)
    pl, ml, vl = [np.zeros(n)], [np.zeros(n)], [np.zeros(n)]
    pa, ma, va = [np.zeros(n)], [np.zeros(n)], [np.zeros(n)]
    numel = np.asarray([n], np.uint64)
    tr = oracle.lamb_step(numel, [g], pl, ml, vl, step=1, **HP)
    oracle.adam_step(numel, [g], pa, ma, va, step=1, **HP)
    assert tr[0] == 1.0
    assert np.array_equal(pl[0], pa[0]) and np.array_equal(ml[0], ma[0]) and np.array_equal(vl[0], va[0])
    # update = 0 (no gradient history, no decay): p stays, ratio 1, nothing is NaN
    p = [np.asarray([1.0, 2.0])]
    tr = oracle.lamb_step(np.asarray([2], np.uint64), [np.zeros(2, np.float32)], p, [np.zeros(2)], [np.zeros(2)],
                          step=1, **dict(HP, weight_decay=0.0))
    assert tr[0] == 1.0 and np.array_equal(p[0], [1.0, 2.0])


def test_lamb_moments_are_adams_moments():
    numels = [300, 17]
    g = W.normal_tensors(numels, 3, "g", 1e-3)
    mk = lambda: ([x.astype(np.float64) for x in W.normal_tensors(numels, 3, "p", 0.02)],
                  [x.astype(np.float64) for x in W.normal_tensors(numels, 3, "m", 3e-4)],
                  [x.astype(np.float64) for x in W.warm_second_moment(numels, 3)])
    pl, ml, vl = mk()
    pa, ma, va = mk()
    oracle.lamb_step(np.asarray(numels, np.uint64), g, pl, ml, vl, step=9, **HP)
    oracle.adam_step(np.asarray(numels, np.uint64), g, pa, ma, va, step=9, **HP)
    for a, b in zip(ml + vl, ma + va):
        assert np.array_equal(a, b)
    assert not np.array_equal(pl[0], pa[0])


def test_lamb_trust_ratio_counts_the_decay_term_and_uses_the_parameters_before_the_update():
    # definition written out with numpy in fp64 for one warm tensor
    n = 400
    g = W.normal_tensors([n], 4, "g", 1e-3)[0]
    p0 = W.normal_tensors([n], 4, "p", 0.02)[0].astype(np.float64)
    m0 = W.normal_tensors([n], 4, "m", 3e-4)[0].astype(np.float64)
    v0 = W.warm_second_moment([n], 4)[0].astype(np.float64)
    h = dict(HP, weight_decay=0.3)
    p, m, v = [p0.copy()], [m0.copy()], [v0.copy()]
    step = 50
    tr = oracle.lamb_step(np.asarray([n], np.uint64), [g], p, m, v, step=step, **h)
    gd = g.astype(np.float64)
    m1 = h["beta1"] * m0 + (1 - h["beta1"]) * gd
    v1 = h["beta2"] * v0 + (1 - h["beta2"]) * gd * gd
    u = (m1 / (1 - h["beta1"] ** step)) / (np.sqrt(v1 / (1 - h["beta2"] ** step)) + h["eps"]) + h["weight_decay"] * p0
    want_tr = np.linalg.norm(p0) / np.linalg.norm(u)
    assert tr[0] == pytest.approx(want_tr, rel=1e-13)
    assert np.allclose(p[0], p0 - h["lr"] * want_tr * u, rtol=1e-13, atol=0)
    # leaving the decay term out of the norm, or taking ||p|| after the update, gives another number
    r_only = u - h["weight_decay"] * p0
    assert abs(np.linalg.norm(p0) / np.linalg.norm(r_only) - want_tr) > 1e-3 * want_tr
    assert abs(np.linalg.norm(p[0]) / np.linalg.norm(u) - want_tr) > 1e-6 * want_tr


def test_lamb_tensors_are_independent_and_scale_with_their_parameters():
    numels = [64, 64]
    g = W.normal_tensors(numels, 5, "g", 1e-3)
    p32 = W.normal_tensors(numels, 5, "p", 0.02)
    h = dict(HP, weight_decay=0.0)

    def run(gs, scale1=1.0):
        p = [p32[0].astype(np.float64), p32[1].astype(np.float64) * scale1]
        m, v = [np.zeros(64), np.zeros(64)], [np.zeros(64), np.zeros(64)]
        tr = oracle.lamb_step(np.asarray(numels, np.uint64), gs, p, m, v, step=1, **h)
        return p, tr
    base, tr0 = run(g)
    other, tr1 = run([g[0], g[1] * np.float32(8)])
    assert np.array_equal(base[0], other[0]) and tr0[0] == tr1[0]           # tensor 0 does not see tensor 1
    scaled, tr2 = run(g, scale1=4.0)
    assert tr2[1] == pytest.approx(4 * tr0[1], rel=1e-13)                    # ratio grows with ||p||
    d0 = base[1] - p32[1].astype(np.float64)
    d2 = scaled[1] - 4.0 * p32[1].astype(np.float64)
    assert np.allclose(d2, 4 * d0, rtol=1e-12, atol=0)


# ------------------------------------------------------------------ clipping + LAMB


def small():
    numels = W.scaled_bert_numels(32, 2, 64, vocab=200, max_pos=16)
    lay = W.layout_flat_split(numels, 1500)
    g = W.normal_tensors(numels, 6, "g", 1e-3)
    p = [x.astype(np.float64) for x in W.normal_tensors(numels, 6, "p", 0.02)]
    m = [x.astype(np.float64) for x in W.normal_tensors(numels, 6, "m", 3e-4)]
    v = [x.astype(np.float64) for x in W.warm_second_moment(numels, 6)]
    return lay, numels, g, p, m, v


def test_clip_then_lamb_is_lamb_on_the_bucketwise_scaled_gradient():
    lay, numels, g, p, m, v = small()
    norms = oracle.bucket_norms(lay, g)
    thr = (norms * np.where(np.arange(lay.n_buckets) % 2 == 0, 0.5, 2.0)).astype(np.float32)
    p2, m2, v2 = [x.copy() for x in p], [x.copy() for x in m], [x.copy() for x in v]
    g_in = [x.copy() for x in g]
    n1, c1, tr1, st = oracle.bucket_clip_lamb(lay, g_in, p, m, v, thr, step=20, **HP)
    assert st == 0 and np.array_equal(n1, norms)
    assert all(np.array_equal(a, b) for a, b in zip(g_in, g))      # without write-back the gradients are only read
    coefs, _ = oracle.clip_coefs(norms, thr)
    assert np.array_equal(c1, coefs) and (coefs < 1).any() and (coefs == 1).any()
    assert lay.tensors_split() > 0                                 # some tensor sees two different coefficients
    # scaled gradient in fp64, element by element, then plain LAMB written with numpy
    for t in range(len(numels)):
        ghat = np.zeros(numels[t])
        for b in range(lay.n_buckets):
            for tt, beg, ln in lay.segments_of(b):
                if tt == t:
                    ghat[beg:beg + ln] = np.float64(coefs[b]) * g[t][beg:beg + ln].astype(np.float64)
        mm = HP["beta1"] * m2[t] + (1 - HP["beta1"]) * ghat
        vv = HP["beta2"] * v2[t] + (1 - HP["beta2"]) * ghat * ghat
        u = (mm / (1 - HP["beta1"] ** 20)) / (np.sqrt(vv / (1 - HP["beta2"] ** 20)) + HP["eps"]) + HP["weight_decay"] * p2[t]
        trust = np.linalg.norm(p2[t]) / np.linalg.norm(u)
        assert tr1[t] == pytest.approx(trust, rel=1e-12)
        assert np.allclose(p[t], p2[t] - HP["lr"] * trust * u, rtol=1e-12, atol=1e-300)
        assert np.allclose(m[t], mm, rtol=1e-14) and np.allclose(v[t], vv, rtol=1e-14)


def test_clip_then_lamb_without_clipping_is_lamb_step_and_write_back_stores_scaled_gradient():
    lay, numels, g, p, m, v = small()
    pa, ma, va = [x.copy() for x in p], [x.copy() for x in m], [x.copy() for x in v]
    inf = np.full(lay.n_buckets, np.inf, np.float32)
    ga = [x.copy() for x in g]
    _, c, tra, _ = oracle.bucket_clip_lamb(lay, ga, pa, ma, va, inf, step=3, write_back=True, **HP)
    trb = oracle.lamb_step(lay, g, p, m, v, step=3, **HP)
    assert np.all(c == 1) and np.array_equal(tra, trb)
    assert all(np.array_equal(a, b) for a, b in zip(pa + ma + va + ga, p + m + v + g))
    # with clipping and write-back the stored gradient is what bucket_scale stores
    lay, numels, g, p, m, v = small()
    thr = np.full(lay.n_buckets, 0.01, np.float32)
    gw = [x.copy() for x in g]
    _, coefs, _, _ = oracle.bucket_clip_lamb(lay, gw, p, m, v, thr, step=3, write_back=True, **HP)
    gs = [x.copy() for x in g]
    oracle.bucket_scale(lay, gs, coefs)
    assert (coefs < 1).all() and all(np.array_equal(a, b) for a, b in zip(gw, gs))


# ------------------------------------------------------------------ per-tensor weight-decay mask


def test_decay_mask_matches_torch_adamw_with_two_parameter_groups():
    torch = pytest.importorskip("torch")
    numels = [50, 7, 120, 7]
    mask = np.asarray([1, 0, 1, 0], np.uint8)
    p32 = W.normal_tensors(numels, 8, "p", 0.02)
    steps = 3
    gs = [W.normal_tensors(numels, 80 + k, "g", 1e-2) for k in range(steps)]
    p = [x.astype(np.float64) for x in p32]
    m = [np.zeros(n) for n in numels]
    v = [np.zeros(n) for n in numels]
    h = dict(HP, weight_decay=0.2)
    for k in range(steps):
        oracle.adam_step(np.asarray(numels, np.uint64), gs[k], p, m, v, step=k + 1, decay=mask, **h)
    tp = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in p32]
    opt = torch.optim.AdamW([{"params": [tp[0], tp[2]], "weight_decay": 0.2}, {"params": [tp[1], tp[3]], "weight_decay": 0.0}],
                            lr=h["lr"], betas=(h["beta1"], h["beta2"]), eps=h["eps"])
    for k in range(steps):
        for t, x in zip(tp, gs[k]):
            t.grad = torch.tensor(x, dtype=torch.float64)
        opt.step()
    for t in range(4):
        assert np.allclose(p[t], tp[t].detach().numpy(), rtol=1e-12, atol=1e-15)


def test_decay_mask_none_means_all_and_every_entry_point_honours_it():
    lay, numels, g, p, m, v = small()
    nt = len(numels)
    mask = (np.arange(nt) % 3 != 0).astype(np.uint8)
    h0 = dict(HP, weight_decay=0.0)
    h1 = dict(HP, weight_decay=0.25)
    thr = np.full(lay.n_buckets, 0.01, np.float32)

    def cp():
        return [x.copy() for x in p], [x.copy() for x in m], [x.copy() for x in v]

    def runs(fn):
        """fn(state, hyper, decay) -> updated p list"""
        full, none, masked, all_ones = (fn(cp(), h1, None), fn(cp(), h0, None), fn(cp(), h1, mask),
                                        fn(cp(), h1, np.ones(nt, np.uint8)))
        for t in range(nt):
            assert np.array_equal(all_ones[t], full[t])
            assert np.array_equal(masked[t], full[t] if mask[t] else none[t])
        assert any(not np.array_equal(full[t], none[t]) for t in range(nt))

    runs(lambda s, h, d: (oracle.adam_step(lay, g, *s, step=4, decay=d, **h), s[0])[1])
    runs(lambda s, h, d: (oracle.bucket_clip_adam(lay, [x.copy() for x in g], *s, thr, step=4, decay=d, **h), s[0])[1])
    runs(lambda s, h, d: (oracle.whole_clip_adam(lay, [x.copy() for x in g], *s, 0.05, step=4, decay=d, **h), s[0])[1])
    runs(lambda s, h, d: (oracle.lamb_step(lay, g, *s, step=4, decay=d, **h), s[0])[1])
    runs(lambda s, h, d: (oracle.bucket_clip_lamb(lay, [x.copy() for x in g], *s, thr, step=4, decay=d, **h), s[0])[1])
