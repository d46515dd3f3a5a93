"""Pins for the oracle's whole-gradient clipping (the paper's two baselines, Sec. 3.2,
which coincide on one GPU): clipping-by-norm (Sec. 2.3) applied once to the whole
gradient with one threshold, then Adam."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as W

HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-6, weight_decay=0.01)


def make(seed=0, sigma=1e-2):
    numels = W.scaled_bert_numels(32, 2, 64, vocab=200, max_pos=16)
    lay = W.layout_flat_split(numels, 1500)
    g = W.normal_tensors(numels, seed, "g", sigma)
    p = [x.astype(np.float64) for x in W.normal_tensors(numels, seed, "p", 0.02)]
    m = [x.astype(np.float64) for x in W.normal_tensors(numels, seed, "m", 3e-4)]
    v = [x.astype(np.float64) for x in W.warm_second_moment(numels, seed)]
    return lay, numels, g, p, m, v


def test_whole_norm_is_the_exact_root_of_the_sum_over_all_elements_and_of_bucket_squares():
    lay, numels, g, p, m, v = make()
    norms, whole, coef, st = oracle.whole_clip_adam(lay, g, p, m, v, 1e9, step=1, **HP)
    exact = math.sqrt(sum(Fraction(float(x)) ** 2 for t in g for x in t[:400])
                      + sum(Fraction(float(x)) ** 2 for t in g for x in t[400:]))
    assert whole == pytest.approx(exact, rel=1e-13)
    assert np.array_equal(norms, oracle.bucket_norms(lay, g))
    assert whole == pytest.approx(math.sqrt(float(np.sum(norms ** 2))), rel=1e-13)
    assert coef == 1.0 and st == 0


def test_one_coefficient_for_all_buckets_and_post_clip_norm_equals_threshold():
    lay, numels, g, p, m, v = make()
    g0 = [x.copy() for x in g]
    c = 0.05
    norms, whole, coef, st = oracle.whole_clip_adam(lay, g, p, m, v, c, step=3, write_back=True, **HP)
    assert whole > c and coef == np.float32(np.float32(c) / whole)
    for a, b in zip(g, g0):
        assert np.array_equal(a, b * np.float32(coef))           # every element scaled by the same fp32 factor
    after = oracle.bucket_norms(lay, g)
    assert math.sqrt(float(np.sum(after ** 2))) == pytest.approx(c, rel=1e-6)
    # below the threshold nothing changes, bit for bit
    g1 = [x.copy() for x in g0]
    _, whole1, coef1, _ = oracle.whole_clip_adam(lay, g1, p, m, v, whole * 1.01, step=4, write_back=True, **HP)
    assert coef1 == 1.0 and all(np.array_equal(a, b) for a, b in zip(g1, g0))


def test_whole_clip_equals_bucket_wise_clip_when_everything_is_one_bucket():
    lay, numels, g, p, m, v = make(seed=2)
    one = W.layout_flat_split(numels, 10 ** 9)
    assert one.n_buckets == 1
    pa, ma, va = [x.copy() for x in p], [x.copy() for x in m], [x.copy() for x in v]
    _, whole, coef, _ = oracle.whole_clip_adam(lay, [x.copy() for x in g], p, m, v, 0.03, step=7, **HP)
    n1, c1, _ = oracle.bucket_clip_adam(one, [x.copy() for x in g], pa, ma, va, np.asarray([0.03], np.float32), step=7, **HP)
    assert n1[0] == pytest.approx(whole, rel=1e-13) and c1[0] == pytest.approx(coef, rel=2e-7)
    for a, b in zip(p + m + v, pa + ma + va):
        assert np.allclose(a, b, rtol=1e-6, atol=1e-12)


def test_whole_clip_differs_from_bucket_wise_clip_with_alg1_thresholds():
    # Bucket-wise clipping with c/sqrt(B) bounds the whole norm by c but is not the same map:
    # a bucket with a small norm is left alone where whole-gradient clipping would shrink it too.
    lay, numels, g, p, m, v = make(seed=3)
    W.scale_buckets_inplace(lay, g, [0], 1e-3)
    B = lay.n_buckets
    thr = np.full(B, oracle.alg1_threshold(0.05, B), np.float32)
    _, coefs, _ = oracle.bucket_clip_adam(lay, [x.copy() for x in g], [x.copy() for x in p], [x.copy() for x in m],
                                          [x.copy() for x in v], thr, step=1, **HP)
    _, whole, coef, _ = oracle.whole_clip_adam(lay, [x.copy() for x in g], p, m, v, 0.05, step=1, **HP)
    assert coefs[0] == 1.0 and coef < 1.0 and (coefs[1:] < 1).all()


def test_matches_torch_clip_grad_norm_then_adamw_fp64():
    torch = pytest.importorskip("torch")
    lay, numels, g, p, m, v = make(seed=4)
    p0 = [x.copy() for x in p]
    m = [np.zeros_like(x) for x in m]
    v = [np.zeros_like(x) for x in v]
    c = 0.1
    tp = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in p0]
    opt = torch.optim.AdamW(tp, lr=HP["lr"], betas=(HP["beta1"], HP["beta2"]), eps=HP["eps"],
                            weight_decay=HP["weight_decay"])
    for k in range(3):
        gk = W.normal_tensors(numels, 40 + k, "g", 1e-2)
        _, whole, coef, _ = oracle.whole_clip_adam(lay, gk, p, m, v, c, step=k + 1, **HP)
        for t, x in zip(tp, gk):
            t.grad = torch.tensor(x, dtype=torch.float64)
        tn = torch.nn.utils.clip_grad_norm_(tp, c)            # library: coef = c / (norm + 1e-6), clamped to 1
        assert float(tn) == pytest.approx(whole, rel=1e-12)
        opt.step()
    for a, t in zip(p, tp):
        # the library's 1e-6 fudge term in the coefficient moves the update by ~1e-5 relative
        assert np.allclose(a, t.detach().numpy(), rtol=0, atol=2e-8)
