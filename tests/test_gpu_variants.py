"""GPU parity of the optimizer variants: bfloat16 gradient storage, the per-tensor
weight-decay mask, and LAMB (alone and behind bucket-wise clipping), each against
the CPU oracle on the same seeded inputs.  Tolerances as for Adam: norms and trust
ratios rel <= 1e-5; p, m, v rel <= 1e-5, or abs <= 1e-7 where |oracle| < 1e-2."""
import numpy as np
import pytest
import torch

import oracle
import paper_2402_02447_amd as B
import workloads as W
from gpu_util import Device, bits_equal, check_norms, check_state, f64, hp_kwargs, hyper, to_host
from test_gpu_parity import (adversarial_cases, check_scaled_grads, random_layout, run_fused, run_unfused, run_whole,
                             small_bert, state_of)

pytestmark = pytest.mark.gpu


def warm_state(numels, seed):
    return (W.normal_tensors(numels, seed, "p", 0.02, threads=1), W.normal_tensors(numels, seed, "m", 3e-3, threads=1),
            W.warm_second_moment(numels, seed, threads=1))


def alternating_thresholds(lay, g):
    norms = oracle.bucket_norms(lay, g)
    return np.asarray([max(norms[b], 1e-3) * (0.1, 10.0, 0.9)[b % 3] for b in range(lay.n_buckets)], np.float32)


# ------------------------------------------------------------------ bfloat16 gradients


@pytest.mark.parametrize("name", list(adversarial_cases()))
def test_bf16_gradients_adversarial_layouts_fused_and_unfused(name):
    lay, offsets = adversarial_cases()[name]
    numels = [int(n) for n in lay.tensor_numel]
    g = oracle.Bf16(W.normal_bf16_tensors(numels, 7, 1e-2, threads=1))
    p, m, v = warm_state(numels, 7)
    thr = alternating_thresholds(lay, g)
    hp = W.Hyper()
    for flags in (0, B.BCA_WRITE_BACK_GRADS):
        run_fused(lay, g, p, m, v, thr, hp, 3, flags, offsets=offsets)
    run_unfused(lay, g, p, m, v, thr, hp, 3, offsets=offsets)
    run_fused(lay, g, p, m, v, thr, hp, 3, B.BCA_WRITE_BACK_GRADS, offsets=offsets, chunk_norm=2048, chunk_apply=2048,
              group_bytes=20_000, tune_flags=B.BCA_TUNE_MULTI_LAUNCH)


def test_bf16_gradients_small_bert_all_modes():
    w = small_bert("large")
    numels = [int(n) for n in w.layout.tensor_numel]
    g = oracle.Bf16(W.normal_bf16_tensors(numels, 3, 1e-3))
    p, m, v = state_of(w)
    norms = oracle.bucket_norms(w.layout, g)
    thr = (np.median(norms) * np.ones_like(norms)).astype(np.float32)
    r = run_fused(w.layout, g, p, m, v, thr, w.hyper, w.first_step)
    assert r["norm_rel"] < 1e-6
    run_fused(w.layout, g, p, m, v, thr, w.hyper, w.first_step, B.BCA_WRITE_BACK_GRADS)
    run_unfused(w.layout, g, p, m, v, thr, w.hyper, w.first_step)
    whole = float(np.sqrt(np.sum(norms ** 2)))
    run_whole(w.layout, g, p, m, v, 0.3 * whole, w.hyper, w.first_step, B.BCA_WRITE_BACK_GRADS)


def test_bf16_nan_and_inf_gradients_are_flagged():
    lay = W.layout_one_tensor_per_bucket([300, 300])
    bits = W.normal_bf16_tensors([300, 300], 1, 1e-2, threads=1)
    bits[0][17] = 0x7F80                                     # +inf
    bits[1][5] = 0x7FC1                                      # NaN
    z = [np.zeros(300, np.float32), np.zeros(300, np.float32)]
    dev = Device(lay, oracle.Bf16(bits), z, z, z)
    dev.plan.bucket_clip_norms(0, 2, dev.norms)
    dev.plan.bucket_clip_apply(0, 2, dev.thresholds(np.ones(2, np.float32)), dev.norms, dev.coefs, dev.status)
    dev.sync()
    n = dev.norms.cpu().numpy()
    assert np.isinf(n[0]) and np.isnan(n[1])
    assert int(dev.status.item()) & B.BCA_STATUS_NONFINITE
    dev.close()


# ------------------------------------------------------------------ weight-decay mask


def test_decay_mask_small_bert_fused_unfused_whole():
    w = small_bert("base")
    lay = w.layout
    mask = W.bert_decay_mask(2000, 64, 3, 256, 64)
    assert mask.shape[0] == lay.n_tensors and 0 < mask.sum() < lay.n_tensors
    g = w.grads()
    p, m, v = state_of(w)
    norms = oracle.bucket_norms(lay, g)
    thr = (np.median(norms) * np.ones_like(norms)).astype(np.float32)
    hp = W.Hyper(weight_decay=0.3)            # strong decay: a wrong mask moves p far outside the tolerance
    run_fused(lay, g, p, m, v, thr, hp, 9, decay=mask)
    run_fused(lay, g, p, m, v, thr, hp, 9, B.BCA_SKIP_STEP_ON_NONFINITE, decay=mask)
    run_fused(lay, g, p, m, v, thr, hp, 9, decay=mask, tune_flags=B.BCA_TUNE_MULTI_LAUNCH, group_bytes=300_000)
    run_unfused(lay, g, p, m, v, thr, hp, 9, decay=mask)


def test_decay_mask_can_change_on_a_bound_plan_and_none_restores_the_default():
    lay = W.layout_flat_split([3000, 50, 2000, 50], 1800)
    numels = [3000, 50, 2000, 50]
    g = W.normal_tensors(numels, 2, "g", 1e-2, threads=1)
    p, m, v = warm_state(numels, 2)
    hp = W.Hyper(weight_decay=0.5)
    dev = Device(lay, g, p, m, v)
    op, om, ov = f64(p), f64(m), f64(v)
    for step, mask in enumerate([None, [1, 0, 1, 0], [0, 1, 1, 1], None], start=1):
        dev.plan.set_decay_mask(mask)
        dev.plan.adam_step(hyper(hp), step)
        dev.sync()
        oracle.adam_step(lay, g, op, om, ov, step=step, decay=mask, **hp_kwargs(hp))
        check_state(f"p@{step}", to_host(dev.p), op)
    check_state("m", to_host(dev.m), om)
    check_state("v", to_host(dev.v), ov, strict_rel=True)
    dev.close()


# ------------------------------------------------------------------ LAMB


def check_trust(got: np.ndarray, want: np.ndarray):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    rel = np.abs(got - want) / want
    assert rel.size == 0 or rel.max() <= 1e-5, f"trust ratio rel err {rel.max():.3e} at tensor {int(np.argmax(rel))}"


def run_lamb(layout, g, p, m, v, thr, hp, step, flags=0, offsets=None, decay=None, **tuning):
    """bucket_clip_lamb (thr given) or lamb_step (thr None) against the oracle."""
    dev = Device(layout, g, p, m, v, offsets, **tuning)
    if decay is not None:
        dev.plan.set_decay_mask(decay)
    nt = layout.n_tensors
    og = type(g)(x.copy() for x in g)
    op, om, ov = f64(p), f64(m), f64(v)
    if thr is None:
        dev.plan.lamb_step(hyper(hp), step, dev.trust)
        dev.sync()
        otrust = oracle.lamb_step(layout, og, op, om, ov, step=step, decay=decay, **hp_kwargs(hp))
    else:
        dev.plan.bucket_clip_lamb(dev.thresholds(thr), hyper(hp), step, flags, dev.norms, dev.coefs, dev.trust,
                                  dev.status)
        dev.sync()
        onorm, ocoef, otrust, ost = oracle.bucket_clip_lamb(layout, og, op, om, ov, thr, step=step,
                                                            write_back=bool(flags & B.BCA_WRITE_BACK_GRADS),
                                                            decay=decay, **hp_kwargs(hp))
        check_norms(dev.norms.cpu().numpy(), onorm)
        assert np.allclose(dev.coefs.cpu().numpy(), ocoef, rtol=1e-6, atol=0)
        assert int(dev.status.item()) == ost
    check_trust(dev.trust.cpu().numpy()[:nt], otrust)
    out = {"p": check_state("p", to_host(dev.p), op), "m": check_state("m", to_host(dev.m), om),
           "v": check_state("v", to_host(dev.v), ov, strict_rel=True)}
    gg = to_host(dev.g)
    if thr is not None and flags & B.BCA_WRITE_BACK_GRADS:
        check_scaled_grads(gg, og, g, layout, dev.coefs.cpu().numpy())
    else:
        assert bits_equal(gg, g), "gradients must not be written without BCA_WRITE_BACK_GRADS"
    dev.close()
    return out


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("name", list(adversarial_cases()))
def test_lamb_adversarial_layouts(name, dtype):
    lay, offsets = adversarial_cases()[name]
    numels = [int(n) for n in lay.tensor_numel]
    if dtype == "f32":
        g = W.normal_tensors(numels, 7, "g", 1e-2, threads=1)
    elif dtype == "f16":
        g = W.student_t_fp16_tensors(numels, 7, 1e-3, threads=1)
    else:
        g = oracle.Bf16(W.normal_bf16_tensors(numels, 7, 1e-2, threads=1))
    p, m, v = warm_state(numels, 7)
    thr = alternating_thresholds(lay, g)
    hp = W.Hyper()
    run_lamb(lay, g, p, m, v, None, hp, 3, offsets=offsets)
    run_lamb(lay, g, p, m, v, thr, hp, 3, offsets=offsets)
    run_lamb(lay, g, p, m, v, thr, hp, 3, B.BCA_WRITE_BACK_GRADS, offsets=offsets, chunk_norm=2048, chunk_apply=2048)


@pytest.mark.parametrize("kind", ["base", "large", "fp16"])
def test_lamb_small_bert(kind):
    w = small_bert(kind)
    p, m, v = state_of(w)
    g = w.grads()
    thr = w.thresholds
    if kind != "fp16":
        norms = oracle.bucket_norms(w.layout, g)
        thr = (np.median(norms) * np.ones_like(norms)).astype(np.float32)
    mask = W.bert_decay_mask(2000, 64, 3, 256, 64)
    run_lamb(w.layout, g, p, m, v, None, w.hyper, w.first_step)
    run_lamb(w.layout, g, p, m, v, thr, w.hyper, w.first_step)
    run_lamb(w.layout, g, p, m, v, thr, W.Hyper(weight_decay=0.3), w.first_step, B.BCA_WRITE_BACK_GRADS, decay=mask)


def test_lamb_zero_parameters_and_zero_updates_give_ratio_one():
    numels = [2000, 300, 64]
    lay = W.layout_flat_split(numels, 1000)
    g = W.normal_tensors(numels, 4, "g", 1e-2, threads=1)
    g[2][:] = 0                                               # tensor 2: no gradient, no history, no decay -> update 0
    p = W.normal_tensors(numels, 4, "p", 0.02, threads=1)
    p[1][:] = 0                                               # tensor 1: ||p|| = 0
    z = [np.zeros(n, np.float32) for n in numels]
    dev = Device(lay, g, p, z, z)
    hp = W.Hyper(weight_decay=0.0)
    dev.plan.lamb_step(hyper(hp), 1, dev.trust)
    dev.sync()
    tr = dev.trust.cpu().numpy()[:3]
    assert tr[1] == 1.0 and tr[2] == 1.0 and tr[0] != 1.0
    op, om, ov = f64(p), f64(z), f64(z)
    otr = oracle.lamb_step(lay, g, op, om, ov, step=1, **hp_kwargs(hp))
    check_trust(tr, otr)
    check_state("p", to_host(dev.p), op)
    assert np.array_equal(to_host(dev.p)[2], p[2])
    dev.close()


def test_lamb_20_steps_error_accumulation():
    w = small_bert("multistep")
    lay = w.layout
    p, m, v = state_of(w)
    norms0 = oracle.bucket_norms(lay, w.grads(0))
    thr = (norms0 * (w.thresholds / 1.024)).astype(np.float32)
    dev = Device(lay, w.grads(0), p, m, v)
    dthr = dev.thresholds(thr)
    op, om, ov = f64(p), f64(m), f64(v)
    for k in range(w.n_steps):
        g = w.grads(k)
        dev.set_grads(g)
        step = w.first_step + k
        dev.plan.bucket_clip_lamb(dthr, hyper(w.hyper), step, 0, dev.norms, dev.coefs, dev.trust, dev.status)
        dev.sync()
        onorm, ocoef, otrust, _ = oracle.bucket_clip_lamb(lay, g, op, om, ov, thr, step=step, **hp_kwargs(w.hyper))
        check_norms(dev.norms.cpu().numpy(), onorm)
        check_trust(dev.trust.cpu().numpy()[:lay.n_tensors], otrust)
        check_state(f"p@{step}", to_host(dev.p), op)
        check_state(f"m@{step}", to_host(dev.m), om)
        check_state(f"v@{step}", to_host(dev.v), ov, strict_rel=True)
    dev.close()


def test_lamb_is_reproducible_and_the_update_has_length_lr_times_parameter_norm():
    w = small_bert("large")
    g = w.grads()
    p, m, v = state_of(w)
    norms = oracle.bucket_norms(w.layout, g)
    thr = (np.median(norms) * np.ones_like(norms)).astype(np.float32)
    outs = []
    for _ in range(2):
        dev = Device(w.layout, g, p, m, v)
        dev.plan.bucket_clip_lamb(dev.thresholds(thr), hyper(w.hyper), 5, 0, dev.norms, dev.coefs, dev.trust, dev.status)
        dev.sync()
        outs.append((dev.trust.cpu().numpy(), to_host(dev.p), to_host(dev.m), to_host(dev.v)))
        dev.close()
    assert np.array_equal(outs[0][0], outs[1][0])
    assert all(bits_equal(outs[0][i], outs[1][i]) for i in (1, 2, 3))
    for t, (new, old) in enumerate(zip(outs[0][1], p)):
        if old.size >= 64:      # fp32 rounding of p swamps the identity on tiny tensors
            d = np.linalg.norm(new.astype(np.float64) - old.astype(np.float64))
            assert d == pytest.approx(w.hyper.lr * np.linalg.norm(old.astype(np.float64)), rel=2e-3), t


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_lamb_step_in_runs_of_tensors_equals_one_run_bit_for_bit(dtype):
    """lamb_step sweeps a large model run by run (both sweeps of a run of tensors before the next run, the moments stored
    with cacheable stores in between).  Whatever the runs, trust ratios, p, m, v are the bits of a single run over
    everything, over two steps; and they match the oracle."""
    w = small_bert("large")
    lay, hp = w.layout, w.hyper
    numels = [int(n) for n in lay.tensor_numel]
    if dtype == "f32":
        g = w.grads()
    elif dtype == "f16":
        g = W.student_t_fp16_tensors(numels, 9, 1e-3, threads=1)
    else:
        g = oracle.Bf16(W.normal_bf16_tensors(numels, 9, 1e-2, threads=1))
    p, m, v = state_of(w)
    outs = []
    for limit in (2 ** 62, 1, 20_000, 100_000):
        dev = Device(lay, g, p, m, v, lamb_group_elems=limit)
        n_runs = len(dev.plan.lamb_runs())
        assert (n_runs == 1) == (limit == 2 ** 62) and (limit != 1 or n_runs == lay.n_tensors)
        for step in (3, 4):
            dev.plan.lamb_step(hyper(hp), step, dev.trust)
        dev.sync()
        outs.append((dev.trust.cpu().numpy().copy(), to_host(dev.p), to_host(dev.m), to_host(dev.v)))
        assert bits_equal(to_host(dev.g), g)
        dev.close()
    for o in outs[1:]:
        assert np.array_equal(o[0], outs[0][0])
        assert all(bits_equal(o[i], outs[0][i]) for i in (1, 2, 3))
    op, om, ov = f64(p), f64(m), f64(v)
    for step in (3, 4):
        otrust = oracle.lamb_step(lay, g, op, om, ov, step=step, **hp_kwargs(hp))
    check_trust(outs[1][0][:lay.n_tensors], otrust)
    check_state("p", outs[1][1], op), check_state("m", outs[1][2], om), check_state("v", outs[1][3], ov, strict_rel=True)


@pytest.mark.parametrize("seed", range(6))
def test_lamb_random_layouts(seed):
    rng = np.random.default_rng(2000 + seed)
    lay, numels = random_layout(rng)
    kind = seed % 3
    offsets = [int(rng.integers(0, 4)) for _ in numels] if seed % 2 == 0 else None
    if kind == 0:
        g = W.normal_tensors(numels, seed, "g", 1e-2, threads=1)
    elif kind == 1:
        g = W.student_t_fp16_tensors(numels, seed, 1e-3, threads=1)
    else:
        g = oracle.Bf16(W.normal_bf16_tensors(numels, seed, 1e-2, threads=1))
    p, m, v = warm_state(numels, seed)
    norms = oracle.bucket_norms(lay, g)
    thr = np.asarray([max(norms[b], 1e-3) * float(rng.choice([0.05, 0.5, 0.999, 1.5, 50.0]))
                      for b in range(lay.n_buckets)], np.float32)
    hp = W.Hyper(lr=float(rng.choice([1e-3, 1e-2])), beta1=float(rng.choice([0.7, 0.9])),
                 beta2=float(rng.choice([0.85, 0.999])), eps=float(rng.choice([1e-11, 1e-6])),
                 weight_decay=float(rng.choice([0.0, 0.01, 0.1])))
    step = int(rng.choice([1, 2, 77, 100000]))
    mask = rng.integers(0, 2, len(numels)).astype(np.uint8)
    run_lamb(lay, g, p, m, v, None, hp, step, offsets=offsets, decay=mask)
    run_lamb(lay, g, p, m, v, thr, hp, step, B.BCA_WRITE_BACK_GRADS, offsets=offsets, decay=mask,
             chunk_apply=int(rng.choice([1024, 2048, 4096])))
    # and Adam with the same mask and gradient type, all launch variants
    run_fused(lay, g, p, m, v, thr, hp, step, 0, offsets=offsets, decay=mask)
    run_fused(lay, g, p, m, v, thr, hp, step, B.BCA_WRITE_BACK_GRADS, offsets=offsets, decay=mask,
              tune_flags=B.BCA_TUNE_MULTI_LAUNCH, group_bytes=5000)
    run_unfused(lay, g, p, m, v, thr, hp, step, offsets=offsets, decay=mask)


def test_clip_lamb_in_a_hip_graph_replays_like_eager_calls():
    # bucket_clip_lamb is five kernel launches with no host-side state that a capture would freeze and no memset
    # nodes.  Replays are interleaved with eager work and synchronisations; each is compared with an eager twin.
    w = small_bert("multistep")
    lay = w.layout
    p, m, v = state_of(w)
    norms0 = oracle.bucket_norms(lay, w.grads(0))
    thr = (norms0 * (w.thresholds / 1.024)).astype(np.float32)
    eager = Device(lay, w.grads(0), p, m, v)
    graph = Device(lay, w.grads(0), p, m, v)
    ethr, gthr = eager.thresholds(thr), graph.thresholds(thr)
    hp = hyper(w.hyper)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        graph.plan.bucket_clip_lamb(gthr, hp, 7, 0, graph.norms, graph.coefs, graph.trust, graph.status, stream=s)   # warm-up
        eager.plan.bucket_clip_lamb(ethr, hp, 7, 0, eager.norms, eager.coefs, eager.trust, eager.status, stream=s)
        s.synchronize()
        cg = torch.cuda.CUDAGraph()
        with torch.cuda.graph(cg, stream=s):
            graph.plan.bucket_clip_lamb(gthr, hp, 7, 0, graph.norms, graph.coefs, graph.trust, graph.status,
                                        stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for k in range(1, 5):
        gk = w.grads(k)
        eager.set_grads(gk)
        graph.set_grads(gk)
        torch.cuda.synchronize()
        cg.replay()
        eager.plan.bucket_clip_lamb(ethr, hp, 7, 0, eager.norms, eager.coefs, eager.trust, eager.status)
        torch.cuda.synchronize()
        assert int(graph.status.item()) == 0 == int(eager.status.item())
        assert np.array_equal(graph.trust.cpu().numpy(), eager.trust.cpu().numpy())
        assert np.array_equal(graph.coefs.cpu().numpy(), eager.coefs.cpu().numpy())
        assert bits_equal(to_host(graph.p), to_host(eager.p))
        assert bits_equal(to_host(graph.m), to_host(eager.m))
        assert bits_equal(to_host(graph.v), to_host(eager.v))
    op, om, ov = f64(p), f64(m), f64(v)
    for k in [0, 1, 2, 3, 4]:
        oracle.bucket_clip_lamb(lay, w.grads(k), op, om, ov, thr, step=7, **hp_kwargs(w.hyper))
    check_state("p", to_host(eager.p), op)
    check_state("v", to_host(eager.v), ov, strict_rel=True)
    eager.close()
    graph.close()


def test_lamb_step_in_runs_in_a_hip_graph_replays_like_eager_calls():
    """lamb_step in runs of tensors is three launches per run and nothing else: captured once, replayed with new
    gradients and eager work in between, every replay gives the bits of an eager call on a twin."""
    w = small_bert("multistep")
    lay = w.layout
    p, m, v = state_of(w)
    eager = Device(lay, w.grads(0), p, m, v, lamb_group_elems=30_000)
    graph = Device(lay, w.grads(0), p, m, v, lamb_group_elems=30_000)
    assert len(graph.plan.lamb_runs()) >= 5
    hp = hyper(w.hyper)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        graph.plan.lamb_step(hp, 7, graph.trust, stream=s)   # warm-up
        eager.plan.lamb_step(hp, 7, eager.trust, stream=s)
        s.synchronize()
        cg = torch.cuda.CUDAGraph()
        with torch.cuda.graph(cg, stream=s):
            graph.plan.lamb_step(hp, 7, graph.trust, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for k in range(1, 5):
        gk = w.grads(k)
        eager.set_grads(gk)
        graph.set_grads(gk)
        torch.cuda.synchronize()
        cg.replay()
        eager.plan.lamb_step(hp, 7, eager.trust)
        torch.cuda.synchronize()
        assert np.array_equal(graph.trust.cpu().numpy(), eager.trust.cpu().numpy())
        for a, b in ((graph.p, eager.p), (graph.m, eager.m), (graph.v, eager.v)):
            assert bits_equal(to_host(a), to_host(b)), k
    op, om, ov = f64(p), f64(m), f64(v)
    for k in [0, 1, 2, 3, 4]:
        oracle.lamb_step(lay, w.grads(k), op, om, ov, step=7, **hp_kwargs(w.hyper))
    check_state("p", to_host(eager.p), op)
    check_state("v", to_host(eager.v), ov, strict_rel=True)
    eager.close()
    graph.close()


def test_clip_lamb_single_launch_equals_the_separate_launches_bit_for_bit():
    for kind in ("large", "fp16"):
        w = small_bert(kind)
        g = w.grads()
        p, m, v = state_of(w)
        norms = oracle.bucket_norms(w.layout, g)
        thr = (np.median(norms) * np.ones_like(norms)).astype(np.float32)
        outs = []
        for tuning in (dict(), dict(tune_flags=B.BCA_TUNE_MULTI_LAUNCH), dict(group_bytes=300_000), dict(chunk_apply=2048)):
            dev = Device(w.layout, g, p, m, v, **tuning)
            dev.plan.bucket_clip_lamb(dev.thresholds(thr), hyper(w.hyper), 5, B.BCA_WRITE_BACK_GRADS, dev.norms, dev.coefs,
                                      dev.trust, dev.status)
            dev.sync()
            assert int(dev.status.item()) == 0
            outs.append((dev.norms.cpu().numpy(), dev.coefs.cpu().numpy(), dev.trust.cpu().numpy(), to_host(dev.p),
                         to_host(dev.m), to_host(dev.v), to_host(dev.g)))
            dev.close()
        ref = outs[0]
        assert (ref[1] < 1).any()
        for other in outs[1:3]:            # same chunk cuts: everything identical
            assert all(np.array_equal(ref[i], other[i]) for i in (0, 1, 2))
            assert all(bits_equal(ref[i], other[i]) for i in (3, 4, 5, 6))
        # other chunk cuts: other partial sums, so trust ratios may differ in the last bits; moments and gradients do not
        assert np.array_equal(ref[1], outs[3][1]) and bits_equal(ref[4], outs[3][4]) and bits_equal(ref[6], outs[3][6])


# ------------------------------------------------------------------ per-kernel timing


@pytest.mark.parametrize("tuning", [dict(), dict(tune_flags=B.BCA_TUNE_MULTI_LAUNCH, group_bytes=200_000)],
                         ids=["single_launch", "multi_launch_groups"])
def test_profiling_counts_ordinary_calls_only_and_leaves_results_alone(tuning):
    """Profiled calls give the same bits as unprofiled ones; a call that needs every norm first (skip on
    non-finite, whole-gradient clipping) runs as one group and is not recorded, whatever the plan's groups."""
    w = small_bert("large")
    p, m, v = state_of(w)
    g = w.grads()
    norms = oracle.bucket_norms(w.layout, g)
    thr = (np.median(norms) * np.ones_like(norms)).astype(np.float32)

    def run(profiled):
        d = Device(w.layout, g, p, m, v, **tuning)
        if tuning:
            assert d.plan.n_groups > 1
        if profiled:
            d.plan.profile(4)
        t = d.thresholds(thr)
        for step, flags in ((1, 0), (2, B.BCA_SKIP_STEP_ON_NONFINITE), (3, 0), (4, B.BCA_CLIP_WHOLE_GRADIENT)):
            whole = torch.empty(w.layout.n_buckets + 1, dtype=torch.float32, device="cuda")
            d.plan.bucket_clip_adam(t if flags != B.BCA_CLIP_WHOLE_GRADIENT else d.thresholds(np.asarray([1e30])),
                                    hyper(w.hyper), step, flags, norms=whole, coefs=d.coefs, status=d.status)
        d.sync()
        out = None
        if profiled:
            out = d.plan.profile_read()
            assert d.plan.profile_read()[1] == 0          # reading starts a new series
            d.plan.profile(0)
        state = (to_host(d.p), to_host(d.m), to_host(d.v))
        d.close()
        return state, out

    plain, _ = run(False)
    prof, (ms, n) = run(True)
    assert n == 2
    assert all(np.isfinite(x) and x >= 0 for x in ms) and ms[2] > 0
    for a, b in zip(plain, prof):
        assert bits_equal(a, b)


# ------------------------------------------------------------------ hyper-parameters and step in device memory


def device_hyper(hp, step):
    return torch.frombuffer(bytearray(B.pack_device_hyper(hyper(hp), step)), dtype=torch.uint8).cuda()


def test_hyper_parameters_from_device_memory_in_a_replayed_graph_follow_a_schedule():
    """One captured fused step is replayed with the step count and the learning rate rewritten in device
    memory before every replay (the case a captured graph cannot serve with host arguments); the state
    after four steps matches the oracle run with the same schedule.  The host arguments are ignored."""
    w = small_bert("multistep")
    lay = w.layout
    p, m, v = state_of(w)
    norms0 = oracle.bucket_norms(lay, w.grads(0))
    thr = (norms0 * (w.thresholds / 1.024)).astype(np.float32)
    lrs = [1e-3, 2e-3, 5e-4, 1.5e-3]
    d = Device(lay, w.grads(0), p, m, v)
    dthr = d.thresholds(thr)
    import dataclasses
    hp_at = [dataclasses.replace(w.hyper, lr=lr) for lr in lrs]
    dev = device_hyper(hp_at[0], 1)
    d.plan.set_device_hyper(dev)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    scratch = Device(lay, w.grads(0), p, m, v)                       # warm-up happens on a twin, not on the state under test
    scratch.plan.set_device_hyper(dev)
    with torch.cuda.stream(s):
        scratch.plan.bucket_clip_adam(dthr, None, 0, 0, scratch.norms, scratch.coefs, scratch.status, stream=s)
        s.synchronize()
        cg = torch.cuda.CUDAGraph()
        with torch.cuda.graph(cg, stream=s):
            d.plan.bucket_clip_adam(dthr, None, 12345, 0, d.norms, d.coefs, d.status, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    op, om, ov = f64(p), f64(m), f64(v)
    for k in range(4):
        d.set_grads(w.grads(k))
        dev.copy_(device_hyper(hp_at[k], k + 1))
        torch.cuda.synchronize()
        cg.replay()
        torch.cuda.synchronize()
        assert int(d.status.item()) == 0
        oracle.bucket_clip_adam(lay, w.grads(k), op, om, ov, thr, step=k + 1, **hp_kwargs(hp_at[k]))
        check_state("p", to_host(d.p), op)
        check_state("m", to_host(d.m), om)
        check_state("v", to_host(d.v), ov, strict_rel=True)
    scratch.close()
    d.close()


def test_hyper_parameters_from_device_memory_every_entry_point_and_back_to_host_arguments():
    w = small_bert("large")
    lay = w.layout
    p, m, v = state_of(w)
    g = w.grads()
    norms = oracle.bucket_norms(lay, g)
    thr = (np.median(norms) * np.ones_like(norms)).astype(np.float32)
    import dataclasses
    hp = dataclasses.replace(w.hyper, lr=3e-3, beta1=0.8, beta2=0.99, eps=1e-7, weight_decay=0.02)
    dev = device_hyper(hp, 9)
    wrong = hyper(w.hyper)                                             # host arguments that must be ignored

    def fresh():
        d = Device(lay, g, p, m, v)
        d.plan.set_device_hyper(dev)
        return d

    d = fresh()                                                         # adam_step
    d.plan.adam_step(wrong, 77)
    d.sync()
    op, om, ov = f64(p), f64(m), f64(v)
    oracle.adam_step(lay, g, op, om, ov, step=9, **hp_kwargs(hp))
    check_state("p", to_host(d.p), op), check_state("v", to_host(d.v), ov, strict_rel=True)
    d.close()

    for flags in (0, B.BCA_CLIP_WHOLE_GRADIENT, B.BCA_SKIP_STEP_ON_NONFINITE):   # fused Adam: single launch and multi-launch routes
        d = fresh()
        nm = torch.zeros(lay.n_buckets + 1, dtype=torch.float32, device="cuda")
        whole = flags == B.BCA_CLIP_WHOLE_GRADIENT
        t = d.thresholds(np.asarray([0.5 * float(np.sqrt(np.sum(norms ** 2)))], np.float32) if whole else thr)
        d.plan.bucket_clip_adam(t, None, 0, flags, nm, d.coefs, d.status)
        d.sync()
        op, om, ov = f64(p), f64(m), f64(v)
        if flags == B.BCA_CLIP_WHOLE_GRADIENT:
            oracle.whole_clip_adam(lay, g, op, om, ov, 0.5 * float(np.sqrt(np.sum(norms ** 2))), step=9, **hp_kwargs(hp))
        else:
            oracle.bucket_clip_adam(lay, g, op, om, ov, thr, step=9, **hp_kwargs(hp))
        check_state("p", to_host(d.p), op), check_state("m", to_host(d.m), om)
        check_state("v", to_host(d.v), ov, strict_rel=True)
        d.close()

    d = fresh()                                                         # LAMB, alone and behind the clip
    d.plan.lamb_step(None, 0, d.trust)
    d.sync()
    op, om, ov = f64(p), f64(m), f64(v)
    otrust = oracle.lamb_step(lay, g, op, om, ov, step=9, **hp_kwargs(hp))
    check_norms(d.trust.cpu().numpy()[:lay.n_tensors], otrust)
    check_state("p", to_host(d.p), op)
    d.close()
    d = fresh()
    d.plan.bucket_clip_lamb(d.thresholds(thr), wrong, 3, 0, d.norms, d.coefs, d.trust, d.status)
    d.sync()
    op, om, ov = f64(p), f64(m), f64(v)
    oracle.bucket_clip_lamb(lay, g, op, om, ov, thr, step=9, **hp_kwargs(hp))
    check_state("p", to_host(d.p), op), check_state("v", to_host(d.v), ov, strict_rel=True)
    # back to host arguments
    d.plan.set_device_hyper(None)
    d.plan.adam_step(hyper(w.hyper), 10)
    d.sync()
    oracle.adam_step(lay, g, op, om, ov, step=10, **hp_kwargs(w.hyper))
    check_state("p", to_host(d.p), op)
    d.close()
