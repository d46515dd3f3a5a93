"""The randomized GPU parity tests at many more seeds than their own parametrizations run (random layouts with
empty buckets and unaligned tensors, all gradient types, launch variants, LAMB, the load-balancing simulation one
method at a time and all methods at once, bucket_clip over random bucket ranges).  Each case is a few
milliseconds; a failure names its seed."""
import numpy as np
import pytest

import oracle
import workloads as W
from gpu_util import Device, check_norms, to_host
import test_gpu_lbs as TL
import test_gpu_parity as TP
import test_gpu_variants as TV

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("block", range(4))
def test_adam_random_layouts_many_seeds(block):
    for seed in range(12 + 60 * block, 12 + 60 * (block + 1)):
        try:
            TP.test_random_layouts_all_modes(seed)
        except AssertionError as e:
            raise AssertionError(f"seed {seed}: {e}") from e


@pytest.mark.parametrize("block", range(3))
def test_lamb_random_layouts_many_seeds(block):
    for seed in range(6 + 50 * block, 6 + 50 * (block + 1)):
        try:
            TV.test_lamb_random_layouts(seed)
        except AssertionError as e:
            raise AssertionError(f"seed {seed}: {e}") from e


def test_lbs_random_settings_many_seeds():
    for seed in range(8, 200):
        try:
            TL.test_random_settings_all_methods(seed)
        except AssertionError as e:
            raise AssertionError(f"seed {seed}: {e}") from e


def test_lbs_all_methods_at_once_random_power_of_two_settings():
    for seed in range(300):
        rng = np.random.default_rng(9000 + seed)
        n_strata = int(rng.integers(1, 6))
        max_len = int(rng.choice([17, 64, 200, 512, 1000, 1024]))
        ends = sorted(set(int(x) for x in rng.integers(1, max_len, n_strata - 1))) + [max_len] if n_strata > 1 else [max_len]
        cum = W.length_histogram_piecewise_uniform(int(rng.integers(1000, 200_000)), ends, rng.random(len(ends)) + 0.05)
        b = int(rng.choice([1, 2, 4, 8, 16, 32, 64]))
        P = int(rng.choice([1, 2, 4, 8, 16, 32]))
        while P * b > 1024:
            P //= 2
        G = P * int(rng.integers(1, 40))
        quota = [int(q) for q in W.stratum_quota(cum, ends, b)]
        try:
            TL.check_all(cum, ends, b, P, G, quota, seed=int(rng.integers(0, 2 ** 62)), n=int(rng.integers(1, 12)),
                         first=int(rng.integers(0, 2 ** 40)))
        except AssertionError as e:
            raise AssertionError(f"seed {seed}: {e}") from e


def test_bucket_clip_over_random_bucket_ranges():
    for seed in range(300):
        rng = np.random.default_rng(7000 + seed)
        lay, numels = TP.random_layout(rng)
        nb = lay.n_buckets
        if seed % 3 == 0:
            g = W.normal_tensors(numels, seed, "g", 1e-2, threads=1)
        elif seed % 3 == 1:
            g = W.student_t_fp16_tensors(numels, seed, 1e-3, threads=1)
        else:
            g = oracle.Bf16(W.normal_bf16_tensors(numels, seed, 1e-2, threads=1))
        p, m, v = TV.warm_state(numels, seed)
        norms = oracle.bucket_norms(lay, g)
        thr = np.asarray([max(norms[k], 1e-3) * float(rng.choice([0.05, 0.5, 0.999, 1.5, 50.0])) for k in range(nb)], np.float32)
        cuts = sorted(set([0, nb] + [int(x) for x in rng.integers(0, nb + 1, int(rng.integers(0, 4)))]))
        offsets = [int(rng.integers(0, 4)) for _ in numels] if seed % 2 else None
        dev = Device(lay, g, p, m, v, offsets, chunk_norm=int(rng.choice([0, 1024, 4096])), chunk_apply=int(rng.choice([1024, 2048])))
        dthr, st = dev.thresholds(thr), 0
        for a, b in zip(cuts[:-1], cuts[1:]):
            dev.plan.bucket_clip(a, b, dthr, dev.norms, dev.coefs, dev.status)
            st |= int(dev.status.item())
        dev.sync()
        try:
            check_norms(dev.norms.cpu().numpy(), norms)
            ocoef, ost = oracle.clip_coefs(norms, thr)
            assert st == ost
            gcoef = dev.coefs.cpu().numpy()
            assert np.allclose(gcoef, ocoef, rtol=1e-6, atol=0)
            og = type(g)(x.copy() for x in g)
            oracle.bucket_scale(lay, og, ocoef)
            TP.check_scaled_grads(to_host(dev.g), og, g, lay, gcoef)
        except AssertionError as e:
            raise AssertionError(f"seed {seed}: {e}") from e
        finally:
            dev.close()
