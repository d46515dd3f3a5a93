"""Writes tests/golden/tiny_lamb_step.json and tests/golden/small_lbs_table.json from the CPU oracles alone.

Neither fixture pins an oracle against the paper (the paper prints no worked LAMB step, and its Table 5 needs the
Wikipedia length histogram, which it does not print); they freeze what the pinned oracles give, so that a later
change to their arithmetic, to the generator or to the seeded inputs cannot pass unnoticed:
  * one bucket_clip_lamb step on the Tiny configuration (3 buckets of 1000 / 4096 / 12345 fp32 elements, thresholds
    0.1 / 1 / 10, warm moments, step 3, biases-style mask on the middle tensor);
  * the five load-balancing methods on 64 simulated GPUs (local batch 16, nodes of 8, quota 6/3/2/5, seed 7,
    first 20 trials) on the piecewise-uniform stand-in histogram.

Run from the repository root:  python tests/golden/make_variants_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import workloads as W  # noqa: E402
from oracle import lbs  # noqa: E402

SAMPLE = [0, 1, 2, 499, 999]
HERE = os.path.dirname(os.path.abspath(__file__))


def compute_lamb():
    w = W.config_tiny()
    h = w.hyper
    numels = w.layout.tensor_numel
    g = w.grads()
    p = [x.astype(np.float64) for x in w.params()]
    m = [x.astype(np.float64) for x in W.normal_tensors(numels, 0, "m", 3e-4)]
    v = [x.astype(np.float64) for x in W.warm_second_moment(numels, 0)]
    norms, coefs, trust, status = oracle.bucket_clip_lamb(w.layout, g, p, m, v, w.thresholds, h.lr, h.beta1, h.beta2,
                                                          h.eps, h.weight_decay, 3, decay=[1, 0, 1])
    return {"norms": [float(x) for x in norms], "coefs": [float(x) for x in coefs], "trust": [float(x) for x in trust],
            "status": status, "sample_index": SAMPLE,
            "tensors": [{"p": [float(p[t][i]) for i in SAMPLE], "m": [float(m[t][i]) for i in SAMPLE],
                         "v": [float(v[t][i]) for i in SAMPLE], "p_sum": float(np.sum(p[t]))}
                        for t in range(w.layout.n_tensors)]}


def compute_lbs():
    cum = W.length_histogram_piecewise_uniform()
    out = {"setting": {"n_gpus": 64, "local_batch": 16, "gpus_per_node": 8, "quota": [6, 3, 2, 5], "seed": 7, "trials": 20},
           "first_draws_gpu0_trial0": [int(x) for x in lbs.draw(cum, True, W.LENGTH_STRATUM_END, [6, 3, 2, 5], 16, 64, 7, 0, 0)],
           "methods": {}}
    for name, method in (("none", lbs.NONE), ("stratified", lbs.STRATIFIED), ("local_raster", lbs.LOCAL_RASTER),
                         ("local_snake", lbs.LOCAL_SNAKE), ("global", lbs.GLOBAL)):
        tmin, tmax, s0, s1 = lbs.simulate(cum, W.LENGTH_STRATUM_END, [6, 3, 2, 5], 16, 8, 64, method, 7, 20)
        out["methods"][name] = {"trial_min": [int(x) for x in tmin], "trial_max": [int(x) for x in tmax],
                                "sum_min": s0, "sum_max": s1}
    return out


if __name__ == "__main__":
    for name, fn in (("tiny_lamb_step.json", compute_lamb), ("small_lbs_table.json", compute_lbs)):
        with open(os.path.join(HERE, name), "w") as f:
            json.dump(fn(), f, indent=1)
        print("wrote", name)
