"""Writes tests/golden/tiny_fused_step.json from the CPU oracle alone.

The paper prints no worked numeric example of clipping or Adam, so this fixture
is not a pin of the oracle against the paper; it freezes what the pinned oracle
gives on the Tiny configuration (3 buckets of 1000 / 4096 / 12345 fp32 elements,
thresholds 0.1 / 1 / 10, one fused step from m = v = 0), so that a later change to
the oracle's arithmetic or to the seeded inputs cannot pass unnoticed.

Run from the repository root:  python tests/golden/make_tiny_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import workloads as W  # noqa: E402

SAMPLE = [0, 1, 2, 499, 999]


def compute():
    w = W.config_tiny()
    h = w.hyper
    g = w.grads()
    p = [x.astype(np.float64) for x in w.params()]
    m = [x.astype(np.float64) for x in w.exp_avg()]
    v = [x.astype(np.float64) for x in w.exp_avg_sq()]
    norms, coefs, status = oracle.bucket_clip_adam(w.layout, g, p, m, v, w.thresholds, h.lr, h.beta1, h.beta2, h.eps,
                                                   h.weight_decay, w.first_step)
    out = {"norms": [float(x) for x in norms], "coefs": [float(x) for x in coefs], "status": status,
           "sample_index": SAMPLE, "tensors": []}
    for t in range(w.layout.n_tensors):
        out["tensors"].append({"g": [float(g[t][i]) for i in SAMPLE], "p": [float(p[t][i]) for i in SAMPLE],
                               "m": [float(m[t][i]) for i in SAMPLE], "v": [float(v[t][i]) for i in SAMPLE],
                               "p_sum": float(np.sum(p[t])), "m_sum": float(np.sum(m[t])), "v_sum": float(np.sum(v[t]))})
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_fused_step.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=1)
    print("wrote", path)
