"""Helpers for the GPU parity tests: put a workload's host arrays on the device,
run the library through its C ABI binding, bring results back and compare them
with the oracle under the acceptance rule."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

import oracle
import paper_2402_02447_amd as B

REL_TOL = 1e-5      # norms; p, m, v where |oracle| >= 1e-2
ABS_TOL = 1e-7      # p, m, v where |oracle| < 1e-2
SMALL = 1e-2


def gdt_of(grads: Sequence[np.ndarray]) -> int:
    if isinstance(grads, oracle.Bf16):
        return B.BCA_GRAD_BF16
    return B.BCA_GRAD_F16 if len(grads) and grads[0].dtype == np.float16 else B.BCA_GRAD_F32


def to_dev(arrs: Sequence[np.ndarray], offsets: Optional[Sequence[int]] = None) -> List[torch.Tensor]:
    """One device allocation per tensor.  With `offsets`, tensor t instead starts
    offsets[t] elements into its own slightly larger allocation, which gives
    addresses that are only element-aligned."""
    out = []
    for i, a in enumerate(arrs):
        t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a)      # bf16 bit patterns travel as int16
        if offsets is None or offsets[i] == 0:
            out.append(t.cuda())
        else:
            buf = torch.empty(a.shape[0] + offsets[i] + 8, dtype=t.dtype, device="cuda")
            view = buf[offsets[i]:offsets[i] + a.shape[0]]
            view.copy_(t)
            out.append(view)
    return out


def to_host(ts: Sequence[torch.Tensor]) -> List[np.ndarray]:
    return [t.cpu().numpy().view(np.uint16) if t.dtype == torch.int16 else t.cpu().numpy() for t in ts]


class Device:
    """A workload resident on the GPU, bound to a plan."""

    def __init__(self, layout, grads, params, exp_avg, exp_avg_sq, offsets=None, **tuning):
        self.layout = layout
        self.g = to_dev(grads, offsets)
        self.p = to_dev(params, offsets)
        self.m = to_dev(exp_avg, offsets)
        self.v = to_dev(exp_avg_sq, offsets)
        self.plan = B.Plan.from_layout(layout, gdt_of(grads), device=torch.cuda.current_device(), **tuning)
        self.plan.bind(self.g, self.p, self.m, self.v)
        nb = layout.n_buckets
        self.norms = torch.full((nb,), -1.0, dtype=torch.float32, device="cuda")
        self.coefs = torch.full((nb,), -1.0, dtype=torch.float32, device="cuda")
        self.status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        self.trust = torch.full((max(1, layout.n_tensors),), -1.0, dtype=torch.float32, device="cuda")

    def set_grads(self, grads):
        for d, h in zip(self.g, grads):
            d.copy_(torch.from_numpy(h.view(np.int16) if h.dtype == np.uint16 else h))

    def thresholds(self, thr: np.ndarray) -> torch.Tensor:
        return torch.from_numpy(np.ascontiguousarray(thr, np.float32)).cuda()

    def sync(self):
        torch.cuda.synchronize()

    def close(self):
        self.plan.close()


def hyper(h) -> B.AdamHyper:
    return B.AdamHyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay)


def hp_kwargs(h) -> dict:
    return dict(lr=h.lr, beta1=h.beta1, beta2=h.beta2, eps=h.eps, weight_decay=h.weight_decay)


def f64(arrs: Sequence[np.ndarray]) -> List[np.ndarray]:
    return [a.astype(np.float64) for a in arrs]


def check_norms(got: np.ndarray, want: np.ndarray):
    want = np.asarray(want, np.float64)
    got = np.asarray(got, np.float64)
    nz = want != 0
    rel = np.abs(got[nz] - want[nz]) / want[nz]
    assert np.all(got[~nz] == 0), "zero-norm buckets must come out as exactly 0"
    assert rel.size == 0 or rel.max() <= REL_TOL, f"bucket norm rel err {rel.max():.3e} at bucket {int(np.argmax(rel))}"
    return float(rel.max()) if rel.size else 0.0


def check_state(name: str, got: Sequence[np.ndarray], want: Sequence[np.ndarray], strict_rel: bool = False) -> dict:
    """Acceptance rule per element: rel <= 1e-5, or abs <= 1e-7 where |oracle| < 1e-2.
    strict_rel additionally requires rel <= 1e-5 wherever |oracle| > 1e-30 (used
    for v, which has no cancellation and would otherwise only meet the absolute clause)."""
    agg = {"n_bad": 0, "max_rel_big": 0.0, "max_abs_small": 0.0, "max_rel_all": 0.0}
    for t, (g, w) in enumerate(zip(got, want)):
        if g.size == 0:
            continue
        r = oracle.compare_f32(g, w, REL_TOL, ABS_TOL, SMALL)
        assert r["n_bad"] == 0, (f"{name}[{t}]: {r['n_bad']} elements out of tolerance, worst at {r['worst_index']}: "
                                 f"gpu {g[r['worst_index']]!r} oracle {w[r['worst_index']]!r}")
        for k in ("max_rel_big", "max_abs_small", "max_rel_all"):
            agg[k] = max(agg[k], r[k])
    if strict_rel:
        assert agg["max_rel_all"] <= REL_TOL, f"{name}: max relative error {agg['max_rel_all']:.3e}"
    return agg


def bits_equal(a: Sequence[np.ndarray], b: Sequence[np.ndarray]) -> bool:
    return all(np.array_equal(x.view(np.uint8), y.view(np.uint8)) for x, y in zip(a, b))
