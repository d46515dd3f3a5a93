"""Per-bucket clipping as the paper uses it: clip each bucket the moment backward
has produced it, on a side stream, while backward goes on (Sec. 4.2, Fig. 5c;
Alg. 1 marks the clip and the all-reduce "do in parallel" with backward).

There is no model here, so backward is a stand-in: for every bucket, in the
order backward would produce them, a few large fp32 matrix products on the main
stream (compute bound, like backward), then an event.  The side stream waits
for that event and runs bucket_clip on that bucket alone; the all-reduce that
would follow is left out (one GPU).  After the last bucket the main stream waits for the side stream and runs adam_step.

Three timings, K repetitions each: backward alone; backward with the clips
serialised on the same stream; backward with the clips on the side stream.
Prints one JSON line.  Run from the repository root on a GPU machine:
    python -m paper_2402_02447_amd.overlap_timeline --config 3
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=3, choices=[2, 3, 5])
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--matmul-n", type=int, default=4096, help="side of the square fp32 matrices of the stand-in")
    ap.add_argument("--matmuls-per-bucket", type=int, default=4)
    ap.add_argument("--chunk-norm", type=int, default=0, help="elements per squared-norm chunk (0: library default)")
    ap.add_argument("--two-calls", action="store_true", help="bucket_clip_norms + bucket_clip_apply instead of bucket_clip")
    a = ap.parse_args()

    import numpy as np
    import torch

    import paper_2402_02447_amd as B
    import workloads as W

    B.load_library()
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    w = W.CONFIGS[a.config]()
    lay = w.layout
    numels = [int(n) for n in lay.tensor_numel]
    nb = lay.n_buckets
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)
    g0 = [torch.randn(n, generator=gen, device=dev) * w.sigma_g for n in numels]
    g = [x.clone() for x in g0]
    p = [torch.randn(n, generator=gen, device=dev) * 0.02 for n in numels]
    m = [torch.zeros(n, device=dev) for n in numels]
    v = [torch.zeros(n, device=dev) for n in numels]
    thr = torch.from_numpy(w.thresholds).to(dev)
    hp = B.AdamHyper(w.hyper.lr, w.hyper.beta1, w.hyper.beta2, w.hyper.eps, w.hyper.weight_decay)
    plan = B.Plan.from_layout(lay, B.BCA_GRAD_F32, device=0, chunk_norm=a.chunk_norm)
    plan.bind(g, p, m, v)
    norms = torch.zeros(nb, device=dev)
    coefs = torch.zeros(nb, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    xa = torch.randn(a.matmul_n, a.matmul_n, generator=gen, device=dev)
    xb = torch.randn(a.matmul_n, a.matmul_n, generator=gen, device=dev)
    xc = torch.empty_like(xa)

    main_s = torch.cuda.current_stream()
    side = torch.cuda.Stream()

    def backward_piece():
        for _ in range(a.matmuls_per_bucket):
            torch.matmul(xa, xb, out=xc)

    def clip(b, stream):
        if a.two_calls:
            plan.bucket_clip_norms(b, b + 1, norms, stream=stream)
            plan.bucket_clip_apply(b, b + 1, thr, norms, coefs, status, stream=stream)
        else:
            plan.bucket_clip(b, b + 1, thr, norms, coefs, status, stream=stream)

    def iteration(mode):
        """mode: 'backward' | 'serial' | 'overlap'.  Returns (ms until backward is done, ms until all clips are done)."""
        for x, y in zip(g, g0):
            x.copy_(y)
        torch.cuda.synchronize()
        t0, t_bwd, t_end = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        t0.record(main_s)
        for b in range(nb):
            backward_piece()
            if mode == "serial":
                clip(b, main_s)
            elif mode == "overlap":
                ready = torch.cuda.Event()
                ready.record(main_s)
                side.wait_event(ready)
                clip(b, side)
        t_bwd.record(main_s)
        if mode == "overlap":
            main_s.wait_stream(side)
        t_end.record(main_s)
        torch.cuda.synchronize()
        return t0.elapsed_time(t_bwd), t0.elapsed_time(t_end)

    res = {}
    for mode in ("backward", "serial", "overlap"):
        iteration(mode)                                   # warm-up
        runs = [iteration(mode) for _ in range(a.reps)]
        res[mode] = (float(np.median([r[0] for r in runs])), float(np.median([r[1] for r in runs])))
    clipped = int((coefs < 1).sum().item())

    # Adam after the loop, on the clipped gradients (the paper's last line of the iteration)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    plan.adam_step(hp, w.first_step)
    torch.cuda.synchronize()
    e0.record(main_s)
    for k in range(10):
        plan.adam_step(hp, w.first_step + 1 + k)
    e1.record(main_s)
    torch.cuda.synchronize()
    adam_ms = e0.elapsed_time(e1) / 10

    bwd = res["backward"][1]
    serial_extra = res["serial"][1] - bwd
    overlap_extra = res["overlap"][1] - bwd
    out = {
        "workload": f"{w.name}: {lay.n_elements} fp32 gradients in {nb} buckets, clipped one bucket at a time",
        "stand_in_backward": f"{a.matmuls_per_bucket} fp32 matmuls of {a.matmul_n}^3 per bucket",
        "backward_alone_ms": round(bwd, 3),
        "clips_on_same_stream_ms": round(res["serial"][1], 3), "clip_cost_serial_ms": round(serial_extra, 3),
        "clips_on_side_stream_ms": round(res["overlap"][1], 3), "clip_cost_exposed_ms": round(overlap_extra, 3),
        "hidden_fraction": round(1.0 - overlap_extra / serial_extra, 3) if serial_extra > 0 else None,
        "clip_us_per_bucket_serial": round(serial_extra * 1e3 / nb, 1),
        "adam_step_ms": round(adam_ms, 4),
        "adam_step_GBps": round(28 * lay.n_elements / (adam_ms * 1e-3) / 1e9, 1),
        "buckets_clipped": clipped, "status": int(status.item()),
    }
    print(json.dumps(out))
    plan.close()


if __name__ == "__main__":
    main()
