#!/usr/bin/env python3
"""Benchmark of the fused bucket_clip_adam step on one MI355X.

A step is one pass of the whole hot path (per-bucket squared norms, finalize to
norm and clip coefficient, clip-fused Adam sweep) over the BERT-Large fp32
parameter set packed into 50 MiB buckets, with all inputs resident in HBM.

Prints ONE JSON line: ms/step, plus `roofline` for the dominant kernel and
`cpu_baseline` (the fp64 oracle timed on this machine's host cores).  The dominant
kernel is k_step, the one launch that holds the whole fused step.  Its duration
comes from HIP events recorded on the launch stream inside the timed region
itself.  It is priced on the bytes HBM has to move: p, m, v read and written
and the gradients read once, 28 B per element with fp32 gradients (26 with
16-bit ones) -- the method reads the gradients a second time, but that read is
served by the Infinity Cache and is therefore not counted.  The same launch
priced on everything that crosses the L2 / fabric boundary (gradients counted
twice, 32 or 28 B per element) is printed beside it as `frac_through_l2`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E peak
# Bytes crossing the L2 <-> fabric boundary in one launch of the dominant kernel, from two rocprofv3 --pmc
# runs (FETCH_SIZE, WRITE_SIZE) scaled by what the same counters read for libbca's plain copy kernel
# (profiles/k_step_<workload>.txt).  Key: (config, gradient type, single_launch).
MEASURED_TRAFFIC_BYTES = {      # from profiles/k_step_<workload>.txt; a combination without a counter run reports null
    (3, "f32", True): 10803960290, (2, "f32", True): 3529458180, (4, "f16", True): 9465252253,
    (5, "f32", True): 10805399362, (3, "bf16", True): 9463045573}
# The same for the other entry points (all kernels of one call summed), config 3, fp32 gradients
# (profiles/other_entry_points_bert_large_fp32_50MiB.txt).
MEASURED_TRAFFIC_OTHER_OPS = {"adam": 9446939648, "norms": 1346181120, "lamb": 13547380736, "clip_lamb": 14914948096}

def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, choices=[2, 3, 4, 5], help="benchmark configuration: 2 BERT-Base 25 MiB, 3 BERT-Large 50 MiB, 4 fp16 1 MiB, 5 4 MiB")
    ap.add_argument("--op", default="clip_adam", choices=["clip_adam", "adam", "clip_lamb", "lamb", "norms", "whole_clip_adam", "per_bucket", "lbs", "issue_rate"],
                    help="what one step is: the fused bucket_clip_adam (headline, default), adam_step alone, "
                         "bucket_clip_lamb, lamb_step, bucket_clip_norms alone, whole-gradient clipping + Adam, the paper's "
                         "order (bucket_clip bucket by bucket, then adam_step), or (lbs) the load-balancing "
                         "simulation: one step = --lbs-trials trials of each of the five methods")
    ap.add_argument("--lbs-trials", type=int, default=100000)
    ap.add_argument("--lbs-gpus", type=int, default=1024)
    ap.add_argument("--grad-dtype", default="", choices=["", "f32", "f16", "bf16"],
                    help="override the configuration's gradient storage type")
    ap.add_argument("--decay-mask", action="store_true", help="exempt biases and LayerNorm tensors from weight decay")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--chunk-norm", type=int, default=0)
    ap.add_argument("--norm-item-chunks", type=int, default=0, help="fused step: squared-norm chunks per work item (0: automatic)")
    ap.add_argument("--norm-lead", type=int, default=0, help="fused step: bucket groups the squared-norm items run ahead (0: default)")
    ap.add_argument("--chunk-apply", type=int, default=0)
    ap.add_argument("--unroll-apply", type=int, default=0)
    ap.add_argument("--group-mib", type=int, default=0)
    ap.add_argument("--adam-lds-kib", type=int, default=0, help="adam_step: LDS reserved per workgroup, KiB (0: default, -1: none)")
    ap.add_argument("--grid-norm", type=int, default=0)
    ap.add_argument("--grid-apply", type=int, default=0)
    ap.add_argument("--tune-flags", type=int, default=0)
    ap.add_argument("--lamb-group-mi", type=int, default=0, help="lamb_step: run length in Mi elements (0: library default)")
    ap.add_argument("--graph", action="store_true",
                    help="--op other than clip_adam: capture one step in a HIP graph and time its replays instead of eager calls")
    ap.add_argument("--oracle-steps", type=int, default=8)
    ap.add_argument("--calibrate-copy", type=int, default=0,
                    help="also run this many 1 GiB plain copies (k_copy) so that counter runs have a known reference")
    return ap.parse_args()


def other_ops(a, w, plan, g, p, m, v, dev):
    """Steps other than the headline one: timed the same way (K steps between two synchronisations, then each
    step between two events on the launch stream), priced on their own algorithmic bytes.  One JSON line."""
    import torch

    import paper_2402_02447_amd as B
    lay = w.layout
    N = lay.n_elements
    gb = g[0].element_size()
    hp = B.AdamHyper(w.hyper.lr, w.hyper.beta1, w.hyper.beta2, w.hyper.eps, w.hyper.weight_decay)
    thr = torch.from_numpy(w.thresholds).to(dev)
    norms = torch.zeros(lay.n_buckets, dtype=torch.float32, device=dev)
    coefs = torch.zeros_like(norms)
    trust = torch.zeros(max(1, lay.n_tensors), dtype=torch.float32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()
    step = [w.first_step]
    thr_whole = torch.ones(1, dtype=torch.float32, device=dev)
    norms_whole = torch.zeros(lay.n_buckets + 1, dtype=torch.float32, device=dev)

    # per_bucket scales g in place, so a fixed threshold would clip once and never again: the thresholds start at
    # 0.9 x the smallest bucket norm and shrink by 0.9 per step (precomputed, one row per step), so that every
    # bucket clips in every step and the bytes moved stay the same
    n_calls = [0]
    thr_rows = None
    if a.op == "per_bucket":
        plan.bucket_clip_norms(0, lay.n_buckets, norms, stream)
        base = 0.9 * float(norms.min().item())
        rows = a.warmup + 2 * a.steps
        thr_rows = base * (0.9 ** torch.arange(rows, dtype=torch.float64, device=dev)).to(torch.float32)[:, None].repeat(
            1, lay.n_buckets).contiguous()

    thr_now = torch.zeros(lay.n_buckets, dtype=torch.float32, device=dev)    # the row in use (a fixed address for --graph)

    def per_bucket():
        for b in range(lay.n_buckets):
            plan.bucket_clip(b, b + 1, thr_now, norms, coefs, status, stream)
        plan.adam_step(hp, step[0], stream)
    # algorithmic bytes per element: every sweep's reads and writes, nothing assumed cached
    ops = {
        "adam": (lambda: plan.adam_step(hp, step[0], stream), 24 + gb,
                 "adam_step: k_adam, g p m v read, p m v written"),
        "norms": (lambda: plan.bucket_clip_norms(0, lay.n_buckets, norms, stream), gb,
                  "bucket_clip_norms: k_sqnorm + k_finalize, g read"),
        "lamb": (lambda: plan.lamb_step(hp, step[0], trust, stream), (gb + 12 + 8) + (12 + 4),
                 "lamb_step: k_lamb_moments (g p m v read, m v written), k_lamb_trust, k_lamb_update (p m v read, p written)"),
        "clip_lamb": (lambda: plan.bucket_clip_lamb(thr, hp, step[0], 0, norms, coefs, trust, status, stream),
                      gb + (gb + 12 + 8) + (12 + 4), "bucket_clip_lamb: k_sqnorm + k_finalize, then the three LAMB kernels"),
        # the paper's two baselines (Sec. 3.2): one coefficient from the whole gradient's norm, so every norm
        # comes before any update and g crosses HBM twice
        "whole_clip_adam": (lambda: plan.bucket_clip_adam(thr_whole, hp, step[0], B.BCA_CLIP_WHOLE_GRADIENT, norms_whole,
                                                           coefs, status, stream),
                            gb + 24 + gb, "bucket_clip_adam, whole-gradient clipping: k_sqnorm, k_finalize, k_whole_coef, k_adam"),
        # Alg. 1 in the paper's order, without the all-reduce: every bucket clipped by a call of its own (norm, then
        # scale in place: every bucket of this workload clips), then Adam on the stored gradients
        "per_bucket": (per_bucket, gb + 2 * gb + 24 + gb,
                       "bucket_clip per bucket (k_sqnorm + k_clip_scale each), then adam_step (k_adam)"),
    }
    fn, per_elt, what = ops[a.op]

    if a.graph:          # one step captured once; every timed step is a replay (same host arguments, so the same step count)
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        eager_fn = fn
        with torch.cuda.stream(side):
            stream = side
            if thr_rows is not None:
                thr_now.copy_(thr_rows[0])
            eager_fn()                                   # warm-up outside the capture
            side.synchronize()
            cg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(cg, stream=side):
                stream = torch.cuda.current_stream()
                eager_fn()
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()
        fn = cg.replay
        what += "; HIP graph replays"

    def one():
        if thr_rows is not None:
            thr_now.copy_(thr_rows[n_calls[0]])
            n_calls[0] += 1
        fn()
        step[0] += 1
    for _ in range(a.warmup):
        one()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        one()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / a.steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(a.steps)]
    for e0, e1 in evs:
        e0.record(stream)
        one()
        e1.record(stream)
    torch.cuda.synchronize()
    per = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    med = per[len(per) // 2]
    gbps = per_elt * N / (med * 1e-3) / 1e9
    print(json.dumps({
        "metric": f"{a.op} step time (ms/step)", "value": round(ms, 4), "unit": "ms/step", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": round(ms, 4), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if gb == 4 else f"f32 ({a.grad_dtype or w.grad_dtype} gradients)",
        "data": "synthetic",
        "config": {"workload": f"configs[{a.config - 1}]: {w.name}, {N} params, {lay.n_buckets} buckets, op {a.op}"},
        "roofline": {"bound": "hbm", "kernel": what, "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC_OTHER_OPS.get(a.op) if (a.config == 3 and gb == 4) else None,
                     "bytes_per_elt": per_elt,
                     "ms_per_launch": round(med, 4)},
        "cpu_baseline": None, "ms_per_step_median": round(med, 4), "ms_per_step_min": round(per[0], 4),
        "status": int(status.item()), "buckets_clipped_last_step": int((coefs < 1).sum().item()),
    }))


def issue_rate_bench(a, dev):
    """Vector issue rates of the instruction kinds the load-balancing simulation is made of (lbs_issue_rate_probe):
    the evidence for the "alu" peak that k_lbs_all is priced on.  One JSON line."""
    import torch

    from paper_2402_02447_amd import lbs
    grid, iters = 256 * 8 * 4, 2000                      # 8 workgroups per compute unit resident, 4 rounds of them
    out = torch.zeros(grid * 256, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()
    rates = {}
    for kind, (what, n_instr) in lbs.PROBE_KINDS.items():
        lbs.issue_rate_probe(kind, grid, iters, out, stream)
        ts = []
        for _ in range(max(3, a.steps)):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            lbs.issue_rate_probe(kind, grid, iters, out, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        ms = sorted(ts)[len(ts) // 2]
        lane_ops = grid * 256 * iters * 8 * n_instr
        rates[what] = {"ms": round(ms, 3), "T_lane_ops_per_s": round(lane_ops / (ms * 1e-3) / 1e12, 1)}
    peak = 256 * 4 * 32 * 2.4e9 / 1e12
    print(json.dumps({"metric": "vector issue rate per instruction kind (lane-operations per second)", "unit": "T lane-ops/s",
                      "n_gpus": 1, "config": {"workload": f"{grid} workgroups x 256 threads x {iters} rounds x 8 chains per lane"},
                      "peak_taken": round(peak, 1), "rates": rates}))


def lbs_bench(a, dev):
    """Load-balancing simulation (Sec. 5.2, Table 5) at the paper's setting: local batch 16, nodes of 8 GPUs,
    --lbs-gpus GPUs, --lbs-trials trials per method.  One JSON line: simulated sequence draws per second over
    the five methods, the table of average minimum / maximum token counts, and the oracle timed on a sample."""
    import numpy as np
    import torch

    import workloads as W
    from paper_2402_02447_amd import lbs
    cum = W.length_histogram_piecewise_uniform()
    ends = W.LENGTH_STRATUM_END
    quota = [int(q) for q in W.stratum_quota(cum, ends, 16)]
    G, b, P, n = a.lbs_gpus, 16, 8, a.lbs_trials
    names = {lbs.LBS_NONE: "no balancing", lbs.LBS_STRATIFIED: "+ stratification", lbs.LBS_LOCAL_RASTER: "+ local presorting",
             lbs.LBS_LOCAL_SNAKE: "+ snake scanning", lbs.LBS_GLOBAL: "global presorting"}
    ds = lbs.Dataset(cum, ends, device=0)
    stream = torch.cuda.current_stream()
    sums = {m: torch.zeros(2, dtype=torch.int64, device=dev) for m in names}
    sums_all = torch.zeros((5, 2), dtype=torch.int64, device=dev)

    def one_step():     # the five methods of Table 5 on shared draws: one lbs_simulate_all call, one kernel
        ds.lbs_simulate_all(b, P, G, quota, 2024, n, sums_all, stream=stream)
    for _ in range(a.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        one_step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / a.steps
    per_method = {}
    for m in names:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        ds.lbs_simulate(m, b, P, G, quota, 2024, n, sums[m], stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        per_method[m] = e0.elapsed_time(e1)
    assert all(int(sums[m][0]) == int(sums_all[m][0]) and int(sums[m][1]) == int(sums_all[m][1]) for m in names)
    table = {names[m]: {"avg_min": round(int(sums[m][0]) / n, 1), "avg_max": round(int(sums[m][1]) / n, 1),
                        "ms_alone": round(per_method[m], 3)} for m in names}
    draws = 5 * n * G * b
    cpu = None
    if not a.no_cpu_baseline:
        from oracle import lbs as O
        n_cpu = max(1, min(n, 2000 * 1024 // G))
        t1 = time.perf_counter()
        for m in names:
            _, _, s0, s1 = O.simulate(cum, ends, quota, b, P, G, m, 2024, n_cpu)
        dt = time.perf_counter() - t1
        cpu = {"value": round(5 * n_cpu * G * b / dt / 1e6, 2), "unit": "M draws/s", "cores": 1, "kind": "oracle",
               "sample": f"{n_cpu} trials of each of the five methods, same setting, single thread"}
    # The step is one kernel, k_lbs_all.  Vector instructions it executes, from a rocprofv3 --pmc SQ_INSTS_VALU run of
    # this command (profiles/lbs_table5_setting_kernel_stats.txt): 4.235e9 wavefront instructions per 100 000 trials at
    # 1 024 GPUs, i.e. 2 x 1.638e9 draws made (one set from the whole dataset, one stratified) = 82.7 lane-operation
    # slots per draw made (64 lanes per instruction).  Peak: a SIMD issues a 64-lane move, add or xor in 2 cycles and
    # a multiply, minimum or median in 4 (measured); the bound taken is every instruction at the faster rate,
    # 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz = 78.6 T lane-operations/s, which is also the rate behind the chip's
    # 157.3 TFLOP/s of fp32 vector FMAs.
    ops_per_draw_made = 82.7
    draws_made = 2 * n * G * b
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(a.steps):
        one_step()
    e1.record(stream)
    torch.cuda.synchronize()
    t_all = e0.elapsed_time(e1) / a.steps * 1e-3
    achieved = ops_per_draw_made * draws_made / t_all / 1e12
    peak = 256 * 4 * 32 * 2.4e9 / 1e12
    print(json.dumps({
        "metric": "load-balancing simulation throughput (sequence draws simulated per second over the five methods, "
                  "which share two sets of draws)",
        "value": round(draws / (ms * 1e-3) / 1e9, 3), "unit": "G draws/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32/u64",
        "data": "synthetic",
        "config": {"workload": f"Table 5 setting: {G} simulated GPUs, local batch {b}, nodes of {P}, {n} trials per method, "
                               f"piecewise-uniform length histogram with the printed stratum shares, quota {quota}"},
        "roofline": {"bound": "alu", "kernel": "k_lbs_all (both sets of draws, counting sort over all GPUs, bitonic sort of each "
                                               "node's pool in registers, the five methods' deals)",
                     "achieved": round(achieved, 2), "peak": round(peak, 1), "unit": "T lane-ops/s",
                     "frac": round(achieved / peak, 3), "traffic": None, "ops_per_draw_made": ops_per_draw_made,
                     "draws_made_per_step": draws_made, "ms_per_launch": round(t_all * 1e3, 3)},
        "cpu_baseline": cpu, "table": table,
    }))
    ds.close()


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2402_02447_amd as B
    import workloads as W

    B.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if a.op == "lbs":
        lbs_bench(a, dev)
        return
    if a.op == "issue_rate":
        issue_rate_bench(a, dev)
        return

    w = W.CONFIGS[a.config]()
    lay = w.layout
    numels = [int(n) for n in lay.tensor_numel]
    N = lay.n_elements
    gdt_name = a.grad_dtype or w.grad_dtype
    f16 = gdt_name == "f16"
    bf16 = gdt_name == "bf16"

    # ---- synthetic inputs, generated on the device (seeded), one allocation per tensor
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    def randn(n, sigma):
        return torch.randn(n, generator=gen, device=dev, dtype=torch.float32) * sigma
    p = [randn(n, 0.02) for n in numels]
    if w.warm:
        m = [randn(n, 3e-4) for n in numels]
        v = [(torch.rand(n, generator=gen, device=dev, dtype=torch.float32) + 0.5) * 1e-6 for n in numels]
    else:
        m = [torch.zeros(n, device=dev) for n in numels]
        v = [torch.zeros(n, device=dev) for n in numels]
    if f16:
        def t3(n):
            z = torch.randn(4, n, generator=gen, device=dev, dtype=torch.float32)
            return (z[0] / torch.sqrt((z[1] ** 2 + z[2] ** 2 + z[3] ** 2) / 3.0) * w.sigma_g).to(torch.float16)
        g = [t3(n) for n in numels]
    else:
        g = [randn(n, w.sigma_g) for n in numels]
        for b in w.hot_buckets:
            for t, beg, ln in lay.segments_of(b):
                g[t][beg:beg + ln] *= 100.0
        if bf16:
            g = [x.to(torch.bfloat16) for x in g]
    thr = torch.from_numpy(w.thresholds).to(dev)
    hp = B.AdamHyper(w.hyper.lr, w.hyper.beta1, w.hyper.beta2, w.hyper.eps, w.hyper.weight_decay)

    gdt = B.BCA_GRAD_F16 if f16 else B.BCA_GRAD_BF16 if bf16 else B.BCA_GRAD_F32
    plan = B.Plan.from_layout(lay, gdt, device=0, chunk_norm=a.chunk_norm,
                              chunk_apply=a.chunk_apply, grid_norm=a.grid_norm, grid_apply=a.grid_apply,
                              unroll_apply=a.unroll_apply, tune_flags=a.tune_flags, group_bytes=a.group_mib << 20,
                              adam_lds_reserve=1 if a.adam_lds_kib < 0 else a.adam_lds_kib << 10,
                              norm_item_chunks=a.norm_item_chunks, norm_lead=a.norm_lead,
                              lamb_group_elems=a.lamb_group_mi << 20)
    plan.bind(g, p, m, v)
    mask = None
    if a.decay_mask:
        H, L, F = (768, 12, 3072) if a.config == 2 else (1024, 24, 4096)
        mask = W.bert_decay_mask(30522, H, L, F, 512)
        plan.set_decay_mask(mask)
    if a.calibrate_copy:     # a kernel with exactly known traffic, for counter runs
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(7)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(a.calibrate_copy):
            B.copy_bytes(dst, src, 1 << 30, torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert bool((dst[:: 1 << 20] == 7).all())
        del src, dst
    if a.op != "clip_adam":
        other_ops(a, w, plan, g, p, m, v, dev)
        plan.close()
        return
    norms = torch.zeros(lay.n_buckets, dtype=torch.float32, device=dev)
    coefs = torch.zeros_like(norms)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    flags = 0        # gradients are read, never written: the timed steps keep clipping the same way
    stream = torch.cuda.current_stream()

    # host copies for the CPU baseline are taken before the state evolves; and so that the benched configuration is
    # itself held to the oracle, one fused step runs on copies of p, m, v (a second plan), to be compared below
    host = None
    check = None
    if not a.no_cpu_baseline:
        host = [[t.cpu().numpy() for t in xs] for xs in (g, p, m, v)]
        pc, mc, vc = ([x.clone() for x in xs] for xs in (p, m, v))
        plan_c = B.Plan.from_layout(lay, gdt, device=0)
        plan_c.bind(g, pc, mc, vc)
        plan_c.set_decay_mask(mask)
        norms_c, coefs_c, status_c = torch.zeros_like(norms), torch.zeros_like(norms), torch.zeros_like(status)
        plan_c.bucket_clip_adam(thr, hp, w.first_step, flags, norms_c, coefs_c, status_c, stream)
        torch.cuda.synchronize()
        check = [[t.cpu().numpy() for t in xs] for xs in (pc, mc, vc)] + [norms_c.cpu().numpy(), int(status_c.item())]
        plan_c.close()
        del pc, mc, vc

    step = w.first_step
    def one_step():
        nonlocal step
        plan.bucket_clip_adam(thr, hp, step, flags, norms, coefs, status, stream)
        step += 1

    for _ in range(a.warmup):
        one_step()
    plan.profile(a.steps)      # HIP events around the kernels of the next K calls, on the launch stream
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; the per-kernel events are recorded inside it, so the kernel durations
    # ---- reported below are those of the very launches whose wall time is ms_per_step
    t0 = time.perf_counter()
    for _ in range(a.steps):
        one_step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / a.steps
    (ms_norm, ms_fin, ms_adam), n_prof = plan.profile_read()
    plan.profile(0)
    n_waited, n_polls = plan.wait_stats()        # over warm-up and timed steps
    assert n_prof == a.steps
    ms_norm, ms_fin, ms_adam = ms_norm / n_prof, ms_fin / n_prof, ms_adam / n_prof
    st = int(status.item())
    assert st == 0, f"status word {st} after the timed steps"
    n_clipped = int((coefs < 1).sum().item())

    # ---- per-step spread: each step between two events on the launch stream
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(a.steps)]
    for e0, e1 in evs:
        e0.record(stream)
        one_step()
        e1.record(stream)
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    ms_median, ms_min = per_step[len(per_step) // 2], per_step[0]

    # ---- practical ceiling on this machine: plain copy kernel, 1 GiB, read + written bytes
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
    dst = torch.empty_like(src)
    B.copy_bytes(dst, src, 1 << 30, stream)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record(stream)
    for _ in range(5):
        B.copy_bytes(dst, src, 1 << 30, stream)
    c1.record(stream)
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * (1 << 30) / (c0.elapsed_time(c1) * 1e-3) / 1e9
    # and a yardstick that is not this library's: torch's own element-wise kernel over the same gigabyte (read + written)
    a32, b32 = src.view(torch.float32), dst.view(torch.float32)
    torch.add(a32, 1.0, out=b32)
    c0.record(stream)
    for _ in range(5):
        torch.add(a32, 1.0, out=b32)
    c1.record(stream)
    torch.cuda.synchronize()
    torch_gbps = 5 * 2 * (1 << 30) / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst, a32, b32

    gbytes = 2 if (f16 or bf16) else 4
    single = not (a.tune_flags & B.BCA_TUNE_MULTI_LAUNCH)
    pmv_bytes = 24                                         # p, m, v read and written
    hbm_per_elt = pmv_bytes + gbytes                       # what HBM must move: gradients once
    l2_per_elt = pmv_bytes + 2 * gbytes                    # what crosses L2 <-> fabric: gradients read by both passes
    ms_kernel = ms_adam
    if single:
        kname = ("k_step (the whole fused step in one launch: squared norms, finalize, clip-fused Adam sweep); priced on HBM "
                 "bytes, the second read of the gradients being served by the Infinity Cache")
    else:
        kname = "k_adam (clip-fused Adam sweep, summed over bucket groups; gradients still cached from the group's norm pass)"
    achieved = hbm_per_elt * N / (ms_kernel * 1e-3) / 1e9
    through_l2 = (l2_per_elt if single else hbm_per_elt) * N / (ms_kernel * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get((a.config, gdt_name, single))
    roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "bytes_per_elt": hbm_per_elt,
                "ms_per_launch": round(ms_kernel, 4),
                # the counters behind `traffic` sit at the L2 / fabric boundary, in front of the Infinity Cache: they see the
                # gradients twice.  The same launch priced on those bytes:
                "bytes_per_elt_through_l2": l2_per_elt if single else hbm_per_elt,
                "achieved_through_l2": round(through_l2, 1), "frac_through_l2": round(through_l2 / HBM_PEAK_GBPS, 4)}
    extras = {
        "kernels_ms": ({"k_finish": round(ms_norm, 4), "k_step": round(ms_adam, 4)} if single else
                       {"k_sqnorm": round(ms_norm, 4), "k_finalize": round(ms_fin, 4), "k_adam": round(ms_adam, 4)}),
        "ms_per_step_median": round(ms_median, 4), "ms_per_step_min": round(ms_min, 4),
        "plain_copy_kernel_GBps": round(copy_gbps, 1),
        "step_GBps_hbm_bytes": round(hbm_per_elt * N / (ms_per_step * 1e-3) / 1e9, 1),
        "step_frac_of_peak_hbm_bytes": round(hbm_per_elt * N / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "plain_copy_frac_of_peak": round(copy_gbps / HBM_PEAK_GBPS, 4),
        "torch_elementwise_add_GBps": round(torch_gbps, 1),
        "items_that_waited_per_step": round(n_waited / (a.warmup + a.steps), 1),
        "polls_per_waiting_item": round(n_polls / max(n_waited, 1), 1),
        "elements": N, "buckets": lay.n_buckets, "chunks_norm": plan.n_chunks(B.BCA_TABLE_NORM),
        "chunks_apply": plan.n_chunks(B.BCA_TABLE_APPLY), "groups": plan.n_groups, "buckets_clipped": n_clipped,
        "status": st,
    }

    cpu = None
    if host is not None:
        import oracle
        hg, hp_, hm, hv = host
        with ThreadPoolExecutor(max_workers=8) as ex:
            op, om, ov = (list(ex.map(lambda x: x.astype(np.float64), xs)) for xs in (hp_, hm, hv))
        cpu_s = 0.0
        parity = None
        for k in range(a.oracle_steps):
            t1 = time.perf_counter()
            onorm, _, ost = oracle.bucket_clip_adam(lay, hg, op, om, ov, w.thresholds, w.hyper.lr, w.hyper.beta1, w.hyper.beta2,
                                                    w.hyper.eps, w.hyper.weight_decay, w.first_step + k, decay=mask)
            cpu_s += time.perf_counter() - t1
            if k == 0:
                # the GPU's first step on this very workload against the oracle's, every element, BASELINE's tolerances
                # (relative 1e-5, or absolute 1e-7 where |oracle| < 1e-2; norms relative 1e-5)
                cp, cm, cv, cn, cst = check
                worst = {}
                n_bad = 0
                for name, got, want in (("p", cp, op), ("m", cm, om), ("v", cv, ov)):
                    big = small = rel_all = 0.0
                    for t in range(lay.n_tensors):
                        if got[t].size:
                            r = oracle.compare_f32(got[t], want[t])
                            n_bad += r["n_bad"]
                            big, small = max(big, r["max_rel_big"]), max(small, r["max_abs_small"])
                            rel_all = max(rel_all, r["max_rel_all"])
                    worst[name] = {"max_rel_where_oracle_ge_1e-2": float(f"{big:.3g}"),
                                   "max_abs_where_oracle_lt_1e-2": float(f"{small:.3g}")}
                    if name == "v":      # no cancellation in v: the relative error holds everywhere
                        worst[name]["max_rel_everywhere"] = float(f"{rel_all:.3g}")
                        assert rel_all <= 1e-5, rel_all
                norm_rel = float(np.max(np.abs(cn.astype(np.float64) - onorm) / np.maximum(onorm, 1e-300)))
                assert n_bad == 0 and norm_rel <= 1e-5 and cst == ost, (n_bad, norm_rel, cst, ost)
                parity = {"checked": "first fused step of this workload, every element of p, m, v and every bucket norm, "
                                     "against the oracle", "elements_out_of_tolerance": n_bad,
                          "errors": worst,
                          "max_rel_err_norms": float(f"{norm_rel:.3g}")}
        cpu_ms = cpu_s * 1e3 / a.oracle_steps
        cpu = {"value": round(cpu_ms, 1), "unit": "ms/step", "cores": 1, "kind": "oracle",
               "sample": f"{a.oracle_steps} full fused steps of the same workload ({N} elements), single thread, "
                         f"host has {os.cpu_count()} logical cpus"}
        extras["parity_vs_oracle"] = parity

    out = {
        "metric": ("fused bucket_clip_adam step time, BERT-Large fp32 (ms/step; HBM fraction in roofline)"
                   if (a.config == 3 and gdt_name == "f32") else
                   f"fused bucket_clip_adam step time, {w.name}, {gdt_name} gradients (ms/step; HBM fraction in roofline)"),
        "value": round(ms_per_step, 4), "unit": "ms/step", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if gdt_name == "f32" else f"f32 ({gdt_name} gradients)", "data": "synthetic",
        "config": {"workload": f"configs[{a.config - 1}]: {w.name}, {N} params in {lay.n_tensors} tensors, "
                               f"{lay.n_buckets} buckets, grads {gdt_name}"},
        "roofline": roofline, "cpu_baseline": cpu, **extras,
    }
    print(json.dumps(out))
    plan.close()


if __name__ == "__main__":
    main()
