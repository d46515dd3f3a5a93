"""CPU-only checks of libbca's host side: the library loads, exports every symbol
declared in include/bca.h, validates layouts and hyper-parameters, and cuts the
bucket layout into a correct chunk table.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2402_02447_amd as B
from paper_2402_02447_amd import binding
import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_binding_constants_equal_the_headers():
    """Every #define of include/bca.h and include/lbs.h that the bindings mirror has the same value there."""
    import ctypes as C
    from paper_2402_02447_amd import binding, lbs
    for header, module in (("bca.h", binding), ("lbs.h", lbs)):
        text = open(os.path.join(ROOT, "include", header)).read()
        defines = dict(re.findall(r"#define\s+((?:BCA|LBS)_[A-Z0-9_]+)\s+\(?(-?\d+)u?\)?", text))
        mirrored = [k for k in defines if hasattr(module, k)]
        assert len(mirrored) >= 9, (header, mirrored)
        for k in mirrored:
            assert getattr(module, k) == int(defines[k]), (header, k)
        # error codes are mirrored as a code -> name table
        table = binding._ERR_NAMES if module is binding else lbs._ERR
        errs = {int(v): k for k, v in defines.items() if "_ERR_" in k}
        assert errs == table, (header, errs, table)
    # struct layouts the C side and ctypes must agree on (C99 layout rules: natural alignment)
    assert C.sizeof(binding._Segment) == 24 and C.sizeof(binding._Tuning) == 56 and C.sizeof(lbs._Run) == 72


def test_library_loads_and_exports_every_declared_symbol():
    L = B.load_library()
    header = open(os.path.join(ROOT, "include", "bca.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(bca_[a-z0-9_]+|bucket_clip_[a-z]+|bucket_clip|adam_step|lamb_step)\s*\(", header))
    assert {"bucket_clip_norms", "bucket_clip_apply", "bucket_clip", "adam_step", "bucket_clip_adam", "lamb_step",
            "bucket_clip_lamb", "bca_plan_set_decay_mask"} <= declared
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name
    assert L.bca_version() >= 1


def host_plan(layout, grad_dtype=0, **kw):
    return B.Plan.from_layout(layout, grad_dtype, device=-1, **kw)


@pytest.mark.parametrize("table", [B.BCA_TABLE_NORM, B.BCA_TABLE_APPLY])
@pytest.mark.parametrize("chunk", [1024, 4096, 16384])
def test_chunk_table_partitions_the_layout(chunk, table):
    numels = W.scaled_bert_numels(64, 2, 256, vocab=1000, max_pos=32) + [0, 7, 1]
    lay = W.layout_flat_split(numels, 50_000)
    p = host_plan(lay, chunk_norm=chunk, chunk_apply=chunk)
    assert p.n_buckets == lay.n_buckets
    seen = [np.zeros(n, np.int8) for n in numels]
    prev_bucket = 0
    per_bucket = np.zeros(lay.n_buckets, np.int64)
    for i in range(p.n_chunks(table)):
        t, beg, ln, b = p.chunk_info(i, table)
        assert 0 < ln <= chunk
        assert b >= prev_bucket                        # bucket-major order
        prev_bucket = b
        assert beg // chunk == (beg + ln - 1) // chunk  # never straddles a multiple of the chunk size
        seen[t][beg:beg + ln] += 1
        per_bucket[b] += ln
        f, n = p.bucket_chunks(b, table)
        assert f <= i < f + n
    assert all((s == 1).all() for s in seen)
    assert np.array_equal(per_bucket, lay.bucket_numel())
    # chunks stay inside their segment's bucket: elements of bucket b per the layout
    for b in range(lay.n_buckets):
        f, n = p.bucket_chunks(b, table)
        cover = {}
        for i in range(f, f + n):
            t, beg, ln, bb = p.chunk_info(i, table)
            assert bb == b
            cover.setdefault(t, []).append((beg, ln))
        want = {}
        for t, beg, ln in lay.segments_of(b):
            if ln:
                want.setdefault(t, []).append((beg, ln))
        assert set(cover) == set(want)
        for t in want:
            assert sum(l for _, l in cover[t]) == sum(l for _, l in want[t])
            assert min(bg for bg, _ in cover[t]) == min(bg for bg, _ in want[t])


def test_chunk_counts_and_groups_of_the_bert_large_configs():
    N = 335_141_888
    # default cuts: 1 024 elements for the read-write passes, 16 Ki for the squared-norm pass (one set of partial
    # sums per chunk).  A squared-norm work item of the fused step reads the largest power of two in [16 Ki, 64 Ki]
    # elements that leaves an average bucket group at least 160 items: 4 chunks for 50 MiB buckets (one per group),
    # 2 for 1 MiB buckets (32 per group of 8 Mi elements), 2 for BERT-Base's 25 MiB ones
    for make, per_item in ((W.config_bert_large, 4), (W.config_bert_large_fp16, 2)):
        w = make()
        p = host_plan(w.layout)
        assert -(-N // 16384) <= p.n_chunks(B.BCA_TABLE_NORM) <= -(-N // 16384) + 2 * w.layout.n_segments
        assert max(p.chunk_info(i, B.BCA_TABLE_NORM)[2] for i in range(0, p.n_chunks(B.BCA_TABLE_NORM), 7)) == 16384
        assert p.norm_item_chunks == per_item
        assert -(-N // 1024) <= p.n_chunks(B.BCA_TABLE_APPLY) <= -(-N // 1024) + 2 * w.layout.n_segments
    assert host_plan(W.config_bert_base().layout).norm_item_chunks == 2
    assert max(host_plan(W.config_bert_base().layout).chunk_info(i, B.BCA_TABLE_NORM)[2] for i in range(100)) == 16384
    assert max(host_plan(W.config_tiny().layout).chunk_info(i, B.BCA_TABLE_NORM)[2] for i in range(3)) == 12345
    assert host_plan(W.config_tiny().layout).norm_item_chunks == 1
    assert host_plan(W.config_bert_base().layout, chunk_norm=32768).norm_item_chunks == 1       # a named chunk: one per item
    assert host_plan(W.config_bert_base().layout, chunk_norm=8192, norm_item_chunks=3).norm_item_chunks == 3
    with pytest.raises(B.BcaError):
        host_plan(W.config_tiny().layout, norm_item_chunks=5)
    assert host_plan(W.config_bert_base().layout, chunk_norm=4096).n_chunks(B.BCA_TABLE_NORM) > 109_482_240 // 4096
    w = W.config_bert_large()
    assert host_plan(w.layout).n_groups == 26                          # default 8 Mi elements: one 50 MiB bucket per group
    assert host_plan(w.layout, group_bytes=110 << 20).n_groups == 13   # two per group
    assert host_plan(W.config_bert_large_multistep().layout).n_groups == 40    # 4 MiB buckets: eight per group
    assert host_plan(W.config_bert_large_fp16().layout, grad_dtype=B.BCA_GRAD_F16).n_groups == 40
    assert host_plan(w.layout, group_bytes=160 << 20).n_groups == 9    # three per group
    assert host_plan(w.layout, group_bytes=1).n_groups == w.layout.n_buckets   # never less than one bucket per group
    assert host_plan(w.layout, group_bytes=1 << 40).n_groups == 1


def _raw_create(numel, off, segs, gdt=0, device=-1, tuning=None):
    L = B.load_library()
    h = C.c_void_p()
    numel = np.asarray(numel, np.uint64)
    off = np.asarray(off, np.uint64)
    arr = (binding._Segment * max(1, len(segs)))()
    for i, (t, b, l) in enumerate(segs):
        arr[i] = binding._Segment(t, 0, b, l)
    rc = L.bca_plan_create(C.byref(h), device, len(numel), numel.ctypes.data_as(C.POINTER(C.c_uint64)), len(off) - 1,
                           off.ctypes.data_as(C.POINTER(C.c_uint64)), arr, gdt, tuning)
    if rc == 0:
        L.bca_plan_destroy(h)
    return rc, L.bca_last_error().decode()


def test_layout_errors_are_reported_and_nothing_is_created():
    ok = _raw_create([10, 5], [0, 2], [(0, 0, 10), (1, 0, 5)])
    assert ok[0] == 0
    rc, msg = _raw_create([10, 5], [0, 2], [(0, 0, 10), (1, 0, 4)])          # gap at the end
    assert rc == -2 and "cover" in msg
    rc, msg = _raw_create([10, 5], [0, 2], [(0, 0, 6), (0, 5, 5), ])          # overlap + tensor 1 missing
    assert rc == -2 and "overlap" in msg
    rc, msg = _raw_create([10], [0, 2], [(0, 0, 4), (0, 5, 5)])               # hole in the middle
    assert rc == -2 and "gap" in msg
    rc, msg = _raw_create([10], [0, 1], [(0, 5, 6)])                          # runs past the end
    assert rc == -2 and "exceeds" in msg
    rc, msg = _raw_create([10], [0, 1], [(3, 0, 10)])                         # unknown tensor
    assert rc == -2
    rc, msg = _raw_create([10], [0, 1, 0], [(0, 0, 10)])                      # offsets decrease
    assert rc == -2
    rc, msg = _raw_create([10], [1, 1], [(0, 0, 10)])                         # offsets do not start at 0
    assert rc == -2
    rc, msg = _raw_create([10], [0], [])                                      # no bucket at all
    assert rc == -2
    rc, msg = _raw_create([10], [0, 1], [(0, 0, 10)], gdt=5)
    assert rc == -7
    for bad in (binding._Tuning(1000, 0, 0, 0, 0, 0, 0), binding._Tuning(0, 1000, 0, 0, 0, 0, 0),
                binding._Tuning(0, 0, 0, 0, 3, 0, 0), binding._Tuning(0, 0, 0, 0, 0, 8, 0)):
        rc, msg = _raw_create([10], [0, 1], [(0, 0, 10)], tuning=C.byref(bad))   # chunk not a multiple of 1024, ...
        assert rc == -3
    # empty buckets, empty segments and empty tensors are legal
    assert _raw_create([10, 0], [0, 0, 3, 3], [(0, 0, 4), (1, 0, 0), (0, 4, 6)])[0] == 0


def test_null_arguments_and_host_only_plans_are_refused_cleanly():
    L = B.load_library()
    assert L.bca_plan_create(None, -1, 0, None, 1, None, None, 0, None) == -1
    assert L.bucket_clip_norms(None, 0, 0, None, None) == -1
    assert L.adam_step(None, None, 1, None) == -1
    p = host_plan(W.layout_one_tensor_per_bucket([8, 8]))
    with pytest.raises(B.BcaError) as e:
        p.bucket_clip_norms(0, 2, 1234)
    assert e.value.code == -5
    with pytest.raises(B.BcaError) as e:
        p.adam_step(B.AdamHyper(), 1)
    assert e.value.code == -5
    with pytest.raises(B.BcaError) as e:
        p.bind([1, 2], [3, 4], [5, 6], [7, 8])
    assert e.value.code == -5
    with pytest.raises(B.BcaError):
        p.chunk_info(10 ** 6)
    L.bca_plan_destroy(None)     # no-op


def test_argument_errors_come_before_any_launch():
    # argument checks run before the plan is asked to launch anything, so a host-only plan shows them
    p = host_plan(W.layout_one_tensor_per_bucket([8, 8]))
    bad = [dict(beta1=1.0), dict(beta1=-0.1), dict(beta2=1.5), dict(beta2=float("nan")), dict(eps=-1e-8),
           dict(lr=float("inf")), dict(weight_decay=float("nan"))]
    for kw in bad:
        with pytest.raises(B.BcaError) as e:
            p.adam_step(B.AdamHyper(**kw), 1)
        assert e.value.code == -4, kw
        with pytest.raises(B.BcaError) as e:
            p.bucket_clip_adam(1234, B.AdamHyper(**kw), 1)
        assert e.value.code == -4, kw
    with pytest.raises(B.BcaError) as e:
        p.adam_step(B.AdamHyper(), 0)                      # steps count from 1
    assert e.value.code == -4
    with pytest.raises(B.BcaError) as e:
        p.bucket_clip_adam(1234, B.AdamHyper(), 1, flags=8)
    assert e.value.code == -3
    with pytest.raises(B.BcaError) as e:
        p.bucket_clip_adam(None, B.AdamHyper(), 1)
    assert e.value.code == -1
    for b0, b1 in [(2, 1), (0, 3), (3, 3)]:
        with pytest.raises(B.BcaError) as e:
            p.bucket_clip_norms(b0, b1, 1234)
        assert e.value.code == -3
        with pytest.raises(B.BcaError) as e:
            p.bucket_clip_apply(b0, b1, 1234, 1234)
        assert e.value.code == -3
        with pytest.raises(B.BcaError) as e:
            p.bucket_clip(b0, b1, 1234)
        assert e.value.code == -3
    with pytest.raises(B.BcaError) as e:
        p.bucket_clip_norms(0, 2, None)
    assert e.value.code == -1
    with pytest.raises(B.BcaError) as e:
        p.bucket_clip_apply(0, 2, None, 1234)
    assert e.value.code == -1
    with pytest.raises(B.BcaError) as e:
        p.bucket_clip(0, 2, None)
    assert e.value.code == -1
    with pytest.raises(B.BcaError) as e:
        p.bucket_clip(0, 2, 1234)
    assert e.value.code == -5


def test_device_hyper_parameters_need_a_device_plan_and_pack_to_the_c_struct():
    import struct
    p = host_plan(W.layout_one_tensor_per_bucket([8, 8]))
    with pytest.raises(B.BcaError) as e:
        p.set_device_hyper(4096)
    assert e.value.code == -5
    raw = B.pack_device_hyper(B.AdamHyper(2e-3, 0.8, 0.99, 1e-7, 0.05), 41)
    assert len(raw) == 48 and struct.unpack("<5dQ", raw) == (2e-3, 0.8, 0.99, 1e-7, 0.05, 41)
    header = open(os.path.join(ROOT, "include", "bca.h")).read()
    body = re.search(r"typedef struct bca_adam_device \{(.*?)\} bca_adam_device;", header, re.S).group(1)
    assert re.sub(r"/\*.*?\*/", "", body, flags=re.S).split() == "double lr, beta1, beta2, eps, weight_decay; uint64_t step;".split()


def test_a_device_plan_fails_loudly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(B.BcaError) as e:
        B.Plan.from_layout(W.layout_one_tensor_per_bucket([8]), device=0)
    assert e.value.code == -6


def test_alg1_thresholds_come_from_the_library():
    """Alg. 1 compares every bucket with c / sqrt(B) (not c / B): evaluated by the C export, the binding forwards."""
    thr = B.alg1_thresholds(1.0, 16)
    assert thr.dtype == np.float32 and thr.shape == (16,) and np.all(thr == np.float32(0.25))
    assert np.all(B.alg1_thresholds(3.0, 9) == np.float32(1.0))
    thr = B.alg1_thresholds(1.0, 1279)
    assert np.all(thr == np.float32(1.0 / np.sqrt(np.float64(1279))))
    assert float(np.sum(thr.astype(np.float64) ** 2)) == pytest.approx(1.0, rel=1e-6)      # sum_b c_b^2 = c^2
    assert np.all(np.isinf(B.alg1_thresholds(float("inf"), 4)))
    assert B.alg1_thresholds(1.0, 0).shape == (0,)
    L = B.load_library()
    for bad in (0.0, -1.0, float("nan")):
        with pytest.raises(B.BcaError) as e:
            B.alg1_thresholds(bad, 4)
        assert e.value.code == -4
    assert L.bca_alg1_thresholds(1.0, 4, None) == -1
    # the oracle's helper, written separately, agrees
    import oracle
    assert np.float32(oracle.alg1_threshold(1.0, 1279)) == thr[0]


@pytest.mark.parametrize("chunk", [1024, 4096])
def test_tensor_major_table_partitions_every_tensor_in_order_and_keeps_chunks_inside_buckets(chunk):
    numels = W.scaled_bert_numels(64, 2, 256, vocab=1000, max_pos=32) + [0, 7, 1]
    lay = W.layout_flat_split(numels, 50_000)
    assert lay.tensors_split() > 0
    p = host_plan(lay, chunk_apply=chunk)
    T = B.BCA_TABLE_LAMB
    owner = [np.full(n, -1, np.int64) for n in numels]          # bucket of every element per the layout
    for b in range(lay.n_buckets):
        for t, beg, ln in lay.segments_of(b):
            owner[t][beg:beg + ln] = b
    total = 0
    for t, n in enumerate(numels):
        f, cnt = p.bucket_chunks(t, T)
        assert f == total
        pos = 0
        for i in range(f, f + cnt):
            tt, beg, ln, b = p.chunk_info(i, T)
            assert tt == t and beg == pos and 0 < ln <= chunk     # contiguous, in order of position
            assert beg // chunk == (beg + ln - 1) // chunk
            assert (owner[t][beg:beg + ln] == b).all()            # one bucket per chunk: one clip coefficient
            pos += ln
        assert pos == n
        total += cnt
    assert total == p.n_chunks(T) == p.n_chunks(B.BCA_TABLE_APPLY)
    with pytest.raises(B.BcaError):
        p.bucket_chunks(len(numels), T)


def test_decay_mask_is_accepted_on_a_host_plan_and_checked_for_length():
    lay = W.layout_one_tensor_per_bucket([5, 6, 7])
    p = host_plan(lay)
    p.set_decay_mask([1, 0, 1])
    p.set_decay_mask(None)
    with pytest.raises(ValueError):
        p.set_decay_mask([1, 0])


def test_bf16_plans_are_accepted_and_unknown_types_are_not():
    lay = W.layout_one_tensor_per_bucket([5, 6, 7])
    host_plan(lay, B.BCA_GRAD_BF16)
    with pytest.raises(B.BcaError) as e:
        host_plan(lay, 3)
    assert e.value.code == -7


@pytest.mark.parametrize("tuning", [{}, {"norm_lead": 1}, {"norm_lead": 2}, {"norm_lead": 5}, {"norm_item_chunks": 1},
                                    {"norm_item_chunks": 4, "group_bytes": 1}, {"group_bytes": 1 << 40},
                                    {"chunk_norm": 2048, "norm_item_chunks": 3, "norm_lead": 3, "group_bytes": 300_000}])
def test_work_list_of_the_fused_step(tuning):
    """What the fused step's forward progress and completeness rest on, checked on the host: every chunk of the norm
    table is in exactly one squared-norm item, an item's chunks lie in one bucket, every chunk of the apply table is
    exactly one Adam item, every bucket without elements has its stand-in, all squared-norm items of a bucket come
    before all of its Adam items, and the squared norms run `norm_lead` bucket groups ahead, no more."""
    rng = np.random.default_rng(11)
    numels = W.scaled_bert_numels(64, 2, 256, vocab=3000, max_pos=32) + [0, 7, 1, 40_000]
    lay = W.layout_flat_split(numels, 30_000)
    p = host_plan(lay, **tuning)
    items = p.work_items()
    nN, nA, nb = p.n_chunks(B.BCA_TABLE_NORM), p.n_chunks(B.BCA_TABLE_APPLY), lay.n_buckets
    bucket_of_norm = [p.chunk_info(i, B.BCA_TABLE_NORM)[3] for i in range(nN)]
    bucket_of_apply = [p.chunk_info(i, B.BCA_TABLE_APPLY)[3] for i in range(nA)]
    seen_norm, seen_apply = np.zeros(nN, int), np.zeros(nA, int)
    last_norm_pos, first_adam_pos = {}, {}
    for pos, (kind, first, count) in enumerate(items):
        if kind == 0:
            assert 1 <= count <= max(p.norm_item_chunks, 1) and first + count <= nN
            assert len({bucket_of_norm[c] for c in range(first, first + count)}) == 1
            seen_norm[first:first + count] += 1
            last_norm_pos[bucket_of_norm[first]] = pos
        elif kind == 1:
            assert count == 1
            seen_apply[first] += 1
            first_adam_pos.setdefault(bucket_of_apply[first], pos)
        else:
            assert kind == 2 and count == 0 and p.bucket_chunks(first, B.BCA_TABLE_NORM)[1] == 0
            last_norm_pos[first] = pos
    assert np.all(seen_norm == 1) and np.all(seen_apply == 1)
    assert set(last_norm_pos) == set(range(nb))                      # every bucket is finalized by somebody
    for b, pos in first_adam_pos.items():
        assert last_norm_pos[b] < pos, f"bucket {b}: an Adam item before the bucket's last squared-norm item"
    # lead: when the first Adam item of the list appears, the squared-norm items of exactly min(lead, groups) groups precede it
    first_adam = min(first_adam_pos.values())
    buckets_normed = {bucket_of_norm[f] if k == 0 else f for k, f, _ in items[:first_adam] if k != 1}
    lead = tuning.get("norm_lead", 0)
    if lead:
        # groups are runs of consecutive buckets; count how many distinct groups the normed buckets span via the plan
        assert len(buckets_normed) >= 1
        if p.n_groups <= lead:
            assert buckets_normed == set(range(nb))
        else:
            assert len(buckets_normed) < nb


def test_runs_of_tensors_for_the_lamb_sweeps():
    """Runs are consecutive, cover every tensor once, hold at most the limit unless a single tensor exceeds it,
    and are as long as the limit allows (the next tensor would not have fitted)."""
    numels = [10, 0, 5000, 300, 300, 9000, 1, 1, 1, 4000, 999]
    lay = W.layout_flat_split(numels, 2000)
    assert host_plan(lay).lamb_runs() == [(0, len(numels))]                    # default limit: far above this model
    assert host_plan(lay, lamb_group_elems=2 ** 63).lamb_runs() == [(0, len(numels))]
    for limit in (1, 600, 5000, 5310, 9000, 20000):
        runs = host_plan(lay, lamb_group_elems=limit).lamb_runs()
        assert runs[0][0] == 0 and runs[-1][1] == len(numels)
        assert all(a[1] == b[0] for a, b in zip(runs, runs[1:])) and all(a < b for a, b in runs)
        for a, b in runs:
            tot = sum(numels[a:b])
            assert tot <= limit or b - a == 1
            if b < len(numels):
                assert tot + numels[b] > limit
    assert host_plan(lay, lamb_group_elems=1).lamb_runs() == [(t, t + 1) for t in range(len(numels))]
    big = host_plan(W.config_bert_large().layout)
    runs = big.lamb_runs()
    assert len(runs) == 11 and sum(b - a for a, b in runs) == 391


def test_the_packages_bucket_layouts_are_valid_and_match_the_test_generators():
    """paper_2402_02447_amd.buckets (what a user builds plans from) against the layouts the tests are written with
    (workloads.py, written separately): the same arrays for random tensor lists and capacities, empty tensors and
    empty models included; and the library accepts them (every element in exactly one segment)."""
    rng = np.random.default_rng(3)
    cases = [([], 10), ([0, 0], 10), ([7], 7), ([7], 3), ([5, 0, 0, 7], 5), ([5, 0], 100), ([0, 5], 2)]
    for _ in range(60):
        n = int(rng.integers(1, 12))
        numels = [int(x) for x in rng.choice([0, 1, 2, 31, 100, 1024, 5000], n)]
        cases.append((numels, int(rng.choice([1, 7, 100, 1024, 3000, 100000]))))
    fields = ("tensor_numel", "bucket_seg_off", "seg_tensor", "seg_begin", "seg_len")
    for numels, cap in cases:
        for rev in (True, False):
            for mine, ref in ((B.flat_split(numels, cap, rev), W.layout_flat_split(numels, cap, rev)),
                              (B.whole_tensors(numels, cap, rev), W.layout_whole_tensors(numels, cap, rev))):
                for f in fields:
                    a, b = getattr(mine, f), getattr(ref, f)
                    assert a.dtype == b.dtype and np.array_equal(a, b), (numels, cap, rev, f, a, b)
                assert mine.n_buckets == ref.n_buckets and mine.n_elements == ref.n_elements
                with host_plan(mine) as p:
                    assert p.n_buckets == mine.n_buckets
    big = B.flat_split(W.bert_large_numels(), 50 * W.MIB // 4)
    assert big.n_buckets == 26 and int(big.bucket_seg_off[-1]) == 416
    with pytest.raises(ValueError):
        B.flat_split([1, 2], 0)
