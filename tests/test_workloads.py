"""The synthetic layouts: BERT tensor counts and the bucket cuts of the five configurations."""
import numpy as np
import pytest

import workloads as W


def test_bert_tensor_lists_have_the_standard_parameter_counts():
    base, large = W.bert_base_numels(), W.bert_large_numels()
    assert len(base) == 199 and sum(base) == 109_482_240
    assert len(large) == 391 and sum(large) == 335_141_888


@pytest.mark.parametrize("make,B,last,segments,split", [
    (W.config_bert_base, 17, 4_624_640, 215, 14),
    (W.config_bert_large, 26, 7_461_888, 416, 24),
    (W.config_bert_large_fp16, 1279, 121_856, 1668, 147),
    (W.config_bert_large_multistep, 320, 646_144, 710, 146),
])
def test_flat_split_bucket_counts(make, B, last, segments, split):
    w = make()
    lay = w.layout
    assert lay.n_buckets == B and lay.n_segments == segments
    sizes = lay.bucket_numel()
    assert int(sizes[-1]) == last and np.all(sizes[:-1] == sizes[0])
    assert lay.tensors_split() == split
    assert w.thresholds.shape == (B,)


def test_every_element_is_covered_exactly_once_and_order_is_reversed():
    numels = W.scaled_bert_numels(16, 2, 32, vocab=100, max_pos=8)
    for lay in (W.layout_flat_split(numels, 700), W.layout_whole_tensors(numels, 700),
                W.layout_one_tensor_per_bucket(numels)):
        seen = [np.zeros(n, np.int32) for n in numels]
        for b in range(lay.n_buckets):
            for t, beg, ln in lay.segments_of(b):
                seen[t][beg:beg + ln] += 1
        assert all((s == 1).all() for s in seen)
    lay = W.layout_flat_split(numels, 700)
    # bucket 0 starts with the last-registered tensor, the last bucket ends with the first one
    assert int(lay.seg_tensor[0]) == len(numels) - 1 and int(lay.seg_tensor[-1]) == 0


def test_values_are_seeded_and_of_the_stated_scale():
    w = W.config_tiny()
    a, b = w.grads(), w.grads()
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    g = np.concatenate(a)
    assert g.dtype == np.float32 and abs(g.std() - 1e-2) < 5e-4
    p = np.concatenate(w.params())
    assert abs(p.std() - 0.02) < 1e-3
    assert all((x == 0).all() for x in w.exp_avg() + w.exp_avg_sq())
    assert list(w.thresholds) == [np.float32(0.1), np.float32(1.0), np.float32(10.0)]


def test_multistep_gradients_change_every_step_and_thresholds_clip_about_half():
    w = W.config_bert_large_multistep(W.scaled_bert_numels(32, 2, 64, vocab=300, max_pos=16), 4096 * 4)
    g0, g1 = w.grads(0), w.grads(1)
    assert not np.array_equal(g0[0], g1[0])
    assert w.thresholds.min() >= 0.01 and w.thresholds.max() <= 2.0
    full = W.config_bert_large_multistep()
    # expected bucket norm 1e-3*sqrt(2^20) = 1.024: thresholds below it clip
    frac = float(np.mean(full.thresholds < 1.024))
    assert 0.4 < frac < 0.6


def test_fp16_workload_has_many_subnormal_halves():
    w = W.config_bert_large_fp16(W.scaled_bert_numels(32, 2, 64, vocab=300, max_pos=16), 4096)
    g = np.concatenate(w.grads())
    assert g.dtype == np.float16
    sub = np.mean((np.abs(g.astype(np.float32)) < 6.1e-5) & (g != 0))
    assert sub > 0.2
