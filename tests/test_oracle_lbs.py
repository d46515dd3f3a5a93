"""Pins for the load-balancing simulation oracle (Sec. 5.2 "Load balancing effect
simulation", Sec. 4.1, App. C Table 5).

The generator is pinned by SplitMix64's published outputs; sampling by brute force
and degenerate datasets; the scatter patterns by hand-worked examples (Fig. 4's
raster and snake order); the whole simulation by an independent pure-Python
evaluation with exact integer equality, structural identities between the methods,
the bound max - min <= L - 1 that global presorting satisfies by construction, and
the order of the methods in Table 5.  Table 5's absolute numbers need the Wikipedia
length histogram, which the paper does not print: parity unpinned for those."""
import numpy as np
import pytest

import workloads as W
from oracle import lbs

M64 = (1 << 64) - 1
ENDS = W.LENGTH_STRATUM_END


def test_generator_reproduces_published_splitmix64_outputs():
    # first outputs for seed 0 (the values used to seed xoshiro generators in their reference code)
    assert [lbs.splitmix64(0, k) for k in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    # and the widely quoted sequence for seed 1234567
    assert [lbs.splitmix64(1234567, k) for k in range(5)] == [6457827717110365317, 3203168211198807973,
                                                              9817491932198370423, 4593380528125082431,
                                                              16408922859458223821]


def test_length_of_is_the_inverse_of_the_cumulative_histogram():
    hist = [0, 3, 0, 2, 1, 0, 4]                    # lengths 1..6: 3, 0, 2, 1, 0, 4 samples
    cum = np.cumsum(hist)
    expanded = [l for l, n in enumerate(hist) for _ in range(n)]        # the dataset, ordered by length
    assert [lbs.length_of(cum, i) for i in range(len(expanded))] == expanded


def py_draw(cum, stratified, ends, quota, b, G, seed, trial, gpu):
    """Independent statement of the draw in Python integers."""
    def sm(k):
        z = (seed + (k + 1) * 0x9E3779B97F4A7C15) & M64
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
        return z ^ (z >> 31)
    cum = [int(x) for x in cum]
    k0 = (trial * G + gpu) * b
    ranges = [(0, cum[-1])] * b if not stratified else \
        [(cum[0 if s == 0 else ends[s - 1]], cum[ends[s]]) for s in range(len(ends)) for _ in range(int(quota[s]))]
    out = []
    for j, (lo, hi) in enumerate(ranges):
        idx = lo + (((sm(k0 + j) >> 32) * (hi - lo)) >> 32)
        out.append(next(l for l in range(1, len(cum)) if cum[l] > idx))
    return out


def py_simulate(cum, ends, quota, b, P, G, method, seed, n_trials, first=0):
    mins, maxs = [], []
    for trial in range(first, first + n_trials):
        strat = method in (lbs.STRATIFIED, lbs.LOCAL_RASTER, lbs.LOCAL_SNAKE)
        per_gpu = [py_draw(cum, strat, ends, quota, b, G, seed, trial, g) for g in range(G)]
        if method in (lbs.NONE, lbs.STRATIFIED):
            tokens = [sum(x) for x in per_gpu]
        else:
            group = P if method != lbs.GLOBAL else G
            tokens = []
            for n0 in range(0, G, group):
                pool = sorted(x for g in range(n0, n0 + group) for x in per_gpu[g])
                t = [0] * group
                for r in range(b):
                    row = pool[r * group:(r + 1) * group]
                    if method == lbs.LOCAL_SNAKE and r % 2 == 1:
                        row = row[::-1]
                    for c in range(group):
                        t[c] += row[c]
                tokens += t
        mins.append(min(tokens)), maxs.append(max(tokens))
    return mins, maxs


SMALL_CUM = W.length_histogram_piecewise_uniform(20_000, (8, 16, 24, 32), W.LENGTH_STRATUM_SHARE)
SMALL_ENDS = (8, 16, 24, 32)


@pytest.mark.parametrize("stratified", [False, True])
def test_draws_match_the_python_statement_and_respect_the_strata(stratified):
    quota = [3, 1, 0, 4]
    for trial, gpu in [(0, 0), (0, 5), (7, 2), (123456789, 11)]:
        got = lbs.draw(SMALL_CUM, stratified, SMALL_ENDS, quota, 8, 12, 99, trial, gpu)
        assert list(got) == py_draw(SMALL_CUM, stratified, SMALL_ENDS, quota, 8, 12, 99, trial, gpu)
        if stratified:
            want = [s for s, q in enumerate(quota) for _ in range(q)]
            assert [int(np.searchsorted(SMALL_ENDS, l)) for l in got] == want       # quota[s] draws inside stratum s


def test_draws_follow_the_dataset_histogram():
    cum = W.length_histogram_piecewise_uniform()
    got = np.concatenate([lbs.draw(cum, False, ENDS, [16, 0, 0, 0], 16, 64, 5, t, g) for t in range(40) for g in range(64)])
    n = got.size
    hist = np.diff(cum.astype(np.int64)) / float(cum[-1])                 # probability of each length 1..512
    mean = float(np.sum(np.arange(1, 513) * hist))
    var = float(np.sum((np.arange(1, 513) - mean) ** 2 * hist))
    assert abs(got.mean() - mean) < 5 * np.sqrt(var / n)
    share = [np.mean((got > lo) & (got <= hi)) for lo, hi in zip((0,) + ENDS[:-1], ENDS)]
    for s, want in zip(share, W.LENGTH_STRATUM_SHARE):
        assert abs(s - want / sum(W.LENGTH_STRATUM_SHARE)) < 5 * np.sqrt(0.25 / n)
    assert got.min() >= 1 and got.max() <= 512 and len(np.unique(got)) > 500


def test_scatter_hand_worked_raster_and_snake():
    # 16 sequences of lengths 1..16 on 4 GPUs: rows 1-4, 5-8, 9-12, 13-16
    lengths = np.random.default_rng(0).permutation(np.arange(1, 17))
    assert list(lbs.presort_scatter(lengths, 4, 4, snake=False)) == [28, 32, 36, 40]   # column sums
    assert list(lbs.presort_scatter(lengths, 4, 4, snake=True)) == [34, 34, 34, 34]    # rows 2 and 4 reversed
    # three rows on two GPUs: sorted 1 2 | 5 9 | 10 20 -> raster (1+5+10, 2+9+20); snake (1+9+10, 2+5+20)
    assert list(lbs.presort_scatter([9, 1, 20, 5, 2, 10], 2, 3, snake=False)) == [16, 31]
    assert list(lbs.presort_scatter([9, 1, 20, 5, 2, 10], 2, 3, snake=True)) == [20, 27]


def test_scatter_conserves_tokens_and_one_gpu_keeps_everything():
    rng = np.random.default_rng(1)
    for n_group, b in [(8, 16), (3, 5), (1, 7)]:
        lengths = rng.integers(1, 513, n_group * b)
        for snake in (False, True):
            t = lbs.presort_scatter(lengths, n_group, b, snake)
            assert int(t.sum()) == int(lengths.sum())
            if n_group == 1:
                assert int(t[0]) == int(lengths.sum())


@pytest.mark.parametrize("method", [lbs.NONE, lbs.STRATIFIED, lbs.LOCAL_RASTER, lbs.LOCAL_SNAKE, lbs.GLOBAL])
def test_simulation_equals_independent_python_evaluation(method):
    quota = [2, 1, 1, 2]
    tmin, tmax, s0, s1 = lbs.simulate(SMALL_CUM, SMALL_ENDS, quota, 6, 4, 12, method, 2024, 25, first_trial=3)
    wmin, wmax = py_simulate(SMALL_CUM, SMALL_ENDS, quota, 6, 4, 12, method, 2024, 25, first=3)
    assert list(tmin) == wmin and list(tmax) == wmax
    assert s0 == sum(wmin) and s1 == sum(wmax)


def test_structural_identities_between_methods():
    cum, ends = SMALL_CUM, SMALL_ENDS
    one = ([32], [6])                                 # a single stratum holding the whole dataset
    run = lambda method, P, strata=(ends, [2, 1, 1, 2]): lbs.simulate(cum, strata[0], strata[1], 6, P, 12, method, 7, 40)[:2]
    same = lambda a, b: np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert same(run(lbs.STRATIFIED, 4, one), run(lbs.NONE, 4))                  # one stratum = the original dataset
    assert same(run(lbs.LOCAL_RASTER, 12, one), run(lbs.GLOBAL, 4))             # one node spanning all GPUs = global presorting
    assert same(run(lbs.LOCAL_RASTER, 1), run(lbs.STRATIFIED, 4))               # one GPU per node: nothing to redistribute
    assert same(run(lbs.LOCAL_SNAKE, 1), run(lbs.STRATIFIED, 4))
    assert not same(run(lbs.LOCAL_SNAKE, 4), run(lbs.LOCAL_RASTER, 4))
    # trials are independent of how a run is split
    a = lbs.simulate(cum, ends, [2, 1, 1, 2], 6, 4, 12, lbs.LOCAL_SNAKE, 7, 40)
    b1 = lbs.simulate(cum, ends, [2, 1, 1, 2], 6, 4, 12, lbs.LOCAL_SNAKE, 7, 15)
    b2 = lbs.simulate(cum, ends, [2, 1, 1, 2], 6, 4, 12, lbs.LOCAL_SNAKE, 7, 25, first_trial=15)
    assert np.array_equal(a[0], np.concatenate([b1[0], b2[0]])) and a[2] == b1[2] + b2[2] and a[3] == b1[3] + b2[3]


def test_degenerate_dataset_and_bad_arguments():
    cum = np.zeros(513, np.uint32)
    cum[100:] = 1000                                  # every sequence has length 100
    for method in range(5):
        tmin, tmax, s0, s1 = lbs.simulate(cum, [512], [16], 16, 8, 64, method, 1, 5)
        assert list(tmin) == [1600] * 5 == list(tmax) and s0 == s1 == 8000
    with pytest.raises(ValueError):
        lbs.simulate(SMALL_CUM, SMALL_ENDS, [1, 1, 1, 1], 6, 4, 12, lbs.STRATIFIED, 1, 1)     # quota does not add up
    with pytest.raises(ValueError):
        lbs.simulate(SMALL_CUM, SMALL_ENDS, [2, 1, 1, 2], 6, 5, 12, lbs.LOCAL_SNAKE, 1, 1)    # 12 GPUs, nodes of 5
    with pytest.raises(ValueError):
        lbs.simulate(SMALL_CUM, SMALL_ENDS, [2, 1, 1, 2], 6, 4, 12, 5, 1, 1)                  # unknown method


def test_table5_order_of_the_methods_and_global_presorting_bound():
    # 1 024 GPUs, local batch 16, nodes of 8, synthetic histogram with the printed stratum shares
    cum = W.length_histogram_piecewise_uniform()
    quota = W.stratum_quota(cum, ENDS, 16)
    assert list(quota) == [6, 3, 2, 5]
    n = 30
    res = {m: lbs.simulate(cum, ENDS, quota, 16, 8, 1024, m, 11, n) for m in range(5)}
    rng = {m: (res[m][3] - res[m][2]) / n for m in res}            # average max - average min
    assert rng[lbs.NONE] > rng[lbs.STRATIFIED] > rng[lbs.LOCAL_RASTER] > rng[lbs.GLOBAL] > rng[lbs.LOCAL_SNAKE]
    # Table 5's ranges: 4573, 862, 658, 506, 346 -- the stand-in histogram gives the same picture
    assert 3500 < rng[lbs.NONE] < 5500 and 700 < rng[lbs.STRATIFIED] < 1100 and 250 < rng[lbs.LOCAL_SNAKE] < 450
    # dealing a sorted list row by row: a GPU's excess over another is at most the sum of the rows' ranges <= L - 1
    assert np.all(res[lbs.GLOBAL][1].astype(np.int64) - res[lbs.GLOBAL][0] <= 511)
    assert 480 < rng[lbs.GLOBAL] <= 511
    # the paper's quota example (Fig. 3: 5, 2, 3, 6) is accepted too and also narrows the range
    r5 = lbs.simulate(cum, ENDS, [5, 2, 3, 6], 16, 8, 1024, lbs.STRATIFIED, 11, n)
    assert (r5[3] - r5[2]) / n < 0.3 * rng[lbs.NONE]
