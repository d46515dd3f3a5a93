"""A host-side model of the fused step's waiting scheme, run on the work list the library really builds (CPU only).

The kernels cannot be run here, and no GPU test may force the hardware to start workgroups in a bad order.  What can
be checked on the CPU is the scheme itself: the rules by which the items of one launch arrive, wait, give up and are
completed by the finish kernel are restated below as a small discrete-event model (written from the description in
bca.h and the kernels' comments; it shares no code with them), and that model is driven with the plan's own work
list under start orders and residency limits chosen to be as bad as possible: reversed, random, one workgroup at
a time, every slot taken by Adam items whose squared norms have not started.

Claims checked for every schedule: the launch ends (no order lets waiting items block the items they wait for, once
waits are bounded); every squared-norm chunk is summed once and every bucket finalized once; every Adam chunk is carried
out exactly once, either by its own item or by the finish kernel; an Adam item never runs before its bucket's
coefficient exists; the skipped list never holds more than one entry per Adam chunk; the state the next call starts
from (arrival counters, abort word, skipped count, epoch) is what a first call finds.  With unbounded waits the same
model deadlocks under the bad schedules, which shows that the model is able to see the problem the bound removes."""
import numpy as np
import pytest

import paper_2402_02447_amd as B
import workloads as W

N, A, E = 0, 1, 2        # item kinds as bca_plan_work_item reports them


def host_plan(lay, **tuning):
    return B.Plan.from_layout(lay, B.BCA_GRAD_F32, device=-1, **tuning)


class Model:
    """State of one plan across calls, and one launch of the step kernel plus its finish kernel."""

    def __init__(self, plan, n_buckets):
        self.items = plan.work_items()
        nN, nA = plan.n_chunks(B.BCA_TABLE_NORM), plan.n_chunks(B.BCA_TABLE_APPLY)
        self.bucket_of_norm = [plan.chunk_info(i, B.BCA_TABLE_NORM)[3] for i in range(nN)]
        self.bucket_of_apply = [plan.chunk_info(i, B.BCA_TABLE_APPLY)[3] for i in range(nA)]
        self.total = [plan.bucket_chunks(b, B.BCA_TABLE_NORM)[1] for b in range(n_buckets)]
        self.nb, self.nN, self.nA = n_buckets, nN, nA
        # what lives in device memory between calls
        self.arrived = [0] * n_buckets
        self.ready_epoch = [0] * n_buckets
        self.epoch, self.abort, self.skipped = 1, 0, []

    def launch(self, order, slots, spin_limit, norm_ticks=3, max_ticks=10_000_000):
        """Workgroups start in `order` (a permutation of the item indices) as slots become free; at most `slots` are
        resident.  A resident squared-norm item needs `norm_ticks` ticks, then arrives; a resident Adam item looks at
        its bucket's ready word once per tick.  spin_limit None = wait for ever.  Returns False on deadlock."""
        epoch = self.epoch
        summed = np.zeros(self.nN, int)
        applied = np.zeros(self.nA, int)
        finalized = np.zeros(self.nb, int)
        timed_out = False
        resident = []                                   # [item index, ticks or polls so far]
        nxt, tick = 0, 0
        while nxt < len(order) or resident:
            tick += 1
            if tick > max_ticks:
                return None
            while nxt < len(order) and len(resident) < slots:
                resident.append([order[nxt], 0])
                nxt += 1
            progressed = False
            still = []
            for w in resident:
                kind, first, count = self.items[w[0]]
                if kind == A:
                    b = self.bucket_of_apply[first]
                    if self.ready_epoch[b] == epoch:
                        applied[first] += 1             # coefficient exists: carry out and leave
                        progressed = True
                        continue
                    w[1] += 1
                    if (spin_limit is not None and w[1] > spin_limit) or self.abort:
                        self.abort, timed_out = 1, True
                        self.skipped.append(first)
                        progressed = True
                        continue
                    still.append(w)
                else:
                    w[1] += 1
                    progressed = True                   # squared-norm items never wait
                    if kind == N and w[1] < norm_ticks:
                        still.append(w)
                        continue
                    b = self.bucket_of_norm[first] if kind == N else first
                    if kind == N:
                        summed[first:first + count] += 1
                        self.arrived[b] += count
                        last = self.arrived[b] == self.total[b]
                    else:
                        last = True                     # a bucket without elements: its stand-in finalizes at once
                    if last:
                        self.arrived[b] = 0
                        finalized[b] += 1
                        self.ready_epoch[b] = epoch
            resident = still
            if not progressed and spin_limit is None and (nxt >= len(order) or len(resident) >= slots):
                return False                            # everybody resident waits for ever and nobody else can start
        # the finish kernel: one workgroup, after the launch has ended
        assert len(self.skipped) <= self.nA
        for first in self.skipped:
            assert self.ready_epoch[self.bucket_of_apply[first]] == epoch, "a skipped item whose coefficient is missing"
            applied[first] += 1
        self.skipped, self.abort = [], 0
        self.epoch = epoch + 1 if epoch + 1 < 2 ** 32 else 1
        return dict(summed=summed, applied=applied, finalized=finalized, timed_out=timed_out, ticks=tick)

    def check(self, r):
        assert r, "the launch did not end"
        assert np.all(r["summed"] == 1), "a squared-norm chunk summed twice or not at all"
        assert np.all(r["finalized"] == 1), "a bucket finalized twice or not at all"
        assert np.all(r["applied"] == 1), "an Adam chunk carried out twice or not at all"
        assert self.arrived == [0] * self.nb and self.abort == 0 and self.skipped == []


def small_plan(**tuning):
    numels = W.scaled_bert_numels(32, 2, 128, vocab=500, max_pos=16) + [0, 7, 1, 9_000]
    lay = W.layout_flat_split(numels, 12_000)
    return host_plan(lay, chunk_norm=1024, **tuning), lay


def orders(m, rng):
    n = len(m.items)
    ident = list(range(n))
    yield "in order", ident
    yield "reversed", ident[::-1]
    yield "random", [int(i) for i in rng.permutation(n)]
    yield "adam first", adam_first(m)


def adam_first(m):
    """Every Adam item before any squared-norm item."""
    return sorted(range(len(m.items)), key=lambda i: (m.items[i][0] != A, i))


@pytest.mark.parametrize("tuning", [{}, {"norm_lead": 2}, {"norm_item_chunks": 4, "group_bytes": 1}])
def test_every_schedule_ends_and_every_chunk_is_done_once(tuning):
    plan, lay = small_plan(**tuning)
    rng = np.random.default_rng(5)
    m = Model(plan, lay.n_buckets)
    n = len(m.items)
    assert m.nA > 50 and m.nN > 20 and lay.n_buckets >= 5
    for name, order in orders(m, rng):
        for slots in (1, 2, 7, 64, n):
            for spin in (1, 5, 200):
                r = m.launch(order, slots, spin)
                m.check(r)
                # in the intended order with room for everything nobody waits long enough to give up
                if name == "in order" and spin == 200:
                    assert not r["timed_out"], (name, slots)
    # the state carries over: the epoch has moved once per call, and an old ready word is never taken for a new one
    assert m.epoch == 1 + 4 * 5 * 3


def test_in_order_start_never_times_out_whatever_the_residency():
    """When workgroups start in list order, everything an Adam item waits for has already been started, so it is
    resident or done: the wait is bounded by the squared-norm items' own duration and no bound is needed."""
    plan, lay = small_plan()
    m = Model(plan, lay.n_buckets)
    for slots in (1, 3, 16, 1000):
        r = m.launch(list(range(len(m.items))), slots, spin_limit=None)
        m.check(r)
        assert not r["timed_out"]


def test_without_the_bound_a_bad_order_deadlocks_in_the_model():
    """The model sees the problem that the bounded wait removes: Adam items that take every slot before their squared
    norms have started wait for ever."""
    plan, lay = small_plan()
    m = Model(plan, lay.n_buckets)
    assert m.launch(adam_first(m), slots=8, spin_limit=None) is False
    m2 = Model(plan, lay.n_buckets)
    m2.check(m2.launch(adam_first(m2), slots=8, spin_limit=3))


def test_an_old_ready_word_is_not_taken_for_this_calls():
    """Second call on the same plan, Adam items first: the ready words still hold the previous epoch and must not let
    an Adam item through before this call's squared norms exist (the model's applied-before-finalized check is the
    epoch comparison itself, so plant the mistake and see the model object to it)."""
    plan, lay = small_plan()
    m = Model(plan, lay.n_buckets)
    n = len(m.items)
    m.check(m.launch(list(range(n)), 64, 50))
    stale = list(m.ready_epoch)
    r = m.launch(adam_first(m), 8, 2)
    m.check(r)
    assert r["timed_out"]                                    # they had to wait: the old words did not count
    assert all(e == 1 for e in stale) and all(e == 2 for e in m.ready_epoch)
