"""Pins of the scheduler oracle (oracle/scheduler_oracle.py) against things
other than itself: a hand-worked trace, exhaustive search on tiny queues,
closed forms of the running averages."""

import itertools
import os

import numpy as np
import pytest

from conftest import ROOT
from oracle import scheduler_oracle as so


def _hand_ops():
    path = os.path.join(ROOT, "tests", "golden", "scheduler_hand_example.txt")
    ops = []
    for line in open(path):
        line = line.split("#")[0].split()
        if line:
            ops.append(line)
    return ops


def run_hand_example(make):
    """Shared with the C-ABI test: `make(b_min, b_max, max_wait)` returns an
    object with submit(id, t, L, B) and form_batch(now, free)."""
    s = make(2, 3, 100)
    n_forms = 0
    for op in _hand_ops():
        if op[0] == "submit":
            assert s.submit(int(op[1]), int(op[2]), int(op[3]), int(op[4]))
        else:
            want = [] if op[3] == "-" else [int(x) for x in op[3:]]
            assert list(s.form_batch(int(op[1]), int(op[2]))) == want, op
            n_forms += 1
    assert n_forms == 7


def test_hand_worked_trace():
    run_hand_example(so.Scheduler)


@pytest.mark.parametrize("seed", range(20))
def test_largest_batch_that_fits_against_exhaustive_search(seed):
    """Without overdue requests the batch must have the largest number of
    requests of any subset that fits (memory and B_max) and, among those, the
    smallest total need."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 10))
    b_max = int(rng.integers(1, 8))
    s = so.Scheduler(1, b_max, 10**9)
    budgets = rng.integers(1, 200, size=n)
    for i in range(n):
        assert s.submit(i, i, 200, int(budgets[i]))
    free = int(rng.integers(0, 40))
    need = [so.blocks(b) for b in budgets]
    best = (0, 0)
    for k in range(1, min(n, b_max) + 1):
        for sub in itertools.combinations(range(n), k):
            tot = sum(need[i] for i in sub)
            if tot <= free and (k, -tot) > (best[0], -best[1]):
                best = (k, tot)
    batch = s.form_batch(n, free)
    assert len(batch) == best[0]
    assert sum(need[i] for i in batch) == best[1]
    assert batch == sorted(batch)                      # arrival order
    assert len(s.pending) == n - len(batch)


def test_trigger_threshold_and_wait_time():
    s = so.Scheduler(3, 8, 50)
    s.submit(1, 0, 100, 10)
    s.submit(2, 10, 100, 10)
    assert not s.ready(49) and s.form_batch(49, 100) == []
    assert s.ready(50)                                 # oldest has waited max_wait
    s.submit(3, 20, 100, 10)
    assert s.ready(20)                                 # |Q| >= b_target
    assert s.form_batch(20, 100) == [1, 2, 3]
    assert not s.ready(10**9)                          # empty queue never fires


def test_rejected_submissions_change_nothing():
    s = so.Scheduler(1, 4, 10)
    assert s.submit(1, 100, 50, 50)
    assert not s.submit(2, 99, 50, 10)                 # arrival before the last one
    assert not s.submit(3, 100, 50, 51)                # budget above the length
    assert not s.submit(3, 100, 50, 0)
    assert not s.submit(1, 100, 50, 10)                # id still pending
    assert [p[1] for p in s.pending] == [1] and s.gap_avg == 0


def test_running_averages_and_target():
    s = so.Scheduler(2, 16, 10**9)
    for i in range(10):
        s.submit(i, 1000 * i, 64, 16)
    assert s.gap_avg == 1000                           # constant input: the average is the input
    assert s.adjust(4500) == 5                         # ceil(4500 / 1000), first sample sets it
    # step response: avg += floor((x - avg) / 4)
    assert s.adjust(8500) == 6 and s.svc_avg == 5500
    assert s.adjust(100) == 5 and s.svc_avg == 5500 + (100 - 5500) // 4
    for _ in range(40):
        s.adjust(100)
    assert s.b_target == 2                             # clamped below by B_min
    for _ in range(40):
        s.adjust(10**6)
    assert s.b_target == 16                            # and above by B_max
    t = so.Scheduler(3, 9, 0)
    assert t.adjust(500) == 3                          # no arrival gap yet: B_min
