"""The C-ABI scheduler (host code only, so this runs without a GPU) against
the oracle: the hand-worked trace, and identical decisions on seeded random
traces (integer decisions: bit-exact)."""

import numpy as np
import pytest

from oracle import scheduler_oracle as so
from test_oracle_sched_pins import run_hand_example


@pytest.fixture(scope="module")
def Sched():
    from paper_2503_08461_amd import fastcache
    return fastcache.Scheduler


def test_hand_worked_trace_through_the_c_abi(Sched):
    made = []

    def make(*a):
        made.append(Sched(*a))
        return made[-1]

    run_hand_example(make)
    for s in made:
        s.close()


@pytest.mark.parametrize("seed", range(12))
def test_same_decisions_as_the_oracle_on_random_traces(Sched, seed):
    """Poisson-like arrivals, heterogeneous sizes, a pool whose free count
    moves with the batches formed and with releases, service times fed back."""
    rng = np.random.default_rng(500 + seed)
    b_min = int(rng.integers(1, 5))
    b_max = int(rng.integers(b_min, 20))
    max_wait = int(rng.integers(0, 5000))
    g, o = Sched(b_min, b_max, max_wait), so.Scheduler(b_min, b_max, max_wait)
    now, free, next_id = 0, int(rng.integers(50, 400)), 0
    holding = []                                  # (release time, blocks)
    n_batches = 0
    for step in range(400):
        now += int(rng.exponential(300.0))
        while holding and holding[0][0] <= now:
            free += holding.pop(0)[1]
        if rng.random() < 0.75:
            L = int(rng.integers(1, 7200))
            B = max(1, int(L * rng.uniform(0.05, 1.0)))
            t = now if rng.random() < 0.9 else now - 1     # sometimes out of order: rejected
            a, b = g.submit(next_id, t, L, B), o.submit(next_id, t, L, B)
            assert a == b
            next_id += 1
        assert g.ready(now) == o.ready(now)
        assert g.pending() == len(o.pending)
        bg, bo = g.form_batch(now, free), o.form_batch(now, free)
        assert bg == bo, (seed, step)
        if bg:
            n_batches += 1
            service = int(rng.integers(50, 4000))
            assert g.adjust(service) == o.adjust(service)
            assert g.batch_target() == o.b_target
            # the blocks of the batch stay busy for a while, then come back
            blocks_used = int(rng.integers(0, free + 1))
            free -= blocks_used
            holding.append((now + int(rng.integers(100, 3000)), blocks_used))
            holding.sort()
    assert n_batches > 10
    g.close()


def test_errors(Sched):
    from paper_2503_08461_amd import fastcache as fc
    with pytest.raises(fc.FastCacheError):
        Sched(0, 4, 10)
    with pytest.raises(fc.FastCacheError):
        Sched(5, 4, 10)
    s = Sched(1, 4, 10)
    assert s.submit(7, 100, 10, 5) and not s.submit(7, 100, 10, 5)
    assert not s.submit(8, 99, 10, 5) and not s.submit(8, 100, 10, 11)
    assert s.pending() == 1 and s.form_batch(100, 0) == [] and s.pending() == 1
    assert s.form_batch(100, 1) == [7] and s.pending() == 0
    s.close()
