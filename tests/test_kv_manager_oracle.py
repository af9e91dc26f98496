"""Oracle of the cache manager and iteration loop (paper Sections 3.2 and 4.2) against what the
paper and plain bookkeeping fix: hand-worked cases, the swap order of Section 4.2, deferred
release, the idle reserve's behaviour under bursts, and conservation of blocks and slots under
random traffic.  No library code runs here."""
import os

import numpy as np
import pytest

from oracle.kv_manager import (IterationLoop, LEAVING, ProactiveCacheManager, RESIDENT, RETURNING, SWAPPED_OUT)
from oracle.scheduler import SkipJoinMLFQ


# ---- the oracle, pinned by hand-worked cases and invariants -------------------------------
def small(reserve=0, blocks=8, slots=8, **kw):
    s = SkipJoinMLFQ(4, 1.0, 1, 100.0, 2)
    return s, ProactiveCacheManager(s, blocks, slots, 16, 4, reserve_idle_blocks=reserve, **kw)


def test_blocks_are_handed_out_in_order_and_counted_by_the_paper_formula():
    s, k = small()
    assert [k.blocks_needed(t) for t in (0, 1, 16, 17, 64)] == [0, 1, 1, 2, 4]
    assert k.admit(1, 33) and k.jobs[1].blocks == [0, 1, 2]            # 33 tokens: 3 blocks of 16
    assert k.admit(2, 16) and k.jobs[2].blocks == [3]
    assert not k.admit(3, 65)                                           # 5 blocks > table width 4
    assert not k.admit(3, 64 + 16) and 3 not in k.jobs
    k.advance(2, 16)
    assert k.grow(2, 1) and k.jobs[2].blocks == [3, 4]                  # token 17 needs a second block
    assert k.grow(1, 5) and k.jobs[1].blocks == [0, 1, 2]               # room already there: nothing taken
    k.release(1)
    assert k.admit(4, 1) and k.jobs[4].blocks == [0]                    # the lowest free id goes first
    assert k.admit(5, 40) and k.jobs[5].blocks == [1, 2, 5]             # neighbours where there are any


def test_swap_out_takes_the_latest_next_scheduled_job_and_swap_in_the_earliest():
    # three idle jobs in queues 1, 2, 3 (init times 1, 2, 4 with q1 = 1): the job in the lowest
    # queue has the largest estimated next scheduled time and leaves first (Section 4.2)
    s, k = small(blocks=6)
    for j, t in ((1, 1.0), (2, 2.0), (3, 4.0)):
        assert k.admit(j, 32)
        s.add_job(j, t, 1.0)
    assert [s.jobs[j].priority for j in (1, 2, 3)] == [1, 2, 3]
    assert k.start_swaps(running=[], want_free=2) == [("out", 3)]
    assert k.jobs[3].where == LEAVING and k.jobs[3].slots == [0, 1] and not s.jobs[3].ready
    assert len(k.free_blocks) == 0                                      # vacated blocks are not free yet
    assert k.retire() == 1 and k.jobs[3].where == SWAPPED_OUT and sorted(k.free_blocks) == [4, 5]
    assert k.start_swaps(running=[], want_free=4) == [("out", 2)] and k.retire() == 1
    # both are out; room for one: the job in the higher queue returns first
    assert k.start_swaps(running=[], want_free=2) == [("in", 2)]
    assert k.jobs[2].where == RETURNING and not s.jobs[2].ready
    k.retire()
    assert k.jobs[2].where == RESIDENT and s.jobs[2].ready and sorted(k.free_slots) == [2, 3, 4, 5, 6, 7]


def test_running_jobs_never_leave_and_a_job_that_does_not_fit_the_host_is_passed_over():
    s, k = small(blocks=8, slots=2)
    for j, n in ((1, 48), (2, 32), (3, 16)):                            # 3, 2, 1 blocks
        k.admit(j, n)
        s.add_job(j, 1.0, 1.0)
    moves = k.start_swaps(running=[2], want_free=8)
    assert ("out", 2) not in moves and ("out", 1) not in moves          # 2 runs; 1 needs 3 slots of 2
    assert moves == [("out", 3)]


def test_release_during_a_move_waits_for_the_move():
    s, k = small(blocks=4)
    k.admit(1, 32)
    s.add_job(1, 1.0, 1.0)
    k.start_swaps([], 4)
    assert k.jobs[1].where == LEAVING
    k.release(1)
    assert 1 in k.jobs and len(k.free_blocks) == 2 and len(k.free_slots) == 6    # nothing returned yet
    k.retire()
    assert 1 not in k.jobs and len(k.free_blocks) == 4 and len(k.free_slots) == 8


def test_idle_reserve_follows_the_arrival_history():
    # more frequent bursts never reserve less; quiet traffic reserves little; old bursts are forgotten
    def reserve_after(demands, **kw):
        s, k = small(blocks=200, **kw)
        for d in demands:
            k.observe_arrivals(d)
        return k.reserve
    quiet = [2 if i % 10 == 0 else 0 for i in range(50)]
    bursty = [40 if i % 5 == 0 else 0 for i in range(50)]
    assert reserve_after(quiet, reserve_window=50, reserve_quantile=0.9) <= 2
    assert reserve_after(bursty, reserve_window=50, reserve_quantile=0.9) == 40
    last = -1
    for period in (40, 20, 10, 5, 2):
        r = reserve_after([30 if i % period == 0 else 0 for i in range(40)], reserve_window=40, reserve_quantile=0.9)
        assert r >= last
        last = r
    assert last == 30
    assert reserve_after([100] + [0] * 8, reserve_window=8, reserve_quantile=1.0, reserve=1) == 1
    assert reserve_after([500], reserve_window=4, reserve_quantile=1.0) == 100       # never more than half the pool
    assert reserve_after([7, 9], reserve_window=0) == 0                              # no window: the fixed reserve


def check_conservation(k):
    owned = sum(len(c.blocks) for c in k.jobs.values())
    held = sum(len(c.slots) for c in k.jobs.values())
    moving_b = sum(len(m["vacated"]) for m in k.moves if m["out"])
    moving_s = sum(len(m["vacated"]) for m in k.moves if not m["out"])
    assert owned + moving_b + len(k.free_blocks) == k.N
    all_b = list(k.free_blocks) + [b for c in k.jobs.values() for b in c.blocks] + \
        [b for m in k.moves if m["out"] for b in m["vacated"]]
    assert sorted(all_b) == list(range(k.N))                            # every block exactly once
    return held + moving_s


class OracleWorld:
    """The oracle's scheduler and manager behind one event interface."""

    def __init__(self, s, k):
        self.s, self.k = s, k

    def admit(self, j, tokens, init_time):
        ok = self.k.admit(j, tokens)
        if ok:
            self.s.add_job(j, init_time, 1.0)
        return ok

    def grow(self, j, n):
        ok = self.k.grow(j, n)
        if ok:
            self.k.advance(j, n)
        return ok

    def iteration(self, elapsed):
        batch = self.s.schedule()
        self.s.complete_iteration(batch, elapsed, [])
        return batch

    def start_swaps(self, want):
        running = self.s.schedule()
        return running, self.k.start_swaps(running, want)

    def retire(self, n):
        return self.k.retire(n)

    def observe(self, d):
        self.k.observe_arrivals(d)

    def release(self, j):
        self.k.release(j)
        self.s.set_ready(j, True)                  # the scheduler forgets a job through an iteration it finishes in
        self.s.complete_iteration([j], 0.0, [j])


def random_drive(world, rng, steps):
    """Random admissions, growth, scheduler iterations, swaps, completions and releases."""
    k = world.k
    nxt, live = 0, []
    for step in range(steps):
        # admissions while few jobs live, otherwise growth, iterations, swaps, retirements, arrivals, releases
        ev = 0 if len(live) < 4 else int(rng.choice([0, 0, 1, 2, 3, 3, 4, 4, 5, 6, 6]))
        if ev == 0 or not live:
            if world.admit(nxt, int(rng.integers(1, 60)), float(rng.choice([0.5, 1.0, 3.0, 9.0]))):
                live.append(nxt)
            nxt += 1
        elif ev == 1:
            j = int(rng.choice(live))
            if k.jobs[j].where == RESIDENT and not k.jobs[j].released:
                world.grow(j, int(rng.integers(1, 20)))
        elif ev == 2:
            world.iteration(float(rng.choice([0.5, 1.0, 2.0])))
        elif ev == 3:
            world.start_swaps(int(rng.choice([0, 0, 4, 10])))
        elif ev == 4:
            world.retire(int(rng.integers(-1, 3)))
        elif ev == 5:
            world.observe(int(rng.integers(0, 12)))
        else:
            j = int(rng.choice(live))
            live.remove(j)
            world.release(j)
        check_conservation(k)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_oracle_conserves_blocks_and_slots_under_random_traffic(seed):
    s = SkipJoinMLFQ(4, 1.0, 1, 6.0, 3)
    k = ProactiveCacheManager(s, 24, 30, 16, 6, reserve_idle_blocks=2, reserve_window=8, reserve_quantile=0.75)
    random_drive(OracleWorld(s, k), np.random.default_rng(seed), 600)
    k.retire()
    held = check_conservation(k)
    assert held + len(k.free_slots) == 30
    assert k.blocks_out > 0 and k.blocks_in > 0, "the drive did not exercise swapping"
