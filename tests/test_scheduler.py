"""Skip-join MLFQ scheduler and ENST swap order (paper Section 4.1, Algorithm 1, Section
4.2): pins of the Python oracle against hand-worked timelines, closed forms and
invariants, then the C++ scheduler of the library against the oracle decision by
decision on seeded random traffic.  CPU only.

The paper's own worked example (Figure 7: average latencies 4.23 / 5 / 3.3 / 3 under
FCFS / MLFQ / skip-join MLFQ / SRPT) cannot serve as a pin: the job sizes are only in
the figure, which the available text does not contain -- parity unpinned for it."""
import math

import numpy as np
import pytest

from oracle.scheduler import SkipJoinMLFQ, simulate_single_server

INF = 1e30


# ---- oracle pins ------------------------------------------------------------------
def test_skip_join_places_a_job_in_the_first_queue_whose_quantum_covers_its_first_iteration():
    s = SkipJoinMLFQ(6, 1.0, 1, INF, 4)
    assert s.q == [1, 2, 4, 8, 16, 32]
    for t in (0.2, 1.0, 1.01, 2.0, 3.9, 4.0, 4.1, 31.9, 32.0, 500.0):
        want = min(6, max(1, math.ceil(math.log2(t)) + 1)) if t > 1 else 1
        assert s.queue_for(t) == want, t


def test_hand_worked_timeline_three_jobs_quanta_1_2_4_8():
    # J1: first iteration 4, then 2 decode iterations of 1; J2, J3: first iteration 1,
    # then 1 decode iteration of 1.  One job per iteration, no starvation promotion.
    # Skip-join: J1 -> Q3, J2 and J3 -> Q1.  J2 runs [0,1) and is demoted to Q2, J3 runs
    # [1,2) and follows it; Q2: J2 [2,3) done, J3 [3,4) done; Q3: J1 [4,8), demoted to Q4,
    # [8,9), [9,10) done.
    s = SkipJoinMLFQ(4, 1.0, 1, INF, 1)
    jobs = [dict(id=1, init=4, decode=1, n_decode=2), dict(id=2, init=1, decode=1, n_decode=1),
            dict(id=3, init=1, decode=1, n_decode=1)]
    done = simulate_single_server(s, jobs)
    assert done == {2: 3.0, 3: 4.0, 1: 10.0}
    # first come first served (one queue) blocks the short jobs behind J1: 6, 8, 10
    fcfs = simulate_single_server(SkipJoinMLFQ(1, 100.0, 1, INF, 1), jobs)
    assert fcfs == {1: 6.0, 2: 8.0, 3: 10.0}
    assert sum(done.values()) / 3 < sum(fcfs.values()) / 3


def test_single_queue_is_first_come_first_served():
    rng = np.random.default_rng(0)
    jobs = [dict(id=i, init=float(rng.integers(1, 5)), decode=1.0, n_decode=int(rng.integers(0, 4))) for i in range(8)]
    done = simulate_single_server(SkipJoinMLFQ(1, 1000.0, 1, INF, 1), jobs)
    t, want = 0.0, {}
    for j in jobs:
        t += j["init"] + j["n_decode"] * j["decode"]
        want[j["id"]] = t
    assert done == want


def test_quantum_use_demotes_by_eta_and_never_above_the_next_iteration_time():
    s = SkipJoinMLFQ(5, 1.0, 2, INF, 1)
    s.add_job(7, 1.0, 1.0)                     # Q1
    s.complete_iteration([7], 1.0, [])         # used 1 >= q1 -> Q3 (eta = 2)
    assert s.jobs[7].priority == 3 and s.jobs[7].used == 0
    s.complete_iteration([7], 1.0, [])         # used 1 < q3 = 4: stays
    assert s.jobs[7].priority == 3 and s.jobs[7].used == 1
    s2 = SkipJoinMLFQ(5, 1.0, 1, INF, 1)
    s2.add_job(8, 0.5, 7.0)                    # first iteration fits Q1, decode needs q >= 7 -> Q4
    s2.complete_iteration([8], 1.0, [])
    assert s2.jobs[8].priority == 4


def test_starved_jobs_are_promoted_to_the_first_queue():
    s = SkipJoinMLFQ(4, 1.0, 1, 3.0, 1)
    s.add_job(1, 1.0, 1.0)    # Q1
    s.add_job(2, 8.0, 1.0)    # Q4
    for _ in range(2):
        s.complete_iteration(s.schedule(), 1.0, [])
    assert s.jobs[2].priority == 4 and s.jobs[2].starve == 2.0
    s.complete_iteration(s.schedule(), 1.0, [])          # job 2 has now waited 3 = alpha
    assert s.jobs[2].priority == 1 and s.jobs[2].starve == 0.0
    assert s.schedule() == [2]                             # job 1 sits in Q3 by now


def test_enst_hand_example():
    # quanta 1,2,4,8, B = 2, alpha = 10: a in Q1, b in Q2, c in Q4
    s = SkipJoinMLFQ(4, 1.0, 1, 10.0, 2)
    s.add_job(1, 1.0, 1.0), s.add_job(2, 2.0, 1.0), s.add_job(3, 8.0, 1.0)
    assert [s.jobs[i].priority for i in (1, 2, 3)] == [1, 2, 4]
    assert s.t_execute(1) == 0.0
    assert s.t_execute(2) == (1.0) / 2                      # job 1 passes Q1
    assert s.t_execute(3) == ((1 + 2 + 4) + (2 + 4)) / 2    # job 1 passes Q1..Q3, job 2 passes Q2..Q3
    s.jobs[3].starve = 7.0
    assert s.t_promote(3) == 3.0 and s.enst(3) == 3.0       # promotion comes first
    assert s.swap_out_order([1, 2, 3]) == [3, 2, 1]
    assert s.swap_in_order([1, 2, 3]) == [1, 2, 3]


def drive(s, rng, steps, on_step=None):
    next_id = 0
    live = {}
    for it in range(steps):
        for _ in range(int(rng.integers(0, 3))):
            s.add_job(next_id, float(rng.choice([0.3, 1.0, 2.5, 7.0, 30.0])), float(rng.choice([0.5, 1.0, 1.5])))
            live[next_id] = int(rng.integers(1, 12))
            next_id += 1
        for jid in list(live):
            if rng.random() < 0.15:
                s.set_ready(jid, bool(rng.integers(0, 2)))
        batch = s.schedule()
        elapsed = float(rng.choice([0.5, 1.0, 2.0]))
        fin = []
        for jid in batch:
            live[jid] -= 1
            if live[jid] == 0:
                fin.append(jid)
                del live[jid]
        if on_step:
            on_step(batch, elapsed, fin, list(live))
        s.complete_iteration(batch, elapsed, fin)


def test_invariants_under_random_traffic():
    s = SkipJoinMLFQ(5, 1.0, 1, 6.0, 3)
    rng = np.random.default_rng(1)

    def check(batch, elapsed, fin, live):
        assert len(batch) <= 3 and len(set(batch)) == len(batch)
        assert all(s.jobs[j].ready for j in batch)
        placed = [j for Q in s.queues for j in Q]
        assert sorted(placed) == sorted(s.jobs)                       # every job in exactly one queue
        for k, Q in enumerate(s.queues, start=1):
            assert all(s.jobs[j].priority == k for j in Q)
        # priority order: nothing ready and unscheduled sits above a scheduled job's queue
        if batch and len(batch) == 3:
            worst = max(s.jobs[j].priority for j in batch)
            for j in s.jobs:
                if s.jobs[j].ready and j not in batch:
                    assert s.jobs[j].priority >= worst
    drive(s, rng, 300, check)


# ---- the library's scheduler against the oracle ---------------------------------------
@pytest.fixture(scope="module")
def fs_sched():
    import os
    import paper_2305_05920_amd as fs
    if not os.path.exists(fs.LIB_PATH):
        from paper_2305_05920_amd import build
        build.build_library()
    from paper_2305_05920_amd import sched
    return sched


@pytest.mark.parametrize("seed,nq,eta,alpha,B", [(0, 4, 1, 5.0, 2), (1, 6, 2, 3.0, 4), (2, 1, 1, 2.0, 3), (3, 8, 1, 1e9, 8)])
def test_library_scheduler_makes_the_oracles_decisions(fs_sched, seed, nq, eta, alpha, B):
    ora = SkipJoinMLFQ(nq, 1.0, eta, alpha, B)
    lib = fs_sched.Scheduler(nq, 1.0, eta, alpha, B)

    class Both:
        """Feeds both schedulers the same events and compares every decision."""
        jobs = ora.jobs

        def add_job(self, jid, a, b):
            assert lib.add_job(jid, a, b) == ora.add_job(jid, a, b)

        def set_ready(self, jid, r):
            ora.set_ready(jid, r), lib.set_ready(jid, r)

        def schedule(self):
            a, b = ora.schedule(), lib.schedule()
            assert a == b
            return a

        def complete_iteration(self, batch, elapsed, fin):
            ora.complete_iteration(batch, elapsed, fin), lib.complete_iteration(batch, elapsed, fin)
            assert lib.num_jobs() == len(ora.jobs)
            ids = sorted(ora.jobs)
            for j in ids:
                p, used, starve, it = lib.job_info(j)
                o = ora.jobs[j]
                assert (p, used, starve, it) == (o.priority, o.used, o.starve, o.iterations)
                tp, te, en = lib.enst(j)
                assert (tp, te, en) == (ora.t_promote(j), ora.t_execute(j), ora.enst(j))
            assert lib.swap_order(ids, False) == ora.swap_out_order(ids)
            assert lib.swap_order(ids, True) == ora.swap_in_order(ids)

    drive(Both(), np.random.default_rng(seed), 200)
    lib.close()


def test_library_scheduler_rejects_bad_arguments(fs_sched):
    import paper_2305_05920_amd as fs
    with pytest.raises(fs.FsError):
        fs_sched.Scheduler(0, 1.0, 1, 1.0, 1)
    s = fs_sched.Scheduler(3, 1.0, 1, 1.0, 2)
    s.add_job(1, 1.0, 1.0)
    with pytest.raises(fs.FsError):
        s.add_job(1, 1.0, 1.0)                  # duplicate id
    with pytest.raises(fs.FsError):
        s.set_ready(99, True)                   # unknown job
    with pytest.raises(fs.FsError):
        s.complete_iteration([1], 1.0, [2])     # finished job that did not run
    s.close()
