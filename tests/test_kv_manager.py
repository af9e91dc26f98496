"""The library's cache manager and iteration loop (paper Sections 3.2 and 4.2), through the C ABI
and without a GPU (a manager without layer pools keeps the books and issues no copies), against
the oracle decision by decision: the same events go to both, and after every event the free
lists, the reserve, every job's state, length and block ids, and the scheduler's next batch must
agree."""
import os

import numpy as np
import pytest

from oracle.kv_manager import IterationLoop, ProactiveCacheManager, RESIDENT, RETURNING
from oracle.scheduler import SkipJoinMLFQ
from tests.test_kv_manager_oracle import OracleWorld, random_drive


# ---- the library against the oracle ---------------------------------------------------------
@pytest.fixture(scope="module")
def fs():
    import paper_2305_05920_amd as fs
    if not os.path.exists(fs.LIB_PATH):
        from paper_2305_05920_amd import build
        build.build_library()
    return fs


def compare_managers(k, lib_k, lib_s, s):
    assert lib_k.free_blocks == len(k.free_blocks) and lib_k.free_slots == len(k.free_slots)
    assert lib_k.reserve == k.reserve
    out, back, flying = lib_k.stats()
    assert (out, back, flying) == (k.blocks_out, k.blocks_in, len(k.moves))
    for j, c in k.jobs.items():
        if c.released:
            continue
        state, length, ids = lib_k.job_info(j)
        assert state == c.where and length == c.length
        assert ids == (c.blocks if c.where in (RESIDENT, RETURNING) else c.slots), j
        if c.where == RESIDENT:
            assert lib_k.table_rows([j])[0].tolist() == k.table_row(j)
    assert lib_s.schedule() == s.schedule()


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_library_manager_makes_the_oracles_decisions(fs, seed):
    from paper_2305_05920_amd import kvm, sched
    s = SkipJoinMLFQ(4, 1.0, 1, 6.0, 3)
    k = ProactiveCacheManager(s, 24, 30, 16, 6, reserve_idle_blocks=2, reserve_window=8, reserve_quantile=0.75)
    lib_s = sched.Scheduler(4, 1.0, 1, 6.0, 3)
    lib_k = kvm.KVManager(None, lib_s, 24, 30, 6, reserve_idle_blocks=2, reserve_window=8, reserve_quantile=0.75)

    class BothWorlds(OracleWorld):
        """Every event goes to the oracle and to the library; every answer and the whole state are compared."""

        def admit(self, j, tokens, init_time):
            ok = super().admit(j, tokens, init_time)
            assert lib_k.admit(j, tokens) == ok
            if ok:
                lib_s.add_job(j, init_time, 1.0)
            return self.same(ok)

        def grow(self, j, n):
            ok = super().grow(j, n)
            assert lib_k.grow(j, n) == ok
            if ok:
                lib_k.advance(j, n)
            return self.same(ok)

        def iteration(self, elapsed):
            batch = super().iteration(elapsed)
            lib_s.complete_iteration(batch, elapsed, [])
            return self.same(batch)

        def start_swaps(self, want):
            live = [j for j, c in k.jobs.items() if not c.released]
            before = {j: lib_k.job_info(j)[0] for j in live}
            running, moves = super().start_swaps(want)
            lib_k.start_swaps(running, want)
            changed = {j for j in live if lib_k.job_info(j)[0] != before[j]}
            assert changed == {j for _, j in moves}
            return self.same((running, moves))

        def retire(self, n):
            got = super().retire(n)
            assert lib_k.retire(n) == got
            return self.same(got)

        def observe(self, d):
            super().observe(d)
            lib_k.observe_arrivals(d)
            self.same(None)

        def release(self, j):
            super().release(j)
            lib_k.release(j)
            lib_s.set_ready(j, True)
            lib_s.complete_iteration([j], 0.0, [j])
            self.same(None)

        def same(self, x):
            compare_managers(k, lib_k, lib_s, s)
            return x

    random_drive(BothWorlds(s, k), np.random.default_rng(100 + seed), 500)
    assert k.blocks_out > 0 and k.blocks_in > 0
    lib_k.close()
    lib_s.close()


def make_trace(rng, n):
    prompts = np.clip(np.round(rng.exponential(60.0, n)), 1, 200).astype(int)
    outputs = np.clip(np.floor(rng.pareto(1.2, n) * 6 + 1), 1, 60).astype(int)
    arrival = np.sort(rng.integers(0, 30, size=n))
    return prompts, outputs, arrival


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_library_loop_makes_the_oracles_decisions(fs, seed):
    from paper_2305_05920_amd import kvm
    rng = np.random.default_rng(500 + seed)
    n = 40
    prompts, outputs, arrival = make_trace(rng, n)
    W = 20
    kw = dict(num_blocks=60, num_host_blocks=400, block_size=16, table_width=W, reserve_idle_blocks=4,
              reserve_window=16, reserve_quantile=0.8)
    ora = IterationLoop(5, 1.0, 1, 12.0, 4, 256, **kw)
    lib = kvm.ServeLoop(None, 5, 1.0, 1, 12.0, 4, kw["num_blocks"], kw["num_host_blocks"], W, max_prompt_tokens=256,
                        reserve_idle_blocks=4, reserve_window=16, reserve_quantile=0.8)
    for j in range(n):
        init, dec = float(prompts[j]) / 16.0, 1.0
        ora.submit(j, int(arrival[j]), int(prompts[j]), int(outputs[j]), init, dec)
        lib.submit(j, int(arrival[j]), int(prompts[j]), int(outputs[j]), init, dec)
    its = swaps = 0
    while ora.jobs and its < 5000:
        a, b = ora.plan(), lib.plan()
        assert (a["first"], a["decode"], a["lens_before"]) == (b["first"], b["decode"], b["lens_before"]), its
        assert b["n_waiting"] == len(ora.waiting) and b["n_unfinished"] == len(ora.jobs)
        swaps += len(a["moves"])
        compare_managers(ora.kvm, lib.manager, lib.scheduler, ora.sched)
        ora.complete(), lib.complete()
        its += 1
    st = lib.stats()
    assert not ora.jobs and st["finished_jobs"] == n == ora.finished
    assert st["job_tokens"] == int(outputs.sum()) == ora.job_tokens
    assert st["prompt_tokens"] == int(prompts.sum()) == ora.prompt_tokens
    assert st["iterations"] == its and st["iterations_without_work"] == ora.idle_iterations
    assert swaps > 0 and st["blocks_swapped_out"] == ora.kvm.blocks_out > 0, "the trace did not force swapping"
    lib.close()


def test_library_manager_rejects_bad_arguments(fs):
    from paper_2305_05920_amd import kvm, sched
    with pytest.raises(fs.FsError):
        kvm.KVManager(None, None, 0, 0, 4)                       # no blocks
    s = sched.Scheduler(2, 1.0, 1, 5.0, 2)
    k = kvm.KVManager(None, s, 4, 4, 2)
    assert k.admit(1, 16)
    with pytest.raises(fs.FsError):
        k.admit(1, 16)                                           # id already present
    assert not k.admit(2, 16 * 3)                                # wider than the table
    with pytest.raises(fs.FsError):
        k.grow(9, 1)                                             # unknown job
    with pytest.raises(fs.FsError):
        k.stage_batch([1])                                       # no layer pools: nothing to stage to
    k.close()
    s.close()
