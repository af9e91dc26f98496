"""What the scheduler is for (paper Sections 1 and 4.1): with output lengths unknown and heavy
tailed, preempting at token granularity with skip-join MLFQ gives a lower average job completion
time than first-come-first-served run-to-completion.  A seeded discrete-event simulation on
synthetic lengths, driven by the library's scheduler through its C ABI; no dataset, no GPU.

Model: one engine, batches of at most B jobs per iteration; an iteration lasts as long as its
slowest member (a first iteration costs prompt/32 decode iterations, a decode iteration 1).
Prompts and output lengths are Pareto distributed, arrivals Poisson at 90 % load."""
import numpy as np
import pytest

from paper_2305_05920_amd.sched import Scheduler


def simulate(policy: str, seed: int, njobs: int = 300, B: int = 8, load: float = 0.9):
    rng = np.random.default_rng(seed)
    prompts = np.clip(rng.pareto(1.5, njobs) * 64 + 16, 16, 2048)
    outs = np.clip(np.floor(rng.pareto(1.2, njobs) * 20 + 1), 1, 1500).astype(int)
    init, dec = prompts / 32.0, 1.0
    demand = (init + outs * dec).mean() / B
    arrivals = np.cumsum(rng.exponential(demand / load, njobs))
    if policy == "fcfs":          # one queue, a quantum nobody uses up: strict arrival order
        s = Scheduler(1, 1e18, 1, 1e18, B)
    else:                          # quanta 1, 2, 4, ... 128; no starvation promotion in this run
        s = Scheduler(8, 1.0, 1, 1e18, B)
    t, nxt, left, jct, started, tokens = 0.0, 0, {}, {}, set(), 0
    while len(jct) < njobs:
        while nxt < njobs and arrivals[nxt] <= t:
            s.add_job(nxt, float(init[nxt]), dec)
            left[nxt] = int(outs[nxt])
            nxt += 1
        batch = s.schedule()
        if not batch:
            t = arrivals[nxt]
            continue
        assert len(batch) <= B and len(set(batch)) == len(batch)
        elapsed = max(float(init[j]) if j not in started else dec for j in batch)
        t += elapsed
        finished = []
        for j in batch:
            started.add(j)
            left[j] -= 1
            tokens += 1
            if left[j] == 0:
                finished.append(j)
                jct[j] = t - arrivals[j]
        s.complete_iteration(batch, elapsed, finished)
    s.close()
    assert tokens == int(outs.sum())            # every job produced exactly its tokens
    return float(np.mean(list(jct.values()))), float(np.percentile(list(jct.values()), 50))


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_skip_join_mlfq_beats_run_to_completion_on_heavy_tailed_lengths(seed):
    fcfs_mean, fcfs_p50 = simulate("fcfs", seed)
    mlfq_mean, mlfq_p50 = simulate("skipjoin", seed)
    print(f"[policy] seed {seed}: mean JCT fcfs {fcfs_mean:.1f} skip-join {mlfq_mean:.1f}; "
          f"median fcfs {fcfs_p50:.1f} skip-join {mlfq_p50:.1f}")
    assert mlfq_mean < 0.8 * fcfs_mean
    assert mlfq_p50 < 0.5 * fcfs_p50            # short jobs no longer wait behind long ones
