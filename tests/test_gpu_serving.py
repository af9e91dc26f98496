"""Token-granularity preemptive serving end to end on the GPU: the skip-join MLFQ
scheduler admits a different ragged batch every iteration, new jobs run their initialization
phase (cache fill and prompt attention in one launch per layer), the proactive cache manager
moves the blocks of waiting jobs -- of both layers of the two-layer model, which share one
block table -- to host memory and back on a side stream while the decode step of the running
batch executes, and every generated token's attention output
is checked against the CPU oracle's logical caches (which know nothing of blocks,
preemption or swapping)."""
import numpy as np
import pytest
import torch

import fs_workload as wl
import oracle
from tests import harness as hs

pytestmark = pytest.mark.gpu


def test_serving_loop_with_preemption_and_swapping_matches_oracle():
    import paper_2305_05920_amd as fs
    from paper_2305_05920_amd.kvm import ServeLoop

    H, D, W = 4, 128, 16                       # up to 256 tokens per job
    rng = np.random.default_rng(2305)
    njobs, max_batch = 16, 4
    prompts = rng.integers(20, 150, size=njobs)
    outputs = rng.integers(3, 12, size=njobs)
    arrival = np.sort(rng.integers(0, 12, size=njobs))
    # HBM pool of 36 blocks (576 tokens) for ~1800 tokens of live cache: swapping is forced
    NL = 2                                     # two layers: one pool each, one table for both
    pools = [fs.Pool("bf16", H, D, 36, num_host_blocks=160) for _ in range(NL)]
    # scheduler, cache manager (reserve following the arrivals) and the loop itself are the library's
    loop = ServeLoop(pools, 4, 1.0, 1, 6.0, max_batch, 36, 160, W, max_prompt_tokens=600, reserve_idle_blocks=4,
                     reserve_window=8, reserve_quantile=0.75)
    for j in range(njobs):
        loop.submit(j, int(arrival[j]), int(prompts[j]), int(outputs[j]), float(prompts[j]) / 32.0, 1.0)

    def rand_bits(shape):
        return wl.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))

    def dev(shape):
        return torch.zeros(shape, dtype=torch.bfloat16, device="cuda")

    pq, pk, pv = dev((600, H, D)), dev((600, H, D)), dev((600, H, D))
    dq, dk, dv = dev((max_batch, H, D)), dev((max_batch, H, D)), dev((max_batch, H, D))
    pout = torch.zeros((600, H, D), dtype=torch.float32, device="cuda")
    dout = torch.zeros((max_batch, H, D), dtype=torch.float32, device="cuda")
    bufs = ServeLoop.buffers(pq, pk, pv, pout, dq, dk, dv, dout)

    # logical caches (oracle side), one per layer and job
    K = {(l, j): np.zeros((256, H, D), np.uint16) for l in range(NL) for j in range(njobs)}
    V = {(l, j): np.zeros((256, H, D), np.uint16) for l in range(NL) for j in range(njobs)}
    length = {j: 0 for j in range(njobs)}
    last_ran, preempted = {}, set()
    checked = prompt_rows = it = 0
    while True:
        assert it < 600, "serving loop does not terminate"
        plan = loop.plan()
        if plan["n_unfinished"] == 0:
            loop.complete()
            break
        first, decode, offs = plan["first"], plan["decode"], plan["token_offsets"]
        assert plan["lens_before"] == [length[j] for j in decode]
        for l in range(NL):                                      # a model: one launch per layer, its own projections
            T = plan["prompt_tokens"]
            if first:
                hq, hk, hv = (rand_bits((T, H, D)) for _ in range(3))
                pq[:T].copy_(hs.to_torch("bf16", hq)), pk[:T].copy_(hs.to_torch("bf16", hk))
                pv[:T].copy_(hs.to_torch("bf16", hv))
                pout.fill_(float("nan"))
            if decode:
                n = len(decode)
                q, kn, vn = (rand_bits((n, H, D)) for _ in range(3))
                dq[:n].copy_(hs.to_torch("bf16", q)), dk[:n].copy_(hs.to_torch("bf16", kn))
                dv[:n].copy_(hs.to_torch("bf16", vn))
                dout.fill_(float("nan"))
            if first or decode:
                loop.launch(bufs, layer=l)
            torch.cuda.synchronize()
            pools[l].check()
            if first:
                pgot = pout.cpu().numpy()
                for r, j in enumerate(first):
                    a, b = offs[r], offs[r + 1]
                    assert b - a == prompts[j]
                    K[l, j][:b - a], V[l, j][:b - a] = hk[a:b], hv[a:b]
                    ref = oracle.prefill_attention_job(np.ascontiguousarray(hq[a:b]), np.ascontiguousarray(hk[a:b]),
                                                       np.ascontiguousarray(hv[a:b]), "bf16")
                    hs.assert_parity(pgot[a:b], ref, f"iteration {it} layer {l} prompt of job {j} ({b - a} tokens)")
                    prompt_rows += b - a
            if decode:
                got = dout.cpu().numpy()
                for r, j in enumerate(decode):
                    K[l, j][length[j]], V[l, j][length[j]] = kn[r], vn[r]
                    ref = oracle.attention_job(q[r], K[l, j], V[l, j], "bf16", length=length[j] + 1)
                    err = np.abs(got[r] - ref).max()
                    rel = np.linalg.norm(got[r] - ref) / np.linalg.norm(ref)
                    assert err <= hs.MAX_ABS_TOL and rel <= hs.REL_L2_TOL, (it, l, j, err, rel)
                    checked += 1
        for j in first:
            length[j] = int(prompts[j])
        for j in decode:
            length[j] += 1
        for j in first + decode:
            if j in last_ran and last_ran[j] < it - 1:
                preempted.add(j)                                  # it waited while others ran
            last_ran[j] = it
        loop.complete()
        it += 1
    st = loop.stats()
    loop.manager.retire(wait=True)
    print(f"[serving] {it} iterations, {prompt_rows} prompt rows and {checked} decode outputs checked, "
          f"{len(preempted)} jobs preempted, {st['blocks_swapped_out']} blocks swapped out, "
          f"{st['blocks_swapped_in']} swapped in", flush=True)
    assert st["finished_jobs"] == njobs and st["job_tokens"] == int(outputs.sum())
    assert checked == NL * int((outputs - 1).sum()) and prompt_rows == NL * int(prompts.sum())
    assert st["blocks_swapped_out"] > 0 and st["blocks_swapped_in"] > 0, "the test did not exercise swapping"
    assert preempted, "no job was ever preempted"
    assert loop.manager.free_blocks == 36 and loop.manager.free_slots == 160
    loop.close()
    for p in pools:
        p.close()


def test_compiled_loop_runs_a_trace_to_completion_without_host_waits():
    # fs_serve_run: the whole multi-iteration run inside the library (no Python between iterations);
    # afterwards every job has finished, every block and slot is back, no kernel met a bad table
    import paper_2305_05920_amd as fs
    from paper_2305_05920_amd.kvm import ServeLoop
    H, D, W, max_batch = 8, 128, 24, 8
    rng = np.random.default_rng(77)
    njobs = 48
    prompts = np.clip(np.round(rng.exponential(96.0, njobs)), 8, 300).astype(int)
    outputs = np.clip(np.floor(rng.pareto(1.2, njobs) * 8 + 2), 2, 64).astype(int)
    arrival = np.sort(rng.integers(0, 40, size=njobs))
    nblocks = 96                                                   # ~1500 tokens of HBM for ~8000 tokens of live cache
    pool = fs.Pool("bf16", H, D, nblocks, num_host_blocks=1200)
    loop = ServeLoop([pool], 6, 1.0, 1, 30.0, max_batch, nblocks, 1200, W, max_prompt_tokens=1024,
                     reserve_idle_blocks=8)
    for j in range(njobs):
        loop.submit(j, int(arrival[j]), int(prompts[j]), int(outputs[j]), float(prompts[j]) / 64.0, 1.0)
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    pq, pk, pv = (torch.randn((1024, H, D), generator=g, device="cuda").to(torch.bfloat16) for _ in range(3))
    dq, dk, dv = (torch.randn((max_batch, H, D), generator=g, device="cuda").to(torch.bfloat16) for _ in range(3))
    pout = torch.full((1024, H, D), float("nan"), dtype=torch.float32, device="cuda")
    dout = torch.full((max_batch, H, D), float("nan"), dtype=torch.float32, device="cuda")
    st = loop.run(ServeLoop.buffers(pq, pk, pv, pout, dq, dk, dv, dout), 20000)
    torch.cuda.synchronize()
    pool.check()
    loop.manager.retire(wait=True)
    print(f"[serving] compiled loop: {st}", flush=True)
    assert st["finished_jobs"] == njobs and st["job_tokens"] == int(outputs.sum())
    assert st["prompt_tokens"] == int(prompts.sum())
    assert st["blocks_swapped_out"] > 0 and st["blocks_swapped_in"] > 0
    assert loop.manager.free_blocks == nblocks and loop.manager.free_slots == 1200
    assert torch.isfinite(dout[:1]).all()
    loop.close()
    pool.close()


def test_iteration_time_profile_feeds_skip_join():
    # the job profiler of Section 3.2 / 4.1, measured with the library's own kernels: first-iteration
    # time grows with the prompt, and skip-join sends long prompts to lower-priority queues
    from paper_2305_05920_amd.profiler import IterationTimeProfile
    from paper_2305_05920_amd.sched import Scheduler
    prof = IterationTimeProfile("bf16", 8, 128, prompt_lengths=(16, 128, 1024, 4096), cache_lengths=(16, 2048), reps=3)
    t = [prof.init_time(s) for s in (16, 128, 1024, 4096, 8192)]
    print("[profile]", prof.as_dict(), flush=True)
    assert all(x > 0 for x in t) and t[3] > 2 * t[0] and t[4] > t[3]
    assert prof.decode_time(2048) >= prof.decode_time(16) > 0
    q1 = prof.min_iteration_time()
    assert 0 < q1 <= min(t)
    sched = Scheduler(8, q1, 1, 1e9, 4)
    queues = [sched.add_job(i, prof.init_time(s), prof.decode_time(s)) for i, s in enumerate((16, 1024, 8192))]
    sched.close()
    assert 1 <= queues[0] <= 2 and queues[0] <= queues[1] <= queues[2] and queues[2] > queues[0]
