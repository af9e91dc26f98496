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
    from paper_2305_05920_amd.kv_manager import ArrivalReserve, KVManager
    from paper_2305_05920_amd.sched import Scheduler

    H, D, W = 4, 128, 16                       # up to 256 tokens per job
    cfg = wl.CONFIGS[1].scaled(num_heads=H, head_dim=D)
    rng = np.random.default_rng(2305)
    njobs = 16
    prompts = rng.integers(20, 150, size=njobs)
    outputs = rng.integers(3, 12, size=njobs)
    arrival = np.sort(rng.integers(0, 12, size=njobs))
    # HBM pool of 36 blocks (576 tokens) for ~1800 tokens of live cache: swapping is forced
    NL = 2                                     # two layers: one pool each, one table for both
    pools = [fs.Pool("bf16", H, D, 36, num_host_blocks=160) for _ in range(NL)]
    pool = pools[0]
    sched = Scheduler(4, 1.0, 1, 6.0, 4)
    kv = KVManager(pools, sched, W, reserve_idle_blocks=4)
    kv.arrival_reserve = ArrivalReserve(window=8, quantile=0.75, floor=4)   # the reserve follows the arrivals

    def rand_bits(shape):
        return wl.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))

    # logical caches (oracle side), one per layer and job
    K = {(l, j): np.zeros((256, H, D), np.uint16) for l in range(NL) for j in range(njobs)}
    V = {(l, j): np.zeros((256, H, D), np.uint16) for l in range(NL) for j in range(njobs)}
    length = {j: 0 for j in range(njobs)}
    produced = {j: 0 for j in range(njobs)}
    waiting, done = [], set()
    last_ran, preempted = {}, set()
    checked = 0
    prompt_rows = 0
    it = 0
    while len(done) < njobs:
        assert it < 600, "serving loop does not terminate"
        new = [j for j in range(njobs) if arrival[j] == it]
        kv.observe_arrivals(sum(kv.blocks_needed(int(prompts[j]) + 1) for j in new))
        waiting += new
        for j in list(waiting):                                  # admission: prompt must fit beside the reserve
            if kv.blocks_needed(int(prompts[j]) + 1) + kv.reserve <= len(kv.free_blocks):
                kv.admit(j, int(prompts[j]) + 1)
                sched.add_job(j, float(prompts[j]) / 32.0, 1.0)
                waiting.remove(j)
        batch = [j for j in sched.schedule()]
        # a decoding job needs room for one more token; if HBM is full it sits this one out
        runnable = [j for j in batch if length[j] == 0 or kv.grow(j, 1)]
        kv.start_swaps(runnable, want_free=len(batch) - len(runnable) + len(waiting))
        first = [j for j in runnable if length[j] == 0]
        decode = [j for j in runnable if length[j] > 0]
        if first:                                                # initialization phase, all new jobs in one launch per layer
            ns = [int(prompts[j]) for j in first]
            offs = np.zeros(len(first) + 1, dtype=np.int32)
            offs[1:] = np.cumsum(ns)
            d_table, d_offs = torch.from_numpy(kv.table_rows(first)).cuda(), torch.from_numpy(offs).cuda()
            for l in range(NL):
                pq, pk, pv = (rand_bits((int(offs[-1]), H, D)) for _ in range(3))
                pout = torch.full((int(offs[-1]), H, D), float("nan"), dtype=torch.float32, device="cuda")
                fs.fs_prefill_step(pools[l], d_table, d_offs, hs.to_torch("bf16", pk), hs.to_torch("bf16", pv),
                                   hs.to_torch("bf16", pq), pout)
                torch.cuda.synchronize()
                pgot = pout.cpu().numpy()
                for r, j in enumerate(first):
                    a, b = int(offs[r]), int(offs[r + 1])
                    K[l, j][:ns[r]], V[l, j][:ns[r]] = pk[a:b], pv[a:b]
                    ref = oracle.prefill_attention_job(np.ascontiguousarray(pq[a:b]), np.ascontiguousarray(pk[a:b]),
                                                       np.ascontiguousarray(pv[a:b]), "bf16")
                    hs.assert_parity(pgot[a:b], ref, f"iteration {it} layer {l} prompt of job {j} ({ns[r]} tokens)")
                    prompt_rows += ns[r]
            for r, j in enumerate(first):
                kv.advance(j, ns[r])
                length[j] = ns[r]
        layer_out = []
        if decode:                                               # decoding phase: one fused step per layer
            lens_before = np.array([length[j] for j in decode], dtype=np.int32)
            d_table, d_lens = torch.from_numpy(kv.table_rows(decode)).cuda(), torch.from_numpy(lens_before).cuda()
            for l in range(NL):
                q, kn, vn = (rand_bits((len(decode), H, D)) for _ in range(3))
                out = torch.full((len(decode), H, D), float("nan"), dtype=torch.float32, device="cuda")
                fs.fs_decode_step(pools[l], d_table, d_lens, hs.to_torch("bf16", kn), hs.to_torch("bf16", vn),
                                  hs.to_torch("bf16", q), out)
                layer_out.append((q, kn, vn, out))
        kv.finish_swaps()
        torch.cuda.synchronize()
        for p in pools:
            p.check()
        if decode:
            for l, (q, kn, vn, out) in enumerate(layer_out):
                got = out.cpu().numpy()
                for r, j in enumerate(decode):
                    K[l, j][length[j]], V[l, j][length[j]] = kn[r], vn[r]
                    ref = oracle.attention_job(q[r], K[l, j], V[l, j], "bf16", length=length[j] + 1)
                    err = np.abs(got[r] - ref).max()
                    assert err <= hs.MAX_ABS_TOL, (it, l, j, err)
                    checked += 1
            for j in decode:
                length[j] += 1
                kv.advance(j, 1)
        finished = []
        for j in runnable:
            produced[j] += 1
            if j in last_ran and last_ran[j] < it - 1:
                preempted.add(j)                                  # it waited while others ran
            last_ran[j] = it
            if produced[j] == outputs[j]:
                finished.append(j)
        elapsed = max([float(prompts[j]) / 32.0 if j in first else 1.0 for j in runnable], default=1.0)
        sched.complete_iteration(runnable, elapsed, finished)
        for j in finished:
            kv.release(j)
            done.add(j)
        it += 1
    print(f"[serving] {it} iterations, {prompt_rows} prompt rows and {checked} decode outputs checked, "
          f"{len(preempted)} jobs preempted, "
          f"{kv.swapped_out_blocks} blocks swapped out, {kv.swapped_in_blocks} swapped in", flush=True)
    assert checked == NL * int((outputs - 1).sum()) and prompt_rows == NL * int(prompts.sum())
    assert kv.swapped_out_blocks > 0 and kv.swapped_in_blocks > 0, "the test did not exercise swapping"
    assert preempted, "no job was ever preempted"
    assert len(kv.free_blocks) == pool.num_blocks and len(kv.free_slots) == pool.num_host_blocks
    sched.close()
    for p in pools:
        p.close()


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
