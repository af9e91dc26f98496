#!/usr/bin/env python3
"""Benchmark of the paged decode step on one MI355X.

A step is one pass of the whole hot path over one admitted batch: KV append of
every job's new token (fs_kv_append), then one-query-per-job attention over every
job's paged cache (fs_decode_attention: partition pass + combine).  The fused entry
point fs_decode_step (append inside the attention kernel) is timed beside it.  Inputs are synthetic and seeded
(fs_workload), resident in HBM before the timed region.  To keep the 256 MB
last-level cache from serving the reads, the steps rotate over several replicas
of the pool.

Prints ONE JSON line; see --help for the knobs.
"""
from __future__ import annotations

import argparse
from concurrent.futures import ThreadPoolExecutor
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "decode-attention achieved HBM GB/s (% of MI355X peak); job-tokens/s per step"
HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published


def algorithmic_bytes(cfg, lens) -> int:
    """Bytes one attention launch has to move: every cached K and V element once,
    q once, out once, each job's table entries and length once."""
    H, D, e = cfg.num_heads, cfg.head_dim, cfg.elem_bytes
    total = int(lens.astype(np.int64).sum())
    nb = int(((lens.astype(np.int64) + cfg.block_size - 1) // cfg.block_size).sum())
    J = len(lens)
    return 2 * H * D * e * total + J * H * D * e + J * H * D * 4 + 4 * nb + 4 * J


class Replicas:
    """R copies of one workload's pool in HBM, each behind its own fs_pool."""

    def __init__(self, fs, torch, wl, cfg, rep, min_footprint_bytes, pool_kw, log):
        self.fs, self.torch, self.cfg = fs, torch, cfg
        step = wl.make_step(cfg, rep)
        self.step = step
        bt = step.tables
        H, D = cfg.num_heads, cfg.head_dim
        block_elems = 2 * H * cfg.block_size * D
        pool_bytes = bt.num_blocks * block_elems * cfg.elem_bytes
        self.alg_bytes = algorithmic_bytes(cfg, step.lens)
        R = max(2, int(np.ceil(min_footprint_bytes / max(self.alg_bytes, 1))))
        R = min(R, max(2, int(24e9 // pool_bytes)))
        self.R = R
        tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[cfg.dtype]
        self.mem = torch.empty((R, bt.num_blocks, block_elems), dtype=tdt, device="cuda")
        self.pools = [fs.Pool(cfg.dtype, H, D, bt.num_blocks, device_mem=self.mem[r], **pool_kw) for r in range(R)]
        self.table = torch.from_numpy(bt.table).cuda()
        self.lens = torch.from_numpy(step.lens).cuda()
        lens_before = (step.lens - 1).astype(np.int32)
        self.lens_before = torch.from_numpy(lens_before).cuda()
        self.max_len = int(step.lens.max())
        # host caches -> packed prefix tokens -> bulk write into replica 0 -> copy to the rest
        t0 = time.time()
        with ThreadPoolExecutor(max_workers=8) as ex:      # numpy's generators release the GIL
            self.caches = list(ex.map(step.cache, range(cfg.num_jobs)))
        log(f"generated {cfg.name}: J={cfg.num_jobs} sum(L)={step.total_tokens} "
            f"pool={pool_bytes / 1e9:.2f} GB x{R} in {time.time() - t0:.1f}s")
        offs = np.zeros(cfg.num_jobs + 1, dtype=np.int32)
        offs[1:] = np.cumsum(lens_before)
        self.q = self._dev(step.q)
        self.k_new = self._dev(np.stack([K[-1] for K, _ in self.caches]))
        self.v_new = self._dev(np.stack([V[-1] for _, V in self.caches]))
        # bulk write in slices of jobs so that the packed staging copy stays small
        j = 0
        while j < cfg.num_jobs:
            j1, tok = j, 0
            while j1 < cfg.num_jobs and (tok == 0 or tok + lens_before[j1] <= (1 << 21)):
                tok += int(lens_before[j1])
                j1 += 1
            if tok > 0:
                K = np.concatenate([self.caches[i][0][:lens_before[i]] for i in range(j, j1)])
                V = np.concatenate([self.caches[i][1][:lens_before[i]] for i in range(j, j1)])
                o = (offs[j:j1 + 1] - offs[j]).astype(np.int32)
                fs.fs_kv_prefill(self.pools[0], self.table[j:j1].contiguous(),
                                 torch.zeros(j1 - j, dtype=torch.int32, device="cuda"),
                                 torch.from_numpy(o).cuda(), tok, self._dev(K), self._dev(V))
                torch.cuda.synchronize()
            j = j1
        self.pools[0].check()
        for r in range(1, R):
            self.mem[r].copy_(self.mem[0])
        self.out = torch.empty((cfg.num_jobs, H, D), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()

    def _dev(self, a):
        t = self.torch
        if self.cfg.dtype in ("bf16", "f16"):
            return t.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(
                t.bfloat16 if self.cfg.dtype == "bf16" else t.float16)
        return t.from_numpy(np.ascontiguousarray(a)).cuda()

    fused = False

    def run_step(self, i):
        pool = self.pools[i % self.R]
        if self.fused:
            self.fs.fs_decode_step(pool, self.table, self.lens_before, self.k_new, self.v_new, self.q,
                                   self.out, max_len_hint=self.max_len)
        else:
            self.fs.fs_kv_append(pool, self.table, self.lens_before, self.k_new, self.v_new)
            self.fs.fs_decode_attention(self.q, pool, self.table, self.lens, self.out,
                                        max_len_hint=self.max_len)

    def close(self):
        for p in self.pools:
            p.close()


def swap_overlap(fs, torch, wl, cfg, log, steps=150, warmup=20, waiting_jobs=48, waiting_tokens=1024):
    """Decode steps of the preset's batch while the cache manager (C++, fs_kvm_*) swaps WAITING jobs
    between HBM and pinned host memory on its side stream, in the order of their estimated next
    scheduled time (paper Section 4.2): every other step it is asked for `rate` more free blocks
    (jobs leave), in between for none (jobs return).  The rate is swept from nothing to more than
    the host link carries; copies that do not finish within a step simply stay in flight (their
    events are polled).  Reported per rate: the step time, the attention kernel's own duration
    and the bytes that crossed the link per second of the timed region."""
    from paper_2305_05920_amd.kvm import KVManager
    from paper_2305_05920_amd.sched import Scheduler
    if cfg.dtype == "f32":
        return None
    H, D, B = cfg.num_heads, cfg.head_dim, cfg.block_size
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float16
    lens = wl.job_lens(cfg, wl.seed_for(cfg.index, 0)).astype(np.int64)
    J = cfg.num_jobs
    W = int(max((lens.max() + B - 1) // B, (waiting_tokens + B - 1) // B)) + 1
    nb_run = int(((lens + B - 1) // B).sum())
    nb_wait = waiting_jobs * ((waiting_tokens + B - 1) // B)
    nblocks, nslots = nb_run + nb_wait + 64, nb_wait + 64
    # the cache contents do not matter for time, but they must be finite numbers: zeros
    mem = torch.zeros((nblocks, 2 * H * B * D), dtype=tdt, device="cuda")
    pool = fs.Pool(cfg.dtype, H, D, nblocks, num_host_blocks=nslots, device_mem=mem)
    sched = Scheduler(6, 1.0, 1, 1e9, J)
    kvm = KVManager([pool], sched, nblocks, nslots, W, max_batch=J)
    running = list(range(J))
    for j in running:
        assert kvm.admit(j, int(lens[j]))
        sched.add_job(j, 0.5, 0.5)
        kvm.advance(j, int(lens[j]) - 1)                  # the step appends the last token
    rng = np.random.default_rng(11)
    for w in range(waiting_jobs):                         # waiting jobs spread over the lower queues
        jid = J + w
        assert kvm.admit(jid, waiting_tokens)
        sched.add_job(jid, float(rng.choice([1.5, 3.0, 6.0, 12.0])), 1.0)
        kvm.advance(jid, waiting_tokens)
    block_bytes = pool.block_bytes
    table = torch.from_numpy(kvm.table_rows(running)).cuda()
    d_before = torch.from_numpy((lens - 1).astype(np.int32)).cuda()
    d_lens = torch.from_numpy(lens.astype(np.int32)).cuda()
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    q, k_new, v_new = (torch.randn((J, H, D), generator=g, device="cuda").to(tdt) for _ in range(3))
    out = torch.empty((J, H, D), dtype=torch.float32, device="cuda")
    lens_max = int(lens.max())

    def step():
        fs.fs_kv_append(pool, table, d_before, k_new, v_new)
        fs.fs_decode_attention(q, pool, table, d_lens, out, max_len_hint=lens_max)

    def drive(rate, n):
        for i in range(n):
            if rate:
                kvm.retire()
                # even steps ask for `rate` blocks more than are free or on their way out: waiting
                # jobs leave, latest next scheduled time first; odd steps ask for nothing: those
                # whose blocks have arrived in host memory come back, earliest first
                kvm.start_swaps(running, want_free=(kvm.free_blocks + rate) if i % 2 == 0 else 0)
            yield i
            step()

    def timed(rate):
        bo0, bi0, _ = kvm.stats()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in drive(rate, steps):
            marks[i].record()
        marks[steps].record()
        torch.cuda.current_stream().synchronize()
        wall = time.perf_counter() - t0
        kvm.retire(wait=True)
        t_all = time.perf_counter() - t0
        per = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(steps)])
        bo, bi, _ = kvm.stats()
        # the kernels' own durations from a second, shorter pass with launch-attached events
        # (recording them costs host time, so the step time above is taken without)
        pool.profile_enable(True)
        for _ in drive(rate, steps // 3):
            pass
        torch.cuda.synchronize()
        kvm.retire(wait=True)
        prof = pool.profile_collect()
        pool.profile_enable(False)
        return {"blocks_asked_per_swap_step": rate, "ms_per_step_median": float(np.median(per)),
                "ms_per_step_mean_wall": wall * 1e3 / steps,
                "attention_kernel_ms": prof["attention"]["ms"] / max(prof["attention"]["launches"], 1),
                "gb_per_s_to_host": (bo - bo0) * block_bytes / t_all / 1e9,
                "gb_per_s_from_host": (bi - bi0) * block_bytes / t_all / 1e9,
                "blocks_out": bo - bo0, "blocks_in": bi - bi0, "seconds_until_copies_done": t_all}

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    rows = [timed(0)]
    base = rows[0]["ms_per_step_median"]
    per_job = (waiting_tokens + B - 1) // B
    for jobs_at_once in (1, 2, 4, 8, 16, 32):           # from a trickle to more than the link carries
        rows.append(timed(per_job * jobs_at_once))
    for r in rows:
        r["step_time_vs_no_swaps"] = r["ms_per_step_median"] / base
    pool.check()
    kvm.close()
    sched.close()
    pool.close()
    res = {"workload": f"{cfg.name} batch decoding while {waiting_jobs} waiting jobs of {waiting_tokens} tokens are swapped "
                       f"by the cache manager in ENST order", "block_bytes": block_bytes, "rates": rows}
    log(json.dumps(res))
    return res


MIN_TIMED_STEPS = 50


def time_steps(torch, reps, steps, warmup):
    """`warmup` untimed steps, then max(steps, 50) timed ones between two synchronisations.  Every
    step is bracketed by events on the stream the kernels run on; returns the median step time,
    the wall-clock mean over the same steps, the minimum and the number of steps timed."""
    n = max(int(steps), MIN_TIMED_STEPS)
    for i in range(warmup):
        reps.run_step(i)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n):
        marks[i].record()
        reps.run_step(warmup + i)
    marks[n].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / n
    per_step = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(n)])
    return {"median_ms": float(np.median(per_step)), "mean_wall_ms": wall_ms, "min_ms": float(per_step.min()),
            "timed_steps": n}


def read_ceiling(fs, torch, nbytes=4 << 30, reps=5):
    """Practical HBM read rate of this machine: a plain streaming read kernel (non-temporal loads,
    like the decode kernel's cache reads) over 4 GiB, best of several grid sizes."""
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    src.zero_()
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    best = 0.0
    for wgs in (256, 512, 8192, 16384):
        fs.fs_stream_read(src, sink, wgs)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fs.fs_stream_read(src, sink, wgs)
        torch.cuda.synchronize()
        best = max(best, nbytes * reps / (time.perf_counter() - t0) / 1e9)
    del src
    torch.cuda.empty_cache()
    return best


def same_bytes_read(fs, torch, sizes, reps=40):
    """What a kernel that does nothing but read costs at the presets' own sizes: for every byte
    count in `sizes`, the median duration of fs_stream_read's kernel over that many bytes, on the
    attention kernel's grid (one 256-thread workgroup per compute unit), every launch on the
    next region of a buffer of 4 GiB or more (a size far beyond the caches is simply read
    again).  The duration comes from events attached to the launch, as the attention kernel's."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    big = torch.empty(max(4 << 30, max(int(n) for n in sizes) + 4096), dtype=torch.uint8, device="cuda")
    big.zero_()
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    out = []
    for n in sizes:
        nbytes = max(4096, int(n) // 4096 * 4096)
        step = (nbytes + (64 << 20)) // 4096 * 4096
        off, ts = 0, []
        for _ in range(reps + 5):
            if off + nbytes > big.numel():
                off = 0
            ts.append(fs.fs_stream_read_timed(big[off:off + nbytes], sink, cus))
            off += step
        ts = sorted(ts[5:])
        us = ts[len(ts) // 2]
        out.append({"bytes": nbytes, "kernel_us": us, "kernel_us_min": ts[0], "gbps": nbytes / us / 1e3})
    del big
    torch.cuda.empty_cache()
    return out


def time_steps_warm(torch, reps, steps, warmup):
    """The same step on ONE pool every time: its blocks stay in the 256 MB last-level cache
    between steps.  Reported beside the headline and labelled as such, never as the headline."""
    for i in range(warmup):
        reps.run_step(0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        reps.run_step(0)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def serving_run(fs, torch, wl, cfg, log, njobs=96, max_batch=8, seed=7):
    """Token-granularity preemptive serving over many iterations on the preset's layer shape, the
    whole loop inside the library (fs_serve_run, C++): the skip-join MLFQ scheduler picks the batch
    of every iteration, new jobs run their initialization phase (fs_prefill_step), running jobs one
    fused decode step (fs_decode_step), the cache manager keeps the block tables, stages them to
    the GPU ahead of the kernels and moves waiting jobs' blocks to pinned host memory and back on
    a side stream.  The host never waits for the GPU inside the run.  wall_s: from the call to
    the moment the GPU has drained; gpu_ms: the sum of the kernels' own durations (second run of
    the same trace with launch-attached events)."""
    from paper_2305_05920_amd.kvm import ServeLoop
    from paper_2305_05920_amd.profiler import IterationTimeProfile
    H, D = cfg.num_heads, cfg.head_dim
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16}.get(cfg.dtype)
    if tdt is None:
        return None
    rng = np.random.default_rng(seed)
    prompts = np.clip(np.round(rng.exponential(256.0, njobs)), 16, 1024).astype(int)
    outputs = np.clip(np.floor(rng.pareto(1.2, njobs) * 16 + 4), 4, 192).astype(int)
    arrival = np.sort(rng.integers(0, 24, size=njobs))
    W = int((prompts.max() + outputs.max() + 15) // 16 + 1)
    live_tokens = int((prompts + outputs).sum())
    nblocks = max(W * 4, int(0.25 * live_tokens / 16))          # HBM holds a quarter of all caches: swapping is forced
    nslots = int(live_tokens / 16) + njobs
    prof_t = IterationTimeProfile(cfg.dtype, H, D, prompt_lengths=(16, 64, 256, 1024), cache_lengths=(16, 1024), reps=3)
    q1 = prof_t.min_iteration_time()               # Section 4.1: the first quantum is the minimum iteration time
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    maxtok = int(prompts.max()) * 2
    pq, pk, pv = (torch.randn((maxtok, H, D), generator=g, device="cuda").to(tdt) for _ in range(3))
    pout = torch.empty((maxtok, H, D), dtype=torch.float32, device="cuda")
    dq, dk, dv = (torch.randn((max_batch, H, D), generator=g, device="cuda").to(tdt) for _ in range(3))
    dout = torch.empty((max_batch, H, D), dtype=torch.float32, device="cuda")

    def one_run(profile):
        pool = fs.Pool(cfg.dtype, H, D, nblocks, num_host_blocks=nslots)
        loop = ServeLoop([pool], 6, q1, 1, 40.0 * q1, max_batch, nblocks, nslots, W, max_prompt_tokens=maxtok,
                         reserve_idle_blocks=W)
        for j in range(njobs):
            loop.submit(j, int(arrival[j]), int(prompts[j]), int(outputs[j]), prof_t.init_time(int(prompts[j])),
                        prof_t.decode_time(int(prompts[j])))
        bufs = ServeLoop.buffers(pq, pk, pv, pout, dq, dk, dv, dout)
        pool.profile_enable(profile)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        st = loop.run(bufs, 100000)
        t_host = time.perf_counter() - t0
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        gpu_ms = None
        if profile:
            gpu_ms = sum(rec["ms"] for rec in pool.profile_collect().values())
            pool.profile_enable(False)
        pool.check()
        loop.manager.retire(wait=True)
        loop.close()
        pool.close()
        return st, wall, t_host, gpu_ms

    one_run(False)                                  # warm-up of the same trace
    # The run's course depends on when its swaps retire, which is a matter of timing: iteration
    # counts and host times differ from run to run.  Three runs; the one with the median wall
    # time is reported, all three wall times are listed.
    runs = sorted((one_run(False) for _ in range(3)), key=lambda r: r[1])
    st, wall, t_host, _ = runs[1]
    _, _, _, gpu_ms = one_run(True)
    tokens = st["job_tokens"]
    res = {"workload": f"{njobs} jobs on the {cfg.name} layer shape ({H} heads x {D}, {cfg.dtype}): prompts Exp(256) in "
                       f"[16,1024], outputs Pareto in [4,192], batches of at most {max_batch}, HBM pool of {nblocks} blocks",
           "driver": "fs_serve_run (C++ loop inside the library: scheduler, cache manager, table staging, launches)",
           "iterations": st["iterations"], "job_tokens": tokens, "prompt_tokens": st["prompt_tokens"],
           "finished_jobs": st["finished_jobs"], "iterations_without_work": st["iterations_without_work"],
           "wall_s": wall, "wall_s_of_three_runs": [r[1] for r in runs], "host_loop_s": t_host,
           "host_seconds": {k: st[k] for k in ("host_seconds_plan", "host_seconds_launch", "host_seconds_complete")}, "job_tokens_per_s_wall": tokens / wall, "gpu_ms": gpu_ms,
           "job_tokens_per_s_gpu_time": tokens / (gpu_ms / 1e3) if gpu_ms else None,
           "wall_over_gpu_time": wall / (gpu_ms / 1e3) if gpu_ms else None,
           "blocks_swapped_out": st["blocks_swapped_out"], "blocks_swapped_in": st["blocks_swapped_in"],
           "iteration_time_profile_ms": prof_t.as_dict(), "first_quantum_ms": q1}
    log(json.dumps(res))
    return res


def kernel_times(torch, reps, steps):
    """Average duration of each kernel, from HIP events the library records on the
    launch stream around every launch."""
    for p in reps.pools:
        p.profile_enable(True)
    for i in range(steps):
        reps.run_step(i)
    torch.cuda.synchronize()
    tot = {}
    for p in reps.pools:
        for kind, rec in p.profile_collect().items():
            a = tot.setdefault(kind, {"ms": 0.0, "launches": 0})
            a["ms"] += rec["ms"]
            a["launches"] += rec["launches"]
        p.profile_enable(False)
    return {k: (v["ms"] / v["launches"] if v["launches"] else None) for k, v in tot.items()}


def graph_ms(torch, reps, steps):
    """The same steps replayed from one captured HIP graph (R steps per replay)."""
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        for i in range(reps.R):
            reps.run_step(i)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        for i in range(reps.R):
            reps.run_step(i)
    n = max(1, steps // reps.R)
    g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        g.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / (n * reps.R)


def cpu_baseline(reps, budget_s=12.0):
    """The fp64 oracle, as it stands, on this host: whole step (append + attention)."""
    import oracle
    cfg, step = reps.cfg, reps.step
    k_new = np.stack([K[-1] for K, _ in reps.caches])
    v_new = np.stack([V[-1] for _, V in reps.caches])

    def fresh():
        lc = oracle.LogicalCaches(cfg.dtype, cfg.num_heads, cfg.head_dim)
        for K, V in reps.caches:
            lc.add_job(np.ascontiguousarray(K[:-1]), np.ascontiguousarray(V[:-1]))
        return lc

    times, out, spent = [], None, 0.0
    while (spent < budget_s and len(times) < 200) or not times:
        lc = fresh()
        t0 = time.perf_counter()
        out = lc.decode_step(k_new, v_new, step.q)
        dt = time.perf_counter() - t0
        times.append(dt)
        spent += dt
    best = min(times)
    return {"value": cfg.num_jobs / best, "unit": "job-tokens/s", "cores": 1, "kind": "oracle",
            "sample": f"whole {cfg.name} step (append + attention, {cfg.num_jobs} jobs, "
                      f"{step.total_tokens} cached tokens), best of {len(times)} runs, "
                      f"{spent:.1f}s of CPU work",
            "seconds_per_step": best}, out


MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 / fp16 matrix-core peak


def prefill_cpu_baseline(wl, cfg, budget_s=8.0):
    """The oracle's prompt attention on a bounded sample of the same workload: one prompt of the
    preset's median length, as many heads as fit the time budget (single thread)."""
    import oracle
    lens = wl.job_lens(cfg, wl.seed_for(cfg.index, 0)).astype(np.int64)
    n = int(np.sort(lens)[len(lens) // 2])
    rng = np.random.default_rng(wl.seed_for(cfg.index, 0))
    conv = wl.f32_to_bf16_bits if cfg.dtype == "bf16" else wl.f32_to_f16_bits
    q, k, v = (conv(rng.standard_normal((n, cfg.num_heads, cfg.head_dim), dtype=np.float32)) for _ in range(3))
    heads, spent = 0, 0.0
    while heads < cfg.num_heads and spent < budget_s:
        t0 = time.perf_counter()
        oracle.prefill_attention_job(q, k, v, cfg.dtype, heads=(heads, heads + 1))
        spent += time.perf_counter() - t0
        heads += 1
    flops = 4.0 * cfg.head_dim * heads * n * (n + 1) / 2
    return {"value": flops / spent / 1e12, "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
            "sample": f"one prompt of {n} tokens (the preset's median), {heads} of {cfg.num_heads} heads, "
                      f"{spent:.1f}s of CPU work", "prompt_tokens_per_s": n * heads / cfg.num_heads / spent}


def prefill_phase(fs, torch, wl, cfg, reps, log, with_cpu=True):
    """Initialization phase on the preset's shape: the jobs' lengths taken as prompt lengths,
    packed q, k, v [T][H][D]; fs_kv_prefill writes the cache blocks, fs_prefill_attention
    computes the causal attention of every prompt token.  Kernel times from launch-attached
    events; flops = 4*D per (query, visible key) pair and head."""
    if cfg.dtype == "f32":
        return None
    lens = wl.job_lens(cfg, wl.seed_for(cfg.index, 0)).astype(np.int64)
    H, D = cfg.num_heads, cfg.head_dim
    T = int(lens.sum())
    offs = np.zeros(cfg.num_jobs + 1, dtype=np.int32)
    offs[1:] = np.cumsum(lens)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float16
    g = torch.Generator(device="cuda")
    g.manual_seed(wl.seed_for(cfg.index, 0))
    q, k, v = (torch.randn((T, H, D), generator=g, device="cuda", dtype=torch.float32).to(tdt) for _ in range(3))
    out = torch.empty((T, H, D), dtype=torch.float32, device="cuda")
    nblk = (lens + cfg.block_size - 1) // cfg.block_size
    W = int(nblk.max())
    table = np.full((cfg.num_jobs, W), -1, dtype=np.int32)
    nb = 0
    for j in range(cfg.num_jobs):
        table[j, :nblk[j]] = np.arange(nb, nb + nblk[j])
        nb += int(nblk[j])
    pool = fs.Pool(cfg.dtype, H, D, nb)
    try:
        d_table, d_offs = torch.from_numpy(table).cuda(), torch.from_numpy(offs).cuda()
        d_starts = torch.zeros(cfg.num_jobs, dtype=torch.int32, device="cuda")

        def two_calls():
            fs.fs_kv_prefill(pool, d_table, d_starts, d_offs, T, k, v)
            fs.fs_prefill_attention(pool, q, k, v, d_offs, out)

        def fused():
            fs.fs_prefill_step(pool, d_table, d_offs, k, v, q, out)

        def timed(fn):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            pool.profile_enable(True)
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            wall_ms = (time.perf_counter() - t0) * 1e3 / reps
            prof = pool.profile_collect()
            pool.profile_enable(False)
            pool.check()
            return wall_ms, {kind: rec["ms"] / max(rec["launches"], 1) for kind, rec in prof.items() if rec["launches"]}

        wall_ms, kms = timed(two_calls)
        wall_f, kms_f = timed(fused)
        attn_ms = kms["prefill_attention"]
        flops = float(4 * D * H * (lens * (lens + 1) // 2).sum())
        hbm_bytes = float(T * H * D * (3 * cfg.elem_bytes + 4))
        res = {"workload": f"{cfg.name} lengths as prompts: {cfg.num_jobs} prompts, {T} tokens, {H} heads x {D}, {cfg.dtype}",
               "ms_per_pass": wall_ms, "prompt_tokens_per_s": T / (wall_ms / 1e3),
               "kernel_ms": {"prefill_attention": attn_ms, "kv_write": kms["prefill"], "work_list": kms["prefill_plan"]},
               "fused_step": {"ms_per_pass": wall_f, "prompt_tokens_per_s": T / (wall_f / 1e3),
                              "kernel_ms": {"prefill_attention": kms_f["prefill_attention"],
                                            "work_list": kms_f["prefill_plan"]}},
               "roofline": {"bound": "mfma", "achieved": flops / (attn_ms * 1e-3) / 1e12, "peak": MFMA_PEAK_TFLOPS,
                            "unit": "TFLOP/s", "frac": flops / (attn_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                            "traffic": None, "kernel": "fs_prefill_attn_kernel", "flops_per_launch": flops,
                            "alg_bytes_per_launch": hbm_bytes,
                            "alg_gbps": hbm_bytes / (attn_ms * 1e-3) / 1e9},
               "cpu_baseline": prefill_cpu_baseline(wl, cfg) if with_cpu else None}
        log(json.dumps(res))
        return res
    finally:
        pool.close()


def load_traffic(cfg_name):
    """HBM bytes per attention launch measured with rocprofv3 --pmc on this preset (the committed
    summary of that run: profiles/attn_partition_<preset>_traffic.txt), or None."""
    path = os.path.join(ROOT, "profiles", f"attn_partition_{cfg_name}_traffic.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for ln in open(path):
        if "=" in ln and not ln.lstrip().startswith("#"):
            k, v = ln.split("=", 1)
            vals[k.strip()] = v.strip()
    try:
        return float(vals["hbm_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def roofline_of(cfg, alg_bytes, attn_ms):
    achieved = alg_bytes / (attn_ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS, "traffic": load_traffic(cfg.name),
            "kernel": "fs_attn_partition_kernel", "kernel_ms": attn_ms, "alg_bytes_per_launch": alg_bytes}


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", type=int, default=1, help="workload preset timed as the headline (default 1)")
    ap.add_argument("--dtype", type=str, default="", choices=["", "bf16", "f16", "f32"],
                    help="override the presets' storage type (default: the preset's own, bf16)")
    ap.add_argument("--also", type=str, default="2,3,4", help="other presets reported under 'other_workloads'")
    ap.add_argument("--footprint-gb", type=float, default=2.0, help="bytes touched between reuses of a replica")
    ap.add_argument("--wgs-per-cu", type=int, default=0)
    ap.add_argument("--set", action="append", default=[], metavar="NAME=VALUE",
                    help="pool knob for every pool of the run (fs_pool_set_param), e.g. merge_in_kernel=1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-swap-overlap", action="store_true", help="skip the steps timed beside block swaps")
    ap.add_argument("--no-warm-cache", action="store_true", help="skip the steps repeated on one pool")
    ap.add_argument("--no-merge-in-kernel", action="store_true",
                    help="skip the steps timed with the combine merged into the attention kernel")
    ap.add_argument("--no-prefill", action="store_true", help="skip the initialization-phase measurement")
    ap.add_argument("--only-prefill", action="store_true", help="measure the initialization phase alone")
    ap.add_argument("--no-serving-run", action="store_true", help="skip the multi-iteration scheduler-driven run")
    ap.add_argument("--only-serving-run", action="store_true", help="run the scheduler-driven loop alone")
    ap.add_argument("--only-swap-overlap", action="store_true", help="time the steps beside the cache manager's swaps alone")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch the plain stream read/copy kernels over 1 GiB (scale of hardware byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards by head, with no exchange "
              "between GPUs); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import fs_workload as wl
    import paper_2305_05920_amd as fs
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    def log(msg):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    pool_kw = {}
    if args.calibrate_copy:
        n = 1 << 30
        src = torch.zeros(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty(n, dtype=torch.uint8, device="cuda")
        sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
        for _ in range(3):
            fs.fs_stream_read(src, sink, 2048)
            fs.fs_stream_copy(dst, src, 2048)
        torch.cuda.synchronize()
        log("calibration: 3x fs_stream_read_kernel and 3x fs_stream_copy_kernel over 1 GiB")
        del src, dst

    def config_of(idx):
        return wl.CONFIGS[idx] if not args.dtype else wl.CONFIGS[idx].scaled(dtype=args.dtype)

    def measure(idx, steps, warmup, cpu_budget_s, extras):
        """One preset: the two-call step (the headline form) and the fused step, each timed over at
        least 50 steps; kernel durations from launch-attached events; its own roofline object and
        its own CPU baseline (the oracle's whole step on the same inputs, one thread)."""
        cfg = config_of(idx)
        reps = Replicas(fs, torch, wl, cfg, 0, args.footprint_gb * 1e9, pool_kw, log)
        try:
            if args.wgs_per_cu:
                for p in reps.pools:
                    p.set_param("wgs_per_cu", args.wgs_per_cu)
            for kv in args.set:
                name, val = kv.split("=")
                for p in reps.pools:
                    p.set_param(name, int(val))
            nk = max(reps.R * 4, min(max(steps, MIN_TIMED_STEPS), 200))
            reps.fused = True
            t_f = time_steps(torch, reps, steps, warmup)
            kt_f = kernel_times(torch, reps, nk)
            reps.fused = False
            t = time_steps(torch, reps, steps, warmup)
            kt = kernel_times(torch, reps, nk)
            ms = t["median_ms"]
            res = {"workload": f"configs[{cfg.index}] {cfg.name}", "ms_per_step": ms, "step_timing": t,
                   "job_tokens_per_s": cfg.num_jobs / (ms / 1e3),
                   "kernel_ms": kt, "sum_len": int(reps.step.total_tokens), "replicas": reps.R,
                   "roofline": roofline_of(cfg, reps.alg_bytes, kt["attention"]),
                   "fused_step": {"ms_per_step": t_f["median_ms"], "step_timing": t_f,
                                  "job_tokens_per_s": cfg.num_jobs / (t_f["median_ms"] / 1e3), "kernel_ms": kt_f,
                                  "attention_gbps": reps.alg_bytes / (kt_f["attention"] * 1e-3) / 1e9}}
            if not args.no_merge_in_kernel:
                # the same two step forms with the cut pairs merged by the attention kernel
                # itself (no combine launch); the library's default is the combine launch
                for p in reps.pools:
                    p.set_param("merge_in_kernel", 1)
                reps.fused = True
                t_mf = time_steps(torch, reps, steps, warmup)
                reps.fused = False
                t_m = time_steps(torch, reps, steps, warmup)
                kt_m = kernel_times(torch, reps, nk)
                for p in reps.pools:
                    p.set_param("merge_in_kernel", 0)
                res["merge_in_kernel"] = {"ms_per_step": t_m["median_ms"], "fused_ms_per_step": t_mf["median_ms"],
                                          "kernel_ms": kt_m}
            if extras and not args.no_warm_cache:
                res["ms_per_step_warm_cache"] = time_steps_warm(torch, reps, steps, warmup)
            if not args.no_graph:
                try:
                    res["ms_per_step_graph"] = graph_ms(torch, reps, max(steps, MIN_TIMED_STEPS))
                except Exception as e:  # graph capture is an extra, never the headline
                    log(f"graph replay skipped: {e}")
            # the result of the last step against the oracle, and the oracle's own speed
            got = reps.out.cpu().numpy()
            if cpu_budget_s > 0:
                base, ref = cpu_baseline(reps, cpu_budget_s)
                res["cpu_baseline"] = base
                diff = got.astype(np.float64) - ref
                res["max_abs_err"] = float(np.abs(diff).max())
                res["rel_l2_err"] = float(np.linalg.norm(diff) / np.linalg.norm(ref))
                rows = np.linalg.norm(diff, axis=-1) / np.maximum(np.linalg.norm(ref, axis=-1), 1e-300)
                res["worst_row_rel_l2_err"] = float(rows.max())      # worst single (job, head) row
            else:
                res["cpu_baseline"] = None
            for p in reps.pools:
                p.check()
            log(json.dumps(res))
            return res
        finally:
            reps.close()

    cfg = config_of(args.config)
    if args.only_serving_run:
        print(json.dumps(serving_run(fs, torch, wl, cfg, log)), flush=True)
        return
    if args.only_prefill:
        print(json.dumps(prefill_phase(fs, torch, wl, cfg, 20, log, not args.no_cpu_baseline)), flush=True)
        return
    if args.only_swap_overlap:
        print(json.dumps(swap_overlap(fs, torch, wl, cfg, log)), flush=True)
        return
    with_cpu = not args.no_cpu_baseline
    main_res = measure(args.config, args.steps, args.warmup, 12.0 if with_cpu else 0.0, True)
    others = []
    for tok in [t for t in args.also.split(",") if t.strip()]:
        idx = int(tok)
        if idx == args.config:
            continue
        others.append(measure(idx, max(MIN_TIMED_STEPS, args.steps // 4), max(10, args.warmup // 4),
                              3.0 if with_cpu else 0.0, False))

    worst = min([main_res] + others, key=lambda r: r["roofline"]["frac"])
    line = {
        "metric": METRIC,
        "value": main_res["job_tokens_per_s"],
        "unit": "job-tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "ms_per_step_is": f"median over {main_res['step_timing']['timed_steps']} steps, each bracketed by events on the "
                          "kernels' stream (at least 50 whatever --steps says); step_timing.mean_wall_ms is the wall "
                          "clock over the same steps",
        "step_timing": main_res["step_timing"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"configs[{cfg.index}] {cfg.name}: {cfg.num_jobs} jobs, {cfg.num_heads} heads x "
                               f"{cfg.head_dim}, {cfg.dtype}, block 16, sum(L)={main_res['sum_len']}",
                   "step": "fs_kv_append + fs_decode_attention (partition pass + combine)",
                   "pool_replicas": main_res["replicas"]},
        "roofline": main_res["roofline"],
        # the lowest fraction of the HBM peak among the presets of this line, and whose it is
        "worst_roofline": {"workload": worst["workload"], "frac": worst["roofline"]["frac"],
                           "achieved": worst["roofline"]["achieved"], "kernel_ms": worst["roofline"]["kernel_ms"]},
        "cpu_baseline": main_res["cpu_baseline"],
        "kernel_ms": main_res["kernel_ms"],
        "fused_step": main_res["fused_step"],
        "merge_in_kernel": main_res.get("merge_in_kernel"),
        "ms_per_step_graph": main_res.get("ms_per_step_graph"),
        "ms_per_step_warm_cache": main_res.get("ms_per_step_warm_cache"),
        "max_abs_err": main_res.get("max_abs_err"),
        "rel_l2_err": main_res.get("rel_l2_err"),
        "worst_row_rel_l2_err": main_res.get("worst_row_rel_l2_err"),
        "other_workloads": others,
    }
    if not args.no_warm_cache:
        ceil = read_ceiling(fs, torch)
        for r in [line] + others:
            r["roofline"]["practical_read_ceiling_gbps"] = ceil
            r["roofline"]["frac_of_practical_ceiling"] = r["roofline"]["achieved"] / ceil
        # the same bytes read by a kernel that does nothing else: what the size itself allows
        rows = [line] + others
        for r, sr in zip(rows, same_bytes_read(fs, torch, [r["roofline"]["alg_bytes_per_launch"] for r in rows])):
            sr["attention_kernel_over_plain_read"] = r["roofline"]["kernel_ms"] * 1e3 / sr["kernel_us"]
            r["roofline"]["plain_read_of_same_bytes"] = sr
    if not args.no_swap_overlap:
        line["swap_overlap"] = [swap_overlap(fs, torch, wl, config_of(i), log) for i in (1, 3)
                                if config_of(i).dtype != "f32"]
    if not args.no_serving_run:
        line["serving_run"] = serving_run(fs, torch, wl, cfg, log)
    if not args.no_prefill:
        line["prefill_phase"] = prefill_phase(fs, torch, wl, cfg, 20, log, with_cpu)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
