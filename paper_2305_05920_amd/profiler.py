"""Iteration-time profile for the scheduler (FastServe, Section 4.1: the skip-join MLFQ
assigns a new job to a queue by the time of its first iteration, which "the job profiler"
supplies from the prompt length; Section 3.2 names the profiler as a component).

The profile is measured on this GPU with the library's own kernels: the initialization
phase of one job (``fs_prefill_step``) for a range of prompt lengths, and one decode step
(``fs_decode_step``) for a range of cache lengths, each as the sum of the kernels' own
durations from launch-attached events.  Times are for ONE layer's attention path -- the
part of the model this library implements; a model with l identical layers scales them by l,
which leaves the queue a job skip-joins unchanged when the quanta are scaled the same way.
"""
from __future__ import annotations

from typing import Dict, Sequence

import numpy as np
import torch

from . import Pool, fs_decode_step, fs_prefill_step


class IterationTimeProfile:
    def __init__(self, dtype: str, num_heads: int, head_dim: int,
                 prompt_lengths: Sequence[int] = (16, 32, 64, 128, 256, 512, 1024, 2048),
                 cache_lengths: Sequence[int] = (16, 256, 2048), reps: int = 5, seed: int = 0):
        self.prompt_lengths = np.array(sorted(prompt_lengths), dtype=np.float64)
        self.cache_lengths = np.array(sorted(cache_lengths), dtype=np.float64)
        H, D = num_heads, head_dim
        tdt = {"bf16": torch.bfloat16, "f16": torch.float16}[dtype]
        smax = int(max(self.prompt_lengths.max(), self.cache_lengths.max())) + 1
        nblk = (smax + 15) // 16 + 1
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        q, k, v = (torch.randn((smax, H, D), generator=g, device="cuda").to(tdt) for _ in range(3))
        out = torch.empty((smax, H, D), dtype=torch.float32, device="cuda")
        table = torch.arange(nblk, dtype=torch.int32, device="cuda").reshape(1, nblk)
        with Pool(dtype, H, D, nblk) as pool:
            def timed(fn) -> float:
                # median over single calls: one slow outlier (first use of a kernel, a clock ramp)
                # must not end up in the table
                for _ in range(2):
                    fn()
                torch.cuda.synchronize()
                vals = []
                for _ in range(reps):
                    pool.profile_enable(True)
                    fn()
                    torch.cuda.synchronize()
                    prof = pool.profile_collect()
                    pool.profile_enable(False)
                    vals.append(sum(r["ms"] for r in prof.values()))
                return float(np.median(vals))

            self.init_ms = []
            for s in self.prompt_lengths.astype(int):
                offs = torch.tensor([0, s], dtype=torch.int32, device="cuda")
                self.init_ms.append(timed(lambda: fs_prefill_step(pool, table, offs, k[:s], v[:s], q[:s], out[:s])))
            self.decode_ms = []
            for L in self.cache_lengths.astype(int):
                lens = torch.tensor([L], dtype=torch.int32, device="cuda")
                self.decode_ms.append(timed(lambda: fs_decode_step(pool, table, lens, k[:1], v[:1], q[:1], out[:1])))
            pool.check()
        self.init_ms = np.array(self.init_ms)
        self.decode_ms = np.array(self.decode_ms)

    def init_time(self, prompt_tokens: int) -> float:
        """Milliseconds of the first iteration of a job with that many prompt tokens
        (piecewise linear between the measured lengths, linear extrapolation beyond)."""
        x, y = self.prompt_lengths, self.init_ms
        if prompt_tokens >= x[-1] and len(x) > 1:
            slope = (y[-1] - y[-2]) / (x[-1] - x[-2])
            return float(y[-1] + slope * (prompt_tokens - x[-1]))
        return float(np.interp(prompt_tokens, x, y))

    def decode_time(self, cache_tokens: int = 0) -> float:
        """Milliseconds of one decode iteration of a job with that many cached tokens."""
        return float(np.interp(cache_tokens, self.cache_lengths, self.decode_ms))

    def min_iteration_time(self) -> float:
        """The quantum of the highest-priority queue (Section 4.1: q_1 is the minimum
        iteration time)."""
        return float(min(self.init_ms.min(), self.decode_ms.min()))

    def as_dict(self) -> Dict[str, list]:
        return {"prompt_lengths": self.prompt_lengths.astype(int).tolist(), "init_ms": self.init_ms.tolist(),
                "cache_lengths": self.cache_lengths.astype(int).tolist(), "decode_ms": self.decode_ms.tolist()}
