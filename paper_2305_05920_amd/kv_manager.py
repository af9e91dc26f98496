"""Proactive key-value cache manager (FastServe, Section 4.2) on top of the block pool.

Host-side bookkeeping only: which job owns which pool blocks, which jobs sit in the
pinned host mirror, and in which order jobs move (the ENST order of the scheduler).
The copies themselves are the library's ``fs_pool_offload`` / ``fs_pool_upload`` on a
side stream, so that the transfer of waiting jobs overlaps the decode kernels of the
running batch; the decode kernels see nothing of this but the block table.

Blocks are owned by jobs in whole; a job is either resident (all its blocks in HBM) or
swapped out (all its blocks in host slots).  A model has one pool per layer; the manager
takes them all (``layers``): block ids and host slots are shared by the layers, so one
table serves every layer and a job's whole key-value tensor -- all layers, as the paper's
cache size 4*l*h*(s+t) counts it -- moves together.  ``reserve_idle_blocks`` HBM blocks are
kept free for new arrivals (Section 4.2, "Handling a burst of new jobs").
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Union

import numpy as np
import torch

from . import Pool, fs_pool_offload, fs_pool_upload
from .sched import Scheduler


class ArrivalReserve:
    """How many HBM blocks to keep idle for new jobs (Section 4.2, "Handling a burst of new
    jobs": the number of idle slots follows the historical arrival pattern, more for more
    frequent bursts).  The paper gives no formula; this one keeps the demand -- blocks asked
    for by the jobs that arrived in one iteration -- of the last `window` iterations and
    reserves a high quantile of it, never less than `floor` blocks."""

    def __init__(self, window: int = 64, quantile: float = 0.9, floor: int = 0):
        if window < 1 or not 0.0 <= quantile <= 1.0 or floor < 0:
            raise ValueError("window >= 1, 0 <= quantile <= 1, floor >= 0")
        self.window, self.quantile, self.floor = window, quantile, floor
        self.history: List[int] = []

    def observe(self, blocks_demanded: int) -> None:
        """Record one iteration (0 when nothing arrived)."""
        self.history.append(int(blocks_demanded))
        if len(self.history) > self.window:
            del self.history[0]

    def blocks(self) -> int:
        if not self.history:
            return self.floor
        ordered = sorted(self.history)
        k = min(len(ordered) - 1, int(np.ceil(self.quantile * len(ordered))) - 1 if self.quantile > 0 else 0)
        return max(self.floor, ordered[max(k, 0)])


@dataclass
class JobBlocks:
    length: int = 0                                         # tokens cached
    blocks: List[int] = field(default_factory=list)         # pool block ids (when resident)
    host_slots: List[int] = field(default_factory=list)     # host slots (when swapped out)
    resident: bool = True


class KVManager:
    def __init__(self, pool: Union[Pool, Sequence[Pool]], sched: Scheduler, table_width: int,
                 reserve_idle_blocks: int = 0):
        self.layers: List[Pool] = [pool] if isinstance(pool, Pool) else list(pool)
        pool = self.layers[0]
        if any(p.num_blocks != pool.num_blocks or p.num_host_blocks != pool.num_host_blocks or
               p.block_size != pool.block_size for p in self.layers):
            raise ValueError("the layers' pools must have the same numbers of blocks and host slots")
        self.pool, self.sched = pool, sched
        self.B = pool.block_size
        self.W = table_width
        self.reserve = reserve_idle_blocks          # blocks kept free for new arrivals; see observe_arrivals
        self.arrival_reserve: Optional[ArrivalReserve] = None
        self.free_blocks: List[int] = list(range(pool.num_blocks - 1, -1, -1))
        self.free_slots: List[int] = list(range(pool.num_host_blocks - 1, -1, -1))
        self.jobs: Dict[int, JobBlocks] = {}
        self.side = torch.cuda.Stream()
        self.swapped_out_blocks = 0      # statistics
        self.swapped_in_blocks = 0

    def observe_arrivals(self, blocks_demanded: int) -> None:
        """Once per iteration: the blocks the jobs that arrived in it ask for.  With an
        ArrivalReserve attached (``arrival_reserve``), the reserve follows the arrival history."""
        if self.arrival_reserve is not None:
            self.arrival_reserve.observe(blocks_demanded)
            self.reserve = min(self.arrival_reserve.blocks(), self.pool.num_blocks // 2)

    # -- allocation ---------------------------------------------------------------------
    def blocks_needed(self, tokens: int) -> int:
        return (tokens + self.B - 1) // self.B

    def can_admit(self, tokens: int) -> bool:
        return self.blocks_needed(tokens) <= len(self.free_blocks)

    def admit(self, job_id: int, tokens: int) -> None:
        """Allocate blocks for a new job's `tokens` tokens (its prompt)."""
        n = self.blocks_needed(tokens)
        if n > len(self.free_blocks) or n > self.W:
            raise MemoryError("no room for the job")
        self.jobs[job_id] = JobBlocks(length=0, blocks=[self.free_blocks.pop() for _ in range(n)])

    def grow(self, job_id: int, new_tokens: int = 1) -> bool:
        """Make room for `new_tokens` more tokens of a resident job; False if HBM is full."""
        jb = self.jobs[job_id]
        need = self.blocks_needed(jb.length + new_tokens) - len(jb.blocks)
        if need > len(self.free_blocks) or len(jb.blocks) + need > self.W:
            return False
        for _ in range(need):
            jb.blocks.append(self.free_blocks.pop())
        return True

    def advance(self, job_id: int, tokens: int = 1) -> None:
        self.jobs[job_id].length += tokens

    def release(self, job_id: int) -> None:
        jb = self.jobs.pop(job_id)
        self.free_blocks.extend(jb.blocks)
        self.free_slots.extend(jb.host_slots)

    def table_rows(self, job_ids: Sequence[int]) -> np.ndarray:
        t = np.full((len(job_ids), self.W), -1, dtype=np.int32)
        for r, j in enumerate(job_ids):
            b = self.jobs[j].blocks
            t[r, :len(b)] = b
        return t

    # -- swapping -----------------------------------------------------------------------
    def _offload(self, job_id: int) -> None:
        jb = self.jobs[job_id]
        slots = [self.free_slots.pop() for _ in jb.blocks]
        for layer in self.layers:
            fs_pool_offload(layer, jb.blocks, slots, stream=self.side)
        self.swapped_out_blocks += len(slots) * len(self.layers)
        self._pending_free.extend(jb.blocks)      # reusable once the copy has run
        jb.host_slots, jb.blocks, jb.resident = slots, [], False
        self.sched.set_ready(job_id, False)

    def _upload(self, job_id: int) -> None:
        jb = self.jobs[job_id]
        blocks = [self.free_blocks.pop() for _ in jb.host_slots]
        for layer in self.layers:
            fs_pool_upload(layer, jb.host_slots, blocks, stream=self.side)
        self.swapped_in_blocks += len(blocks) * len(self.layers)
        self._pending_slots.extend(jb.host_slots)
        self._pending_ready.append(job_id)         # schedulable once the copy has run
        jb.blocks, jb.host_slots, jb.resident = blocks, [], True

    def start_swaps(self, running: Sequence[int], want_free: int = 0) -> None:
        """Issue this iteration's swaps on the side stream (they overlap the decode step
        of `running`, which the caller launches next on its own stream).

        Swap out, largest ENST first, resident jobs that are not running until
        `reserve_idle_blocks + want_free` blocks are free (counting blocks whose offload
        is in flight); then swap in, smallest ENST first, jobs whose return leaves that
        margin intact."""
        self._pending_free: List[int] = []
        self._pending_slots: List[int] = []
        self._pending_ready: List[int] = []
        # the copies must see everything the compute stream has written so far
        self.side.wait_stream(torch.cuda.current_stream())
        margin = self.reserve + want_free
        running = set(running)
        out_cand = [j for j, jb in self.jobs.items() if jb.resident and j not in running and jb.blocks]
        free_after = len(self.free_blocks)
        for j in self.sched.swap_order(out_cand, swap_in=False):
            if free_after >= margin:
                break
            if len(self.jobs[j].blocks) > len(self.free_slots):
                continue
            free_after += len(self.jobs[j].blocks)
            self._offload(j)
        in_cand = [j for j, jb in self.jobs.items() if not jb.resident]
        for j in self.sched.swap_order(in_cand, swap_in=True):
            n = len(self.jobs[j].host_slots)
            if len(self.free_blocks) - n < margin:
                break
            self._upload(j)

    def finish_swaps(self) -> None:
        """Wait for the side stream; blocks and slots vacated by the copies become free
        and uploaded jobs become schedulable."""
        self.side.synchronize()
        self.free_blocks.extend(self._pending_free)
        self.free_slots.extend(self._pending_slots)
        for j in self._pending_ready:
            if j in self.jobs:
                self.sched.set_ready(j, True)
        self._pending_free, self._pending_slots, self._pending_ready = [], [], []
