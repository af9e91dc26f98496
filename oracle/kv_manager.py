"""Oracle of the proactive key-value cache manager and of the iteration loop around it
(test infrastructure only; plain Python, the paper's steps in the paper's order).

Manager: paper Section 4.2.  Key-value tensors of inactive jobs are swapped out to host
memory and swapped back before the job is scheduled ("Proactive key-value cache
management"); the order follows the estimated next scheduled time, latest out first,
earliest in first ("Job swapping order"); some blocks stay idle for newly arrived jobs, their
number following the arrival history ("Handling a burst of new jobs").  Loop: Section 3.2
(scheduler picks a batch, the engine runs one iteration on it, finished jobs leave) and
Algorithm 1.

Where the paper leaves room, this file takes these readings: a job moves as a whole; the lowest
free block id (host slot) is handed out first; a move is "in flight" until the caller says it completed (retire), and only then do
vacated blocks or slots return and does a returning job become ready; the idle reserve is
the ceil(quantile*n)-th smallest of the last n per-iteration demands, at least the fixed
reserve, at most half the pool; a job that leaves while a move of it is in flight is
forgotten when that move retires.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

from .scheduler import SkipJoinMLFQ

RESIDENT, LEAVING, SWAPPED_OUT, RETURNING = 0, 1, 2, 3


@dataclass
class CacheOfJob:
    length: int = 0
    blocks: List[int] = field(default_factory=list)
    slots: List[int] = field(default_factory=list)
    where: int = RESIDENT
    released: bool = False


class ProactiveCacheManager:
    def __init__(self, sched: Optional[SkipJoinMLFQ], num_blocks: int, num_host_blocks: int, block_size: int,
                 table_width: int, reserve_idle_blocks: int = 0, reserve_window: int = 0,
                 reserve_quantile: float = 0.0):
        self.sched = sched
        self.N, self.B, self.W = num_blocks, block_size, table_width
        self.fixed_reserve, self.window, self.quantile = reserve_idle_blocks, reserve_window, reserve_quantile
        self.reserve = reserve_idle_blocks
        self.history: List[int] = []
        self.free_blocks = set(range(num_blocks))
        self.free_slots = set(range(num_host_blocks))
        self.jobs: Dict[int, CacheOfJob] = {}
        self.moves: List[dict] = []          # in flight, oldest first
        self.blocks_out = self.blocks_in = 0

    def blocks_needed(self, tokens: int) -> int:
        return -(-tokens // self.B)

    @staticmethod
    def take(free: set, n: int) -> List[int]:
        """The n lowest free ids, in rising order."""
        ids = sorted(free)[:max(n, 0)]
        free.difference_update(ids)
        return ids

    # -- "Handling a burst of new jobs" ---------------------------------------------
    def observe_arrivals(self, demand: int) -> None:
        if self.window <= 0:
            return
        self.history = (self.history + [demand])[-self.window:]
        n = len(self.history)
        rank = min(n, max(1, math.ceil(self.quantile * n)))      # 1-based
        wanted = max(self.fixed_reserve, sorted(self.history)[rank - 1])
        self.reserve = min(wanted, max(self.fixed_reserve, self.N // 2))

    # -- block-grained allocation (Section 2.2) ---------------------------------------
    def admit(self, job: int, tokens: int) -> bool:
        n = self.blocks_needed(tokens)
        if n > len(self.free_blocks) or n > self.W:
            return False
        self.jobs[job] = CacheOfJob(blocks=self.take(self.free_blocks, n))
        return True

    def grow(self, job: int, new_tokens: int = 1) -> bool:
        c = self.jobs[job]
        assert c.where == RESIDENT
        need = self.blocks_needed(c.length + new_tokens) - len(c.blocks)
        if need > len(self.free_blocks) or len(c.blocks) + need > self.W:
            return False
        c.blocks += self.take(self.free_blocks, need)
        return True

    def advance(self, job: int, tokens: int) -> None:
        self.jobs[job].length += tokens

    def release(self, job: int) -> None:
        c = self.jobs[job]
        if c.where in (LEAVING, RETURNING):
            c.released = True
            return
        self.free_blocks.update(c.blocks)
        self.free_slots.update(c.slots)
        del self.jobs[job]

    # -- "Job swapping order" ---------------------------------------------------------
    def start_swaps(self, running: Sequence[int], want_free: int) -> List[tuple]:
        """Returns the moves issued, in order: ("out" | "in", job)."""
        margin = self.reserve + want_free
        issued = []
        out = [j for j, c in self.jobs.items()
               if c.where == RESIDENT and not c.released and c.blocks and j not in running]
        soon = len(self.free_blocks) + sum(len(m["vacated"]) for m in self.moves if m["out"])
        for j in self.sched.swap_out_order(out):
            if soon >= margin:
                break
            c = self.jobs[j]
            if len(c.blocks) > len(self.free_slots):
                continue
            soon += len(c.blocks)
            slots = self.take(self.free_slots, len(c.blocks))
            self.moves.append({"job": j, "out": True, "vacated": c.blocks})
            self.blocks_out += len(slots)
            c.slots, c.blocks, c.where = slots, [], LEAVING
            self.sched.set_ready(j, False)
            issued.append(("out", j))
        back = [j for j, c in self.jobs.items() if c.where == SWAPPED_OUT and not c.released]
        for j in self.sched.swap_in_order(back):
            c = self.jobs[j]
            if len(self.free_blocks) - len(c.slots) < margin:
                break
            blocks = self.take(self.free_blocks, len(c.slots))
            self.moves.append({"job": j, "out": False, "vacated": c.slots})
            self.blocks_in += len(blocks)
            c.blocks, c.slots, c.where = blocks, [], RETURNING
            issued.append(("in", j))
        return issued

    def retire(self, how_many: int = -1) -> int:
        n = 0
        while self.moves and (how_many < 0 or n < how_many):
            m = self.moves.pop(0)
            (self.free_blocks if m["out"] else self.free_slots).update(m["vacated"])
            c = self.jobs.get(m["job"])
            if c is not None:
                if c.released:
                    self.free_blocks.update(c.blocks)
                    self.free_slots.update(c.slots)
                    del self.jobs[m["job"]]
                elif m["out"]:
                    c.where = SWAPPED_OUT
                else:
                    c.where = RESIDENT
                    self.sched.set_ready(m["job"], True)
            n += 1
        return n

    def table_row(self, job: int) -> List[int]:
        b = self.jobs[job].blocks
        return b + [-1] * (self.W - len(b))


class IterationLoop:
    """Section 3.2 / Algorithm 1 around the manager: arrivals wait until their blocks fit beside
    the idle reserve; every iteration the scheduler picks a batch, decoding jobs take room for
    one more token (one that finds none sits out), swaps for the waiting and the sat-out are
    started, every job that ran produces one token, finished jobs leave."""

    def __init__(self, num_queues: int, q1: float, eta: int, alpha: float, max_batch: int,
                 max_prompt_tokens: int, **manager_kw):
        self.sched = SkipJoinMLFQ(num_queues, q1, eta, alpha, max_batch)
        self.kvm = ProactiveCacheManager(self.sched, **manager_kw)
        self.q1, self.max_prompt_tokens = q1, max_prompt_tokens
        self.jobs: Dict[int, dict] = {}
        self.future: List[int] = []
        self.waiting: List[int] = []
        self.iteration = 0
        self.job_tokens = self.prompt_tokens = self.finished = self.idle_iterations = 0

    def submit(self, job, arrival, prompt, outputs, init_time, decode_time):
        self.jobs[job] = dict(arrival=arrival, prompt=prompt, outputs=outputs, produced=0,
                              init=init_time, decode=decode_time)
        self.future.append(job)

    def plan(self):
        k = self.kvm
        arrived = [j for j in self.future if self.jobs[j]["arrival"] <= self.iteration]
        self.future = [j for j in self.future if j not in arrived]
        self.waiting += arrived
        k.observe_arrivals(sum(k.blocks_needed(self.jobs[j]["prompt"] + 1) for j in arrived))
        k.retire()
        for j in list(self.waiting):
            need = k.blocks_needed(self.jobs[j]["prompt"] + 1)
            if need + k.reserve <= len(k.free_blocks) and k.admit(j, self.jobs[j]["prompt"] + 1):
                self.sched.add_job(j, self.jobs[j]["init"], self.jobs[j]["decode"])
                self.waiting.remove(j)
        batch = self.sched.schedule()
        first, decode, lens, sat_out, packed = [], [], [], 0, 0
        for j in batch:
            if k.jobs[j].length == 0:
                p = self.jobs[j]["prompt"]
                if self.max_prompt_tokens > 0 and packed + p > self.max_prompt_tokens and first:
                    sat_out += 1
                    continue
                first.append(j)
                packed += p
            elif k.grow(j, 1):
                decode.append(j)
                lens.append(k.jobs[j].length)
            else:
                sat_out += 1
        self.ran = [j for j in batch if j in first or j in decode]
        want = sat_out + sum(k.blocks_needed(self.jobs[j]["prompt"] + 1) for j in self.waiting)
        moves = k.start_swaps(self.ran, min(want, k.N // 2))
        return dict(first=first, decode=decode, lens_before=lens, moves=moves)

    def complete(self):
        finished, elapsed = [], 0.0
        for j in self.ran:
            job = self.jobs[j]
            is_first = job["produced"] == 0
            self.kvm.advance(j, job["prompt"] if is_first else 1)
            if is_first:
                self.prompt_tokens += job["prompt"]
            job["produced"] += 1
            self.job_tokens += 1
            elapsed = max(elapsed, job["init"] if is_first else job["decode"])
            if job["produced"] == job["outputs"]:
                finished.append(j)
        if not self.ran:
            elapsed = self.q1
            self.idle_iterations += 1
        self.sched.complete_iteration(self.ran, elapsed, finished)
        for j in finished:
            self.kvm.release(j)
            del self.jobs[j]
            self.finished += 1
        self.iteration += 1
