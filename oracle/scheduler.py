"""Oracle of the skip-join MLFQ scheduler and of the swap-order estimate (test
infrastructure only; plain Python, follows the paper's steps and notation).

Scheduler: paper Section 4.1 and Algorithm 1.  n priority queues Q_1..Q_n with
quanta q_1 < ... < q_n, q_{k+1} = 2 q_k, q_1 = the minimum iteration time.  A new
job skip-joins the highest-priority queue whose quantum covers its first
(initialization) iteration; a job that uses up its quantum is demoted; a job that
has waited alpha or longer is promoted to Q_1; each call hands out at most
MaxBatchSize ready jobs in priority order.

Swap order: paper Section 4.2, "Job swapping order": ENST(i) =
min(T_promote(i), T_execute(i)).

Where the paper leaves room, this file takes these readings: a job that ran is charged
the iteration's elapsed time; a demoted job moves eta queues down, further if its next
iteration would not fit that quantum; waiting time counts from the last run, arrival or
promotion; jobs are visited Q_1 first, first-in first-out inside a queue; in the ENST sum
a job j of a higher-priority queue passes the quanta of its own queue and of every queue
between it and job i's queue.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional


@dataclass
class Job:
    job_id: int
    init_time: float          # profiled time of the first (initialization) iteration
    decode_time: float        # profiled time of a decoding iteration
    priority: int = 1         # queue index, 1 = highest
    used: float = 0.0         # time consumed of the current queue's quantum
    starve: float = 0.0       # time waited since it last ran (or arrived, or was promoted)
    iterations: int = 0       # iterations executed so far
    ready: bool = True        # key-value tensors resident in GPU memory

    def next_iter_time(self) -> float:
        return self.init_time if self.iterations == 0 else self.decode_time


class SkipJoinMLFQ:
    def __init__(self, num_queues: int, q1: float, eta: int, alpha: float, max_batch: int):
        assert num_queues >= 1 and q1 > 0 and eta >= 1 and max_batch >= 1
        self.n = num_queues
        self.q = [q1 * (2 ** k) for k in range(num_queues)]     # q[k-1] = quantum of Q_k
        self.eta, self.alpha, self.B = eta, alpha, max_batch
        self.queues: List[List[int]] = [[] for _ in range(num_queues)]   # job ids, FIFO
        self.jobs: Dict[int, Job] = {}

    # -- Algorithm 1, "skip-join newly arrived jobs" -----------------------------
    def queue_for(self, t: float) -> int:
        """min i such that q_i >= t (the lowest queue if none)."""
        for i, qi in enumerate(self.q, start=1):
            if qi >= t:
                return i
        return self.n

    def add_job(self, job_id: int, init_time: float, decode_time: float) -> int:
        assert job_id not in self.jobs
        p = self.queue_for(init_time)
        self.jobs[job_id] = Job(job_id, init_time, decode_time, priority=p)
        self.queues[p - 1].append(job_id)
        return p

    def set_ready(self, job_id: int, ready: bool) -> None:
        self.jobs[job_id].ready = ready

    # -- Algorithm 1, the loop over all queued jobs after an iteration ------------
    def complete_iteration(self, ran: List[int], elapsed: float, finished: List[int]) -> None:
        ran_set, fin = set(ran), set(finished)
        order = [jid for Q in self.queues for jid in Q]            # Q_1 .. Q_n, FIFO inside
        for jid in order:
            job = self.jobs[jid]
            p = job.priority
            if jid in ran_set:
                job.iterations += 1                                 # outputNewGeneratedToken
                job.used += elapsed
                job.starve = 0.0
                if jid in fin:                                      # isFinished
                    self.queues[p - 1].remove(jid)
                    del self.jobs[jid]
                    continue
                if job.used >= self.q[p - 1]:                       # depleteQuantum: demote
                    target = min(self.n, max(p + self.eta, self.queue_for(job.next_iter_time())))
                    self.queues[p - 1].remove(jid)
                    self.queues[target - 1].append(jid)
                    job.priority, job.used = target, 0.0
            else:
                job.starve += elapsed
                if job.starve >= self.alpha and p != 1:             # promote starved jobs
                    self.queues[p - 1].remove(jid)
                    self.queues[0].append(jid)
                    job.priority, job.used, job.starve = 1, 0.0, 0.0
                elif job.starve >= self.alpha:
                    job.starve = 0.0

    # -- Algorithm 1, "schedule jobs to execute" -----------------------------------
    def schedule(self) -> List[int]:
        out: List[int] = []
        for Q in self.queues:
            for jid in Q:
                if len(out) >= self.B:
                    return out
                if self.jobs[jid].ready:
                    out.append(jid)
        return out

    # -- Section 4.2, estimated next scheduled time --------------------------------
    def t_promote(self, job_id: int) -> float:
        return max(0.0, self.alpha - self.jobs[job_id].starve)

    def t_execute(self, job_id: int) -> float:
        """(1/B) * sum over jobs j of higher priority of the quanta j passes through
        while it is demoted, queue by queue, down to job i's queue."""
        pi = self.jobs[job_id].priority
        total = 0.0
        for other in self.jobs.values():
            if other.priority < pi:
                total += sum(self.q[k - 1] for k in range(other.priority, pi))
        return total / self.B

    def enst(self, job_id: int) -> float:
        return min(self.t_promote(job_id), self.t_execute(job_id))

    def swap_out_order(self, candidates: List[int]) -> List[int]:
        """Largest ENST first (ties: lower priority first, then larger id)."""
        return sorted(candidates, key=lambda j: (-self.enst(j), -self.jobs[j].priority, -j))

    def swap_in_order(self, candidates: List[int]) -> List[int]:
        """Smallest ENST first (ties: higher priority first, then smaller id)."""
        return sorted(candidates, key=lambda j: (self.enst(j), self.jobs[j].priority, j))


# ---------------------------------------------------------------------------------
# Reference policies for the pins (not part of the method): run a single-server,
# batch-size-1 timeline where a job is (init_time, n_decode * decode_time).
# ---------------------------------------------------------------------------------
def simulate_single_server(sched: Optional[SkipJoinMLFQ], jobs: List[dict]) -> Dict[int, float]:
    """Completion times with the scheduler driving a batch of one; jobs:
    {id, init, decode, n_decode}, all arriving at t=0 in list order."""
    t = 0.0
    left = {j["id"]: 1 + j["n_decode"] for j in jobs}
    for j in jobs:
        sched.add_job(j["id"], j["init"], j["decode"])
    done: Dict[int, float] = {}
    while left:
        batch = sched.schedule()
        assert len(batch) == 1
        jid = batch[0]
        dt = sched.jobs[jid].next_iter_time()
        t += dt
        left[jid] -= 1
        fin = [jid] if left[jid] == 0 else []
        if fin:
            done[jid] = t
            del left[jid]
        sched.complete_iteration([jid], dt, fin)
    return done
