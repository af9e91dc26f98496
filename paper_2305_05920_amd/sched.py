"""Binding of the host-side serving policy (C ABI in include/fastserve_sched.h):
skip-join MLFQ scheduler and ENST swap order.  Argument marshalling only."""
from __future__ import annotations

import ctypes
from typing import List, Sequence, Tuple

from . import FsError, load_library

SCHED_EXPORTS = (
    "fs_sched_create", "fs_sched_destroy", "fs_sched_add_job", "fs_sched_set_ready", "fs_sched_schedule",
    "fs_sched_complete_iteration", "fs_sched_job_info", "fs_sched_num_jobs", "fs_sched_enst",
    "fs_sched_swap_order",
)


def _lib():
    lib = load_library()
    if getattr(lib, "_fs_sched_ready", False):
        return lib
    vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
    P = ctypes.POINTER
    lib.fs_sched_create.argtypes = [i32, dbl, i32, dbl, i32, P(vp)]
    lib.fs_sched_destroy.argtypes = [vp]
    lib.fs_sched_add_job.argtypes = [vp, i64, dbl, dbl, P(i32)]
    lib.fs_sched_set_ready.argtypes = [vp, i64, i32]
    lib.fs_sched_schedule.argtypes = [vp, P(i64), i32, P(i32)]
    lib.fs_sched_complete_iteration.argtypes = [vp, P(i64), i32, dbl, P(i64), i32]
    lib.fs_sched_job_info.argtypes = [vp, i64, P(i32), P(dbl), P(dbl), P(i64)]
    lib.fs_sched_num_jobs.argtypes = [vp]
    lib.fs_sched_enst.argtypes = [vp, i64, P(dbl), P(dbl), P(dbl)]
    lib.fs_sched_swap_order.argtypes = [vp, P(i64), i32, i32, P(i64)]
    for name in SCHED_EXPORTS:
        getattr(lib, name).restype = ctypes.c_int
    lib._fs_sched_ready = True
    return lib


def _ok(status: int, where: str) -> None:
    if status != 0:
        raise FsError(status, where)


def _ids(seq: Sequence[int]):
    arr = (ctypes.c_int64 * max(len(seq), 1))(*seq)
    return arr


class Scheduler:
    def __init__(self, num_queues: int, q1: float, eta: int, alpha: float, max_batch: int, _handle=None):
        self._lib = _lib()
        self._owned = _handle is None
        if _handle is not None:                     # a scheduler some other object of the library owns
            self._h, self.max_batch = ctypes.c_void_p(_handle), max_batch
            return
        h = ctypes.c_void_p()
        _ok(self._lib.fs_sched_create(num_queues, q1, eta, alpha, max_batch, ctypes.byref(h)), "fs_sched_create")
        self._h, self.max_batch = h, max_batch

    def close(self) -> None:
        if getattr(self, "_h", None) and self._owned:
            self._lib.fs_sched_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def add_job(self, job_id: int, init_time: float, decode_time: float) -> int:
        q = ctypes.c_int32()
        _ok(self._lib.fs_sched_add_job(self._h, job_id, init_time, decode_time, ctypes.byref(q)), "fs_sched_add_job")
        return q.value

    def set_ready(self, job_id: int, ready: bool) -> None:
        _ok(self._lib.fs_sched_set_ready(self._h, job_id, 1 if ready else 0), "fs_sched_set_ready")

    def schedule(self) -> List[int]:
        out = (ctypes.c_int64 * self.max_batch)()
        n = ctypes.c_int32()
        _ok(self._lib.fs_sched_schedule(self._h, out, self.max_batch, ctypes.byref(n)), "fs_sched_schedule")
        return list(out[:n.value])

    def complete_iteration(self, ran: Sequence[int], elapsed: float, finished: Sequence[int]) -> None:
        _ok(self._lib.fs_sched_complete_iteration(self._h, _ids(ran), len(ran), elapsed, _ids(finished),
                                                  len(finished)), "fs_sched_complete_iteration")

    def job_info(self, job_id: int) -> Tuple[int, float, float, int]:
        p, used, starve, it = ctypes.c_int32(), ctypes.c_double(), ctypes.c_double(), ctypes.c_int64()
        _ok(self._lib.fs_sched_job_info(self._h, job_id, ctypes.byref(p), ctypes.byref(used), ctypes.byref(starve),
                                        ctypes.byref(it)), "fs_sched_job_info")
        return p.value, used.value, starve.value, it.value

    def num_jobs(self) -> int:
        return int(self._lib.fs_sched_num_jobs(self._h))

    def enst(self, job_id: int) -> Tuple[float, float, float]:
        a, b, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        _ok(self._lib.fs_sched_enst(self._h, job_id, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "fs_sched_enst")
        return a.value, b.value, c.value

    def swap_order(self, candidates: Sequence[int], swap_in: bool) -> List[int]:
        n = len(candidates)
        out = (ctypes.c_int64 * max(n, 1))()
        _ok(self._lib.fs_sched_swap_order(self._h, _ids(candidates), n, 1 if swap_in else 0, out), "fs_sched_swap_order")
        return list(out[:n])
