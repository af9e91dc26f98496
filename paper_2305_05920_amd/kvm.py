"""Binding of the proactive key-value cache manager and of the iteration loop (C ABI in
include/fastserve_kvm.h).  Argument marshalling only: every decision is taken in the library."""
from __future__ import annotations

import ctypes
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import FsError, Pool, load_library
from . import sched as _sched

KVM_EXPORTS = (
    "fs_kvm_create", "fs_kvm_destroy", "fs_kvm_blocks_needed", "fs_kvm_free_blocks", "fs_kvm_free_slots",
    "fs_kvm_reserve", "fs_kvm_observe_arrivals", "fs_kvm_admit", "fs_kvm_grow", "fs_kvm_advance", "fs_kvm_release",
    "fs_kvm_start_swaps", "fs_kvm_retire", "fs_kvm_job_info", "fs_kvm_stats", "fs_kvm_table_rows",
    "fs_kvm_stage_batch", "fs_serve_create", "fs_serve_destroy", "fs_serve_scheduler", "fs_serve_manager",
    "fs_serve_submit", "fs_serve_plan", "fs_serve_launch", "fs_serve_complete", "fs_serve_run", "fs_serve_get_stats",
)

RESIDENT, LEAVING, SWAPPED_OUT, RETURNING = 0, 1, 2, 3


class fs_kvm_config(ctypes.Structure):
    _fields_ = [("num_blocks", ctypes.c_int32), ("num_host_blocks", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("table_width", ctypes.c_int32), ("reserve_idle_blocks", ctypes.c_int32),
                ("reserve_window", ctypes.c_int32), ("reserve_quantile", ctypes.c_double),
                ("max_batch", ctypes.c_int32), ("max_staged_extra", ctypes.c_int32)]


class fs_serve_config(ctypes.Structure):
    _fields_ = [("num_queues", ctypes.c_int32), ("q1", ctypes.c_double), ("eta", ctypes.c_int32),
                ("alpha", ctypes.c_double), ("max_batch", ctypes.c_int32), ("max_prompt_tokens", ctypes.c_int64),
                ("kvm", fs_kvm_config)]


class fs_serve_buffers(ctypes.Structure):
    _fields_ = [("prompt_q", ctypes.c_void_p), ("prompt_k", ctypes.c_void_p), ("prompt_v", ctypes.c_void_p),
                ("prompt_out", ctypes.c_void_p), ("max_prompt_tokens", ctypes.c_int64),
                ("decode_q", ctypes.c_void_p), ("decode_k", ctypes.c_void_p), ("decode_v", ctypes.c_void_p),
                ("decode_out", ctypes.c_void_p)]


class fs_serve_iteration(ctypes.Structure):
    _fields_ = [("iteration", ctypes.c_int64), ("n_first", ctypes.c_int32),
                ("first_ids", ctypes.POINTER(ctypes.c_int64)), ("token_offsets", ctypes.POINTER(ctypes.c_int32)),
                ("prompt_tokens", ctypes.c_int64), ("n_decode", ctypes.c_int32),
                ("decode_ids", ctypes.POINTER(ctypes.c_int64)), ("lens_before", ctypes.POINTER(ctypes.c_int32)),
                ("n_waiting", ctypes.c_int32), ("n_unfinished", ctypes.c_int32)]


class fs_serve_stats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("iterations", "job_tokens", "prompt_tokens", "finished_jobs",
                                               "blocks_swapped_out", "blocks_swapped_in", "iterations_without_work")] + \
               [(n, ctypes.c_double) for n in ("host_seconds_plan", "host_seconds_launch", "host_seconds_complete")]


def _lib():
    lib = load_library()
    if getattr(lib, "_fs_kvm_ready", False):
        return lib
    vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
    P = ctypes.POINTER
    lib.fs_kvm_create.argtypes = [P(fs_kvm_config), P(vp), i32, vp, P(vp)]
    lib.fs_kvm_destroy.argtypes = [vp]
    lib.fs_kvm_blocks_needed.argtypes = [vp, i64]
    lib.fs_kvm_free_blocks.argtypes = [vp]
    lib.fs_kvm_free_slots.argtypes = [vp]
    lib.fs_kvm_reserve.argtypes = [vp]
    lib.fs_kvm_observe_arrivals.argtypes = [vp, i32]
    lib.fs_kvm_admit.argtypes = [vp, i64, i64]
    lib.fs_kvm_grow.argtypes = [vp, i64, i32, P(i32)]
    lib.fs_kvm_advance.argtypes = [vp, i64, i32]
    lib.fs_kvm_release.argtypes = [vp, i64]
    lib.fs_kvm_start_swaps.argtypes = [vp, P(i64), i32, i32, vp]
    lib.fs_kvm_retire.argtypes = [vp, i32, i32, P(i32)]
    lib.fs_kvm_job_info.argtypes = [vp, i64, P(i32), P(i64), vp, i32, P(i32)]
    lib.fs_kvm_stats.argtypes = [vp, P(i64), P(i64), P(i32)]
    lib.fs_kvm_table_rows.argtypes = [vp, P(i64), i32, vp]
    lib.fs_kvm_stage_batch.argtypes = [vp, P(i64), i32, vp, i32, vp, P(vp), P(vp), P(vp)]
    lib.fs_serve_create.argtypes = [P(fs_serve_config), P(vp), i32, P(vp)]
    lib.fs_serve_destroy.argtypes = [vp]
    lib.fs_serve_scheduler.argtypes = [vp]
    lib.fs_serve_scheduler.restype = vp
    lib.fs_serve_manager.argtypes = [vp]
    lib.fs_serve_manager.restype = vp
    lib.fs_serve_submit.argtypes = [vp, i64, i64, i32, i32, dbl, dbl]
    lib.fs_serve_plan.argtypes = [vp, vp, P(fs_serve_iteration)]
    lib.fs_serve_launch.argtypes = [vp, i32, P(fs_serve_buffers), vp]
    lib.fs_serve_complete.argtypes = [vp]
    lib.fs_serve_run.argtypes = [vp, P(fs_serve_buffers), vp, i64, P(fs_serve_stats)]
    lib.fs_serve_get_stats.argtypes = [vp, P(fs_serve_stats)]
    for name in KVM_EXPORTS:
        if name not in ("fs_serve_scheduler", "fs_serve_manager"):
            getattr(lib, name).restype = ctypes.c_int
    lib._fs_kvm_ready = True
    return lib


def _ok(status: int, where: str) -> None:
    if status != 0:
        raise FsError(status, where)


def _ids(seq: Sequence[int]):
    return (ctypes.c_int64 * max(len(seq), 1))(*seq)


def _pools(layers) -> Tuple[object, int]:
    layers = [layers] if isinstance(layers, Pool) else list(layers or [])
    arr = (ctypes.c_void_p * max(len(layers), 1))(*[p._h for p in layers])
    return arr, len(layers)


def _stream(stream):
    import torch
    from . import _stream_ptr
    if stream is None and not torch.cuda.is_available():
        return None                                 # a manager without layer pools issues nothing on it
    return _stream_ptr(stream)


class KVManager:
    """fs_kvm_*: block ownership, residency, idle reserve and swaps of the jobs' caches."""

    def __init__(self, layers, sched, num_blocks: int, num_host_blocks: int, table_width: int, block_size: int = 16,
                 reserve_idle_blocks: int = 0, reserve_window: int = 0, reserve_quantile: float = 0.0,
                 max_batch: int = 0, max_staged_extra: int = 0, _handle=None):
        self._lib = _lib()
        self._owned = _handle is None
        self.table_width = table_width
        if _handle is not None:
            self._h = ctypes.c_void_p(_handle)
            return
        cfg = fs_kvm_config(num_blocks, num_host_blocks, block_size, table_width, reserve_idle_blocks,
                            reserve_window, reserve_quantile, max_batch, max_staged_extra)
        arr, n = _pools(layers)
        self._layers = layers                       # keep the pools alive
        h = ctypes.c_void_p()
        _ok(self._lib.fs_kvm_create(ctypes.byref(cfg), arr, n, sched._h if sched is not None else None,
                                    ctypes.byref(h)), "fs_kvm_create")
        self._h = h

    def close(self) -> None:
        if getattr(self, "_h", None) and self._owned:
            self._lib.fs_kvm_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def blocks_needed(self, tokens: int) -> int:
        return int(self._lib.fs_kvm_blocks_needed(self._h, int(tokens)))

    @property
    def free_blocks(self) -> int:
        return int(self._lib.fs_kvm_free_blocks(self._h))

    @property
    def free_slots(self) -> int:
        return int(self._lib.fs_kvm_free_slots(self._h))

    @property
    def reserve(self) -> int:
        return int(self._lib.fs_kvm_reserve(self._h))

    def observe_arrivals(self, blocks_demanded: int) -> None:
        _ok(self._lib.fs_kvm_observe_arrivals(self._h, int(blocks_demanded)), "fs_kvm_observe_arrivals")

    def admit(self, job_id: int, tokens: int) -> bool:
        rc = self._lib.fs_kvm_admit(self._h, int(job_id), int(tokens))
        if rc == -2:                                # FS_ERR_OOM: no room, nothing changed
            return False
        _ok(rc, "fs_kvm_admit")
        return True

    def grow(self, job_id: int, new_tokens: int = 1) -> bool:
        ok = ctypes.c_int32()
        _ok(self._lib.fs_kvm_grow(self._h, int(job_id), int(new_tokens), ctypes.byref(ok)), "fs_kvm_grow")
        return bool(ok.value)

    def advance(self, job_id: int, tokens: int = 1) -> None:
        _ok(self._lib.fs_kvm_advance(self._h, int(job_id), int(tokens)), "fs_kvm_advance")

    def release(self, job_id: int) -> None:
        _ok(self._lib.fs_kvm_release(self._h, int(job_id)), "fs_kvm_release")

    def start_swaps(self, running: Sequence[int], want_free: int = 0, stream=None) -> None:
        _ok(self._lib.fs_kvm_start_swaps(self._h, _ids(running), len(running), int(want_free), _stream(stream)),
            "fs_kvm_start_swaps")

    def retire(self, max_swaps: int = -1, wait: bool = False) -> int:
        n = ctypes.c_int32()
        _ok(self._lib.fs_kvm_retire(self._h, int(max_swaps), 1 if wait else 0, ctypes.byref(n)), "fs_kvm_retire")
        return n.value

    def job_info(self, job_id: int):
        state, length, n = ctypes.c_int32(), ctypes.c_int64(), ctypes.c_int32()
        ids = np.zeros(self.table_width, dtype=np.int32)
        _ok(self._lib.fs_kvm_job_info(self._h, int(job_id), ctypes.byref(state), ctypes.byref(length),
                                      ids.ctypes.data, len(ids), ctypes.byref(n)), "fs_kvm_job_info")
        return state.value, length.value, ids[:n.value].tolist()

    def stats(self):
        a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32()
        _ok(self._lib.fs_kvm_stats(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "fs_kvm_stats")
        return a.value, b.value, c.value

    def table_rows(self, job_ids: Sequence[int]) -> np.ndarray:
        rows = np.zeros((len(job_ids), self.table_width), dtype=np.int32)
        _ok(self._lib.fs_kvm_table_rows(self._h, _ids(job_ids), len(job_ids), rows.ctypes.data), "fs_kvm_table_rows")
        return rows

    def stage_batch(self, job_ids: Sequence[int], extra: Optional[np.ndarray] = None, stream=None):
        """Device addresses (ints) of the staged table rows, lengths and extra words."""
        ex = np.ascontiguousarray(extra if extra is not None else np.zeros(0), dtype=np.int32)
        t, l, e = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        _ok(self._lib.fs_kvm_stage_batch(self._h, _ids(job_ids), len(job_ids), ex.ctypes.data if len(ex) else None,
                                         len(ex), _stream(stream), ctypes.byref(t), ctypes.byref(l), ctypes.byref(e)),
            "fs_kvm_stage_batch")
        return t.value, l.value, e.value


class ServeLoop:
    """fs_serve_*: the iteration loop over scheduler, cache manager and attention kernels."""

    def __init__(self, layers, num_queues: int, q1: float, eta: int, alpha: float, max_batch: int,
                 num_blocks: int, num_host_blocks: int, table_width: int, block_size: int = 16,
                 max_prompt_tokens: int = 0, reserve_idle_blocks: int = 0, reserve_window: int = 0,
                 reserve_quantile: float = 0.0):
        self._lib = _lib()
        cfg = fs_serve_config()
        cfg.num_queues, cfg.q1, cfg.eta, cfg.alpha, cfg.max_batch = num_queues, q1, eta, alpha, max_batch
        cfg.max_prompt_tokens = max_prompt_tokens
        cfg.kvm = fs_kvm_config(num_blocks, num_host_blocks, block_size, table_width, reserve_idle_blocks,
                                reserve_window, reserve_quantile, 0, 0)
        arr, n = _pools(layers)
        self._layers = layers
        h = ctypes.c_void_p()
        _ok(self._lib.fs_serve_create(ctypes.byref(cfg), arr, n, ctypes.byref(h)), "fs_serve_create")
        self._h = h
        self.max_batch = max_batch
        # views of the scheduler and the manager the loop owns (never destroyed through them)
        self.manager = KVManager(None, None, 0, 0, table_width, _handle=self._lib.fs_serve_manager(h))
        self.scheduler = _sched.Scheduler(num_queues, q1, eta, alpha, max_batch,
                                          _handle=self._lib.fs_serve_scheduler(h))

    def close(self) -> None:
        if getattr(self, "_h", None):
            self.manager.close()
            self.scheduler.close()
            self._lib.fs_serve_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def submit(self, job_id: int, arrival_iteration: int, prompt_tokens: int, output_tokens: int,
               init_time: float, decode_time: float) -> None:
        _ok(self._lib.fs_serve_submit(self._h, int(job_id), int(arrival_iteration), int(prompt_tokens),
                                      int(output_tokens), float(init_time), float(decode_time)), "fs_serve_submit")

    def plan(self, stream=None) -> dict:
        it = fs_serve_iteration()
        _ok(self._lib.fs_serve_plan(self._h, _stream(stream), ctypes.byref(it)), "fs_serve_plan")
        return {"iteration": it.iteration, "first": [it.first_ids[i] for i in range(it.n_first)],
                "token_offsets": [it.token_offsets[i] for i in range(it.n_first + 1)],
                "prompt_tokens": it.prompt_tokens, "decode": [it.decode_ids[i] for i in range(it.n_decode)],
                "lens_before": [it.lens_before[i] for i in range(it.n_decode)], "n_waiting": it.n_waiting,
                "n_unfinished": it.n_unfinished}

    @staticmethod
    def buffers(prompt_q, prompt_k, prompt_v, prompt_out, decode_q, decode_k, decode_v, decode_out) -> fs_serve_buffers:
        b = fs_serve_buffers()
        b.prompt_q, b.prompt_k, b.prompt_v = prompt_q.data_ptr(), prompt_k.data_ptr(), prompt_v.data_ptr()
        b.prompt_out, b.max_prompt_tokens = prompt_out.data_ptr(), prompt_q.shape[0]
        b.decode_q, b.decode_k, b.decode_v = decode_q.data_ptr(), decode_k.data_ptr(), decode_v.data_ptr()
        b.decode_out = decode_out.data_ptr()
        b._keep = (prompt_q, prompt_k, prompt_v, prompt_out, decode_q, decode_k, decode_v, decode_out)
        return b

    def launch(self, buffers: fs_serve_buffers, layer: int = -1, stream=None) -> None:
        _ok(self._lib.fs_serve_launch(self._h, int(layer), ctypes.byref(buffers), _stream(stream)), "fs_serve_launch")

    def complete(self) -> None:
        _ok(self._lib.fs_serve_complete(self._h), "fs_serve_complete")

    def run(self, buffers: fs_serve_buffers, max_iterations: int, stream=None) -> dict:
        st = fs_serve_stats()
        _ok(self._lib.fs_serve_run(self._h, ctypes.byref(buffers), _stream(stream), int(max_iterations),
                                   ctypes.byref(st)), "fs_serve_run")
        return {n: getattr(st, n) for n, _ in fs_serve_stats._fields_}

    def stats(self) -> dict:
        st = fs_serve_stats()
        _ok(self._lib.fs_serve_get_stats(self._h, ctypes.byref(st)), "fs_serve_get_stats")
        return {n: getattr(st, n) for n, _ in fs_serve_stats._fields_}
