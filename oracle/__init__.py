"""CPU oracle (test infrastructure only): ctypes front end of ``fs_oracle.c``.

Nothing here is part of the product path.  Only the tests, the smoke check and
the bench's ``cpu_baseline`` leg may import this package, and it imports
nothing from the GPU package.

The oracle keeps every job's cache as one contiguous logical array
``K[t][h][d]`` (paper Section 2.2: the cache holds the keys and values of all
preceding tokens); blocks and block tables do not exist on this side.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fs_oracle.c")
_LIB = os.path.join(_HERE, "libfs_oracle.so")

DTYPE_CODE = {"bf16": 0, "f32": 1, "f64": 2, "f16": 3}
_NP_OF = {"bf16": np.uint16, "f16": np.uint16, "f32": np.float32, "f64": np.float64}

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, dbl, lng, i32 = ctypes.c_void_p, ctypes.c_double, ctypes.c_long, ctypes.c_int
        lib.fso_append.argtypes = [vp, vp, i32, lng, i32, i32, vp, vp]
        lib.fso_append.restype = i32
        lib.fso_attention_job.argtypes = [vp, vp, vp, i32, lng, i32, i32, dbl, i32, i32, vp, vp]
        lib.fso_attention_job.restype = i32
        lib.fso_decode_step.argtypes = [vp, vp, vp, i32, i32, i32, i32, dbl, vp, vp, vp, vp]
        lib.fso_decode_step.restype = i32
        lib.fso_prefill_attention_job.argtypes = [vp, vp, vp, i32, lng, i32, i32, dbl, i32, i32, vp]
        lib.fso_prefill_attention_job.restype = i32
        _lib = lib
    return _lib


def _check(a: np.ndarray, dtype: str, name: str) -> np.ndarray:
    want = _NP_OF[dtype]
    if a.dtype != want or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: need C-contiguous {np.dtype(want).name}, got {a.dtype}")
    return a


def attention_job(q: np.ndarray, K: np.ndarray, V: np.ndarray, dtype: str,
                  length: Optional[int] = None, scale: float = 0.0,
                  heads: Optional[Sequence[int]] = None, want_weights: bool = False):
    """Attention of one job's new token.  q [H][D]; K, V [>=L][H][D] in `dtype`
    storage (bf16 and f16 as uint16 bits).  Returns out [H][D] float64 (rows outside
    `heads`=(h0,h1) are zero) and, if asked, the weights [H][L]."""
    lib = _load()
    H, D = q.shape
    L = K.shape[0] if length is None else int(length)
    _check(q, dtype, "q")
    if L > 0:
        _check(K, dtype, "K"), _check(V, dtype, "V")
        assert K.shape[1:] == (H, D) and V.shape[1:] == (H, D) and K.shape[0] >= L
    h0, h1 = (0, H) if heads is None else (int(heads[0]), int(heads[1]))
    out = np.zeros((H, D), dtype=np.float64)
    w = np.zeros((H, max(L, 1)), dtype=np.float64) if want_weights else None
    rc = lib.fso_attention_job(q.ctypes.data, K.ctypes.data if L > 0 else None,
                               V.ctypes.data if L > 0 else None, DTYPE_CODE[dtype], L, H, D,
                               float(scale), h0, h1, out.ctypes.data,
                               w.ctypes.data if want_weights else None)
    if rc:
        raise RuntimeError(f"fso_attention_job failed: {rc}")
    return (out, w[:, :L]) if want_weights else out


def prefill_attention_job(Q: np.ndarray, K: np.ndarray, V: np.ndarray, dtype: str,
                          scale: Optional[float] = None, heads: Optional[Tuple[int, int]] = None) -> np.ndarray:
    """Initialization-phase attention of one job's prompt.  Q, K, V [s][H][D] in `dtype`
    storage; returns out [s][H][D] float64 (heads outside `heads` stay zero): token i
    attends to tokens 0..i."""
    lib = _load()
    _check(Q, dtype, "Q"), _check(K, dtype, "K"), _check(V, dtype, "V")
    if Q.shape != K.shape or Q.shape != V.shape or Q.ndim != 3:
        raise ValueError("Q, K, V must share the shape [s][H][D]")
    s, H, D = Q.shape
    h0, h1 = heads if heads is not None else (0, H)
    out = np.zeros((s, H, D), dtype=np.float64)
    rc = lib.fso_prefill_attention_job(Q.ctypes.data if s else None, K.ctypes.data if s else None,
                                       V.ctypes.data if s else None, DTYPE_CODE[dtype], s, H, D,
                                       -1.0 if scale is None else float(scale), h0, h1, out.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"fso_prefill_attention_job failed ({rc})")
    return out


class LogicalCaches:
    """Per-job contiguous caches K_j[t][h][d], V_j[t][h][d] with spare capacity."""

    def __init__(self, dtype: str, num_heads: int, head_dim: int):
        self.dtype, self.H, self.D = dtype, num_heads, head_dim
        self.K: list[np.ndarray] = []
        self.V: list[np.ndarray] = []
        self.lens: list[int] = []

    def add_job(self, K: np.ndarray, V: np.ndarray, spare: int = 1) -> None:
        """Adopt a job whose cache already holds K.shape[0] tokens."""
        _check(K, self.dtype, "K"), _check(V, self.dtype, "V")
        L = K.shape[0]
        cap = (L + spare, self.H, self.D)
        k = np.zeros(cap, dtype=K.dtype)
        v = np.zeros(cap, dtype=V.dtype)
        k[:L], v[:L] = K, V
        self.K.append(k), self.V.append(v), self.lens.append(L)

    def append(self, k_new: np.ndarray, v_new: np.ndarray) -> None:
        """Decode-phase append: row L_j of job j's cache := k_new[j], v_new[j]."""
        lib = _load()
        _check(k_new, self.dtype, "k_new"), _check(v_new, self.dtype, "v_new")
        for j in range(len(self.K)):
            if self.lens[j] >= self.K[j].shape[0]:
                raise ValueError("cache capacity exhausted")
            rc = lib.fso_append(self.K[j].ctypes.data, self.V[j].ctypes.data,
                                DTYPE_CODE[self.dtype], self.lens[j], self.H, self.D,
                                k_new[j].ctypes.data, v_new[j].ctypes.data)
            if rc:
                raise RuntimeError(f"fso_append failed: {rc}")
            self.lens[j] += 1

    def attention(self, q: np.ndarray, scale: float = 0.0) -> np.ndarray:
        out = np.zeros((len(self.K), self.H, self.D), dtype=np.float64)
        for j in range(len(self.K)):
            out[j] = attention_job(q[j], self.K[j], self.V[j], self.dtype, self.lens[j], scale)
        return out

    def decode_step(self, k_new: np.ndarray, v_new: np.ndarray, q: np.ndarray,
                    scale: float = 0.0) -> np.ndarray:
        """Append then attend, through the single C entry point (this is what
        the bench times as the CPU baseline)."""
        lib = _load()
        J = len(self.K)
        _check(k_new, self.dtype, "k_new"), _check(v_new, self.dtype, "v_new"), _check(q, self.dtype, "q")
        for j in range(J):
            if self.lens[j] >= self.K[j].shape[0]:
                raise ValueError("cache capacity exhausted")
        kp = (ctypes.c_void_p * J)(*[a.ctypes.data for a in self.K])
        vp = (ctypes.c_void_p * J)(*[a.ctypes.data for a in self.V])
        lens = (ctypes.c_long * J)(*self.lens)
        out = np.zeros((J, self.H, self.D), dtype=np.float64)
        rc = lib.fso_decode_step(kp, vp, lens, J, DTYPE_CODE[self.dtype], self.H, self.D,
                                 float(scale), k_new.ctypes.data, v_new.ctypes.data,
                                 q.ctypes.data, out.ctypes.data)
        if rc:
            raise RuntimeError(f"fso_decode_step failed: {rc}")
        for j in range(J):
            self.lens[j] += 1
        return out
