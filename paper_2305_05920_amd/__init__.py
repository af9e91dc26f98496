"""MI355X-native paged decode step (FastServe hot path): Python binding.

Thin ctypes layer over ``libfastserve.so`` (C ABI in ``include/fastserve.h``).
It only marshals arguments -- tensor addresses, sizes, the current HIP stream --
and every step of the path runs in the library's HIP kernels.  PyTorch is used
for device memory and streams only.  There is no CPU fallback: without the
built library or without a GPU the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # first: the library binds to the HIP runtime torch has loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FS_LIBRARY") or os.path.join(_HERE, "libfastserve.so")

FS_BF16, FS_F32, FS_F16 = 0, 1, 2
FS_OK = 0
FS_ERR_INVALID_ARG, FS_ERR_OOM, FS_ERR_BAD_TABLE, FS_ERR_HIP, FS_ERR_UNSUPPORTED = -1, -2, -3, -4, -5
KERNEL_KINDS = ("append", "attention", "combine", "prefill", "prefill_attention", "prefill_plan")

EXPORTS = (
    "fs_pool_create", "fs_pool_destroy", "fs_pool_block_bytes", "fs_pool_device_ptr",
    "fs_pool_write_block", "fs_pool_read_block", "fs_pool_check", "fs_kv_append", "fs_kv_prefill",
    "fs_prefill_attention", "fs_prefill_step",
    "fs_decode_attention", "fs_decode_attention_static", "fs_decode_step", "fs_pool_offload", "fs_pool_upload", "fs_profile_enable",
    "fs_profile_collect", "fs_pool_set_param", "fs_pool_get_param", "fs_pool_last_plan",
    "fs_stream_read", "fs_stream_read_timed", "fs_stream_copy", "fs_strerror", "fs_version",
)


class FsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


class fs_pool_config(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int32), ("num_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("block_size", ctypes.c_int32), ("num_blocks", ctypes.c_int32),
        ("num_host_blocks", ctypes.c_int32), ("max_jobs", ctypes.c_int32),
        ("max_workgroups", ctypes.c_int32), ("scale", ctypes.c_float), ("reserved", ctypes.c_int32),
        ("device_mem", ctypes.c_void_p), ("device_bytes", ctypes.c_size_t),
    ]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built (see build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2305_05920_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    P = ctypes.POINTER
    lib.fs_pool_create.argtypes = [P(fs_pool_config), P(vp)]
    lib.fs_pool_destroy.argtypes = [vp]
    lib.fs_pool_block_bytes.argtypes = [vp]
    lib.fs_pool_block_bytes.restype = ctypes.c_size_t
    lib.fs_pool_device_ptr.argtypes = [vp]
    lib.fs_pool_device_ptr.restype = vp
    lib.fs_pool_write_block.argtypes = [vp, i32, vp]
    lib.fs_pool_read_block.argtypes = [vp, i32, vp]
    lib.fs_pool_check.argtypes = [vp, vp]
    lib.fs_kv_append.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp]
    lib.fs_kv_prefill.argtypes = [vp, vp, i32, vp, vp, i32, i64, vp, vp, vp]
    lib.fs_prefill_attention.argtypes = [vp, vp, vp, vp, vp, i32, i64, vp, vp]
    lib.fs_prefill_step.argtypes = [vp, vp, i32, vp, i32, i64, vp, vp, vp, vp, vp]
    lib.fs_decode_attention.argtypes = [vp, vp, vp, i32, vp, i32, i32, vp, vp]
    lib.fs_decode_attention_static.argtypes = [vp, vp, vp, i32, vp, i32, i32, vp, vp]
    lib.fs_decode_step.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp, i32, vp, vp]
    lib.fs_pool_offload.argtypes = [vp, vp, vp, i32, vp]
    lib.fs_pool_upload.argtypes = [vp, vp, vp, i32, vp]
    lib.fs_profile_enable.argtypes = [vp, i32]
    lib.fs_profile_collect.argtypes = [vp, P(ctypes.c_float), P(i32)]
    lib.fs_pool_set_param.argtypes = [vp, ctypes.c_char_p, i32]
    lib.fs_pool_get_param.argtypes = [vp, ctypes.c_char_p, P(i32)]
    lib.fs_pool_last_plan.argtypes = [vp, i32, vp, vp]
    lib.fs_stream_read.argtypes = [vp, ctypes.c_size_t, vp, i32, vp]
    lib.fs_stream_read_timed.argtypes = [vp, ctypes.c_size_t, vp, i32, vp, ctypes.POINTER(ctypes.c_float)]
    lib.fs_stream_copy.argtypes = [vp, vp, ctypes.c_size_t, i32, vp]
    lib.fs_strerror.argtypes = [ctypes.c_int]
    lib.fs_strerror.restype = ctypes.c_char_p
    lib.fs_version.restype = ctypes.c_char_p
    for name in EXPORTS:
        fn = getattr(lib, name)
        if name not in ("fs_pool_block_bytes", "fs_pool_device_ptr", "fs_strerror", "fs_version"):
            fn.restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().fs_strerror(int(status)).decode()


def version() -> str:
    return load_library().fs_version().decode()


def _ok(status: int, where: str) -> None:
    if status != FS_OK:
        raise FsError(status, where)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def _dev(t: torch.Tensor, name: str, dtype=None) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: need a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name}: need a contiguous tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: need dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _host_i32(a, name: str):
    import numpy as np
    arr = np.ascontiguousarray(a, dtype=np.int32)
    if arr.ndim != 1:
        raise ValueError(f"{name}: need a 1-d array")
    return arr


class Pool:
    """A block pool plus the library's scratch (``fs_pool_create``)."""

    def __init__(self, dtype: str, num_heads: int, head_dim: int, num_blocks: int,
                 block_size: int = 16, num_host_blocks: int = 0, max_jobs: int = 0,
                 max_workgroups: int = 0, scale: float = 0.0,
                 device_mem: Optional[torch.Tensor] = None):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the decode path runs on the GPU only")
        lib = load_library()
        self.dtype = dtype
        self.torch_dtype = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[dtype]
        self.num_heads, self.head_dim, self.block_size = num_heads, head_dim, block_size
        self.num_blocks, self.num_host_blocks = num_blocks, num_host_blocks
        cfg = fs_pool_config()
        cfg.dtype = {"bf16": FS_BF16, "f16": FS_F16, "f32": FS_F32}[dtype]
        cfg.num_heads, cfg.head_dim, cfg.block_size = num_heads, head_dim, block_size
        cfg.num_blocks, cfg.num_host_blocks = num_blocks, num_host_blocks
        cfg.max_jobs, cfg.max_workgroups, cfg.scale, cfg.reserved = max_jobs, max_workgroups, scale, 0
        self._device_mem = device_mem          # keep the caller's tensor alive
        if device_mem is not None:
            cfg.device_mem = _dev(device_mem, "device_mem")
            cfg.device_bytes = device_mem.numel() * device_mem.element_size()
        handle = ctypes.c_void_p()
        _ok(lib.fs_pool_create(ctypes.byref(cfg), ctypes.byref(handle)), "fs_pool_create")
        self._h = handle
        self._lib = lib

    # -- lifetime ---------------------------------------------------------
    def close(self) -> None:
        if getattr(self, "_h", None):
            self._lib.fs_pool_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # -- facts ------------------------------------------------------------
    @property
    def block_bytes(self) -> int:
        return int(self._lib.fs_pool_block_bytes(self._h))

    @property
    def device_ptr(self) -> int:
        return int(self._lib.fs_pool_device_ptr(self._h))

    def get_param(self, name: str) -> int:
        v = ctypes.c_int32()
        _ok(self._lib.fs_pool_get_param(self._h, name.encode(), ctypes.byref(v)), "fs_pool_get_param")
        return v.value

    def set_param(self, name: str, value: int) -> None:
        _ok(self._lib.fs_pool_set_param(self._h, name.encode(), int(value)), "fs_pool_set_param")

    # -- raw blocks -------------------------------------------------------
    def write_block(self, block_id: int, host_array) -> None:
        import numpy as np
        a = np.ascontiguousarray(host_array)
        if a.nbytes != self.block_bytes:
            raise ValueError("write_block: need exactly one block of bytes")
        _ok(self._lib.fs_pool_write_block(self._h, int(block_id), a.ctypes.data), "fs_pool_write_block")

    def read_block(self, block_id: int, np_dtype):
        import numpy as np
        a = np.empty(self.block_bytes // np.dtype(np_dtype).itemsize, dtype=np_dtype)
        _ok(self._lib.fs_pool_read_block(self._h, int(block_id), a.ctypes.data), "fs_pool_read_block")
        return a

    def check(self, stream=None) -> None:
        _ok(self._lib.fs_pool_check(self._h, _stream_ptr(stream)), "fs_pool_check")

    # -- profiling --------------------------------------------------------
    def profile_enable(self, on: bool) -> None:
        _ok(self._lib.fs_profile_enable(self._h, 1 if on else 0), "fs_profile_enable")

    def profile_collect(self) -> dict:
        n = len(KERNEL_KINDS)
        ms = (ctypes.c_float * n)()
        cnt = (ctypes.c_int32 * n)()
        _ok(self._lib.fs_profile_collect(self._h, ms, cnt), "fs_profile_collect")
        return {k: {"ms": float(ms[i]), "launches": int(cnt[i])} for i, k in enumerate(KERNEL_KINDS)}

    def last_plan(self, num_jobs: int, stream=None):
        import numpy as np
        base = np.zeros(num_jobs + 1, dtype=np.int32)
        _ok(self._lib.fs_pool_last_plan(self._h, int(num_jobs), base.ctypes.data, _stream_ptr(stream)),
            "fs_pool_last_plan")
        return base


def fs_pool_create(**kw) -> Pool:
    return Pool(**kw)


def fs_kv_append(pool: Pool, block_table: torch.Tensor, job_lens: torch.Tensor,
                 k: torch.Tensor, v: torch.Tensor, stream=None) -> None:
    """k, v [J][H][D] join every job's cache at position job_lens[j] (pre-append length)."""
    J = job_lens.numel()
    if block_table.dim() != 2 or block_table.shape[0] != J:
        raise ValueError("block_table: need [num_jobs][table_stride]")
    shape = (J, pool.num_heads, pool.head_dim)
    if tuple(k.shape) != shape or tuple(v.shape) != shape:
        raise ValueError(f"k, v: need shape {shape}")
    _ok(pool._lib.fs_kv_append(pool._h, _dev(block_table, "block_table", torch.int32), block_table.shape[1],
                               _dev(job_lens, "job_lens", torch.int32), J,
                               _dev(k, "k", pool.torch_dtype), _dev(v, "v", pool.torch_dtype),
                               _stream_ptr(stream)), "fs_kv_append")


def fs_kv_prefill(pool: Pool, block_table: torch.Tensor, job_starts: torch.Tensor,
                  token_offsets: torch.Tensor, total_tokens: int, k: torch.Tensor, v: torch.Tensor,
                  stream=None) -> None:
    """Packed tokens k, v [T][H][D]; job j gets rows token_offsets[j]..token_offsets[j+1]."""
    J = job_starts.numel()
    if block_table.dim() != 2 or block_table.shape[0] != J or token_offsets.numel() != J + 1:
        raise ValueError("block_table / token_offsets: wrong shape")
    shape = (int(total_tokens), pool.num_heads, pool.head_dim)
    if tuple(k.shape) != shape or tuple(v.shape) != shape:
        raise ValueError(f"k, v: need shape {shape}")
    _ok(pool._lib.fs_kv_prefill(pool._h, _dev(block_table, "block_table", torch.int32), block_table.shape[1],
                                _dev(job_starts, "job_starts", torch.int32),
                                _dev(token_offsets, "token_offsets", torch.int32), J, int(total_tokens),
                                _dev(k, "k", pool.torch_dtype), _dev(v, "v", pool.torch_dtype),
                                _stream_ptr(stream)), "fs_kv_prefill")


def fs_prefill_attention(pool: Pool, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                         token_offsets: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    """Prompt-phase attention over packed prompts q, k, v [T][H][D]: token i of a job attends
    to tokens 0..i of the same job; out [T][H][D] float32."""
    J = token_offsets.numel() - 1
    T = q.shape[0]
    shape = (T, pool.num_heads, pool.head_dim)
    if J < 0 or tuple(q.shape) != shape or tuple(k.shape) != shape or tuple(v.shape) != shape or \
            tuple(out.shape) != shape:
        raise ValueError(f"q, k, v, out: need shape {shape}; token_offsets [num_jobs+1]")
    _ok(pool._lib.fs_prefill_attention(pool._h, _dev(q, "q", pool.torch_dtype), _dev(k, "k", pool.torch_dtype),
                                       _dev(v, "v", pool.torch_dtype),
                                       _dev(token_offsets, "token_offsets", torch.int32), J, int(T),
                                       _dev(out, "out", torch.float32), _stream_ptr(stream)),
        "fs_prefill_attention")


def fs_prefill_step(pool: Pool, block_table: torch.Tensor, token_offsets: torch.Tensor, k: torch.Tensor,
                    v: torch.Tensor, q: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    """The whole initialization phase of new jobs: their prompt tokens' k, v [T][H][D] fill the
    jobs' cache blocks from position 0 and out [T][H][D] receives the prompt attention."""
    J = token_offsets.numel() - 1
    T = q.shape[0]
    shape = (T, pool.num_heads, pool.head_dim)
    if J < 0 or block_table.dim() != 2 or block_table.shape[0] != J:
        raise ValueError("block_table: need [num_jobs][table_stride]; token_offsets [num_jobs+1]")
    if tuple(q.shape) != shape or tuple(k.shape) != shape or tuple(v.shape) != shape or tuple(out.shape) != shape:
        raise ValueError(f"q, k, v, out: need shape {shape}")
    _ok(pool._lib.fs_prefill_step(pool._h, _dev(block_table, "block_table", torch.int32), block_table.shape[1],
                                  _dev(token_offsets, "token_offsets", torch.int32), J, int(T),
                                  _dev(k, "k", pool.torch_dtype), _dev(v, "v", pool.torch_dtype),
                                  _dev(q, "q", pool.torch_dtype), _dev(out, "out", torch.float32),
                                  _stream_ptr(stream)), "fs_prefill_step")


def fs_decode_attention(q: torch.Tensor, pool: Pool, block_table: torch.Tensor, job_lens: torch.Tensor,
                        out: torch.Tensor, max_len_hint: int = 0, stream=None) -> None:
    """out[j][h] = attention of q[j][h] over the first job_lens[j] cached tokens of job j."""
    J = job_lens.numel()
    shape = (J, pool.num_heads, pool.head_dim)
    if block_table.dim() != 2 or block_table.shape[0] != J:
        raise ValueError("block_table: need [num_jobs][table_stride]")
    if tuple(q.shape) != shape or tuple(out.shape) != shape:
        raise ValueError(f"q, out: need shape {shape}")
    _ok(pool._lib.fs_decode_attention(_dev(q, "q", pool.torch_dtype), pool._h,
                                      _dev(block_table, "block_table", torch.int32), block_table.shape[1],
                                      _dev(job_lens, "job_lens", torch.int32), J, int(max_len_hint),
                                      _dev(out, "out", torch.float32), _stream_ptr(stream)),
        "fs_decode_attention")


def fs_decode_attention_static(q: torch.Tensor, pool: Pool, block_table: torch.Tensor, job_lens: torch.Tensor,
                               out: torch.Tensor, max_len_hint: int = 0, stream=None) -> None:
    """fs_decode_attention on the library's fixed device scratch: allocates nothing; at most 1024 jobs."""
    J = job_lens.numel()
    shape = (J, pool.num_heads, pool.head_dim)
    if block_table.dim() != 2 or block_table.shape[0] != J:
        raise ValueError("block_table: need [num_jobs][table_stride]")
    if tuple(q.shape) != shape or tuple(out.shape) != shape:
        raise ValueError(f"q, out: need shape {shape}")
    _ok(pool._lib.fs_decode_attention_static(_dev(q, "q", pool.torch_dtype), pool._h,
                                             _dev(block_table, "block_table", torch.int32), block_table.shape[1],
                                             _dev(job_lens, "job_lens", torch.int32), J, int(max_len_hint),
                                             _dev(out, "out", torch.float32), _stream_ptr(stream)),
        "fs_decode_attention_static")


def fs_decode_step(pool: Pool, block_table: torch.Tensor, job_lens: torch.Tensor, k: torch.Tensor,
                   v: torch.Tensor, q: torch.Tensor, out: torch.Tensor, max_len_hint: int = 0,
                   stream=None) -> None:
    """Append k, v at position job_lens[j] and attend over job_lens[j] + 1 tokens, one launch fewer."""
    J = job_lens.numel()
    shape = (J, pool.num_heads, pool.head_dim)
    if block_table.dim() != 2 or block_table.shape[0] != J:
        raise ValueError("block_table: need [num_jobs][table_stride]")
    for name, t in (("k", k), ("v", v), ("q", q), ("out", out)):
        if tuple(t.shape) != shape:
            raise ValueError(f"{name}: need shape {shape}")
    _ok(pool._lib.fs_decode_step(pool._h, _dev(block_table, "block_table", torch.int32), block_table.shape[1],
                                 _dev(job_lens, "job_lens", torch.int32), J, _dev(k, "k", pool.torch_dtype),
                                 _dev(v, "v", pool.torch_dtype), _dev(q, "q", pool.torch_dtype),
                                 int(max_len_hint), _dev(out, "out", torch.float32), _stream_ptr(stream)),
        "fs_decode_step")


def fs_pool_offload(pool: Pool, block_ids, host_slots, stream=None) -> None:
    b, s = _host_i32(block_ids, "block_ids"), _host_i32(host_slots, "host_slots")
    if len(b) != len(s):
        raise ValueError("block_ids and host_slots differ in length")
    _ok(pool._lib.fs_pool_offload(pool._h, b.ctypes.data, s.ctypes.data, len(b), _stream_ptr(stream)),
        "fs_pool_offload")


def fs_pool_upload(pool: Pool, host_slots, block_ids, stream=None) -> None:
    b, s = _host_i32(block_ids, "block_ids"), _host_i32(host_slots, "host_slots")
    if len(b) != len(s):
        raise ValueError("block_ids and host_slots differ in length")
    _ok(pool._lib.fs_pool_upload(pool._h, s.ctypes.data, b.ctypes.data, len(b), _stream_ptr(stream)),
        "fs_pool_upload")


def fs_stream_read(src: torch.Tensor, sink: torch.Tensor, workgroups: int, stream=None) -> None:
    """Reads every byte of `src` once (measurement helper)."""
    _ok(load_library().fs_stream_read(_dev(src, "src"), src.numel() * src.element_size(), _dev(sink, "sink"),
                                      int(workgroups), _stream_ptr(stream)), "fs_stream_read")


def fs_stream_read_timed(src: torch.Tensor, sink: torch.Tensor, workgroups: int, stream=None) -> float:
    """fs_stream_read, waited for; returns the kernel's own duration in microseconds."""
    us = ctypes.c_float(0.0)
    _ok(load_library().fs_stream_read_timed(_dev(src, "src"), src.numel() * src.element_size(), _dev(sink, "sink"),
                                            int(workgroups), _stream_ptr(stream), ctypes.byref(us)),
        "fs_stream_read_timed")
    return float(us.value)


def fs_stream_copy(dst: torch.Tensor, src: torch.Tensor, workgroups: int, stream=None) -> None:
    """Copies `src` to `dst` with a plain kernel (measurement helper)."""
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < n:
        raise ValueError("dst smaller than src")
    _ok(load_library().fs_stream_copy(_dev(dst, "dst"), _dev(src, "src"), n, int(workgroups),
                                      _stream_ptr(stream)), "fs_stream_copy")
