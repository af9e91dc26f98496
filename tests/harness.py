"""Shared plumbing of the GPU parity tests: moves one seeded decode step through
the C-ABI library and through the CPU oracle.  No method arithmetic lives here."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

import fs_workload as wl
import oracle
from oracle.layout_model import PoolLayout

# tolerance for attention outputs against the fp64 oracle (bf16 KV, fp32 accumulation)
MAX_ABS_TOL = 1e-2
REL_L2_TOL = 5e-3


def to_torch(cfg_dtype: str, a: np.ndarray, device="cuda") -> torch.Tensor:
    """Host array in storage form (bf16, f16 as uint16 bits) -> device tensor of the pool dtype."""
    if cfg_dtype in ("bf16", "f16"):
        t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device)
        return t.view(torch.bfloat16 if cfg_dtype == "bf16" else torch.float16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def from_torch(cfg_dtype: str, t: torch.Tensor) -> np.ndarray:
    if cfg_dtype in ("bf16", "f16"):
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def layout_of(cfg: wl.WorkloadConfig) -> PoolLayout:
    return PoolLayout(cfg.num_heads, cfg.head_dim, cfg.block_size, cfg.elem_bytes)


def sentinel_of(cfg: wl.WorkloadConfig):
    return np.uint16(0x7FC1) if cfg.dtype in ("bf16", "f16") else np.float32(-12345.678)


@dataclass
class Case:
    step: wl.Step
    caches: list            # per job (K, V) host arrays [L][H][D]
    lens_before: np.ndarray
    k_new: np.ndarray
    v_new: np.ndarray

    @property
    def cfg(self):
        return self.step.cfg


def make_case(cfg: wl.WorkloadConfig, rep: int = 0, lens: Optional[np.ndarray] = None,
              width: Optional[int] = None) -> Case:
    step = wl.make_step(cfg, rep, width=width)
    if lens is not None:
        lens = np.asarray(lens, dtype=np.int32)
        assert len(lens) == cfg.num_jobs
        step.lens = lens
        step.tables = wl.block_tables(cfg, lens, step.seed, width)
    with ThreadPoolExecutor(max_workers=8) as ex:      # numpy's generators release the GIL
        caches = list(ex.map(step.cache, range(cfg.num_jobs)))
    shape = (cfg.num_jobs, cfg.num_heads, cfg.head_dim)
    k_new = np.zeros(shape, dtype=cfg.np_dtype)
    v_new = np.zeros(shape, dtype=cfg.np_dtype)
    for j, (K, V) in enumerate(caches):
        if step.lens[j] > 0:
            k_new[j], v_new[j] = K[-1], V[-1]
    return Case(step, caches, np.maximum(step.lens - 1, 0).astype(np.int32), k_new, v_new)


def oracle_step(case: Case) -> np.ndarray:
    """Append + attention on the logical caches (float64 [J][H][D])."""
    cfg = case.cfg
    lc = oracle.LogicalCaches(cfg.dtype, cfg.num_heads, cfg.head_dim)
    for j, (K, V) in enumerate(case.caches):
        n = int(case.lens_before[j])
        lc.add_job(np.ascontiguousarray(K[:n]), np.ascontiguousarray(V[:n]))
    active = case.step.lens > 0
    if active.all():
        return lc.decode_step(case.k_new, case.v_new, case.step.q)
    # jobs with nothing to attend over take no append; the oracle gives them zeros
    out = np.zeros((cfg.num_jobs, cfg.num_heads, cfg.head_dim))
    for j in range(cfg.num_jobs):
        if active[j]:
            one = oracle.LogicalCaches(cfg.dtype, cfg.num_heads, cfg.head_dim)
            one.add_job(lc.K[j][:lc.lens[j]], lc.V[j][:lc.lens[j]])
            out[j] = one.decode_step(case.k_new[j:j + 1], case.v_new[j:j + 1], case.step.q[j:j + 1])[0]
    return out


def expected_image(case: Case, table: np.ndarray, num_blocks: int, upto: str = "append") -> np.ndarray:
    """Pool image the layout model predicts: sentinel everywhere except written cells."""
    cfg = case.cfg
    lay = layout_of(cfg)
    img = np.full((num_blocks, lay.block_elems), sentinel_of(cfg), dtype=cfg.np_dtype)
    for j, (K, V) in enumerate(case.caches):
        n = int(case.lens_before[j])
        lay.write_tokens(img, table[j], 0, K[:n], V[:n])
    if upto == "append":
        append_into(img, case, table)
    return img


def append_into(img: np.ndarray, case: Case, table: np.ndarray) -> np.ndarray:
    """Adds this step's appended tokens to a prefix image (in place)."""
    lay = layout_of(case.cfg)
    for j, (K, V) in enumerate(case.caches):
        n = int(case.lens_before[j])
        if case.step.lens[j] > 0:
            lay.write_tokens(img, table[j], n, K[n:n + 1], V[n:n + 1])
    return img


class DeviceRun:
    """One pool on the GPU holding a case; drives the library through the binding."""

    def __init__(self, case: Case, fill: str = "image", table: Optional[np.ndarray] = None,
                 num_host_blocks: int = 0, prefix_image: Optional[np.ndarray] = None, **pool_kw):
        import paper_2305_05920_amd as fs
        self.fs = fs
        self.case = case
        cfg = case.cfg
        bt = case.step.tables
        self.table_np = bt.table if table is None else table
        self.num_blocks = bt.num_blocks
        lay = layout_of(cfg)
        if fill == "image":
            img = prefix_image if prefix_image is not None else \
                expected_image(case, self.table_np, self.num_blocks, upto="prefix")
            self.mem = to_torch(cfg.dtype, img)
        else:
            self.mem = to_torch(cfg.dtype, np.full((self.num_blocks, lay.block_elems), sentinel_of(cfg),
                                                   dtype=cfg.np_dtype))
        self.pool = fs.Pool(cfg.dtype, cfg.num_heads, cfg.head_dim, self.num_blocks,
                            block_size=cfg.block_size, num_host_blocks=num_host_blocks,
                            device_mem=self.mem, **pool_kw)
        self.table = torch.from_numpy(self.table_np).cuda()
        self.lens_before = torch.from_numpy(case.lens_before).cuda()
        self.lens = torch.from_numpy(case.step.lens).cuda()
        self.q = to_torch(cfg.dtype, case.step.q)
        self.k_new = to_torch(cfg.dtype, case.k_new)
        self.v_new = to_torch(cfg.dtype, case.v_new)
        self.out = torch.full((cfg.num_jobs, cfg.num_heads, cfg.head_dim), float("nan"),
                              dtype=torch.float32, device="cuda")
        if fill == "prefill":
            self.prefill()

    def prefill(self):
        cfg = self.case.cfg
        ns = self.case.lens_before.astype(np.int64)
        offs = np.zeros(cfg.num_jobs + 1, dtype=np.int32)
        offs[1:] = np.cumsum(ns)
        total = int(offs[-1])
        if total == 0:
            return
        K = np.concatenate([K[:n] for (K, _), n in zip(self.case.caches, ns)])
        V = np.concatenate([V[:n] for (_, V), n in zip(self.case.caches, ns)])
        self.fs.fs_kv_prefill(self.pool, self.table, torch.zeros(cfg.num_jobs, dtype=torch.int32, device="cuda"),
                              torch.from_numpy(offs).cuda(), total, to_torch(cfg.dtype, K),
                              to_torch(cfg.dtype, V))
        torch.cuda.synchronize()

    def append(self):
        # jobs with post-append length 0 do not take part in the step
        self.fs.fs_kv_append(self.pool, self.table, self.lens_before, self.k_new, self.v_new)

    def attention(self, max_len_hint: int = 0) -> np.ndarray:
        self.fs.fs_decode_attention(self.q, self.pool, self.table, self.lens, self.out,
                                    max_len_hint=max_len_hint)
        torch.cuda.synchronize()
        return self.out.cpu().numpy()

    def fused_step(self, max_len_hint: int = 0) -> np.ndarray:
        """Append + attention through the single fused entry point."""
        self.fs.fs_decode_step(self.pool, self.table, self.lens_before, self.k_new, self.v_new, self.q,
                               self.out, max_len_hint=max_len_hint)
        torch.cuda.synchronize()
        return self.out.cpu().numpy()

    def image(self) -> np.ndarray:
        torch.cuda.synchronize()
        return from_torch(self.case.cfg.dtype, self.mem)

    def close(self):
        self.pool.close()


def errors(gpu: np.ndarray, ref: np.ndarray):
    diff = gpu.astype(np.float64) - ref
    max_abs = float(np.abs(diff).max(initial=0.0))
    denom = float(np.linalg.norm(ref.ravel()))
    rel_l2 = float(np.linalg.norm(diff.ravel()) / denom) if denom > 0 else float(np.linalg.norm(diff.ravel()))
    return max_abs, rel_l2


def assert_parity(gpu: np.ndarray, ref: np.ndarray, what: str = ""):
    assert np.isfinite(gpu).all(), f"{what}: non-finite output"
    max_abs, rel_l2 = errors(gpu, ref)
    print(f"[parity] {what}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}", flush=True)
    assert max_abs <= MAX_ABS_TOL, f"{what}: max abs error {max_abs:.3e} > {MAX_ABS_TOL}"
    assert rel_l2 <= REL_L2_TOL, f"{what}: relative L2 error {rel_l2:.3e} > {REL_L2_TOL}"
    return max_abs, rel_l2
