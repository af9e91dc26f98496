"""Seeded synthetic workloads for the paged decode step (inputs only).

This module draws the *inputs* of one decode iteration: per-job KV lengths,
block tables over a block pool, and Q/K/V values.  It contains none of the
method's arithmetic (no dot products, no softmax, no pool addressing): both the
CPU oracle and the GPU path consume what it returns, and neither is imported
here.

The five presets follow the shapes of the paper's evaluation models (Table 1:
OPT-13B 40 heads / hidden 5120, OPT-175B 96 heads / hidden 12288, so
head_dim 128) and its description of serving workloads as long-tailed and
skewed (Section 2.3, Figure 1); the datasets themselves are not used.

Storage convention: bf16 and f16 tensors are carried as numpy ``uint16`` bit patterns
(round-to-nearest-even of an fp32 N(0,1) draw, done once here), fp32 tensors as
``float32``.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Optional

import numpy as np

BASE_SEED = 0xF5E00000
BLOCK_SIZE = 16

# stream tags: every array comes from its own SeedSequence([seed, tag, ...])
_TAG_LENS, _TAG_TABLE, _TAG_KV, _TAG_Q, _TAG_SWAP = 1, 2, 3, 4, 5


@dataclass(frozen=True)
class WorkloadConfig:
    index: int
    name: str
    num_heads: int
    head_dim: int
    dtype: str          # "bf16", "f16" or "f32"
    num_jobs: int
    lens_recipe: str    # see job_lens()
    table_recipe: str   # see block_tables()
    block_size: int = BLOCK_SIZE
    max_len: int = 2048  # upper clip of the length recipe

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype in ("bf16", "f16") else 4

    @property
    def np_dtype(self):
        return np.uint16 if self.dtype in ("bf16", "f16") else np.float32

    def scaled(self, **kw) -> "WorkloadConfig":
        """A copy with some fields replaced (smaller job counts for CPU tests)."""
        return dataclasses.replace(self, **kw)


CONFIGS = (
    WorkloadConfig(0, "tiny", 8, 64, "f32", 4, "uniform_1_256", "perm128", max_len=256),
    WorkloadConfig(1, "opt13b_layer", 40, 128, "bf16", 32, "exp512", "shuffled"),
    WorkloadConfig(2, "opt175b_tp8_share", 12, 128, "bf16", 256, "pareto1.5", "fragmented"),
    WorkloadConfig(3, "skipjoin_mixed", 40, 128, "bf16", 128, "bimodal", "shuffled"),
    WorkloadConfig(4, "long_context", 64, 128, "bf16", 8, "uniform_16k_32k", "shuffled",
                   max_len=32768),
)


def seed_for(config_index: int, rep: int = 0) -> int:
    return BASE_SEED + 16 * int(config_index) + int(rep)


def _rng(seed: int, *tags: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), *map(int, tags)])))


# ----------------------------------------------------------------------------
# lengths
# ----------------------------------------------------------------------------
def job_lens(cfg: WorkloadConfig, seed: int) -> np.ndarray:
    """Post-append KV length L_j of every admitted job (int32, >= 1)."""
    rng = _rng(seed, _TAG_LENS)
    J = cfg.num_jobs
    r = cfg.lens_recipe
    if r == "uniform_1_256":
        lens = rng.integers(1, min(256, cfg.max_len) + 1, size=J)
    elif r == "exp512":
        lens = np.clip(np.rint(rng.exponential(512.0, size=J)), 16, cfg.max_len)
    elif r == "pareto1.5":
        u = 1.0 - rng.random(size=J)            # (0, 1]
        lens = np.clip(np.floor(32.0 * u ** (-1.0 / 1.5)), 32, cfg.max_len)
    elif r == "bimodal":
        short = rng.random(size=J) < 0.7
        a = rng.integers(32, 128 + 1, size=J)
        b = rng.integers(min(1536, cfg.max_len), cfg.max_len + 1, size=J)
        lens = np.where(short, a, b)
    elif r == "uniform_16k_32k":
        lens = rng.integers(cfg.max_len // 2, cfg.max_len + 1, size=J)
    else:
        raise ValueError(f"unknown lens recipe {r!r}")
    return lens.astype(np.int32)


# ----------------------------------------------------------------------------
# block tables
# ----------------------------------------------------------------------------
@dataclass
class SwapPlan:
    """Blocks that leave HBM for host slots and come back under new ids."""
    jobs: np.ndarray        # job indices that are swapped
    old_ids: np.ndarray     # their block ids before the swap (flattened, job order)
    new_ids: np.ndarray     # ids they are uploaded into (same order)
    host_slots: np.ndarray  # host slot used for each block


@dataclass
class BlockTables:
    table: np.ndarray            # int32 [J][W], unused entries -1 (state after any swap)
    num_blocks: int              # pool size in blocks
    width: int                   # W
    table_before_swap: Optional[np.ndarray] = None
    swap: Optional[SwapPlan] = None


def _blocks_of(lens: np.ndarray, block_size: int) -> np.ndarray:
    return (lens.astype(np.int64) + block_size - 1) // block_size


def block_tables(cfg: WorkloadConfig, lens: np.ndarray, seed: int,
                 width: Optional[int] = None) -> BlockTables:
    rng = _rng(seed, _TAG_TABLE)
    B = cfg.block_size
    nb = _blocks_of(lens, B)
    total = int(nb.sum())
    J = len(lens)
    W = int(width) if width is not None else max(1, (cfg.max_len + B - 1) // B)
    if nb.max(initial=0) > W:
        raise ValueError("table width too small")
    table = np.full((J, W), -1, dtype=np.int32)
    r = cfg.table_recipe
    if r == "perm128":
        num_blocks = 128
        if total > num_blocks:
            raise ValueError("perm128 pool too small for these lengths")
        ids = rng.permutation(num_blocks)[:total]
        _deal(table, nb, ids)
        return BlockTables(table, num_blocks, W)
    num_blocks = max(1, int(np.ceil(1.5 * total)))
    if r == "shuffled":
        ids = rng.permutation(num_blocks)[:total]
        _deal(table, nb, ids)
        return BlockTables(table, num_blocks, W)
    if r == "fragmented":
        # jobs grow block by block in a random interleaving; ids handed out in rising order
        owner = np.repeat(np.arange(J), nb)
        rng.shuffle(owner)
        fill = np.zeros(J, dtype=np.int64)
        for bid, j in enumerate(owner):
            table[j, fill[j]] = bid
            fill[j] += 1
        before = table.copy()
        # a quarter of the jobs are offloaded, then uploaded into freed or spare ids
        srng = _rng(seed, _TAG_SWAP)
        n_swap = max(1, J // 4)
        jobs = np.sort(srng.choice(J, size=n_swap, replace=False))
        old_ids = np.concatenate([before[j, :nb[j]] for j in jobs]).astype(np.int32)
        free = np.concatenate([old_ids, np.arange(total, num_blocks, dtype=np.int32)])
        new_ids = srng.permutation(free)[:len(old_ids)].astype(np.int32)
        host_slots = srng.permutation(len(old_ids)).astype(np.int32)
        pos = 0
        for j in jobs:
            table[j, :nb[j]] = new_ids[pos:pos + nb[j]]
            pos += nb[j]
        return BlockTables(table, num_blocks, W, before,
                           SwapPlan(jobs, old_ids, new_ids, host_slots))
    raise ValueError(f"unknown table recipe {r!r}")


def _deal(table: np.ndarray, nb: np.ndarray, ids: np.ndarray) -> None:
    pos = 0
    for j, n in enumerate(nb):
        table[j, :n] = ids[pos:pos + n]
        pos += int(n)


# ----------------------------------------------------------------------------
# values
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> IEEE binary16 bit patterns."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of binary16 bit patterns to fp32."""
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float32)


def to_f64(cfg_or_dtype, x: np.ndarray) -> np.ndarray:
    """Exact widening of a stored tensor to float64."""
    dtype = cfg_or_dtype if isinstance(cfg_or_dtype, str) else cfg_or_dtype.dtype
    if dtype == "bf16":
        return bf16_bits_to_f32(x).astype(np.float64)
    if dtype == "f16":
        return f16_bits_to_f32(x).astype(np.float64)
    return np.asarray(x, dtype=np.float32).astype(np.float64)


def _normal(cfg: WorkloadConfig, rng: np.random.Generator, shape) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if cfg.dtype == "bf16":
        return f32_to_bf16_bits(x)
    return f32_to_f16_bits(x) if cfg.dtype == "f16" else x


def job_cache(cfg: WorkloadConfig, seed: int, job: int, length: int):
    """K and V of one job, logical layout [L][H][D]; the last row is the token
    appended in this step, rows before it are what the cache already held."""
    rng = _rng(seed, _TAG_KV, job)
    shape = (int(length), cfg.num_heads, cfg.head_dim)
    k = _normal(cfg, rng, shape)
    v = _normal(cfg, rng, shape)
    return k, v


def queries(cfg: WorkloadConfig, seed: int, num_jobs: Optional[int] = None) -> np.ndarray:
    """q[J][H][D] of the new token of every job."""
    rng = _rng(seed, _TAG_Q)
    J = cfg.num_jobs if num_jobs is None else num_jobs
    return _normal(cfg, rng, (J, cfg.num_heads, cfg.head_dim))


@dataclass
class Step:
    cfg: WorkloadConfig
    seed: int
    lens: np.ndarray          # post-append lengths L_j
    tables: BlockTables
    q: np.ndarray             # [J][H][D]

    def cache(self, job: int):
        return job_cache(self.cfg, self.seed, job, int(self.lens[job]))

    @property
    def total_tokens(self) -> int:
        return int(self.lens.astype(np.int64).sum())


def make_step(cfg: WorkloadConfig, rep: int = 0, seed: Optional[int] = None,
              width: Optional[int] = None) -> Step:
    seed = seed_for(cfg.index, rep) if seed is None else seed
    lens = job_lens(cfg, seed)
    tables = block_tables(cfg, lens, seed, width)
    return Step(cfg, seed, lens, tables, queries(cfg, seed))
