"""The seeded generator: determinism, the stated length recipes, valid tables."""
import numpy as np
import pytest

import fs_workload as wl


@pytest.mark.parametrize("cfg", wl.CONFIGS[:4], ids=lambda c: c.name)
def test_lens_follow_their_recipe(cfg):
    lens = wl.job_lens(cfg, wl.seed_for(cfg.index))
    assert lens.dtype == np.int32 and lens.shape == (cfg.num_jobs,)
    lo = {0: 1, 1: 16, 2: 32, 3: 32}[cfg.index]
    assert lens.min() >= lo and lens.max() <= cfg.max_len
    if cfg.index == 3:
        short = (lens <= 128).sum()
        assert ((lens <= 128) | (lens >= 1536)).all() and 0.5 < short / len(lens) < 0.9


def test_long_context_lens():
    cfg = wl.CONFIGS[4]
    lens = wl.job_lens(cfg, wl.seed_for(4))
    assert lens.min() >= 16384 and lens.max() <= 32768 and len(lens) == 8


def test_expected_total_tokens_are_near_the_planned_workload_sizes():
    # mean lengths of the recipes: ~503, ~88, ~594 tokens (averaged over seeds)
    for idx, mean in ((1, 503), (2, 88), (3, 594)):
        cfg = wl.CONFIGS[idx]
        tot = np.mean([wl.job_lens(cfg, wl.seed_for(idx, r)).mean() for r in range(16)])
        assert abs(tot - mean) / mean < 0.15, (idx, tot)


@pytest.mark.parametrize("cfg", wl.CONFIGS, ids=lambda c: c.name)
def test_tables_are_valid_and_disjoint(cfg):
    seed = wl.seed_for(cfg.index)
    lens = wl.job_lens(cfg, seed)
    bt = wl.block_tables(cfg, lens, seed)
    nb = (lens + cfg.block_size - 1) // cfg.block_size
    used = np.concatenate([bt.table[j, :nb[j]] for j in range(len(lens))])
    assert used.min() >= 0 and used.max() < bt.num_blocks
    assert len(np.unique(used)) == len(used)                     # no block shared
    for j in range(len(lens)):
        assert (bt.table[j, nb[j]:] == -1).all()
    if cfg.index == 0:
        assert bt.num_blocks == 128
    else:
        assert bt.num_blocks == int(np.ceil(1.5 * nb.sum()))
    if cfg.table_recipe == "fragmented":
        sw = bt.swap
        assert len(sw.jobs) == cfg.num_jobs // 4
        before = np.concatenate([bt.table_before_swap[j, :nb[j]] for j in range(len(lens))])
        assert len(np.unique(before)) == len(before)
        assert len(np.unique(sw.host_slots)) == len(sw.old_ids) == len(sw.new_ids)
        untouched = np.setdiff1d(np.arange(len(lens)), sw.jobs)
        assert np.array_equal(bt.table[untouched], bt.table_before_swap[untouched])


def test_everything_is_deterministic_in_the_seed():
    cfg = wl.CONFIGS[1].scaled(num_jobs=4)
    a, b = wl.make_step(cfg, rep=1), wl.make_step(cfg, rep=1)
    c = wl.make_step(cfg, rep=2)
    assert np.array_equal(a.lens, b.lens) and np.array_equal(a.tables.table, b.tables.table)
    assert np.array_equal(a.q, b.q)
    ka, va = a.cache(2)
    kb, vb = b.cache(2)
    assert np.array_equal(ka, kb) and np.array_equal(va, vb) and not np.array_equal(ka, va)
    assert not np.array_equal(a.lens, c.lens)


def test_values_are_standard_normal_and_bf16_exact():
    cfg = wl.CONFIGS[1]
    k, _ = wl.job_cache(cfg, 123, 0, 64)
    assert k.dtype == np.uint16 and k.shape == (64, 40, 128)
    f = wl.bf16_bits_to_f32(k)
    assert abs(f.mean()) < 0.01 and abs(f.std() - 1.0) < 0.01
    assert np.array_equal(wl.f32_to_bf16_bits(f), k)             # already representable
