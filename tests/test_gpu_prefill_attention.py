"""GPU parity of the prompt-phase attention (matrix-core kernel, called through the C ABI)
against the CPU oracle's causal definition, prompt by prompt."""
import os

import numpy as np
import pytest
import torch

import fs_workload as wl
import oracle
from tests import harness as hs

pytestmark = pytest.mark.gpu


def make_prompts(dtype, lens, H, D, seed):
    rng = np.random.default_rng(seed)
    T = int(sum(lens))
    conv = wl.f32_to_bf16_bits if dtype == "bf16" else wl.f32_to_f16_bits
    q, k, v = (conv(rng.standard_normal((T, H, D), dtype=np.float32)) for _ in range(3))
    offs = np.zeros(len(lens) + 1, dtype=np.int32)
    offs[1:] = np.cumsum(lens)
    return q, k, v, offs


def run_device(dtype, H, D, q, k, v, offs, guard=3):
    import paper_2305_05920_amd as fs
    T = q.shape[0]
    pool = fs.Pool(dtype, H, D, 4)
    try:
        # rows past T must stay untouched; rows inside must all be written
        out = torch.full((T + guard, H, D), float("nan"), dtype=torch.float32, device="cuda")
        fs.fs_prefill_attention(pool, hs.to_torch(dtype, q), hs.to_torch(dtype, k), hs.to_torch(dtype, v),
                                torch.from_numpy(offs).cuda(), out[:T])
        torch.cuda.synchronize()
        pool.check()
        got = out.cpu().numpy()
    finally:
        pool.close()
    assert np.isnan(got[T:]).all(), "rows past the last token were written"
    return got[:T]


def oracle_prompts(dtype, q, k, v, offs):
    ref = np.zeros(q.shape, dtype=np.float64)
    for j in range(len(offs) - 1):
        a, b = int(offs[j]), int(offs[j + 1])
        if b > a:
            ref[a:b] = oracle.prefill_attention_job(np.ascontiguousarray(q[a:b]), np.ascontiguousarray(k[a:b]),
                                                    np.ascontiguousarray(v[a:b]), dtype)
    return ref


EDGE_LENS = [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 257, 0, 5]


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("bf16", 64), ("f16", 128), ("f16", 64)])
def test_tile_boundaries_and_ragged_prompts(dtype, D):
    print(f"[case] prefill attention edges {dtype} D={D}", flush=True)
    H = 3
    q, k, v, offs = make_prompts(dtype, EDGE_LENS, H, D, 11)
    got = run_device(dtype, H, D, q, k, v, offs)
    assert np.isfinite(got).all()
    ref = oracle_prompts(dtype, q, k, v, offs)
    hs.assert_parity(got, ref, f"prefill attention edges {dtype} D={D}")
    # the first token of every prompt returns its own value row (its only weight is 1 up to
    # the rounding of the fused scale-and-subtract in front of the exponential)
    for j, n in enumerate(EDGE_LENS):
        if n:
            np.testing.assert_allclose(got[offs[j]].astype(np.float64), wl.to_f64(dtype, v[offs[j]]), rtol=5e-7, atol=0)


@pytest.mark.parametrize("rep", [0, 1])
def test_prompt_lengths_of_the_headline_preset(rep):
    # prompt lengths drawn as the cache lengths of preset 1 (exponential, mean 512), fewer heads
    cfg = wl.CONFIGS[1].scaled(num_jobs=6, num_heads=4)
    lens = wl.job_lens(cfg, wl.seed_for(cfg.index, rep)).tolist()
    print(f"[case] prefill attention preset-1 lengths {lens}", flush=True)
    q, k, v, offs = make_prompts("bf16", lens, cfg.num_heads, cfg.head_dim, 77 + rep)
    got = run_device("bf16", cfg.num_heads, cfg.head_dim, q, k, v, offs)
    hs.assert_parity(got, oracle_prompts("bf16", q, k, v, offs), f"prefill attention preset 1 rep {rep}")


def test_long_prompt_spans_many_key_tiles():
    lens = [1500, 700]
    q, k, v, offs = make_prompts("bf16", lens, 2, 128, 5)
    got = run_device("bf16", 2, 128, q, k, v, offs)
    hs.assert_parity(got, oracle_prompts("bf16", q, k, v, offs), "prefill attention long")


def test_zero_jobs_and_all_prompts_empty():
    import paper_2305_05920_amd as fs
    pool = fs.Pool("bf16", 2, 64, 4)
    x = torch.zeros((5, 2, 64), dtype=torch.bfloat16, device="cuda")
    o = torch.full((5, 2, 64), 7.0, dtype=torch.float32, device="cuda")
    # three jobs without a token: nothing to do, nothing written
    fs.fs_prefill_attention(pool, x, x, x, torch.zeros(4, dtype=torch.int32, device="cuda"), o)
    torch.cuda.synchronize()
    pool.check()
    assert (o == 7.0).all()
    e = torch.zeros((0, 2, 64), dtype=torch.bfloat16, device="cuda")
    fs.fs_prefill_attention(pool, e, e, e, torch.zeros(1, dtype=torch.int32, device="cuda"),
                            torch.zeros((0, 2, 64), dtype=torch.float32, device="cuda"))
    pool.check()
    pool.close()


def test_bad_offsets_raise_the_flag():
    import paper_2305_05920_amd as fs
    H, D = 2, 64
    q, k, v, offs = make_prompts("bf16", [40, 300], H, D, 7)
    for bad_offs in (np.array([0, 40, 999], np.int32),        # job 1 runs past the arrays
                     np.array([0, 60, 40], np.int32)):        # job 1 decreasing
        pool = fs.Pool("bf16", H, D, 4)
        out = torch.zeros((340, H, D), dtype=torch.float32, device="cuda")
        fs.fs_prefill_attention(pool, hs.to_torch("bf16", q), hs.to_torch("bf16", k), hs.to_torch("bf16", v),
                                torch.from_numpy(bad_offs).cuda(), out)
        torch.cuda.synchronize()
        with pytest.raises(fs.FsError):
            pool.check()
        pool.close()


def test_a_bad_job_leaves_the_valid_ones_served():
    import paper_2305_05920_amd as fs
    H, D = 2, 64
    q, k, v, offs = make_prompts("bf16", [40, 300], H, D, 7)
    ref = oracle_prompts("bf16", q, k, v, offs)
    pool = fs.Pool("bf16", H, D, 4)
    out = torch.full((340, H, D), float("nan"), dtype=torch.float32, device="cuda")
    fs.fs_prefill_attention(pool, hs.to_torch("bf16", q), hs.to_torch("bf16", k), hs.to_torch("bf16", v),
                            torch.tensor([0, 40, 999], dtype=torch.int32, device="cuda"), out)
    torch.cuda.synchronize()
    with pytest.raises(fs.FsError):
        pool.check()
    pool.close()
    got = out.cpu().numpy()
    hs.assert_parity(got[:40], ref[:40], "valid job beside a bad one")
    assert np.isnan(got[40:]).all(), "rows of the bad job were written"


def test_more_jobs_than_one_launch_slice():
    # 1100 prompts of 1..5 tokens: two launches (1024 jobs each at most)
    rng = np.random.default_rng(3)
    lens = rng.integers(1, 6, size=1100).tolist()
    q, k, v, offs = make_prompts("bf16", lens, 2, 64, 8)
    got = run_device("bf16", 2, 64, q, k, v, offs)
    hs.assert_parity(got, oracle_prompts("bf16", q, k, v, offs), "prefill attention 1100 short prompts")


def test_float_pools_are_refused():
    import paper_2305_05920_amd as fs
    pool = fs.Pool("f32", 2, 64, 4)
    x = torch.zeros((8, 2, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(fs.FsError) as ei:
        fs.fs_prefill_attention(pool, x, x, x, torch.tensor([0, 8], dtype=torch.int32, device="cuda"), x.clone())
    assert ei.value.status == fs.FS_ERR_UNSUPPORTED
    pool.close()


# ---- the whole initialization phase in one launch: cache fill + attention ---------------
def shuffled_tables(lens, block_size, spare, seed):
    """Every job owns ceil(len/block) blocks drawn without order from a pool with `spare` extra."""
    nblk = [(n + block_size - 1) // block_size for n in lens]
    total = sum(nblk) + spare
    ids = np.random.default_rng(seed).permutation(total).astype(np.int32)
    W = max(max(nblk), 1)
    table = np.full((len(lens), W), -1, dtype=np.int32)
    at = 0
    for j, nb in enumerate(nblk):
        table[j, :nb] = ids[at:at + nb]
        at += nb
    return table, total


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f16", 64), ("bf16", 64)])
def test_prefill_step_fills_the_cache_bit_exactly_and_matches_the_oracle(dtype, D):
    import paper_2305_05920_amd as fs
    from oracle.layout_model import PoolLayout
    H = 3
    lens = [1, 15, 16, 17, 63, 64, 65, 128, 129, 200, 0, 300]
    print(f"[case] prefill step {dtype} D={D}", flush=True)
    q, k, v, offs = make_prompts(dtype, lens, H, D, 21)
    table, nb = shuffled_tables(lens, 16, 5, 22)
    lay = PoolLayout(H, D, 16, 2)
    sentinel = np.uint16(0x7FC1)
    want = np.full((nb, lay.block_elems), sentinel, dtype=np.uint16)
    for j, n in enumerate(lens):
        lay.write_tokens(want, table[j], 0, k[offs[j]:offs[j + 1]], v[offs[j]:offs[j + 1]])
    mem = hs.to_torch(dtype, np.full((nb, lay.block_elems), sentinel, dtype=np.uint16))
    pool = fs.Pool(dtype, H, D, nb, device_mem=mem)
    T = q.shape[0]
    out = torch.full((T, H, D), float("nan"), dtype=torch.float32, device="cuda")
    fs.fs_prefill_step(pool, torch.from_numpy(table).cuda(), torch.from_numpy(offs).cuda(),
                       hs.to_torch(dtype, k), hs.to_torch(dtype, v), hs.to_torch(dtype, q), out)
    torch.cuda.synchronize()
    pool.check()
    img = hs.from_torch(dtype, mem)
    pool.close()
    assert np.array_equal(img, want), "pool image differs from the layout model"
    hs.assert_parity(out.cpu().numpy(), oracle_prompts(dtype, q, k, v, offs), f"prefill step {dtype} D={D}")


def test_prefill_step_then_decode_steps_match_the_oracle():
    # the two phases of a job back to back: prompts through fs_prefill_step, then three fused
    # decode steps over the blocks it filled
    import paper_2305_05920_amd as fs
    H, D, dtype = 4, 128, "bf16"
    lens = [37, 128, 5, 260]
    q, k, v, offs = make_prompts(dtype, lens, H, D, 31)
    table, nb = shuffled_tables([n + 3 for n in lens], 16, 2, 32)
    pool = fs.Pool(dtype, H, D, nb)
    d_table = torch.from_numpy(table).cuda()
    out = torch.empty((q.shape[0], H, D), dtype=torch.float32, device="cuda")
    fs.fs_prefill_step(pool, d_table, torch.from_numpy(offs).cuda(), hs.to_torch(dtype, k), hs.to_torch(dtype, v),
                       hs.to_torch(dtype, q), out)
    lc = oracle.LogicalCaches(dtype, H, D)
    for j in range(len(lens)):
        lc.add_job(np.ascontiguousarray(k[offs[j]:offs[j + 1]]), np.ascontiguousarray(v[offs[j]:offs[j + 1]]),
                   spare=3)
    rng = np.random.default_rng(33)
    cur = np.array(lens, dtype=np.int32)
    for stepno in range(3):
        qn, kn, vn = (wl.f32_to_bf16_bits(rng.standard_normal((len(lens), H, D), dtype=np.float32)) for _ in range(3))
        got = torch.empty((len(lens), H, D), dtype=torch.float32, device="cuda")
        fs.fs_decode_step(pool, d_table, torch.from_numpy(cur).cuda(), hs.to_torch(dtype, kn), hs.to_torch(dtype, vn),
                          hs.to_torch(dtype, qn), got)
        torch.cuda.synchronize()
        pool.check()
        ref = lc.decode_step(kn, vn, qn)
        hs.assert_parity(got.cpu().numpy(), ref, f"decode step {stepno} after prefill step")
        cur += 1
    pool.close()


def test_prefill_step_flags_a_table_that_is_too_short():
    import paper_2305_05920_amd as fs
    H, D = 2, 64
    q, k, v, offs = make_prompts("bf16", [40], H, D, 41)
    table = np.array([[0, 1]], dtype=np.int32)                 # 32 tokens of room for 40
    pool = fs.Pool("bf16", H, D, 4)
    out = torch.empty((40, H, D), dtype=torch.float32, device="cuda")
    fs.fs_prefill_step(pool, torch.from_numpy(table).cuda(), torch.from_numpy(offs).cuda(), hs.to_torch("bf16", k),
                       hs.to_torch("bf16", v), hs.to_torch("bf16", q), out)
    torch.cuda.synchronize()
    with pytest.raises(fs.FsError):
        pool.check()
    pool.close()


def test_initialization_phase_at_the_benchmarked_size_sampled():
    # The workload bench.py times for the initialization phase: the headline preset's 32 lengths
    # taken as prompts, 40 heads x 128, bf16 (18.6 k tokens), through fs_prefill_step with
    # shuffled block tables.  The oracle recomputes sampled (token, head) rows one by one (a
    # decode-style attention over the first i+1 tokens); every other row must be finite and
    # inside the bound that holds for any attention output (|out| <= max |v| over the prompt);
    # sampled blocks are read back through the C ABI against the layout model.
    import paper_2305_05920_amd as fs
    from oracle.layout_model import PoolLayout
    cfg = wl.CONFIGS[1]
    H, D, dtype = cfg.num_heads, cfg.head_dim, cfg.dtype
    lens = wl.job_lens(cfg, wl.seed_for(cfg.index, 0)).tolist()
    print(f"[case] initialization phase full size: {len(lens)} prompts, {sum(lens)} tokens", flush=True)
    q, k, v, offs = make_prompts(dtype, lens, H, D, 51)
    table, nb = shuffled_tables(lens, 16, 7, 52)
    lay = PoolLayout(H, D, 16, 2)
    T = q.shape[0]
    with fs.Pool(dtype, H, D, nb) as pool:
        out = torch.full((T, H, D), float("nan"), dtype=torch.float32, device="cuda")
        fs.fs_prefill_step(pool, torch.from_numpy(table).cuda(), torch.from_numpy(offs).cuda(),
                           hs.to_torch(dtype, k), hs.to_torch(dtype, v), hs.to_torch(dtype, q), out)
        torch.cuda.synchronize()
        pool.check()
        got = out.cpu().numpy()
        rng = np.random.default_rng(53)
        for j in rng.choice(len(lens), size=6, replace=False):
            for bi in {0, (lens[j] - 1) // 16, int(rng.integers(0, (lens[j] + 15) // 16))}:
                blk = pool.read_block(int(table[j, bi]), np.uint16)[None]
                n = min(16, lens[j] - bi * 16)
                k1, v1 = lay.read_tokens(blk, np.zeros(1, dtype=np.int32), 0, n)
                a = int(offs[j]) + bi * 16
                assert np.array_equal(k1, k[a:a + n]) and np.array_equal(v1, v[a:a + n]), (j, bi)
    assert np.isfinite(got).all()
    for j in range(len(lens)):
        a, b = int(offs[j]), int(offs[j + 1])
        vmax = np.abs(wl.bf16_bits_to_f32(v[a:b])).max(axis=0)            # [H][D]
        assert (np.abs(got[a:b]) <= vmax + 1e-6).all()
    worst = 0.0
    for _ in range(160):
        j = int(rng.integers(len(lens)))
        i, h = int(rng.integers(lens[j])), int(rng.integers(H))
        a = int(offs[j])
        ref = oracle.attention_job(np.ascontiguousarray(q[a + i]), np.ascontiguousarray(k[a:a + i + 1]),
                                   np.ascontiguousarray(v[a:a + i + 1]), dtype, heads=(h, h + 1))[h]
        err = np.abs(got[a + i, h] - ref).max()
        rel = np.linalg.norm(got[a + i, h] - ref) / np.linalg.norm(ref)
        worst = max(worst, err)
        # the relative bar is stated for whole tensors; a single 128-element row gets some slack
        assert err <= hs.MAX_ABS_TOL and rel <= 4 * hs.REL_L2_TOL, (j, i, h, err, rel)
    print(f"[parity] initialization phase full size: worst sampled max_abs={worst:.3e}", flush=True)


@pytest.mark.parametrize("seed", range(int(os.environ.get("FS_RANDOM_SEEDS", "6"))))
def test_random_prompt_batches_both_entry_points(seed):
    # random job counts, head counts, head_dim, 2-byte dtype and length mixes (zeros included);
    # the attention-only entry point and the fused initialization step against the oracle, the
    # filled pool against the layout model
    import paper_2305_05920_amd as fs
    from oracle.layout_model import PoolLayout
    rng = np.random.default_rng(2000 + seed)
    D = int(rng.choice([64, 128]))
    dtype = str(rng.choice(["bf16", "f16"]))
    H = int(rng.integers(1, 10))
    J = int(rng.integers(1, 24))
    mix = str(rng.choice(["short", "long", "mixed"]))
    hi = {"short": 70, "long": 700, "mixed": 400}[mix]
    lens = rng.integers(0, hi, size=J)
    if mix == "mixed":
        lens = np.where(rng.random(J) < 0.5, rng.integers(0, 20, size=J), lens)
    lens = [int(n) for n in lens]
    print(f"[case] random prompts seed {seed}: J={J} H={H} D={D} {dtype} mix={mix} tokens={sum(lens)}", flush=True)
    if sum(lens) == 0:
        lens[0] = 3
    q, k, v, offs = make_prompts(dtype, lens, H, D, 3000 + seed)
    ref = oracle_prompts(dtype, q, k, v, offs)
    got = run_device(dtype, H, D, q, k, v, offs)
    hs.assert_parity(got, ref, f"random prompts {seed} attention only")
    table, nb = shuffled_tables(lens, 16, 3, 4000 + seed)
    lay = PoolLayout(H, D, 16, 2)
    sentinel = np.uint16(0x7FC1)
    want = np.full((nb, lay.block_elems), sentinel, dtype=np.uint16)
    for j in range(J):
        lay.write_tokens(want, table[j], 0, k[offs[j]:offs[j + 1]], v[offs[j]:offs[j + 1]])
    mem = hs.to_torch(dtype, np.full((nb, lay.block_elems), sentinel, dtype=np.uint16))
    pool = fs.Pool(dtype, H, D, nb, device_mem=mem)
    out = torch.full((q.shape[0], H, D), float("nan"), dtype=torch.float32, device="cuda")
    fs.fs_prefill_step(pool, torch.from_numpy(table).cuda(), torch.from_numpy(offs).cuda(), hs.to_torch(dtype, k),
                       hs.to_torch(dtype, v), hs.to_torch(dtype, q), out)
    torch.cuda.synchronize()
    pool.check()
    img = hs.from_torch(dtype, mem)
    pool.close()
    assert np.array_equal(img, want), "pool image differs from the layout model"
    fused = out.cpu().numpy()
    hs.assert_parity(fused, ref, f"random prompts {seed} fused step")
    assert np.array_equal(fused, got), "the fused step and the attention-only call differ"


def test_very_long_prompt_sampled():
    # one prompt of 20 000 tokens (157 query tiles, 313 key tiles for the last one) beside a short
    # one; sampled rows against the oracle's decode-style attention over the first i+1 tokens
    import paper_2305_05920_amd as fs
    H, D, dtype = 2, 128, "bf16"
    lens = [20000, 77]
    print("[case] prefill attention, 20 000-token prompt", flush=True)
    q, k, v, offs = make_prompts(dtype, lens, H, D, 61)
    got = run_device(dtype, H, D, q, k, v, offs)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(62)
    rows = [0, 1, 127, 128, 19999, 19998, 12345] + [int(x) for x in rng.integers(0, 20000, size=40)]
    worst = 0.0
    for i in rows:
        h = int(rng.integers(H))
        ref = oracle.attention_job(np.ascontiguousarray(q[i]), np.ascontiguousarray(k[:i + 1]),
                                   np.ascontiguousarray(v[:i + 1]), dtype, heads=(h, h + 1))[h]
        err = np.abs(got[i, h] - ref).max()
        worst = max(worst, err)
        assert err <= hs.MAX_ABS_TOL, (i, h, err)
    a = int(offs[1])
    ref = oracle.prefill_attention_job(np.ascontiguousarray(q[a:]), np.ascontiguousarray(k[a:]),
                                       np.ascontiguousarray(v[a:]), dtype)
    hs.assert_parity(got[a:], ref, "short prompt beside the long one")
    print(f"[parity] 20 000-token prompt: worst sampled max_abs={worst:.3e}", flush=True)
