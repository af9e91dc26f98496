"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle
(attention: max-abs <= 1e-2, relative L2 <= 5e-3) and the layout model (placement, bit-exact)."""
import os

import numpy as np
import pytest
import torch

import fs_workload as wl
import oracle
from tests import harness as hs

pytestmark = pytest.mark.gpu


def run_full_step(case, fill="image", prefix_image=None, **pool_kw):
    run = hs.DeviceRun(case, fill=fill, prefix_image=prefix_image, **pool_kw)
    try:
        run.append()
        got = run.attention(max_len_hint=int(case.step.lens.max(initial=0)))
        run.pool.check()
        img = run.image()
    finally:
        run.close()
    return got, img


# ---- whole step on the five workload presets -------------------------------------
@pytest.mark.parametrize("idx,rep", [(0, 0), (0, 1), (0, 2), (1, 0), (1, 1), (1, 2), (2, 0), (2, 1), (2, 2),
                                     (3, 0), (3, 1), (3, 2)])
def test_step_matches_oracle_and_layout(idx, rep):
    cfg = wl.CONFIGS[idx]
    print(f"[case] preset {cfg.name} rep {rep}", flush=True)
    case = hs.make_case(cfg, rep)
    bt = case.step.tables
    if rep == 0:
        # pool filled from the layout model's image; the whole pool is compared after the append
        want_img = hs.expected_image(case, bt.table, bt.num_blocks, upto="prefix")
        got, img = run_full_step(case, fill="image", prefix_image=want_img)
        hs.append_into(want_img, case, bt.table)
        assert np.array_equal(img.view(np.uint8), want_img.view(np.uint8)), "pool image differs from the layout model"
    else:
        # pool filled by the bulk-write kernel; the appended cells are read back through the model
        got, img = run_full_step(case, fill="prefill")
        lay = hs.layout_of(cfg)
        for j in range(cfg.num_jobs):
            k1, v1 = lay.read_tokens(img, bt.table[j], int(case.lens_before[j]), 1)
            assert np.array_equal(k1[0], case.k_new[j]) and np.array_equal(v1[0], case.v_new[j])
    hs.assert_parity(got, hs.oracle_step(case), f"{cfg.name} rep {rep}")


@pytest.mark.parametrize("idx,fused", [(1, False), (1, True), (2, False), (3, True)])
def test_half_precision_pool_matches_oracle_and_layout(idx, fused):
    # IEEE half storage, the precision of the paper's own runs (Section 6.1)
    cfg = wl.CONFIGS[idx].scaled(dtype="f16")
    print(f"[case] f16 preset {cfg.name} fused={fused}", flush=True)
    case = hs.make_case(cfg, 0)
    bt = case.step.tables
    want_img = hs.expected_image(case, bt.table, bt.num_blocks, upto="prefix")
    if fused:
        run = hs.DeviceRun(case, fill="image", prefix_image=want_img)
        try:
            got = run.fused_step(max_len_hint=int(case.step.lens.max()))
            run.pool.check()
            img = run.image()
        finally:
            run.close()
    else:
        got, img = run_full_step(case, fill="image", prefix_image=want_img)
    hs.append_into(want_img, case, bt.table)
    assert np.array_equal(img.view(np.uint8), want_img.view(np.uint8)), "pool image differs from the layout model"
    hs.assert_parity(got, hs.oracle_step(case), f"f16 {cfg.name}")


@pytest.mark.parametrize("rep", [0, 1, 2])
def test_long_context_reduced_job_count(rep):
    # preset 4 with 2 of its 8 jobs at a quarter of the length: same heads, same
    # kernels, several partitions per job and the combine kernel, oracle in seconds
    cfg = wl.CONFIGS[4].scaled(num_jobs=2, max_len=8192, num_heads=16)
    print(f"[case] long context reduced rep {rep}", flush=True)
    case = hs.make_case(cfg, rep)
    got, img = run_full_step(case, fill="prefill")
    want_img = hs.expected_image(case, case.step.tables.table, case.step.tables.num_blocks)
    assert np.array_equal(img.view(np.uint8), want_img.view(np.uint8))
    hs.assert_parity(got, hs.oracle_step(case), f"long_context reduced rep {rep}")


@pytest.mark.parametrize("rep", [0, 1, 2])
def test_long_context_full_size_every_row(rep):
    # preset 4 at its full size (8 jobs of 16k-32k tokens, 64 heads: ~6 GB of KV) in the
    # launch configuration bench.py times; every one of the 8 x 64 x 128 outputs is compared
    # with the oracle (one oracle call per job, the jobs on separate host threads).  Seed 0
    # also runs the fused step on the same pool: it rewrites the appended rows with the same
    # bits and must agree with the oracle as well.
    from concurrent.futures import ThreadPoolExecutor
    import paper_2305_05920_amd as fs
    cfg = wl.CONFIGS[4]
    print(f"[case] preset long_context full size rep {rep}", flush=True)
    case = hs.make_case(cfg, rep)
    bt = case.step.tables
    H, D = cfg.num_heads, cfg.head_dim
    lay = hs.layout_of(cfg)
    mem = torch.empty((bt.num_blocks, lay.block_elems), dtype=torch.bfloat16, device="cuda")
    table = torch.from_numpy(bt.table).cuda()
    lens_max = int(case.step.lens.max())
    with fs.Pool(cfg.dtype, H, D, bt.num_blocks, device_mem=mem) as pool:
        for j, (K, V) in enumerate(case.caches):          # bulk write job by job
            n = int(case.lens_before[j])
            fs.fs_kv_prefill(pool, table[j:j + 1].contiguous(), torch.zeros(1, dtype=torch.int32, device="cuda"),
                             torch.tensor([0, n], dtype=torch.int32, device="cuda"), n,
                             hs.to_torch(cfg.dtype, K[:n]), hs.to_torch(cfg.dtype, V[:n]))
            torch.cuda.synchronize()
        d_before = torch.from_numpy(case.lens_before).cuda()
        d_k, d_v, d_q = (hs.to_torch(cfg.dtype, a) for a in (case.k_new, case.v_new, case.step.q))
        fs.fs_kv_append(pool, table, d_before, d_k, d_v)
        out = torch.full((cfg.num_jobs, H, D), float("nan"), dtype=torch.float32, device="cuda")
        fs.fs_decode_attention(d_q, pool, table, torch.from_numpy(case.step.lens).cuda(), out, max_len_hint=lens_max)
        pool.check()
        got = out.cpu().numpy()
        got_fused = None
        if rep == 0:
            out.fill_(float("nan"))
            fs.fs_decode_step(pool, table, d_before, d_k, d_v, d_q, out, max_len_hint=lens_max)
            pool.check()
            got_fused = out.cpu().numpy()
        # placement: sampled blocks read back through the C ABI against the layout model
        rng = np.random.default_rng(4 + rep)
        for j in rng.choice(cfg.num_jobs, size=3, replace=False):
            K, V = case.caches[j]
            for bi in (0, int(case.step.lens[j] - 1) // 16, int(rng.integers(0, case.step.lens[j] // 16))):
                blk = pool.read_block(int(bt.table[j, bi]), np.uint16)[None]
                n = min(16, int(case.step.lens[j]) - bi * 16)
                k1, v1 = lay.read_tokens(blk, np.zeros(1, dtype=np.int32), 0, n)
                assert np.array_equal(k1, K[bi * 16:bi * 16 + n]) and np.array_equal(v1, V[bi * 16:bi * 16 + n])
    # the caches' last rows are the appended tokens: attention over the whole logical cache
    with ThreadPoolExecutor(max_workers=cfg.num_jobs) as ex:
        ref = np.stack(list(ex.map(lambda j: oracle.attention_job(case.step.q[j], *case.caches[j], cfg.dtype),
                                   range(cfg.num_jobs))))
    hs.assert_parity(got, ref, f"long_context full size rep {rep}, all {got.size} outputs")
    if got_fused is not None:
        hs.assert_parity(got_fused, ref, f"long_context full size rep {rep}, fused step")


# ---- fused step: append inside the attention kernel -------------------------------
@pytest.mark.parametrize("idx,rep,append_in_attention", [(0, 0, 0), (0, 1, 1), (1, 0, 0), (1, 0, 1), (2, 1, 0), (3, 2, 0),
                                                         (3, 2, 1)])
def test_fused_step_matches_oracle_and_layout(idx, rep, append_in_attention):
    cfg = wl.CONFIGS[idx]
    print(f"[case] fused preset {cfg.name} rep {rep} append_in_attention {append_in_attention}", flush=True)
    case = hs.make_case(cfg, rep)
    bt = case.step.tables
    want_img = hs.expected_image(case, bt.table, bt.num_blocks, upto="prefix")
    run = hs.DeviceRun(case, fill="image", prefix_image=want_img)
    try:
        run.pool.set_param("append_in_attention", append_in_attention)
        got = run.fused_step(max_len_hint=int(case.step.lens.max()))
        run.pool.check()
        img = run.image()
    finally:
        run.close()
    hs.append_into(want_img, case, bt.table)
    assert np.array_equal(img.view(np.uint8), want_img.view(np.uint8)), "pool image differs from the layout model"
    hs.assert_parity(got, hs.oracle_step(case), f"fused {cfg.name} rep {rep}")


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128), ("f16", 128), ("f16", 64)])
@pytest.mark.parametrize("append_in_attention", [0, 1])
def test_fused_step_boundaries(dtype, D, append_in_attention):
    # lengths after the append; 1 means an empty cache before the step, 65 a cache of
    # exactly one full 64-token unit, 17 a new token that opens a new block.
    # append_in_attention: the new rows are written by the launch after the attention kernel
    # (0, the default) or by the attention kernel itself (1)
    lens = [1, 2, 16, 17, 64, 65, 66, 128, 129, 1000, 1024, 1025]
    cfg = wl.CONFIGS[1].scaled(num_jobs=len(lens), num_heads=5, head_dim=D, dtype=dtype, max_len=1040)
    case = hs.make_case(cfg, 1, lens=lens)
    run = hs.DeviceRun(case, fill="image")
    try:
        run.pool.set_param("append_in_attention", append_in_attention)
        got = run.fused_step()
        run.pool.check()
        img = run.image()
    finally:
        run.close()
    want = hs.expected_image(case, case.step.tables.table, case.step.tables.num_blocks)
    assert np.array_equal(img.view(np.uint8), want.view(np.uint8))
    hs.assert_parity(got, hs.oracle_step(case), f"fused edges {dtype} D={D}")
    assert np.array_equal(got[0].astype(np.float64), wl.to_f64(dtype, case.v_new[0]))   # L = 1: its own value


def test_fused_step_agrees_with_the_two_call_form():
    cfg = wl.CONFIGS[3].scaled(num_jobs=16, num_heads=6)
    case = hs.make_case(cfg, 0)
    a = hs.DeviceRun(case)
    b = hs.DeviceRun(case)
    try:
        a.append()
        two = a.attention()
        one = b.fused_step()
        a.pool.check(), b.pool.check()
        assert np.array_equal(a.image(), b.image())
        np.testing.assert_allclose(one, two, rtol=0, atol=2e-6)
        # an empty-cache garbage guard: stale NaN bit patterns in never-written slots must not leak
        assert np.isfinite(one).all()
    finally:
        a.close(), b.close()


def test_fused_step_flags_a_full_table_row():
    import paper_2305_05920_amd as fs
    cfg = wl.CONFIGS[1].scaled(num_jobs=2, num_heads=2, max_len=64)
    case = hs.make_case(cfg, 0, lens=[40, 64], width=4)
    run = hs.DeviceRun(case)
    try:
        run.fused_step()
        run.pool.check()
        full = torch.tensor([39, 64], dtype=torch.int32, device="cuda")     # job 1: no room for a 65th token
        fs.fs_decode_step(run.pool, run.table, full, run.k_new, run.v_new, run.q, run.out)
        with pytest.raises(fs.FsError):
            run.pool.check()
    finally:
        run.close()


# ---- placement alone ---------------------------------------------------------------
@pytest.mark.parametrize("idx", [0, 1, 2])
def test_prefill_then_append_is_bit_exact_and_touches_nothing_else(idx):
    cfg = wl.CONFIGS[idx].scaled(num_jobs=min(wl.CONFIGS[idx].num_jobs, 24))
    case = hs.make_case(cfg, 1)
    run = hs.DeviceRun(case, fill="prefill")
    try:
        after_prefill = run.image()
        want = hs.expected_image(case, run.table_np, run.num_blocks, upto="prefix")
        assert np.array_equal(after_prefill.view(np.uint8), want.view(np.uint8))
        run.append()
        run.pool.check()
        want = hs.expected_image(case, run.table_np, run.num_blocks, upto="append")
        assert np.array_equal(run.image().view(np.uint8), want.view(np.uint8))
    finally:
        run.close()


def test_append_copies_any_bit_pattern():
    # NaN and infinity patterns included: the append is a copy, not arithmetic
    cfg = wl.CONFIGS[1].scaled(num_jobs=5, num_heads=3)
    case = hs.make_case(cfg, 0, lens=[1, 16, 17, 33, 100])
    rng = np.random.default_rng(5)
    case.k_new = rng.integers(0, 65536, size=case.k_new.shape).astype(np.uint16)
    case.v_new = rng.integers(0, 65536, size=case.v_new.shape).astype(np.uint16)
    for j, (K, V) in enumerate(case.caches):
        K[-1], V[-1] = case.k_new[j], case.v_new[j]
    run = hs.DeviceRun(case, fill="image")
    try:
        run.append()
        run.pool.check()
        want = hs.expected_image(case, run.table_np, run.num_blocks)
        assert np.array_equal(run.image(), want)
    finally:
        run.close()


# ---- edge cases of the attention kernels -------------------------------------------
EDGE_LENS = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1000]


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128), ("f16", 128), ("f16", 64)])
def test_block_and_step_boundaries(dtype, D):
    cfg = wl.CONFIGS[1].scaled(num_jobs=len(EDGE_LENS), num_heads=5, head_dim=D, dtype=dtype, max_len=1024)
    case = hs.make_case(cfg, 0, lens=EDGE_LENS)
    got, _ = run_full_step(case)
    ref = hs.oracle_step(case)
    hs.assert_parity(got, ref, f"edges {dtype} D={D}")
    # a one-token cache returns its value row exactly
    v0 = wl.to_f64(dtype, case.caches[0][1][0])
    assert np.array_equal(got[0].astype(np.float64), v0)


@pytest.mark.parametrize("wgs", [1, 2, 7, 33, 0])
def test_grid_size_does_not_change_the_result(wgs):
    # the batch's 64-token steps are dealt evenly to the waves of the grid: with one
    # workgroup four waves walk many (job, head) pairs each; with the full grid most
    # pairs are cut across several waves and merged by the combine pass
    cfg = wl.CONFIGS[3].scaled(num_jobs=9, num_heads=4)
    case = hs.make_case(cfg, 2, lens=[64, 65, 640, 641, 2048, 2047, 1, 1537, 300])
    got, _ = run_full_step(case, max_workgroups=wgs)
    hs.assert_parity(got, hs.oracle_step(case), f"max_workgroups={wgs}")


@pytest.mark.parametrize("wgs_per_cu", [0, 1, 2])
def test_default_and_explicit_persistent_grids_on_a_full_preset(wgs_per_cu):
    # 0: the default grid, which on a batch of this size (12 units per wave) leaves every eighth
    # workgroup idle; 1, 2: that many workgroups per compute unit, all of them working
    case = hs.make_case(wl.CONFIGS[1], 1)
    run = hs.DeviceRun(case)
    try:
        run.pool.set_param("wgs_per_cu", wgs_per_cu)
        run.append()
        got = run.attention(max_len_hint=int(case.step.lens.max()))
        run.pool.check()
    finally:
        run.close()
    hs.assert_parity(got, hs.oracle_step(case), f"wgs_per_cu={wgs_per_cu}")


def test_step_plan_is_the_prefix_sum_of_64_token_steps():
    cfg = wl.CONFIGS[3].scaled(num_jobs=9, num_heads=4)
    lens = np.array([64, 65, 640, 641, 2048, 2047, 1, 1537, 300], dtype=np.int32)
    case = hs.make_case(cfg, 2, lens=lens)
    run = hs.DeviceRun(case)
    try:
        run.append()
        run.attention()
        base = run.pool.last_plan(cfg.num_jobs)
        assert np.array_equal(base, np.concatenate([[0], np.cumsum((lens + 63) // 64)]))
    finally:
        run.close()


def test_empty_jobs_give_zero_rows():
    cfg = wl.CONFIGS[1].scaled(num_jobs=4, num_heads=3)
    case = hs.make_case(cfg, 0, lens=[0, 40, 0, 7])
    import paper_2305_05920_amd as fs
    img = hs.expected_image(case, case.step.tables.table, case.step.tables.num_blocks, upto="append")
    mem = hs.to_torch(cfg.dtype, img)
    with fs.Pool(cfg.dtype, cfg.num_heads, cfg.head_dim, case.step.tables.num_blocks, device_mem=mem) as pool:
        out = torch.full((4, 3, 128), float("nan"), dtype=torch.float32, device="cuda")
        fs.fs_decode_attention(hs.to_torch(cfg.dtype, case.step.q), pool,
                               torch.from_numpy(case.step.tables.table).cuda(),
                               torch.from_numpy(case.step.lens).cuda(), out)
        pool.check()
        got = out.cpu().numpy()
    assert not got[0].any() and not got[2].any()
    hs.assert_parity(got, hs.oracle_step(case), "empty jobs")


def test_all_jobs_empty():
    import paper_2305_05920_amd as fs
    with fs.Pool("bf16", 2, 128, 4) as pool:
        out = torch.full((3, 2, 128), float("nan"), dtype=torch.float32, device="cuda")
        q = torch.zeros((3, 2, 128), dtype=torch.bfloat16, device="cuda")
        table = torch.full((3, 2), -1, dtype=torch.int32, device="cuda")
        fs.fs_decode_attention(q, pool, table, torch.zeros(3, dtype=torch.int32, device="cuda"), out)
        pool.check()
        assert not out.cpu().numpy().any()
        # zero jobs: a no-op that must not launch anything
        fs.fs_decode_attention(q[:0], pool, table[:0], torch.zeros(0, dtype=torch.int32, device="cuda"), out[:0])
        fs.fs_kv_append(pool, table[:0], torch.zeros(0, dtype=torch.int32, device="cuda"), q[:0], q[:0])


def test_same_job_twice_in_a_batch_gives_identical_rows():
    # two table rows naming the same blocks (shared prefix read by two queries)
    cfg = wl.CONFIGS[1].scaled(num_jobs=2, num_heads=4)
    case = hs.make_case(cfg, 0, lens=[333, 50])
    import paper_2305_05920_amd as fs
    bt = case.step.tables
    img = hs.expected_image(case, bt.table, bt.num_blocks, upto="append")
    table = np.stack([bt.table[0], bt.table[1], bt.table[0]])
    lens = np.array([333, 50, 333], dtype=np.int32)
    q = np.stack([case.step.q[0], case.step.q[1], case.step.q[0]])
    with fs.Pool(cfg.dtype, 4, 128, bt.num_blocks, device_mem=hs.to_torch("bf16", img)) as pool:
        out = torch.empty((3, 4, 128), dtype=torch.float32, device="cuda")
        fs.fs_decode_attention(hs.to_torch("bf16", q), pool, torch.from_numpy(table).cuda(),
                               torch.from_numpy(lens).cuda(), out)
        pool.check()
        got = out.cpu().numpy()
    assert np.array_equal(got[0], got[2])
    hs.assert_parity(got[:2], hs.oracle_step(case), "duplicate job")


def test_more_jobs_than_one_launch_slice():
    # max_jobs=8 forces three slices of the batch through the same scratch
    cfg = wl.CONFIGS[2].scaled(num_jobs=20, num_heads=3)
    case = hs.make_case(cfg, 0)
    got, _ = run_full_step(case, max_jobs=8, max_workgroups=3)
    hs.assert_parity(got, hs.oracle_step(case), "sliced batch")


def test_fused_step_over_several_launch_slices():
    # every slice runs the attention kernel and the combine + append launch on its own jobs
    cfg = wl.CONFIGS[2].scaled(num_jobs=20, num_heads=3)
    case = hs.make_case(cfg, 1)
    run = hs.DeviceRun(case, max_jobs=8, max_workgroups=3)
    try:
        got = run.fused_step()
        run.pool.check()
        img = run.image()
    finally:
        run.close()
    want = hs.expected_image(case, case.step.tables.table, case.step.tables.num_blocks)
    assert np.array_equal(img.view(np.uint8), want.view(np.uint8))
    hs.assert_parity(got, hs.oracle_step(case), "sliced batch, fused")


def test_widest_table_of_the_long_context_preset():
    # W = 2048 table entries per job, one job at the full 32768 tokens, 2 heads
    cfg = wl.CONFIGS[4].scaled(num_jobs=1, num_heads=2)
    case = hs.make_case(cfg, 0, lens=[32768])
    assert case.step.tables.table.shape[1] == 2048
    got, _ = run_full_step(case, fill="prefill")
    hs.assert_parity(got, hs.oracle_step(case), "max length")


# ---- seeded random shapes --------------------------------------------------------------
@pytest.mark.parametrize("seed", range(int(os.environ.get("FS_RANDOM_SEEDS", "6"))))
def test_random_batches_grids_and_entry_points(seed):
    # random job counts, head counts, head_dim, dtype, length mixes (zeros included for the
    # two-call form) and grid caps; both entry points against the oracle
    rng = np.random.default_rng(1000 + seed)
    D = int(rng.choice([64, 128]))
    dtype = str(rng.choice(["bf16", "f32", "f16"]))
    H = int(rng.integers(1, 9))
    J = int(rng.integers(1, 40))
    mix = rng.choice(["short", "long", "mixed"])
    hi = {"short": 80, "long": 1500, "mixed": 700}[mix]
    lens = rng.integers(1, hi, size=J)
    if mix == "mixed":
        short = rng.random(J) < 0.5
        lens = np.where(short, rng.integers(1, 20, size=J), lens)
    cfg = wl.CONFIGS[1].scaled(num_jobs=J, num_heads=H, head_dim=D, dtype=dtype, max_len=1536)
    case = hs.make_case(cfg, seed, lens=lens)
    wgs = int(rng.choice([0, 1, 3, 17, 200]))
    print(f"[case] random seed {seed}: J={J} H={H} D={D} {dtype} mix={mix} max_workgroups={wgs}", flush=True)
    ref = hs.oracle_step(case)
    a = hs.DeviceRun(case, max_workgroups=wgs)
    b = hs.DeviceRun(case, max_workgroups=wgs)
    try:
        a.append()
        two = a.attention(max_len_hint=int(lens.max()))
        one = b.fused_step(max_len_hint=int(lens.max()))
        a.pool.check(), b.pool.check()
        assert np.array_equal(a.image().view(np.uint8), b.image().view(np.uint8))
    finally:
        a.close(), b.close()
    hs.assert_parity(two, ref, f"random {seed} two-call")
    hs.assert_parity(one, ref, f"random {seed} fused")


# ---- offload / upload ----------------------------------------------------------------
def test_offload_upload_round_trip_and_bitwise_stable_attention():
    # preset 2's recipe: a quarter of the jobs leave for host slots and return under
    # other block ids.  Blocks must arrive bit-exact, and since the work split depends
    # on lengths only, attention must be bitwise the same before and after.
    cfg = wl.CONFIGS[2].scaled(num_jobs=64)
    case = hs.make_case(cfg, 0)
    bt = case.step.tables
    sw = bt.swap
    import paper_2305_05920_amd as fs
    run = hs.DeviceRun(case, fill="image", table=bt.table_before_swap, num_host_blocks=len(sw.old_ids))
    try:
        run.append()
        before = run.attention()
        img_before = run.image().copy()
        fs.fs_pool_offload(run.pool, sw.old_ids, sw.host_slots)
        torch.cuda.synchronize()
        # scribble over the vacated blocks so that a stale read would show
        view = run.mem.view(torch.int16) if cfg.dtype == "bf16" else run.mem
        view[torch.from_numpy(sw.old_ids.astype(np.int64)).cuda()] = 0x7FC1 if cfg.dtype == "bf16" else -1.0
        fs.fs_pool_upload(run.pool, sw.host_slots, sw.new_ids)
        torch.cuda.synchronize()
        img_after = run.image()
        assert np.array_equal(img_after[sw.new_ids], img_before[sw.old_ids])
        run.table = torch.from_numpy(bt.table).cuda()
        after = run.attention()
        run.pool.check()
        assert np.array_equal(before.view(np.uint32), after.view(np.uint32))
        hs.assert_parity(after, hs.oracle_step(case), "after swap")
    finally:
        run.close()


# ---- errors are reported, not faulted on -----------------------------------------------
def test_bad_tables_and_lengths_raise_the_flag():
    import paper_2305_05920_amd as fs
    cfg = wl.CONFIGS[1].scaled(num_jobs=3, num_heads=2)
    case = hs.make_case(cfg, 0, lens=[20, 40, 60])
    run = hs.DeviceRun(case)
    try:
        run.append()
        run.attention()
        run.pool.check()
        bad = run.table.clone()
        bad[1, 0] = run.num_blocks + 5                    # block id beyond the pool
        fs.fs_decode_attention(run.q, run.pool, bad, run.lens, run.out)
        with pytest.raises(fs.FsError) as e:
            run.pool.check()
        assert e.value.status == fs.FS_ERR_BAD_TABLE
        run.pool.check()                                  # flag was cleared
        bad[1, 0] = -1
        fs.fs_kv_append(run.pool, bad, torch.zeros(3, dtype=torch.int32, device="cuda"), run.k_new, run.v_new)
        with pytest.raises(fs.FsError):
            run.pool.check()
        too_long = torch.tensor([20, 10 ** 6, 60], dtype=torch.int32, device="cuda")
        fs.fs_decode_attention(run.q, run.pool, run.table, too_long, run.out)
        with pytest.raises(fs.FsError):
            run.pool.check()
        fs.fs_kv_append(run.pool, run.table, too_long, run.k_new, run.v_new)
        with pytest.raises(fs.FsError):
            run.pool.check()
        # host-checkable mistakes are refused before any launch
        with pytest.raises(fs.FsError) as e:
            fs.fs_pool_offload(run.pool, [0], [0])        # pool has no host slots
        assert e.value.status == fs.FS_ERR_INVALID_ARG
        with pytest.raises(fs.FsError):
            run.pool.write_block(run.num_blocks, np.zeros(run.pool.block_bytes, np.uint8))
    finally:
        run.close()


def test_library_allocated_pool_and_raw_block_copies():
    import paper_2305_05920_amd as fs
    with fs.Pool("f32", 2, 64, 6, num_host_blocks=2) as pool:
        assert pool.block_bytes == 2 * 2 * 16 * 64 * 4
        rng = np.random.default_rng(0)
        a = rng.standard_normal(pool.block_bytes // 4).astype(np.float32)
        pool.write_block(3, a)
        assert np.array_equal(pool.read_block(3, np.float32), a)
        fs.fs_pool_offload(pool, [3], [1])
        fs.fs_pool_upload(pool, [1], [5])
        torch.cuda.synchronize()
        assert np.array_equal(pool.read_block(5, np.float32), a)


@pytest.mark.parametrize("engine", [0, 1])
def test_block_copies_in_rising_falling_and_broken_runs(engine):
    # pairs that step together (up or down) travel as one copy each; every block must still land
    # in the slot it was paired with, and come back into the block it is paired with
    import paper_2305_05920_amd as fs
    with fs.Pool("bf16", 3, 64, 24, num_host_blocks=16) as pool:
        pool.set_param("swap_engine", engine)
        rng = np.random.default_rng(5)
        words = pool.block_bytes // 2
        data = {b: rng.integers(0, 1 << 16, size=words, dtype=np.uint16) for b in range(24)}
        for b, a in data.items():
            pool.write_block(b, a)
        blocks = [7, 6, 5, 4, 10, 11, 12, 20, 2, 1, 15, 17, 16]   # falling, rising, single, falling, broken, falling
        slots = [9, 8, 7, 6, 0, 1, 2, 15, 4, 3, 10, 12, 11]
        fs.fs_pool_offload(pool, blocks, slots)
        torch.cuda.synchronize()
        for b in blocks:
            pool.write_block(b, np.zeros(words, dtype=np.uint16))
        back = [b + 1 if b in (20,) else b for b in blocks][::-1]    # same blocks, pairs listed the other way round
        fs.fs_pool_upload(pool, slots[::-1], back)
        torch.cuda.synchronize()
        for b_src, b_dst in zip(blocks[::-1], back):
            assert np.array_equal(pool.read_block(b_dst, np.uint16), data[b_src]), (b_src, b_dst)
        for b in set(range(24)) - set(blocks) - set(back):
            assert np.array_equal(pool.read_block(b, np.uint16), data[b])


def test_kernel_timing_records():
    cfg = wl.CONFIGS[0]
    case = hs.make_case(cfg, 0)
    run = hs.DeviceRun(case)
    try:
        run.pool.profile_enable(True)
        run.append()
        run.attention()
        run.attention()
        rec = run.pool.profile_collect()
        assert rec["append"]["launches"] == 1 and rec["attention"]["launches"] == 2
        assert rec["combine"]["launches"] == 2 and rec["attention"]["ms"] > 0
        run.pool.profile_enable(False)
        run.attention()
        assert run.pool.profile_collect()["attention"]["launches"] == 0
    finally:
        run.close()


def test_plain_read_kernel_reports_its_own_duration():
    # the measurement helper: a read of 256 MiB takes a time that a GPU's memory can deliver
    # (between 2 and 16 TB/s on any HBM part), a bad argument is refused before any launch
    import paper_2305_05920_amd as fs
    src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    fs.fs_stream_read(src, sink, 256)
    torch.cuda.synchronize()
    us = [fs.fs_stream_read_timed(src, sink, 256) for _ in range(3)]
    assert all(16.0 < t < 130.0 for t in us), us
    assert not sink.cpu().numpy().any()
    with pytest.raises(fs.FsError):
        fs.fs_stream_read_timed(src[:24], sink, 256)   # not a multiple of 16 bytes
    with pytest.raises(fs.FsError):
        fs.fs_stream_read_timed(src, sink, 0)


def test_two_pools_on_two_streams_at_once_match_their_serial_results():
    # a pool is not thread-safe, but different pools may run at the same time: the decode step of
    # two batches on two streams, launched back to back without a wait in between, ten times
    # over, must give each batch bit for bit what it gets alone
    import paper_2305_05920_amd as fs
    cases = [hs.make_case(wl.CONFIGS[1].scaled(num_jobs=12, num_heads=8), 0),
             hs.make_case(wl.CONFIGS[3].scaled(num_jobs=10, num_heads=6), 1)]
    alone = []
    for c in cases:
        run = hs.DeviceRun(c)
        try:
            run.append()
            alone.append(run.attention())
        finally:
            run.close()
    runs = [hs.DeviceRun(c) for c in cases]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    try:
        torch.cuda.synchronize()
        for rep in range(10):
            for run, st in zip(runs, streams):
                if rep == 0:
                    fs.fs_kv_append(run.pool, run.table, run.lens_before, run.k_new, run.v_new, stream=st)
                fs.fs_decode_attention(run.q, run.pool, run.table, run.lens, run.out, stream=st)
            if rep % 3 == 2:
                torch.cuda.synchronize()
                for run, want in zip(runs, alone):
                    assert np.array_equal(run.out.cpu().numpy(), want), f"repetition {rep}"
        torch.cuda.synchronize()
        for run, want in zip(runs, alone):
            run.pool.check()
            assert np.array_equal(run.out.cpu().numpy(), want)
    finally:
        for run in runs:
            run.close()


def test_graph_replays_of_both_step_forms_match_the_eager_results():
    # The step is captured into a HIP graph (as a serving loop would, to shed launch overhead) in
    # both forms and replayed several times, with eager work of the library and synchronisations
    # between the replays; every replay must reproduce the eager output bit for bit.  (The library
    # clears nothing with memset nodes: all scratch is written by its kernels before it is read.)
    import paper_2305_05920_amd as fs
    case = hs.make_case(wl.CONFIGS[1].scaled(num_jobs=10, num_heads=8), 2)
    other = hs.make_case(wl.CONFIGS[2].scaled(num_jobs=16, num_heads=4), 0)
    eager_two = hs.DeviceRun(case)
    eager_two.append()
    want_two = eager_two.attention()
    eager_two.close()
    eager_fused = hs.DeviceRun(case)
    want_fused = eager_fused.fused_step()
    eager_fused.close()
    a, b, c = hs.DeviceRun(case), hs.DeviceRun(case), hs.DeviceRun(other)
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                      # warm-up outside capture
            a.append()
            fs.fs_decode_attention(a.q, a.pool, a.table, a.lens, a.out)
            fs.fs_decode_step(b.pool, b.table, b.lens_before, b.k_new, b.v_new, b.q, b.out)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fs.fs_kv_append(a.pool, a.table, a.lens_before, a.k_new, a.v_new)
            fs.fs_decode_attention(a.q, a.pool, a.table, a.lens, a.out)
            fs.fs_decode_step(b.pool, b.table, b.lens_before, b.k_new, b.v_new, b.q, b.out)
        for rep in range(4):
            a.out.fill_(float("nan"))
            b.out.fill_(float("nan"))
            g.replay()
            torch.cuda.synchronize()
            assert np.array_equal(a.out.cpu().numpy(), want_two), f"two-call form, replay {rep}"
            assert np.array_equal(b.out.cpu().numpy(), want_fused), f"fused form, replay {rep}"
            c.append()                                     # eager work between the replays
            c.attention()
            a.pool.check(), b.pool.check(), c.pool.check()
    finally:
        a.close(), b.close(), c.close()
