"""GPU tests of the single-launch form of decode attention (pool knob ``merge_in_kernel``):
the attention kernel itself merges the (job, head) pairs whose cache was cut across waves,
instead of a combine launch.  Checked against the CPU oracle (max-abs <= 1e-2, relative
L2 <= 5e-3) and, bit for bit, against the two-launch form: the merge is the same arithmetic
in the same order whichever wave performs it."""
import os

import numpy as np
import pytest
import torch

import fs_workload as wl
from tests import harness as hs

pytestmark = pytest.mark.gpu


def both_forms(case, fused, repeats=3, **pool_kw):
    """Output of the two-launch form, then `repeats` outputs of the single-launch form from
    the same pool (the per-pair counters must be back at zero after every call)."""
    run = hs.DeviceRun(case, **pool_kw)
    hint = int(case.step.lens.max(initial=0))
    try:
        if not fused:
            run.append()
        step = (lambda: run.fused_step(max_len_hint=hint)) if fused else (lambda: run.attention(max_len_hint=hint))
        # (the fused step rewrites the appended rows with the same bytes on every call)
        plain = step()
        run.pool.set_param("merge_in_kernel", 1)
        assert run.pool.get_param("merge_in_kernel") == 1
        merged = []
        for _ in range(repeats):
            run.out.fill_(float("nan"))
            merged.append(step())
        run.pool.check()
    finally:
        run.close()
    return plain, merged


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


@pytest.mark.parametrize("idx,fused", [(0, False), (1, False), (1, True), (2, False), (2, True), (3, False), (3, True)])
def test_presets_single_launch_equals_two_launch_and_oracle(idx, fused):
    cfg = wl.CONFIGS[idx]
    print(f"[case] merge in kernel: preset {cfg.name} fused={fused}", flush=True)
    case = hs.make_case(cfg, 0)
    plain, merged = both_forms(case, fused)
    for m in merged:
        assert np.array_equal(bits(m), bits(plain))
    hs.assert_parity(merged[-1], hs.oracle_step(case), f"{cfg.name} merged fused={fused}")


def test_long_context_pairs_cut_many_times():
    # few (job, head) pairs, each spread over several waves: every pair is merged in the kernel
    cfg = wl.CONFIGS[4].scaled(num_jobs=2, num_heads=6)
    print(f"[case] merge in kernel: {cfg.name} reduced to 2 jobs x 6 heads", flush=True)
    case = hs.make_case(cfg, 0)
    plain, merged = both_forms(case, False, repeats=2)
    for m in merged:
        assert np.array_equal(bits(m), bits(plain))
    hs.assert_parity(merged[-1], hs.oracle_step(case), "long context merged")


EDGE_LENS = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1000]


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128), ("f16", 128), ("f16", 64)])
@pytest.mark.parametrize("fused", [False, True])
def test_block_and_step_boundaries(dtype, D, fused):
    cfg = wl.CONFIGS[1].scaled(num_jobs=len(EDGE_LENS), num_heads=5, head_dim=D, dtype=dtype, max_len=1024)
    case = hs.make_case(cfg, 0, lens=EDGE_LENS)
    plain, merged = both_forms(case, fused, repeats=2)
    for m in merged:
        assert np.array_equal(bits(m), bits(plain))
    hs.assert_parity(merged[-1], hs.oracle_step(case), f"edges merged {dtype} D={D} fused={fused}")


@pytest.mark.parametrize("wgs", [1, 2, 7, 33, 0])
def test_any_grid_size(wgs):
    # one workgroup: four waves, nearly every pair whole; the full grid on this small batch:
    # more waves than 64-token steps, every step of a pair in a wave of its own
    cfg = wl.CONFIGS[3].scaled(num_jobs=9, num_heads=4)
    case = hs.make_case(cfg, 2, lens=[64, 65, 640, 641, 2048, 2047, 1, 1537, 300])
    for fused in (False, True):
        plain, merged = both_forms(case, fused, max_workgroups=wgs)
        for m in merged:
            assert np.array_equal(bits(m), bits(plain))
        hs.assert_parity(merged[-1], hs.oracle_step(case), f"merged max_workgroups={wgs} fused={fused}")


def test_jobs_without_tokens_get_their_zeros_from_the_attention_kernel():
    cfg = wl.CONFIGS[1].scaled(num_jobs=6, num_heads=3)
    case = hs.make_case(cfg, 0, lens=[0, 40, 0, 700, 0, 0])
    import paper_2305_05920_amd as fs
    img = hs.expected_image(case, case.step.tables.table, case.step.tables.num_blocks, upto="append")
    mem = hs.to_torch(cfg.dtype, img)
    with fs.Pool(cfg.dtype, cfg.num_heads, cfg.head_dim, case.step.tables.num_blocks, device_mem=mem) as pool:
        pool.set_param("merge_in_kernel", 1)
        out = torch.full((6, 3, 128), float("nan"), dtype=torch.float32, device="cuda")
        q = hs.to_torch(cfg.dtype, case.step.q)
        table = torch.from_numpy(case.step.tables.table).cuda()
        fs.fs_decode_attention(q, pool, table, torch.from_numpy(case.step.lens).cuda(), out)
        pool.check()
        got = out.cpu().numpy()
        for j in (0, 2, 4, 5):
            assert not got[j].any()
        hs.assert_parity(got, hs.oracle_step(case), "empty jobs, merged")
        # every job empty: nothing but the zeros
        out.fill_(float("nan"))
        fs.fs_decode_attention(q, pool, table, torch.zeros(6, dtype=torch.int32, device="cuda"), out)
        pool.check()
        assert not out.cpu().numpy().any()
        with pytest.raises(fs.FsError):
            pool.set_param("merge_in_kernel", 2)


def test_more_jobs_than_one_launch_slice():
    # three slices of the batch share the scratch and the counters, one after the other
    cfg = wl.CONFIGS[2].scaled(num_jobs=20, num_heads=3)
    case = hs.make_case(cfg, 0)
    plain, merged = both_forms(case, False, max_jobs=8, max_workgroups=3)
    for m in merged:
        assert np.array_equal(bits(m), bits(plain))
    hs.assert_parity(merged[-1], hs.oracle_step(case), "sliced batch, merged")


@pytest.mark.parametrize("seed", range(int(os.environ.get("FS_RANDOM_SEEDS", "6"))))
def test_random_batches(seed):
    rng = np.random.default_rng(7000 + seed)
    D = int(rng.choice([64, 128]))
    dtype = str(rng.choice(["bf16", "f32", "f16"]))
    H = int(rng.integers(1, 9))
    J = int(rng.integers(1, 40))
    mix = rng.choice(["short", "long", "mixed"])
    hi = {"short": 80, "long": 1500, "mixed": 700}[mix]
    lens = rng.integers(1, hi, size=J)
    if mix == "mixed":
        lens = np.where(rng.random(J) < 0.5, rng.integers(1, 20, size=J), lens)
    cfg = wl.CONFIGS[1].scaled(num_jobs=J, num_heads=H, head_dim=D, dtype=dtype, max_len=1536)
    case = hs.make_case(cfg, seed, lens=lens)
    wgs = int(rng.choice([0, 1, 3, 17, 200]))
    print(f"[case] merged random seed {seed}: J={J} H={H} D={D} {dtype} mix={mix} max_workgroups={wgs}", flush=True)
    ref = hs.oracle_step(case)
    for fused in (False, True):
        plain, merged = both_forms(case, fused, repeats=2, max_workgroups=wgs)
        for m in merged:
            assert np.array_equal(bits(m), bits(plain))
        hs.assert_parity(merged[-1], ref, f"merged random {seed} fused={fused}")


def test_graph_replays_match_the_eager_result():
    # the counters are set back by the kernel itself (no memset node): replays of a captured
    # call, with eager calls on the same pool between them, give the eager bits every time
    cfg = wl.CONFIGS[1].scaled(num_jobs=12, num_heads=8)
    case = hs.make_case(cfg, 1)
    import paper_2305_05920_amd as fs
    run = hs.DeviceRun(case)
    try:
        run.append()
        run.pool.set_param("merge_in_kernel", 1)
        eager = run.attention()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                      # warm-up outside capture
            fs.fs_decode_attention(run.q, run.pool, run.table, run.lens, run.out)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fs.fs_decode_attention(run.q, run.pool, run.table, run.lens, run.out)
        for i in range(4):
            run.out.fill_(float("nan"))
            g.replay()
            torch.cuda.synchronize()
            assert np.array_equal(bits(run.out.cpu().numpy()), bits(eager)), f"replay {i}"
            assert np.array_equal(bits(run.attention()), bits(eager))
        run.pool.check()
    finally:
        run.close()
    hs.assert_parity(eager, hs.oracle_step(case), "merged, graph")
