"""fs_decode_attention_static (the entry point that allocates nothing: its partial results and
plan live in a fixed device array of the library) against fs_decode_attention on the same
inputs, through the C ABI: two calls in a row, the second on a smaller batch, so that what
the first call left in the shared array is still there when the second runs."""
import numpy as np
import pytest
import torch

import fs_workload as wl
from tests import harness as hs

pytestmark = pytest.mark.gpu


def _both(run, fs):
    lens_max = int(run.case.step.lens.max(initial=0))
    ref = run.attention(max_len_hint=lens_max).copy()
    out = torch.full_like(run.out, float("nan"))
    fs.fs_decode_attention_static(run.q, run.pool, run.table, run.lens, out, max_len_hint=lens_max)
    torch.cuda.synchronize()
    run.pool.check()
    return ref, out.cpu().numpy()


def test_static_scratch_entry_point_matches_the_allocating_one_twice_in_a_row():
    import paper_2305_05920_amd as fs
    big = wl.CONFIGS[3].scaled(num_jobs=48)                      # long and short jobs: many cut pairs
    small = wl.CONFIGS[1].scaled(num_jobs=5, num_heads=8)        # fewer jobs, fewer heads, other lengths
    for n, cfg in enumerate((big, small)):
        print(f"[case] static scratch call {n}: {cfg.name} J={cfg.num_jobs} H={cfg.num_heads}", flush=True)
        case = hs.make_case(cfg, n)
        run = hs.DeviceRun(case, fill="image")
        try:
            run.append()
            ref, got = _both(run, fs)
        finally:
            run.close()
        # same kernels, same grid, same order of sums: the same bits
        assert np.array_equal(ref.view(np.uint32), got.view(np.uint32)), f"call {n}: differs from fs_decode_attention"
        hs.assert_parity(got, hs.oracle_step(case), f"static scratch call {n}")


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import paper_2305_05920_amd as fs
    cfg = wl.CONFIGS[0]
    with fs.Pool(cfg.dtype, cfg.num_heads, cfg.head_dim, 16) as pool:
        J = 1025                                                  # one job more than the array is sized for
        q = torch.zeros((J, cfg.num_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
        out = torch.zeros_like(q)
        table = torch.zeros((J, 1), dtype=torch.int32, device="cuda")
        lens = torch.zeros(J, dtype=torch.int32, device="cuda")
        with pytest.raises(fs.FsError) as e:
            fs.fs_decode_attention_static(q, pool, table, lens, out)
        assert e.value.status == fs.FS_ERR_INVALID_ARG
        fs.fs_decode_attention(q, pool, table, lens, out)         # the allocating entry point slices such a batch
        torch.cuda.synchronize()
        pool.check()
