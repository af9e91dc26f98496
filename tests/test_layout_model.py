"""The pool layout model: a bijection inside a block, the stated formulas, and
the paper's cache-size closed form (Section 4.2) and model shapes (Table 1)."""
import os

import numpy as np
import pytest

from oracle.layout_model import PoolLayout, kv_bytes_per_job

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


@pytest.mark.parametrize("H,D,B,e", [(8, 64, 16, 4), (40, 128, 16, 2), (12, 128, 16, 2), (3, 64, 16, 2)])
def test_offsets_tile_the_block_exactly_once(H, D, B, e):
    lay = PoolLayout(H, D, B, e)
    k, v = lay.token_offsets()
    allo = np.concatenate([k.ravel(), v.ravel()])
    assert np.array_equal(np.sort(allo), np.arange(lay.block_elems))
    assert lay.block_bytes == 2 * H * B * D * e


def test_stated_formulas_on_hand_picked_elements():
    lay = PoolLayout(40, 128, 16, 2)          # x = 8 elements per 16 bytes
    assert lay.k_offset(0, 0, 0) == 0
    assert lay.k_offset(0, 1, 0) == 8          # next slot: next 16-byte vector
    assert lay.k_offset(0, 0, 8) == 16 * 8     # next dim group: 16 slots further
    assert lay.k_offset(1, 0, 0) == 16 * 128   # next head: one 4 KiB chunk
    assert lay.k_offset(2, 5, 77) == ((2 * 16 + 9) * 16 + 5) * 8 + 5
    assert lay.v_offset(0, 0, 0) == 40 * 16 * 128
    assert lay.v_offset(2, 5, 77) == 40 * 16 * 128 + (2 * 16 + 5) * 128 + 77
    # one (block, head) chunk of K or V is a whole 4 KiB
    assert (lay.k_offset(1, 0, 0) - lay.k_offset(0, 0, 0)) * 2 == 4096


def test_write_then_read_round_trips_and_touches_nothing_else():
    lay = PoolLayout(3, 64, 16, 2)
    rng = np.random.default_rng(0)
    image = np.full((10, lay.block_elems), 0xABCD, dtype=np.uint16)
    table = np.array([7, 2, 9, -1], dtype=np.int32)
    K = rng.integers(0, 0xABCD, size=(37, 3, 64)).astype(np.uint16)
    V = rng.integers(0, 0xABCD, size=(37, 3, 64)).astype(np.uint16)
    lay.write_tokens(image, table, 0, K, V)
    k2, v2 = lay.read_tokens(image, table, 0, 37)
    assert np.array_equal(k2, K) and np.array_equal(v2, V)
    assert (image[[0, 1, 3, 4, 5, 6, 8]] == 0xABCD).all()        # blocks not in the table
    written = (image != 0xABCD).sum()
    assert written <= 2 * 37 * 3 * 64                             # only token cells
    with pytest.raises(ValueError):
        lay.write_tokens(image, table, 40, K[:10], V[:10])        # runs into the -1 entry


def test_cache_bytes_closed_form_matches_the_papers_worked_example():
    (l, h, s, t, quoted), = rows("kv_bytes.txt")
    n = kv_bytes_per_job(int(l), int(h), int(s), int(t))
    assert n == 4 * 96 * 12288 * 513 == 2420637696
    # the paper's "2.3 GB" is this number in binary gigabytes, rounded
    assert round(n / 2 ** 30, 1) == float(quoted)
    # the same count, from the pool layout: per layer, a token costs block_bytes/B over all heads
    lay = PoolLayout(96, 128, 16, 2)
    assert lay.block_bytes // 16 * 96 * 513 == n


def test_model_shapes_give_head_dim_128():
    for name, layers, heads, hidden in rows("opt_shapes.txt"):
        assert int(hidden) % int(heads) == 0 and int(hidden) // int(heads) == 128, name
