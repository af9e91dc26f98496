"""Pins of the initialization-phase (prompt) attention oracle against what the paper and
the mathematics fix (Section 2.2, Figure 3: the first iteration processes all prompt
tokens; token i sees tokens 0..i)."""
import math

import numpy as np
import pytest

import oracle
from fs_workload import bf16_bits_to_f32, f32_to_bf16_bits


def rand_prompt(seed, s, H, D):
    r = np.random.default_rng(seed)
    return tuple(r.standard_normal((s, H, D)) for _ in range(3))


@pytest.mark.parametrize("s,H,D", [(1, 2, 64), (19, 4, 64), (130, 3, 128), (65, 2, 32)])
def test_matches_torch_cpu_causal_sdpa_fp64(s, H, D):
    import torch
    Q, K, V = rand_prompt(300 + s, s, H, D)
    out = oracle.prefill_attention_job(Q, K, V, "f64")
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (Q, K, V))      # [1][H][s][D]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)


def test_row_i_is_the_decode_attention_over_the_first_i_plus_1_tokens():
    # the prompt phase gives every token what a decode step would give it with the cache
    # cut after that token
    s, H, D = 37, 3, 16
    Q, K, V = rand_prompt(5, s, H, D)
    out = oracle.prefill_attention_job(Q, K, V, "f64")
    for i in range(s):
        ref = oracle.attention_job(np.ascontiguousarray(Q[i]), K, V, "f64", length=i + 1)
        np.testing.assert_allclose(out[i], ref, rtol=0, atol=1e-14)


def test_first_token_returns_its_own_value_exactly():
    Q, K, V = rand_prompt(6, 9, 2, 8)
    out = oracle.prefill_attention_job(Q, K, V, "f64")
    assert np.array_equal(out[0], V[0])


def test_hand_computed_two_tokens():
    # D = 1, scale 1: token 1 sees keys (0, ln 3) with query 1 -> weights 1/4, 3/4
    Q = np.array([[[5.0]], [[1.0]]])
    K = np.array([[[0.0]], [[math.log(3.0)]]])
    V = np.array([[[4.0]], [[8.0]]])
    out = oracle.prefill_attention_job(Q, K, V, "f64", scale=1.0)
    assert out[0, 0, 0] == 4.0
    np.testing.assert_allclose(out[1, 0, 0], 0.25 * 4.0 + 0.75 * 8.0, rtol=1e-15)


def test_later_tokens_do_not_change_earlier_rows():
    s, H, D = 24, 2, 8
    Q, K, V = rand_prompt(7, s, H, D)
    a = oracle.prefill_attention_job(Q, K, V, "f64")
    Q2, K2, V2 = Q.copy(), K.copy(), V.copy()
    Q2[10:], K2[10:], V2[10:] = 3.0, -7.0, 11.0
    b = oracle.prefill_attention_job(Q2, K2, V2, "f64")
    assert np.array_equal(a[:10], b[:10])
    assert not np.array_equal(a[10:], b[10:])


def test_a_prefix_of_the_prompt_gives_the_prefix_of_the_output():
    Q, K, V = rand_prompt(8, 30, 2, 8)
    a = oracle.prefill_attention_job(Q, K, V, "f64")
    b = oracle.prefill_attention_job(np.ascontiguousarray(Q[:13]), np.ascontiguousarray(K[:13]),
                                     np.ascontiguousarray(V[:13]), "f64")
    assert np.array_equal(a[:13], b)


def test_identical_keys_give_running_means_of_the_values():
    s, H, D = 12, 2, 4
    Q, K, V = rand_prompt(9, s, H, D)
    K[:] = K[0]
    out = oracle.prefill_attention_job(Q, K, V, "f64")
    want = np.cumsum(V, axis=0) / np.arange(1, s + 1)[:, None, None]
    np.testing.assert_allclose(out, want, rtol=1e-13, atol=1e-14)


def test_default_scale_is_inverse_sqrt_head_dim():
    Q, K, V = rand_prompt(10, 6, 1, 16)
    a = oracle.prefill_attention_job(Q, K, V, "f64")
    b = oracle.prefill_attention_job(Q, K, V, "f64", scale=0.25)
    assert np.array_equal(a, b)
    c = oracle.prefill_attention_job(Q, K, V, "f64", scale=1.0)
    assert not np.allclose(a[1:], c[1:])


def test_heads_are_independent():
    Q, K, V = rand_prompt(11, 8, 3, 8)
    a = oracle.prefill_attention_job(Q, K, V, "f64")
    for h in range(3):
        one = oracle.prefill_attention_job(np.ascontiguousarray(Q[:, h:h + 1]), np.ascontiguousarray(K[:, h:h + 1]),
                                           np.ascontiguousarray(V[:, h:h + 1]), "f64")
        assert np.array_equal(a[:, h:h + 1], one)
    part = oracle.prefill_attention_job(Q, K, V, "f64", heads=(1, 2))
    assert np.array_equal(part[:, 1], a[:, 1]) and not part[:, 0].any() and not part[:, 2].any()


def test_empty_prompt_gives_an_empty_result():
    e = np.zeros((0, 2, 8))
    assert oracle.prefill_attention_job(e, e, e, "f64").shape == (0, 2, 8)


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_stored_types_widen_exactly(dtype):
    Q, K, V = rand_prompt(12, 21, 2, 16)
    if dtype == "bf16":
        st = [f32_to_bf16_bits(a.astype(np.float32)) for a in (Q, K, V)]
        wd = [bf16_bits_to_f32(a).astype(np.float64) for a in st]
    elif dtype == "f16":
        st = [a.astype(np.float16).view(np.uint16) for a in (Q, K, V)]
        wd = [a.view(np.float16).astype(np.float64) for a in st]
    else:
        st = [a.astype(np.float32) for a in (Q, K, V)]
        wd = [a.astype(np.float64) for a in st]
    assert np.array_equal(oracle.prefill_attention_job(*st, dtype), oracle.prefill_attention_job(*wd, "f64"))
