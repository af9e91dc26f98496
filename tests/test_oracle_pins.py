"""Pins of the CPU oracle against things other than itself.

The paper (Section 2.2) names the operator -- masked self-attention of the one
new token over the job's cached keys and values -- and prints no formula and no
worked numbers for it, so the pins are: values computed by hand, closed forms,
invariants of softmax attention, a stock library routine (PyTorch CPU
scaled_dot_product_attention in fp64), and a brute-force evaluation without
max-subtraction in extended precision.  Each is chosen so that a plausible slip
in the oracle (dropped scale, wrong sign, swapped K/V, transposed head/dim
index, off-by-one length, missing normalisation) fails at least one.
"""
import math

import numpy as np
import pytest

import oracle
from fs_workload import bf16_bits_to_f32, f32_to_bf16_bits


def rng(seed):
    return np.random.default_rng(seed)


def rand_job(seed, L, H, D):
    r = rng(seed)
    return (r.standard_normal((H, D)), r.standard_normal((L, H, D)), r.standard_normal((L, H, D)))


# ---- values worked by hand -------------------------------------------------
def test_hand_computed_two_tokens():
    # D=4, q=(1,1,1,1), k0=(2,0,0,0), k1=0: s0 = 2/sqrt(4) = 1, s1 = 0
    # w0 = e/(1+e) = 0.7310585786300049, out = w0*v0 + (1-w0)*v1
    q = np.ones((1, 4))
    K = np.zeros((2, 1, 4)); K[0, 0, 0] = 2.0
    V = np.zeros((2, 1, 4)); V[0, 0] = [1, 2, 3, 4]; V[1, 0] = [-1, 0, 1, 2]
    out, w = oracle.attention_job(q, K, V, "f64", want_weights=True)
    w0 = 0.7310585786300049
    assert abs(w[0, 0] - w0) < 1e-15 and abs(w[0, 1] - (1 - w0)) < 1e-15
    np.testing.assert_allclose(out[0], w0 * V[0, 0] + (1 - w0) * V[1, 0], rtol=0, atol=1e-15)


def test_default_scale_is_inverse_sqrt_head_dim():
    # D=64: one key equal to q = all ones gives s = 64/8 = 8; the other key is zero.
    q = np.ones((1, 64))
    K = np.zeros((2, 1, 64)); K[1, 0] = 1.0
    V = np.zeros((2, 1, 64)); V[1, 0] = 1.0
    out = oracle.attention_job(q, K, V, "f64")
    w1 = 1.0 / (1.0 + math.exp(-8.0))
    np.testing.assert_allclose(out[0], w1, rtol=1e-15)
    # explicit scale overrides it
    out2 = oracle.attention_job(q, K, V, "f64", scale=1.0 / 64)
    np.testing.assert_allclose(out2[0], 1.0 / (1.0 + math.exp(-1.0)), rtol=1e-15)


# ---- invariants ------------------------------------------------------------
def test_single_token_cache_returns_its_value_exactly():
    q, K, V = rand_job(1, 1, 3, 8)
    out = oracle.attention_job(q, K, V, "f64")
    assert np.array_equal(out, V[0])


def test_identical_keys_give_mean_of_values():
    q, K, V = rand_job(2, 37, 3, 8)
    K[:] = K[0]
    out = oracle.attention_job(q, K, V, "f64")
    np.testing.assert_allclose(out, V.mean(axis=0), rtol=0, atol=1e-14)


def test_zero_query_gives_mean_of_values():
    q, K, V = rand_job(3, 21, 2, 16)
    out = oracle.attention_job(np.zeros_like(q), K, V, "f64")
    np.testing.assert_allclose(out, V.mean(axis=0), rtol=0, atol=1e-14)


def test_weights_sum_to_one_and_are_positive():
    q, K, V = rand_job(4, 100, 4, 16)
    _, w = oracle.attention_job(q, K, V, "f64", want_weights=True)
    assert w.shape == (4, 100)
    assert (w > 0).all()
    np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=0, atol=1e-14)


def test_permuting_cache_positions_leaves_output_unchanged():
    q, K, V = rand_job(5, 50, 3, 8)
    p = rng(55).permutation(50)
    a = oracle.attention_job(q, K, V, "f64")
    b = oracle.attention_job(q, np.ascontiguousarray(K[p]), np.ascontiguousarray(V[p]), "f64")
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)


def test_shifting_every_key_leaves_output_unchanged():
    q, K, V = rand_job(6, 40, 3, 8)
    u = rng(66).standard_normal((3, 8))
    a = oracle.attention_job(q, K, V, "f64")
    b = oracle.attention_job(q, K + u[None], V, "f64")
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)


def test_duplicating_the_cache_leaves_output_unchanged():
    q, K, V = rand_job(7, 33, 2, 8)
    a = oracle.attention_job(q, K, V, "f64")
    b = oracle.attention_job(q, np.concatenate([K, K]), np.concatenate([V, V]), "f64")
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)


def test_output_is_inside_convex_hull_of_values():
    q, K, V = rand_job(8, 64, 3, 8)
    out = oracle.attention_job(q, K, V, "f64")
    assert (out <= V.max(axis=0) + 1e-15).all() and (out >= V.min(axis=0) - 1e-15).all()


def test_identical_values_are_returned():
    q, K, V = rand_job(9, 29, 3, 8)
    V[:] = V[0]
    out = oracle.attention_job(q, K, V, "f64")
    np.testing.assert_allclose(out, V[0], rtol=0, atol=1e-14)


def test_heads_are_independent_and_indexed_head_major():
    # Only head 1 has a key matching q strongly at token 5; H, D, L all differ so a
    # transposed index would read the wrong element or run out of bounds of the pattern.
    H, D, L = 3, 8, 11
    q = np.zeros((H, D)); q[1, 2] = 40.0
    K = np.zeros((L, H, D)); K[5, 1, 2] = 40.0
    V = rng(10).standard_normal((L, H, D))
    out, w = oracle.attention_job(q, K, V, "f64", want_weights=True)
    assert w[1, 5] > 1 - 1e-12                       # 1600/sqrt(8) dominates
    np.testing.assert_allclose(out[1], V[5, 1], atol=1e-10)
    np.testing.assert_allclose(out[0], V[:, 0].mean(axis=0), atol=1e-14)   # untouched heads: uniform
    np.testing.assert_allclose(out[2], V[:, 2].mean(axis=0), atol=1e-14)


def test_head_range_only_writes_requested_rows():
    q, K, V = rand_job(11, 20, 4, 8)
    full = oracle.attention_job(q, K, V, "f64")
    part = oracle.attention_job(q, K, V, "f64", heads=(1, 3))
    assert np.array_equal(part[1:3], full[1:3]) and not part[0].any() and not part[3].any()


def test_empty_cache_gives_zeros():
    q = rng(12).standard_normal((2, 8))
    out = oracle.attention_job(q, np.zeros((0, 2, 8)), np.zeros((0, 2, 8)), "f64")
    assert out.shape == (2, 8) and not out.any()


# ---- closed form -----------------------------------------------------------
def test_two_token_cache_is_a_logistic_blend():
    q, K, V = rand_job(13, 2, 5, 16)
    out = oracle.attention_job(q, K, V, "f64")
    s = np.einsum("hd,thd->th", q, K) / math.sqrt(16)
    sig = 1.0 / (1.0 + np.exp(-(s[0] - s[1])))
    want = sig[:, None] * V[0] + (1 - sig)[:, None] * V[1]
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-14)


# ---- library routine -------------------------------------------------------
@pytest.mark.parametrize("L,H,D", [(1, 2, 64), (17, 8, 64), (130, 5, 128), (257, 3, 32)])
def test_matches_torch_cpu_sdpa_fp64(L, H, D):
    import torch
    q, K, V = rand_job(100 + L, L, H, D)
    out = oracle.attention_job(q, K, V, "f64")
    tq = torch.from_numpy(q)[None, :, None, :]                    # [1][H][1][D]
    tk = torch.from_numpy(K).permute(1, 0, 2)[None]               # [1][H][L][D]
    tv = torch.from_numpy(V).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)


# ---- brute force -----------------------------------------------------------
def test_matches_unnormalised_brute_force_in_extended_precision():
    H, D, L = 2, 8, 23
    q, K, V = rand_job(14, L, H, D)
    out = oracle.attention_job(q, K, V, "f64")
    ld = np.longdouble
    for h in range(H):
        num = np.zeros(D, dtype=ld)
        den = ld(0)
        for t in range(L):
            s = ld(0)
            for d in range(D):
                s += ld(q[h, d]) * ld(K[t, h, d])
            e = np.exp(s / np.sqrt(ld(D)))            # no max subtraction: small scores
            den += e
            for d in range(D):
                num[d] += e * ld(V[t, h, d])
        np.testing.assert_allclose(out[h], (num / den).astype(np.float64), rtol=0, atol=1e-14)


def test_large_scores_do_not_overflow():
    # scores near 1e4 would overflow exp() without the max subtraction
    q = np.full((1, 4), 100.0)
    K = np.zeros((3, 1, 4)); K[0] = 50.0; K[1] = 50.0; K[2] = 49.0
    V = np.array([[[1.0] * 4], [[3.0] * 4], [[100.0] * 4]])
    out = oracle.attention_job(q, K, V, "f64")
    e = math.exp(-200.0)                              # (49-50)*100*4/2
    np.testing.assert_allclose(out[0], (1 + 3 + 100 * e) / (2 + e), rtol=1e-15)


# ---- storage types widen exactly ------------------------------------------
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_stored_types_widen_exactly(dtype):
    H, D, L = 4, 64, 45
    q, K, V = rand_job(15, L, H, D)
    if dtype == "bf16":
        sq, sK, sV = (f32_to_bf16_bits(a.astype(np.float32)) for a in (q, K, V))
        wq, wK, wV = (bf16_bits_to_f32(a).astype(np.float64) for a in (sq, sK, sV))
    elif dtype == "f16":
        sq, sK, sV = (a.astype(np.float16).view(np.uint16) for a in (q, K, V))
        wq, wK, wV = (a.view(np.float16).astype(np.float64) for a in (sq, sK, sV))
    else:
        sq, sK, sV = (a.astype(np.float32) for a in (q, K, V))
        wq, wK, wV = (a.astype(np.float64) for a in (sq, sK, sV))
    a = oracle.attention_job(sq, sK, sV, dtype)
    b = oracle.attention_job(wq, wK, wV, "f64")
    assert np.array_equal(a, b)


def test_every_finite_half_bit_pattern_widens_to_its_ieee_value():
    # a one-token cache returns its value row (weight exactly 1): all 63488 finite binary16
    # patterns, subnormals included, against numpy's float16
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    finite = (bits & 0x7C00) != 0x7C00
    bits = np.where(finite, bits, 0).astype(np.uint16)
    V = bits.reshape(1, 512, 128)
    K = np.zeros_like(V)
    q = np.zeros((512, 128), dtype=np.uint16)
    out = oracle.attention_job(q, K, V, "f16")
    want = bits.view(np.float16).astype(np.float64).reshape(512, 128)
    assert np.array_equal(out, want)
    nz = want != 0                     # a sum that starts at +0 does not keep the sign of -0
    assert np.array_equal(np.signbit(out[nz]), np.signbit(want[nz]))
    # and the known corner values of the format
    corner = np.array([0x0001, 0x03FF, 0x0400, 0x3C00, 0x7BFF, 0xC000], dtype=np.uint16)
    Vc = np.zeros((1, 1, 6), dtype=np.uint16); Vc[0, 0] = corner
    oc = oracle.attention_job(np.zeros((1, 6), np.uint16), np.zeros_like(Vc), Vc, "f16")
    assert oc[0].tolist() == [2.0 ** -24, 1023 * 2.0 ** -24, 2.0 ** -14, 1.0, 65504.0, -2.0]


def test_bf16_rounding_helper_is_round_to_nearest_even():
    # 1 + 2^-8 is a tie between bf16 1.0 (even) and 1.0078125: goes to 1.0;
    # 1 + 3*2^-8 is a tie between 1.0078125 (odd) and 1.015625 (even): goes up.
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5], dtype=np.float32)
    got = bf16_bits_to_f32(f32_to_bf16_bits(x))
    assert got.tolist() == [1.0, 1.015625, 1.0078125, -2.5]


# ---- append and whole step -------------------------------------------------
def test_append_is_a_bit_copy_into_row_L():
    H, D = 3, 8
    r = rng(16)
    caches = oracle.LogicalCaches("bf16", H, D)
    lens = [0, 5, 16]
    olds = []
    for L in lens:
        K = r.integers(0, 65536, size=(L, H, D)).astype(np.uint16)
        V = r.integers(0, 65536, size=(L, H, D)).astype(np.uint16)
        caches.add_job(K, V)
        olds.append((K, V))
    k_new = r.integers(0, 65536, size=(3, H, D)).astype(np.uint16)   # any bit pattern, NaNs included
    v_new = r.integers(0, 65536, size=(3, H, D)).astype(np.uint16)
    caches.append(k_new, v_new)
    for j, L in enumerate(lens):
        assert caches.lens[j] == L + 1
        assert np.array_equal(caches.K[j][:L], olds[j][0]) and np.array_equal(caches.V[j][:L], olds[j][1])
        assert np.array_equal(caches.K[j][L], k_new[j]) and np.array_equal(caches.V[j][L], v_new[j])


def test_new_token_attends_to_itself():
    # empty cache before the step: after append the only token is the new one
    H, D = 2, 8
    r = rng(17)
    caches = oracle.LogicalCaches("f32", H, D)
    caches.add_job(np.zeros((0, H, D), np.float32), np.zeros((0, H, D), np.float32))
    k_new = r.standard_normal((1, H, D)).astype(np.float32)
    v_new = r.standard_normal((1, H, D)).astype(np.float32)
    q = r.standard_normal((1, H, D)).astype(np.float32)
    out = caches.decode_step(k_new, v_new, q)
    assert np.array_equal(out[0], v_new[0].astype(np.float64))


def test_decode_step_equals_append_then_attention():
    H, D = 3, 16
    r = rng(18)
    a = oracle.LogicalCaches("f32", H, D)
    b = oracle.LogicalCaches("f32", H, D)
    for L in (4, 0, 31):
        K = r.standard_normal((L, H, D)).astype(np.float32)
        V = r.standard_normal((L, H, D)).astype(np.float32)
        a.add_job(K, V), b.add_job(K, V)
    k_new, v_new, q = (r.standard_normal((3, H, D)).astype(np.float32) for _ in range(3))
    out_a = a.decode_step(k_new, v_new, q)
    b.append(k_new, v_new)
    out_b = b.attention(q)
    assert np.array_equal(out_a, out_b)
    assert a.lens == b.lens == [5, 1, 32]
