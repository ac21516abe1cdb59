"""Pins for the oracle's building blocks: closed forms, invariants, library routines.

None of these re-type the oracle's own formula: each compares against a value fixed by the
mathematics (a closed form, an identity, a special case) or by an independent library routine.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import verillm_oracle as O

RNG = np.random.default_rng(12345)


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_constant_row_closed_form():
    c, eps = 3.0, 1e-5
    g = RNG.standard_normal(16)
    y = O.rmsnorm(np.full((2, 16), c), g, eps)
    np.testing.assert_allclose(y, np.broadcast_to(g * c / math.sqrt(c * c + eps), (2, 16)), rtol=1e-14)


def test_rmsnorm_output_mean_square_identity():
    x = RNG.standard_normal((5, 64)) * 2.0
    g = 1.0 + 0.1 * RNG.standard_normal(64)
    eps = 1e-5
    y = O.rmsnorm(x, g, eps)
    ms = np.mean(x * x, axis=1)
    np.testing.assert_allclose(np.mean((y / g) ** 2, axis=1), ms / (ms + eps), rtol=1e-12)


def test_rmsnorm_scale_invariance_and_eps_matters():
    x = RNG.standard_normal((3, 32))
    g = np.ones(32)
    np.testing.assert_allclose(O.rmsnorm(1000.0 * x, g, 1e-5), O.rmsnorm(x, g, 1e-5), rtol=1e-4)
    # with a huge eps the output is x / sqrt(eps) to first order: eps sits inside the square root
    y = O.rmsnorm(x, g, 1e6)
    np.testing.assert_allclose(y, x / math.sqrt(1e6), rtol=1e-5)


def test_rmsnorm_matches_torch():
    x = RNG.standard_normal((7, 48))
    g = RNG.standard_normal(48)
    ref = F.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-5).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-5), ref, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- RoPE
def test_rope_literal_values():
    # head_dim 4, base 10000: frequencies 1 and 10000^(-1/2) = 0.01.  Position 1 rotates pair (0,2) by
    # 1 rad and pair (1,3) by 0.01 rad.  cos/sin literals are textbook constants.
    x = np.array([[[1.0, 2.0, 3.0, 4.0]]])
    y = O.apply_rope(x, np.array([1]), 10000.0)[0, 0]
    c1, s1 = 0.5403023058681398, 0.8414709848078965
    c2, s2 = 0.9999500004166653, 0.009999833334166664
    np.testing.assert_allclose(y, [1 * c1 - 3 * s1, 2 * c2 - 4 * s2, 3 * c1 + 1 * s1, 4 * c2 + 2 * s2], rtol=1e-14)


def test_rope_angle_table_closed_form():
    ang = O.rope_angles(np.array([0, 3, 100]), 8, 500000.0)
    assert ang.shape == (3, 4)
    np.testing.assert_allclose(ang[0], 0.0)
    np.testing.assert_allclose(ang[1, 0], 3.0)
    np.testing.assert_allclose(ang[2, 2], 100.0 * 500000.0 ** (-0.5), rtol=1e-14)
    np.testing.assert_allclose(ang[2, 3], 100.0 / 500000.0 ** 0.75, rtol=1e-14)


def test_rope_position_zero_identity_and_norm_preserved():
    x = RNG.standard_normal((4, 3, 16))
    np.testing.assert_allclose(O.apply_rope(x, np.zeros(4, dtype=int), 10000.0), x, rtol=0, atol=0)
    y = O.apply_rope(x, np.array([5, 17, 100, 9000]), 500000.0)
    half = 8
    np.testing.assert_allclose(y[..., :half] ** 2 + y[..., half:] ** 2, x[..., :half] ** 2 + x[..., half:] ** 2,
                               rtol=1e-12)


def test_rope_relative_position_property():
    q = RNG.standard_normal((1, 1, 32))
    k = RNG.standard_normal((1, 1, 32))
    def dot(m, n):
        return float(np.sum(O.apply_rope(q, np.array([m]), 10000.0) * O.apply_rope(k, np.array([n]), 10000.0)))
    np.testing.assert_allclose(dot(37, 12), dot(25, 0), rtol=1e-11)
    np.testing.assert_allclose(dot(1000, 990), dot(10, 0), rtol=1e-10)
    assert abs(dot(37, 12) - dot(36, 12)) > 1e-6     # and it does depend on the offset


# ---------------------------------------------------------------- softmax / attention
def test_softmax_rows_sum_to_one_and_shift_invariant():
    s = RNG.standard_normal((6, 11)) * 5
    p = O.softmax_rows(s)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-14)
    assert (p >= 0).all()
    np.testing.assert_allclose(O.softmax_rows(s + 1000.0), p, rtol=1e-10)
    np.testing.assert_allclose(O.softmax_rows(np.log(np.array([[1.0, 2.0, 5.0]]))), [[0.125, 0.25, 0.625]], rtol=1e-14)


def test_attention_first_position_returns_v0_and_equal_scores_average():
    t, hq, hkv, hd = 6, 4, 2, 8
    v = RNG.standard_normal((t, hkv, hd))
    k = RNG.standard_normal((t, hkv, hd))
    q = RNG.standard_normal((t, hq, hd))
    o = O.causal_attention(q, k, v, np.arange(t))
    for j in range(hq):
        np.testing.assert_allclose(o[0, j], v[0, j // 2], rtol=1e-14)
    # all-zero queries -> equal scores -> running mean of the values
    o = O.causal_attention(np.zeros_like(q), k, v, np.arange(t))
    for i in range(t):
        for j in range(hq):
            np.testing.assert_allclose(o[i, j], v[: i + 1, j // 2].mean(axis=0), rtol=1e-13)


@pytest.mark.parametrize("hq,hkv", [(4, 4), (4, 2), (8, 1)])
def test_attention_matches_torch_sdpa(hq, hkv):
    t, hd = 13, 16
    q = RNG.standard_normal((t, hq, hd))
    k = RNG.standard_normal((t, hkv, hd))
    v = RNG.standard_normal((t, hkv, hd))
    o = O.causal_attention(q, k, v, np.arange(t))
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    # GQA pinned by replicating KV heads explicitly (head j uses kv head j // group)
    rep = hq // hkv
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(rep, dim=0)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(rep, dim=0)[None]
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(o, ref, rtol=1e-11, atol=1e-13)


def test_attention_brute_force_scalar_loops():
    t, hq, hkv, hd = 5, 2, 1, 4
    q = RNG.standard_normal((t, hq, hd))
    k = RNG.standard_normal((t, hkv, hd))
    v = RNG.standard_normal((t, hkv, hd))
    o = O.causal_attention(q, k, v, np.arange(t))
    for i in range(t):
        for j in range(hq):
            w = [math.exp(sum(q[i, j, c] * k[r, 0, c] for c in range(hd)) / math.sqrt(hd)) for r in range(i + 1)]
            z = sum(w)
            for c in range(hd):
                assert abs(o[i, j, c] - sum(w[r] * v[r, 0, c] for r in range(i + 1)) / z) < 1e-12


def test_attention_single_query_against_cache_equals_last_row_of_full():
    t, hq, hkv, hd = 9, 4, 2, 8
    q = RNG.standard_normal((t, hq, hd))
    k = RNG.standard_normal((t, hkv, hd))
    v = RNG.standard_normal((t, hkv, hd))
    full = O.causal_attention(q, k, v, np.arange(t))
    for i in (0, 4, 8):
        one = O.causal_attention(q[i:i + 1], k[: i + 1], v[: i + 1], np.array([i]))
        np.testing.assert_allclose(one[0], full[i], rtol=1e-12)


# ---------------------------------------------------------------- SwiGLU pieces
def test_silu_identities():
    x = RNG.standard_normal(100) * 4
    assert O.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(O.silu(-x), O.silu(x) - x, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(O.silu(np.array([40.0])), [40.0], rtol=1e-15)
    np.testing.assert_allclose(O.silu(x), F.silu(torch.from_numpy(x)).numpy(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(O.silu(np.array([1.0])), [1.0 / (1.0 + math.exp(-1.0))], rtol=1e-15)


# ---------------------------------------------------------------- argmax / upcast
def test_argmax_lowest_index_on_ties():
    z = np.array([[1.0, 5.0, 5.0, 2.0], [7.0, 7.0, 7.0, 7.0], [0.0, -1.0, 3.0, 3.0]])
    assert O.argmax_lowest(z).tolist() == [1, 0, 2]


def test_upcast_bf16_bits_exact():
    # 0x3F80 = 1.0, 0xC000 = -2.0, 0x3DCD = 0.10009765625 (bf16 nearest to 0.1), 0x0000 = 0
    bits = np.array([0x3F80, 0xC000, 0x3DCD, 0x0000], dtype=np.uint16)
    np.testing.assert_array_equal(O.upcast(bits), [1.0, -2.0, 0.10009765625, 0.0])
    f = np.array([1.5, -0.25], dtype=np.float32)
    assert O.upcast(f).dtype == np.float64 and O.upcast(f).tolist() == [1.5, -0.25]


# ---------------------------------------------------------------- bf16 operand rounding (the "bf16 model" reading)
def test_round_bf16_literals_and_ties():
    # 1 + 2^-8 is an exact tie between 1.0 and 1 + 2^-7: even mantissa wins (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    x = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.1, 3.0e38, 1e-30, 0.0])
    y = O.round_bf16(x)
    np.testing.assert_array_equal(y[:4], [1.0, 1.0, 1.015625, -1.0])
    assert y[4] == 0.10009765625 and y[7] == 0.0
    assert abs(y[5] - 3.0e38) / 3.0e38 < 2 ** -8 and abs(y[6] - 1e-30) / 1e-30 < 2 ** -8
    # idempotent, and agrees with torch's conversion
    z = RNG.standard_normal(50000) * 7
    r = O.round_bf16(z)
    np.testing.assert_array_equal(O.round_bf16(r), r)
    ref = torch.from_numpy(z.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(r, ref)
    assert (np.abs(r - z) <= np.abs(z) * 2 ** -8).all()


def test_attention_with_rounded_numerators_stays_close_and_normalised():
    t, hq, hkv, hd = 11, 4, 2, 16
    q = RNG.standard_normal((t, hq, hd))
    k = RNG.standard_normal((t, hkv, hd))
    v = np.ones((t, hkv, hd))
    exact = O.causal_attention(q, k, v, np.arange(t))
    rounded = O.causal_attention(q, k, v, np.arange(t), round_probs=O.round_bf16)
    np.testing.assert_allclose(exact, 1.0, rtol=1e-14)            # weights sum to one
    assert np.abs(rounded - 1.0).max() < 2 ** -8                   # each numerator moved by < 2^-8 relative
    assert np.abs(rounded - 1.0).max() > 0                         # and the rounding is really applied
