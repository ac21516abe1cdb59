"""Pins for the oracle's comparison stage (Section 5.7): closed forms and known tamper masks."""
import math

import numpy as np
import pytest

import synth
from oracle import verillm_oracle as O

RNG = np.random.default_rng(777)


def test_identical_states_accept_with_zero_error():
    h = RNG.standard_normal((9, 32))
    s = O.compare_hidden(h, h.copy(), 1e-3, math.inf)
    assert s["ok"].all() and (s["rel_l2"] == 0).all() and (s["max_abs"] == 0).all() and (s["mean_abs"] == 0).all()


def test_zero_commitment_has_relative_error_one():
    h = RNG.standard_normal((4, 16))
    s = O.compare_hidden(h, np.zeros_like(h), 0.5, math.inf)
    np.testing.assert_allclose(s["rel_l2"], 1.0, rtol=1e-14)
    assert not s["ok"].any()
    np.testing.assert_allclose(s["mean_signed"], h.mean(axis=1), rtol=1e-14)
    np.testing.assert_allclose(s["max_abs"], np.abs(h).max(axis=1), rtol=1e-14)


def test_single_coordinate_offset_closed_form():
    h = RNG.standard_normal((3, 64))
    star = h.copy()
    c = 0.75
    star[1, 17] -= c                                   # Delta = h_hat - h_star = +c at one coordinate
    s = O.compare_hidden(h, star, 1.0, math.inf)
    np.testing.assert_allclose(s["max_abs"], [0, c, 0], rtol=1e-13)
    np.testing.assert_allclose(s["rel_l2"][1], c / np.linalg.norm(h[1]), rtol=1e-13)
    np.testing.assert_allclose(s["mean_abs"][1], c / 64, rtol=1e-13)
    np.testing.assert_allclose(s["mean_signed"][1], c / 64, rtol=1e-13)     # sign: recomputed minus committed


def test_thresholds_are_inclusive_and_both_must_hold():
    h = np.zeros((3, 4))
    h[:, 0] = 2.0                                      # ||h|| = 2
    star = h.copy()
    star[0, 1] = 0.2                                   # rel = 0.1, max_abs = 0.2
    star[1, 1] = 0.2000001
    star[2, 1] = 0.1
    s = O.compare_hidden(h, star, 0.1, math.inf)
    assert s["ok"].tolist() == [True, False, True]
    s = O.compare_hidden(h, star, 1.0, 0.15)           # max_abs gate alone
    assert s["ok"].tolist() == [False, False, True]


def test_nan_and_inf_in_commitment_reject():
    h = RNG.standard_normal((4, 8))
    star = h.copy()
    star[0, 3] = np.nan
    star[1, 2] = np.inf
    s = O.compare_hidden(h, star, 1e9, math.inf)
    assert s["ok"].tolist() == [False, False, True, True]


def test_bf16_commitment_is_upcast_exactly():
    h = RNG.standard_normal((5, 32)).astype(np.float32)
    bits = synth.f32_to_bf16_bits(h)
    back = synth.bf16_bits_to_f32(bits).astype(np.float64)
    s1 = O.compare_hidden(h, bits, 1.0, math.inf)
    s2 = O.compare_hidden(h, back, 1.0, math.inf)
    for k in ("rel_l2", "max_abs", "mean_abs", "mean_signed"):
        np.testing.assert_array_equal(s1[k], s2[k])
    assert (s1["rel_l2"] < 2 ** -8).all() and (s1["rel_l2"] > 0).all()   # bf16 keeps 8 significant bits


def test_token_check_margin_semantics():
    z = np.array([[0.0, 3.0, 2.9, -1.0],
                  [1.0, 1.0, 0.5, 0.0],
                  [5.0, 4.0, 3.0, 2.0],
                  [0.0, 0.0, 0.0, 9.0]])
    a, gap, ok = O.token_check(z, np.array([2, 1, -1, 7]), 0.0)
    assert a.tolist() == [1, 0, 0, 3]
    np.testing.assert_allclose(gap[:3], [0.1, 0.0, 0.0], atol=1e-15)
    assert ok.tolist() == [False, True, True, False]          # tie passes at margin 0; -1 skips; 7 is out of range
    _, _, ok = O.token_check(z, np.array([2, 1, -1, 0]), 0.1 + 1e-12)
    assert ok.tolist() == [True, True, True, False]
    _, _, ok = O.token_check(z, np.array([3, 3, 3, 3]), 4.0)
    assert ok.tolist() == [True, True, True, True]


def test_flags_and_summary_on_a_known_tamper_mask():
    n, d = 40, 64
    h1 = RNG.standard_normal((n, d)) * 3
    h2 = RNG.standard_normal((n, d)) * 5
    c1, c2 = h1 + 1e-4 * RNG.standard_normal((n, d)), h2 + 1e-4 * RNG.standard_normal((n, d))
    bad_hidden = [3, 17]
    for p in bad_hidden:
        c2[p] += 2.0 * RNG.standard_normal(d)
    z = RNG.standard_normal((n, 50))
    cam = np.argmax(z, axis=1)
    cam[[5, 17]] = np.argmin(z, axis=1)[[5, 17]]
    s = [O.compare_hidden(h1, c1, 1e-2, math.inf), O.compare_hidden(h2, c2, 1e-2, math.inf)]
    _, _, tok_ok = O.token_check(z, cam, 0.0)
    f = O.flags([x["ok"] for x in s], tok_ok)
    expect = np.ones(n, np.uint8)
    expect[[3, 5, 17]] = 0
    np.testing.assert_array_equal(f, expect)
    sm = O.summary(s, tok_ok, f)
    assert sm["n_tokens"] == n and sm["n_rejected"] == 3 and sm["n_hidden_reject"] == 2 and sm["n_token_reject"] == 2
    assert sm["max_rel_l2"] == pytest.approx(max(s[1]["rel_l2"][3], s[1]["rel_l2"][17]))
    # T_v with phi = MAE, Psi = mean: equals the plain mean |Delta| over everything compared
    tv = (np.abs(h1 - c1).mean() + np.abs(h2 - c2).mean()) / 2
    assert sm["mean_mae"] == pytest.approx(tv, rel=1e-12)


def test_verify_end_to_end_flags_equal_planted_mask():
    cfg = synth.ModelCfg("v", 2, 32, 4, 2, 8, 48, 64, 1e-5, 10000.0, "f32", 0.3, seed=21)
    wl = synth.small_workload(cfg, [12, 7], [1, 2], tamper_count=3, seed=1)
    m = O.Model(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab,
                cfg.rms_eps, cfg.rope_base, lambda k, l: synth.weight(cfg, k, l, 1))
    x = synth.tokens(wl)
    hid, z = O.decode(m, x, wl.lengths, wl.commit_layers)          # the inferencer's commitments
    committed = np.stack([hid[l] for l in wl.commit_layers]).astype(np.float32)
    cam = O.argmax_lowest(z).astype(np.int32)
    pos = synth.tamper_positions(wl)
    committed_t = synth.tamper_hidden(wl, committed, pos)
    cam_t, changed = synth.tamper_argmax(wl, cam, pos, wrong_tokens=np.argmin(z, axis=1))
    out = O.verify(m, x, wl.lengths, wl.commit_layers, committed_t, cam_t, wl.tol_rel_l2, wl.tol_max_abs,
                   wl.tol_logit_margin)
    expect = np.ones(wl.n_tokens, np.uint8)
    expect[pos] = 0
    np.testing.assert_array_equal(out["flags"], expect)
    assert out["summary"]["n_rejected"] == len(pos)
    assert out["summary"]["n_token_reject"] == len(changed)
    honest = O.verify(m, x, wl.lengths, wl.commit_layers, committed, cam, wl.tol_rel_l2, wl.tol_max_abs,
                      wl.tol_logit_margin)
    assert honest["flags"].all() and honest["summary"]["max_rel_l2"] < 1e-6
