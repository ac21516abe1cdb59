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


# ---------------------------------------------------------------- bit-aware comparison (Section 7) and the offline battery
import struct


def _fields_by_struct(v: float):
    (u,) = struct.unpack("<I", struct.pack("<f", v))
    return u >> 31, (u >> 23) & 0xFF, u & 0x7FFFFF


def test_float32_fields_against_struct_and_frexp():
    vals = np.array([1.0, -1.0, 0.15625, 3.0e38, 1.5e-38, 0.0, -0.0, 7.0, 1.0 - 2.0 ** -24, np.inf], np.float32)
    s, e, m = O.float32_fields(vals)
    for i, v in enumerate(vals.tolist()):
        assert (s[i], e[i], m[i]) == _fields_by_struct(v)
    # textbook values: 1.0 = 0|127|0, 0.15625 = 1.25 * 2^-3 = 0|124|0x200000, 7 = 1.75 * 2^2 = 0|129|0x600000
    assert (s[0], e[0], m[0]) == (0, 127, 0) and (s[1], e[1], m[1]) == (1, 127, 0)
    assert (e[2], m[2]) == (124, 0x200000) and (e[7], m[7]) == (129, 0x600000)
    assert (e[8], m[8]) == (126, 0x7FFFFF) and (e[9], m[9]) == (255, 0)
    # for normal numbers the field is frexp's exponent + 126 (frexp normalises to [0.5, 1))
    x = (RNG.standard_normal(1000) * np.exp(RNG.uniform(-20, 20, 1000))).astype(np.float32)
    _, ex, _ = O.float32_fields(x)
    np.testing.assert_array_equal(ex, np.frexp(x)[1].astype(np.int64) + 126)


def test_bit_compare_hand_worked_row():
    # pair by pair (recomputed, record):
    #  (1, 1)                 identical
    #  (1 - 2^-24, 1)         exponent fields 126 / 127: mismatch, |Delta| = 6e-8 <= e_w -> "close"; also "small"
    #  (2, 1)                 mismatch, same mantissa field, |Delta| = 1: not close, "large"; must NOT count as a match
    #  (1, 1 + 2^-23)         same exponent, mantissa one step apart -> small mantissa deviation; "small"
    #  (0.5, 0.5 + 2^-23)     same exponent (126), mantissa 2 steps apart; "small"
    #  (1 + 8 * 2^-23, 1)     same exponent, 8 steps apart: beyond e_m = 7; |Delta| = 9.5e-7 still "small"
    #  (-1, 1)                fields equal apart from the sign: counts as a mantissa match, Delta = -2 is "large"
    a = np.array([[1.0, 1.0 - 2.0 ** -24, 2.0, 1.0, 0.5, 1.0 + 8 * 2.0 ** -23, -1.0]], np.float32)
    b = np.array([[1.0, 1.0, 1.0, 1.0 + 2.0 ** -23, 0.5 + 2.0 ** -23, 1.0, 1.0]], np.float32)
    c = O.bit_compare(a, b, e_w=1e-2, e_m=7, step_log2=0, q_small=1e-5, tau_large=0.5)
    got = {k: int(v[0]) for k, v in c.items() if k != "d"}
    assert got == {"n_exact": 1, "n_exp_mismatch": 2, "n_mismatch_close": 1, "n_match_small": 4, "n_small": 5, "n_large": 2}
    assert c["d"] == 7
    # one step of a bf16 mantissa is 2^16 float32 steps: with step_log2 = 16 the 8-step pair is well inside
    c16 = O.bit_compare(a, b, 1e-2, 7, 16, 1e-5, 0.5)
    assert int(c16["n_match_small"][0]) == 5


def test_bit_compare_invariants():
    x = (RNG.standard_normal((5, 256)) * 3).astype(np.float32)
    same = O.bit_compare(x, x, 1e-2, 7, 0, 1e-5, 1.0)
    assert (same["n_exact"] == 256).all() and (same["n_exp_mismatch"] == 0).all() and (same["n_match_small"] == 256).all()
    assert (same["n_small"] == 256).all() and (same["n_large"] == 0).all()
    # doubling moves every exponent field by one and leaves every mantissa field alone
    dbl = O.bit_compare(x, 2 * x, 1e-2, 7, 0, 1e-5, 1.0)
    assert (dbl["n_exp_mismatch"] == 256).all() and (dbl["n_match_small"] == 0).all() and (dbl["n_exact"] == 0).all()
    np.testing.assert_array_equal(dbl["n_mismatch_close"], (np.abs(x) <= np.float32(1e-2)).sum(axis=1))
    np.testing.assert_array_equal(dbl["n_large"], (np.abs(x) > 1.0).sum(axis=1))
    # a bf16 record of the same values: at most half a bf16 step away, so every exponent match is a "small" one in
    # bf16 steps, and almost none is within 7 float32 steps; mismatches appear only where rounding carried to 2^k
    rec = synth.f32_to_bf16_bits(x)
    c16 = O.bit_compare(x, rec, 1e-2, 1, 16, 1e-5, 1.0)
    np.testing.assert_array_equal(c16["n_match_small"], 256 - c16["n_exp_mismatch"])
    assert c16["n_exp_mismatch"].sum() <= 8 and (c16["n_mismatch_close"] == c16["n_exp_mismatch"]).all()
    c0 = O.bit_compare(x, rec, 1e-2, 7, 0, 1e-5, 1.0)
    assert c0["n_match_small"].sum() < 0.01 * x.size
    # the recomputation may arrive in float64: it is rounded to float32 first
    np.testing.assert_array_equal(O.bit_compare(x.astype(np.float64), rec, 1e-2, 1, 16, 1e-5, 1.0)["n_match_small"], c16["n_match_small"])


def test_bit_compare_brute_force_with_specials():
    a = (RNG.standard_normal((3, 40)) * np.exp(RNG.uniform(-3, 3, (3, 40)))).astype(np.float32)
    b = (a * (1 + 1e-3 * RNG.standard_normal((3, 40)))).astype(np.float32)
    a[0, 0], b[0, 1], a[1, 2], b[1, 3], a[2, 4], b[2, 4] = np.nan, np.inf, 0.0, -0.0, 1e-40, 2e-40
    e_w, e_m, lg, q, tau = 3e-3, 5, 12, 1e-4, 2e-2
    c = O.bit_compare(a, b, e_w, e_m, lg, q, tau)
    f32 = np.float32
    for r in range(3):
        exact = mis = close = msmall = small = large = 0
        for x, y in zip(a[r].tolist(), b[r].tolist()):
            sx, ex, mx = _fields_by_struct(x)
            sy, ey, my = _fields_by_struct(y)
            with np.errstate(invalid="ignore"):
                dl = abs(float(f32(x) - f32(y)))
            exact += struct.pack("<f", x) == struct.pack("<f", y)
            if ex != ey:
                mis += 1
                close += dl <= float(f32(e_w))
            else:
                msmall += abs(mx - my) <= e_m * 2 ** lg
            small += dl <= float(f32(q))
            large += dl > float(f32(tau))
        assert [int(c[k][r]) for k in ("n_exact", "n_exp_mismatch", "n_mismatch_close", "n_match_small", "n_small", "n_large")] \
            == [exact, mis, close, msmall, small, large]


def test_bit_rule_thresholds_and_empty_sets():
    def counts(d, mis, close, msmall, small=0, large=0):
        return {"d": d, "n_exp_mismatch": np.array([mis]), "n_mismatch_close": np.array([close]),
                "n_match_small": np.array([msmall]), "n_small": np.array([small]), "n_large": np.array([large])}
    rule = dict(pe_max=0.05, pm_min=0.75, pw_min=0.80, eps_max=0.01)
    zero = np.zeros(1)
    assert O.bit_rule(counts(100, 4, 4, 90), zero, **rule)[0]
    assert not O.bit_rule(counts(100, 5, 5, 90), zero, **rule)[0]           # P_e = 0.05 is not < 0.05
    assert not O.bit_rule(counts(100, 4, 3, 90), zero, **rule)[0]           # P_m = 0.75 is not > 0.75
    assert not O.bit_rule(counts(100, 4, 4, 76), zero, **rule)[0]           # P_w = 76/96 < 0.8
    assert O.bit_rule(counts(100, 4, 4, 77), zero, **rule)[0]               # 77/96 = 0.802
    assert O.bit_rule(counts(100, 0, 0, 100), zero, **rule)[0]              # no mismatch: P_m passes on the empty set
    assert O.bit_rule(counts(100, 4, 4, 90), np.array([-0.0099]), **rule)[0]
    assert not O.bit_rule(counts(100, 4, 4, 90), np.array([0.0101]), **rule)[0]
    assert not O.bit_rule(counts(100, 4, 4, 90), np.array([np.nan]), **rule)[0]
    assert not O.bit_rule(counts(100, 4, 4, 90, small=49), zero, q_small_min=0.5, **rule)[0]
    assert O.bit_rule(counts(100, 4, 4, 90, small=50), zero, q_small_min=0.5, **rule)[0]
    assert not O.bit_rule(counts(100, 4, 4, 90, large=3), zero, z_large_max=0.02, **rule)[0]
    assert O.bit_rule(counts(100, 4, 4, 90, large=2), zero, z_large_max=0.02, **rule)[0]
    # d = 100 elements that all mismatch: P_w's set is empty and passes, P_e fails
    assert not O.bit_rule(counts(100, 100, 100, 0), zero, **rule)[0]
    assert O.bit_rule(counts(100, 100, 100, 0), zero, pe_max=1.5, pm_min=0.75, pw_min=0.8, eps_max=0.01)[0]
