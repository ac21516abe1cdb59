"""Pins for the oracle's whole forward pass.

* an independent library implementation (the `transformers` Llama model, float64, CPU) on a tiny
  random model: pins block order, RoPE pairing, GQA head mapping, eps placement, LM head;
* the invariants the method itself rests on (Section 4, Eq. (1) and Section 5.5): token-by-token decode
  with a KV cache reproduces the teacher-forced prefill at every position and layer; later tokens never
  change earlier positions; packed sequences do not interact;
* special cases with known answers; a scalar-loop brute force on a tiny model.
"""
import math

import numpy as np
import pytest
import torch

import synth
from oracle import verillm_oracle as O


def make_model(cfg: synth.ModelCfg, override=None) -> O.Model:
    override = override or {}

    def w(kind, layer):
        if (kind, layer) in override:
            return override[(kind, layer)]
        return synth.weight(cfg, kind, layer, threads=1)

    return O.Model(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn,
                   cfg.vocab, cfg.rms_eps, cfg.rope_base, w)


TINY = synth.ModelCfg("t", 3, 32, 4, 2, 8, 48, 64, 1e-5, 10000.0, "f32", 0.3, seed=5, random_gains=True)
TINY_BF = synth.ModelCfg("tb", 2, 32, 4, 2, 8, 48, 64, 1e-5, 500000.0, "bf16", 0.3, seed=6, random_gains=True)


def toks(n, vocab, seed=0):
    return np.random.default_rng(seed).integers(0, vocab, size=n).astype(np.int32)


# one block at the real 8B evaluation shape (32 / 8 heads of 128, d = 4096, F = 14336, base 500000, bf16 weight values):
# pins whatever depends on the shape itself, e.g. the mapping of 4 query heads onto each KV head
BLOCK_8B = synth.ModelCfg("8b-block", 1, 4096, 32, 8, 128, 14336, 512, 1e-5, 500000.0, "bf16", 0.02, seed=1002)
# the head geometry of the 70B shape (64 / 8 heads of 128, d = 8192) with a narrow feed-forward to keep the test light
HEADS_70B = synth.ModelCfg("70b-heads", 1, 8192, 64, 8, 128, 2048, 512, 1e-5, 500000.0, "bf16", 0.01, seed=1004)


@pytest.mark.parametrize("cfg", [TINY, TINY_BF, BLOCK_8B, HEADS_70B],
                         ids=["f32", "bf16-weights", "8b-shape-block", "70b-head-geometry"])
def test_forward_matches_transformers_llama(cfg):
    transformers = pytest.importorskip("transformers")
    hc = transformers.LlamaConfig(
        vocab_size=cfg.vocab, hidden_size=cfg.d_model, intermediate_size=cfg.d_ffn,
        num_hidden_layers=cfg.n_layers, num_attention_heads=cfg.n_q_heads, num_key_value_heads=cfg.n_kv_heads,
        head_dim=cfg.head_dim, rms_norm_eps=cfg.rms_eps, rope_theta=cfg.rope_base, tie_word_embeddings=False,
        attention_bias=False, mlp_bias=False, max_position_embeddings=256, hidden_act="silu")
    hf = transformers.LlamaForCausalLM(hc).double().eval()
    names = {O.ATTN_NORM: "input_layernorm", O.WQ: "self_attn.q_proj", O.WK: "self_attn.k_proj",
             O.WV: "self_attn.v_proj", O.WO: "self_attn.o_proj", O.FFN_NORM: "post_attention_layernorm",
             O.W_GATE: "mlp.gate_proj", O.W_UP: "mlp.up_proj", O.W_DOWN: "mlp.down_proj"}
    sd = {}
    for l in range(cfg.n_layers):
        for k, nm in names.items():
            sd[f"model.layers.{l}.{nm}.weight"] = torch.from_numpy(synth.weight_values_f32(cfg, k, l, 8)).double()
    sd["model.embed_tokens.weight"] = torch.from_numpy(synth.weight_values_f32(cfg, O.EMBED, 0, 1)).double()
    sd["model.norm.weight"] = torch.from_numpy(synth.weight_values_f32(cfg, O.FINAL_NORM, 0, 1)).double()
    sd["lm_head.weight"] = torch.from_numpy(synth.weight_values_f32(cfg, O.LM_HEAD, 0, 1)).double()
    missing = hf.load_state_dict(sd, strict=False)
    assert not [k for k in missing.missing_keys if "rotary" not in k]
    t = 19
    x = toks(t, cfg.vocab, 3)
    with torch.no_grad():
        out = hf(torch.from_numpy(x.astype(np.int64))[None], output_hidden_states=True)
    hidden, logits = O.prefill(make_model(cfg), x, [t], list(range(1, cfg.n_layers + 1)))
    # hidden_states[l] for 0 < l < L is the residual stream after block l (the last entry is post-norm).
    # The library evaluates its rotary angles in float32 whatever the model dtype, so agreement is at
    # float32 level (values are O(1)); any structural mistake moves the output by O(0.1) or more.
    tol = dict(rtol=2e-5, atol=2e-5)
    for l in range(1, cfg.n_layers):
        np.testing.assert_allclose(hidden[l], out.hidden_states[l][0].numpy(), **tol)
    np.testing.assert_allclose(logits, out.logits[0].numpy(), **tol)
    # the committed last-layer state is the PRE-norm residual: applying the final norm recovers HF's last entry
    g = synth.weight_values_f32(cfg, O.FINAL_NORM, 0, 1)
    np.testing.assert_allclose(O.rmsnorm(hidden[cfg.n_layers], g, cfg.rms_eps),
                               out.hidden_states[cfg.n_layers][0].numpy(), **tol)


def test_decode_equals_prefill_every_position_and_layer():
    m = make_model(TINY)
    lengths = [11, 1, 7]
    x = toks(sum(lengths), TINY.vocab, 1)
    layers = [1, 2, 3]
    hp, zp = O.prefill(m, x, lengths, layers)
    hd, zd = O.decode(m, x, lengths, layers)
    for l in layers:
        np.testing.assert_allclose(hd[l], hp[l], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(zd, zp, rtol=1e-10, atol=1e-12)


def test_causality_appending_tokens_keeps_earlier_positions():
    m = make_model(TINY)
    x = toks(20, TINY.vocab, 2)
    h_long, z_long = O.prefill(m, x, [20], [1, 3])
    h_short, z_short = O.prefill(m, x[:12], [12], [1, 3])
    for l in (1, 3):
        np.testing.assert_allclose(h_long[l][:12], h_short[l], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(z_long[:12], z_short, rtol=1e-12, atol=1e-14)
    # and changing a later token changes later positions only
    y = x.copy()
    y[15] = (y[15] + 1) % TINY.vocab
    h_mod, _ = O.prefill(m, y, [20], [3])
    np.testing.assert_allclose(h_mod[3][:15], h_long[3][:15], rtol=1e-12, atol=1e-14)
    assert np.abs(h_mod[3][15:] - h_long[3][15:]).max() > 1e-6


def test_batch_independence_of_packed_sequences():
    m = make_model(TINY)
    lengths = [5, 9, 3]
    x = toks(sum(lengths), TINY.vocab, 4)
    h_all, z_all = O.prefill(m, x, lengths, [2, 3])
    lo = 0
    for t in lengths:
        h_one, z_one = O.prefill(m, x[lo:lo + t], [t], [2, 3])
        for l in (2, 3):
            np.testing.assert_array_equal(h_all[l][lo:lo + t], h_one[l])
        np.testing.assert_array_equal(z_all[lo:lo + t], z_one)
        lo += t


def test_segment_local_prefill_composes_to_full_prefill():
    # Section 5.6: a verifier of a later segment starts from the recorded upstream states.
    m = make_model(TINY)
    x = toks(10, TINY.vocab, 5)
    h_full, z_full = O.prefill(m, x, [10], [1, 2, 3])
    h_seg, z_seg = O.prefill(m, x, [10], [3], start_layer=1, start_hidden=h_full[1])
    np.testing.assert_allclose(h_seg[3], h_full[3], rtol=1e-13)
    np.testing.assert_allclose(z_seg, z_full, rtol=1e-13)
    h_first, z_first = O.prefill(m, x, [10], [1], end_layer=1)
    np.testing.assert_array_equal(h_first[1], h_full[1])
    assert z_first is None


def test_segment_verifiers_accept_honest_states_and_localise_a_fault():
    # Section 5.6: every segment is judged on its own from the recorded upstream states.  What must hold follows from
    # causality and from the independence of sequences, not from the code: a fault planted in the record of layer 2 at
    # position p of sequence 1 is seen by the verifier of (1,2] at p only; the verifier of (2,3] starts from the
    # faulty record, so its recomputation can differ at p and at later positions of the same sequence, nowhere else;
    # the verifier of (0,1] sees nothing.
    m = make_model(TINY)
    lengths = [6, 9, 4]
    x = toks(sum(lengths), TINY.vocab, 8)
    h, z = O.prefill(m, x, lengths, [1, 2, 3])
    com = {l: h[l].astype(np.float32) for l in (1, 2, 3)}
    cam = O.argmax_lowest(z).astype(np.int32)
    tol = dict(tol_rel_l2=1e-4, tol_max_abs=np.inf, tol_logit_margin=1e-3)
    whole = O.verify(m, x, lengths, [1, 2, 3], np.stack([com[1], com[2], com[3]]), cam, **tol)
    assert whole["flags"].all()
    for lo, hi in ((0, 1), (1, 2), (2, 3)):
        seg = O.verify(m, x, lengths, [hi], com[hi][None], cam if hi == 3 else None, start_layer=lo,
                       upstream_hidden=com[lo] if lo else None, end_layer=hi, **tol)
        assert seg["flags"].all() and seg["stats"][0]["rel_l2"].max() < 1e-6
    p = 6 + 3                                             # position 3 of sequence 1 (rows 6 .. 14)
    bad = com[2].copy()
    bad[p] += 0.05 * np.abs(com[2][p]).max()
    s01 = O.verify(m, x, lengths, [1], com[1][None], None, end_layer=1, **tol)
    s12 = O.verify(m, x, lengths, [2], bad[None], None, start_layer=1, upstream_hidden=com[1], end_layer=2, **tol)
    s23 = O.verify(m, x, lengths, [3], com[3][None], cam, start_layer=2, upstream_hidden=bad, end_layer=3, **tol)
    assert s01["flags"].all()
    expect = np.ones(sum(lengths), np.uint8)
    expect[p] = 0
    np.testing.assert_array_equal(s12["flags"], expect)
    assert s23["flags"][p] == 0
    untouched = np.r_[0:p, 15:19]                         # earlier rows of the sequence and the other sequences
    assert s23["flags"][untouched].all() and s23["stats"][0]["rel_l2"][untouched].max() < 1e-6
    assert (s23["stats"][0]["rel_l2"][p + 1:15] > 1e-6).all()    # later rows do feel the fault through attention
    w = O.verify(m, x, lengths, [1, 2, 3], np.stack([com[1], bad, com[3]]), cam, **tol)
    np.testing.assert_array_equal(w["flags"], expect)     # the whole-model verifier recomputes layer 3 from its own state


def test_gqa_equals_mha_with_replicated_kv_heads():
    gqa = synth.ModelCfg("g", 1, 32, 4, 2, 8, 48, 64, 1e-5, 10000.0, "f32", 0.3, seed=9)
    mha = synth.ModelCfg("m", 1, 32, 4, 4, 8, 48, 64, 1e-5, 10000.0, "f32", 0.3, seed=9)
    wk = synth.weight(gqa, O.WK, 0, 1).reshape(2, 8, 32)
    wv = synth.weight(gqa, O.WV, 0, 1).reshape(2, 8, 32)
    rep = {(O.WK, 0): np.repeat(wk, 2, axis=0).reshape(32, 32), (O.WV, 0): np.repeat(wv, 2, axis=0).reshape(32, 32)}
    for k in (O.WQ, O.WO, O.W_GATE, O.W_UP, O.W_DOWN):
        rep[(k, 0)] = synth.weight(gqa, k, 0, 1)
    for k in (O.EMBED, O.LM_HEAD):
        rep[(k, 0)] = synth.weight(gqa, k, 0, 1)
    x = toks(9, 64, 6)
    h1, z1 = O.prefill(make_model(gqa), x, [9], [1])
    h2, z2 = O.prefill(make_model(mha, rep), x, [9], [1])
    np.testing.assert_allclose(h1[1], h2[1], rtol=1e-12)
    np.testing.assert_allclose(z1, z2, rtol=1e-12)


def test_zero_gate_makes_ffn_a_no_op_and_zero_wo_removes_attention():
    cfg = synth.ModelCfg("z", 1, 32, 4, 2, 8, 48, 64, 1e-5, 10000.0, "f32", 0.3, seed=10)
    x = toks(6, 64, 7)
    emb = synth.weight(cfg, O.EMBED, 0, 1).astype(np.float64)
    ov = {(O.W_GATE, 0): np.zeros((48, 32), np.float32), (O.WO, 0): np.zeros((32, 32), np.float32)}
    h, _ = O.prefill(make_model(cfg, ov), x, [6], [1])
    np.testing.assert_array_equal(h[1], emb[x])        # both residual branches vanish: h^1 = Embed(x)
    ov = {(O.W_GATE, 0): np.zeros((48, 32), np.float32)}
    h_attn_only, _ = O.prefill(make_model(cfg, ov), x, [6], [1])
    assert np.abs(h_attn_only[1] - emb[x]).max() > 1e-3


def test_lm_head_one_hot_rows_give_known_argmax_and_ties_lowest():
    cfg = synth.ModelCfg("o", 1, 16, 2, 2, 8, 24, 10, 1e-5, 10000.0, "f32", 0.3, seed=11)
    # LM-head row v is e_(v mod 16) except rows 3 and 7 which both copy the normalised state's largest axis
    x = toks(5, 10, 8)
    m0 = make_model(cfg)
    h, _ = O.prefill(m0, x, [5], [1])
    u = O.rmsnorm(h[1], np.ones(16), cfg.rms_eps)
    lm = np.zeros((10, 16), np.float32)
    ov = {(O.LM_HEAD, 0): lm}
    for n in range(5):
        j = int(np.argmax(u[n]))
        lm[:] = 0
        lm[3, j] = 1.0
        lm[7, j] = 1.0
        z = O.lm_head(make_model(cfg, ov), h[1][n:n + 1])
        assert z[0, 3] == z[0, 7] == pytest.approx(u[n, j])
        assert O.argmax_lowest(z)[0] == 3


def _scalar_forward(cfg, x):
    """Llama block in pure Python scalar loops (independent of numpy vectorisation)."""
    W = lambda k, l=0: synth.weight_values_f32(cfg, k, l, 1).astype(np.float64).tolist()
    d, hq, hkv, hd, f = cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn
    emb = W(O.EMBED)
    h = [list(emb[int(t)]) for t in x]
    T = len(x)

    def norm(row, g):
        ms = sum(v * v for v in row) / len(row)
        return [v / math.sqrt(ms + cfg.rms_eps) * g[i] for i, v in enumerate(row)]

    def matvec(w, row):
        return [sum(wr[i] * row[i] for i in range(len(row))) for wr in w]

    def rope(vec, pos):
        out = list(vec)
        for hh in range(len(vec) // hd):
            for i in range(hd // 2):
                a = pos * cfg.rope_base ** (-2.0 * i / hd)
                x1, x2 = vec[hh * hd + i], vec[hh * hd + i + hd // 2]
                out[hh * hd + i] = x1 * math.cos(a) - x2 * math.sin(a)
                out[hh * hd + i + hd // 2] = x2 * math.cos(a) + x1 * math.sin(a)
        return out

    for l in range(cfg.n_layers):
        g1, wq, wk, wv, wo = W(O.ATTN_NORM, l), W(O.WQ, l), W(O.WK, l), W(O.WV, l), W(O.WO, l)
        g2, wg, wu, wd = W(O.FFN_NORM, l), W(O.W_GATE, l), W(O.W_UP, l), W(O.W_DOWN, l)
        us = [norm(h[t], g1) for t in range(T)]
        qs = [rope(matvec(wq, us[t]), t) for t in range(T)]
        ks = [rope(matvec(wk, us[t]), t) for t in range(T)]
        vs = [matvec(wv, us[t]) for t in range(T)]
        for t in range(T):
            o = [0.0] * (hq * hd)
            for j in range(hq):
                g = j // (hq // hkv)
                sc = [sum(qs[t][j * hd + c] * ks[r][g * hd + c] for c in range(hd)) / math.sqrt(hd) for r in range(t + 1)]
                mx = max(sc)
                e = [math.exp(s - mx) for s in sc]
                z = sum(e)
                for c in range(hd):
                    o[j * hd + c] = sum(e[r] * vs[r][g * hd + c] for r in range(t + 1)) / z
            att = matvec(wo, o)
            h1 = [h[t][i] + att[i] for i in range(d)]
            xn = norm(h1, g2)
            ga, up = matvec(wg, xn), matvec(wu, xn)
            act = [ga[i] / (1.0 + math.exp(-ga[i])) * up[i] for i in range(f)]
            dn = matvec(wd, act)
            h[t] = [h1[i] + dn[i] for i in range(d)]
    gf, lm = W(O.FINAL_NORM), W(O.LM_HEAD)
    logits = [matvec(lm, norm(h[t], gf)) for t in range(T)]
    return np.array(h), np.array(logits)


def test_forward_matches_scalar_loop_brute_force():
    cfg = synth.ModelCfg("s", 2, 16, 4, 2, 4, 24, 20, 1e-5, 10000.0, "f32", 0.4, seed=12, random_gains=True)
    x = toks(6, 20, 9)
    h_ref, z_ref = _scalar_forward(cfg, x)
    h, z = O.prefill(make_model(cfg), x, [6], [2])
    np.testing.assert_allclose(h[2], h_ref, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(z, z_ref, rtol=1e-11, atol=1e-13)


def test_planted_mistakes_are_caught():
    """The pins above must be able to fail: a wrong RoPE pairing or a wrong GQA mapping moves the output."""
    cfg = TINY
    x = toks(8, cfg.vocab, 10)
    m = make_model(cfg)
    good, _ = O.prefill(m, x, [8], [3])
    orig = O.apply_rope

    def interleaved(xx, pos, base):            # adjacent-pair RoPE instead of half-split
        t, h, hd = xx.shape
        y = xx.reshape(t, h, hd // 2, 2)
        y = np.concatenate([y[..., 0], y[..., 1]], axis=-1)
        r = orig(y, pos, base)
        return np.stack([r[..., : hd // 2], r[..., hd // 2:]], axis=-1).reshape(t, h, hd)

    O.apply_rope = interleaved
    try:
        bad, _ = O.prefill(m, x, [8], [3])
    finally:
        O.apply_rope = orig
    assert np.abs(bad[3] - good[3]).max() > 1e-4


def test_bf16_operand_mode_is_a_small_perturbation_of_the_exact_model():
    """Rounding every matrix-product operand to bf16 (8 significant bits, 2^-8 = 3.9e-3 per rounding) moves the
    states by about 1e-2 per layer on a random model, not more, and the decode == prefill identity still holds to
    rounding noise."""
    cfg = synth.ModelCfg("r", 3, 64, 4, 2, 16, 96, 50, 1e-5, 10000.0, "bf16", 0.2, seed=31)
    x = toks(24, 50, 11)
    w = lambda k, l: synth.weight(cfg, k, l, 1)
    args = (cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab, cfg.rms_eps, cfg.rope_base, w)
    exact, z0 = O.prefill(O.Model(*args), x, [24], [1, 2, 3])
    mr = O.Model(*args, operand_dtype="bf16")
    rnd, z1 = O.prefill(mr, x, [24], [1, 2, 3])
    for l in (1, 2, 3):
        rel = np.linalg.norm(rnd[l] - exact[l], axis=1) / np.linalg.norm(exact[l], axis=1)
        assert 1e-4 < rel.mean() < 2e-2 and rel.max() < 6e-2
    dec, _ = O.decode(mr, x, [24], [3])
    rel = np.linalg.norm(dec[3] - rnd[3], axis=1) / np.linalg.norm(rnd[3], axis=1)
    assert rel.max() < 3e-2
    # operands that are already bf16 values are left alone: a one-hot normalised input survives exactly
    assert (O.round_bf16(np.array([0.5, -2.0, 0.0])) == [0.5, -2.0, 0.0]).all()
