"""GPU parity of the single operations, called through the C ABI, against the CPU oracle."""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2509_24257_amd as P
import synth
from oracle import verillm_oracle as O
from tests import helpers as H

pytestmark = pytest.mark.gpu


def say(msg):
    H.progress("[case] " + msg)


@pytest.fixture(scope="module")
def ctx_small_bf16():
    m = synth.small_model("bf16")
    ctx = H.make_ctx(m, 2048, 16, 1024)
    yield ctx, m
    ctx.close()


@pytest.fixture(scope="module")
def ctx_hd128():
    m = synth.small_model("bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, d_model=512, d_ffn=1024, n_layers=1,
                          vocab=1000, seed=78)
    ctx = H.make_ctx(m, 4096, 16, 2048)
    yield ctx, m
    ctx.close()


# ------------------------------------------------------------------ compare kernel (Section 5.7)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [1, 3, 130, 1027])
def test_compare_matches_oracle(ctx_small_bf16, dtype, n):
    ctx, m = ctx_small_bf16
    d = m.d_model
    say(f"compare dtype={dtype} n={n} d={d}")
    rng = np.random.default_rng(n)
    h = (rng.standard_normal((n, d)) * 3).astype(np.float32)
    star = (h + 0.01 * rng.standard_normal((n, d))).astype(np.float32)
    if n >= 3:
        star[1] += 2.0 * rng.standard_normal(d).astype(np.float32)   # tampered row
        star[2, 5] = np.nan
    if n > 100:
        star[7, 3] = np.inf
        star[9] = 0.0
        h[11] = 0.0
        star[11] = 0.0                                                # 0/0 guarded by the tiny denominator
    st = H.stored(star, dtype)
    tol = P.Tol(0.05, math.inf, 0.0)
    d_h, d_s = H.to_dev(h), H.to_dev(st)
    d_stats = torch.zeros(n * 4, dtype=torch.float32, device=H.DEV)
    d_ok = torch.full((n,), 9, dtype=torch.uint8, device=H.DEV)
    ctx.vl_op_compare(d_h.data_ptr(), d_s.data_ptr(), H.hidden_dtype_code(dtype), n, tol, d_stats.data_ptr(), d_ok.data_ptr())
    got = H.stats_from_dev(d_stats)
    ref = O.compare_hidden(h, st, 0.05, math.inf)
    np.testing.assert_array_equal(d_ok.cpu().numpy().astype(bool), ref["ok"])
    fin = np.isfinite(ref["rel_l2"])
    for k in ("rel_l2", "max_abs", "mean_abs"):
        np.testing.assert_allclose(got[k][fin], ref[k][fin], rtol=2e-5, atol=1e-7)
    np.testing.assert_allclose(got["mean_signed"][fin], ref["mean_signed"][fin], rtol=1e-3, atol=2e-6)
    assert np.isnan(got["max_abs"][~np.isfinite(ref["max_abs"]) & np.isnan(ref["max_abs"])]).all()


def test_compare_is_bit_reproducible(ctx_small_bf16):
    ctx, m = ctx_small_bf16
    n, d = 777, m.d_model
    say("compare reproducibility")
    rng = np.random.default_rng(0)
    h = rng.standard_normal((n, d)).astype(np.float32)
    st = synth.f32_to_bf16_bits(h + 0.1 * rng.standard_normal((n, d)).astype(np.float32))
    d_h, d_s = H.to_dev(h), H.to_dev(st)
    outs = []
    for _ in range(3):
        d_stats = torch.zeros(n * 4, dtype=torch.float32, device=H.DEV)
        d_ok = torch.zeros(n, dtype=torch.uint8, device=H.DEV)
        ctx.vl_op_compare(d_h.data_ptr(), d_s.data_ptr(), P.VL_BF16, n, P.Tol(0.1, math.inf, 0), d_stats.data_ptr(), d_ok.data_ptr())
        outs.append(d_stats.cpu().numpy().tobytes())
    assert outs[0] == outs[1] == outs[2]


# ------------------------------------------------------------------ bit-aware counts and rule (Section 7, Appendix A.1)
BIT_KEYS = ("n_exact", "n_exp_mismatch", "n_mismatch_close", "n_match_small", "n_small", "n_large")


def bits_from_dev(t, n):
    a = t.cpu().numpy().reshape(n, 8)
    out = {k: a[:, i].astype(np.int64) for i, k in enumerate(BIT_KEYS)}
    out["mean_signed"] = a[:, 6].copy().view(np.float32)
    out["ok"] = a[:, 7].astype(bool)
    return out


@pytest.mark.parametrize("dtype,step_log2,e_m", [("f32", 0, 7), ("bf16", 16, 7), ("f32", 12, 3), ("bf16", 23, 1)])
@pytest.mark.parametrize("n", [1, 130, 1027])
def test_compare_bits_counts_are_bit_exact(ctx_small_bf16, dtype, step_log2, e_m, n):
    ctx, m = ctx_small_bf16
    d = m.d_model
    say(f"compare_bits dtype={dtype} step_log2={step_log2} e_m={e_m} n={n}")
    rng = np.random.default_rng(1000 * n + step_log2)
    h = (rng.standard_normal((n, d)) * np.exp(rng.uniform(-2, 2, (n, 1)))).astype(np.float32)
    # rows of different character: cross-device-like relative noise of several sizes, a constant offset (mean shift), a
    # scaled copy (every exponent off by one), exact copies, coarse noise
    kind = rng.integers(0, 6, n)
    noise = np.choose(kind, [1e-7, 1e-4, 3e-3, 0.0, 0.0, 0.3])[:, None]
    star = (h * (1 + noise * rng.standard_normal((n, d)))).astype(np.float32)
    star[kind == 3] += np.float32(0.05)
    star[kind == 4] *= np.float32(2.0)
    if n > 100:
        star[5, 3], star[6, 0], h[7, 9] = np.nan, np.inf, np.nan
        star[8, :40] = 0.0
        h[9, :40] = 0.0
        star[9, :20] = -0.0
        h[10, 0], star[10, 0], h[10, 1], star[10, 1] = 1e-40, 3e-40, 1e-38, 1.3e-38      # denormals, and one next to the border
    st = H.stored(star, dtype)
    rule = P.BitRule(1e-2, e_m, step_log2, 1e-5, 0.1, 0.05, 0.75, 0.80, 0.01, 0.0, 0.3)
    tol = P.Tol(math.inf, math.inf, 0.0)                      # the tolerance test is wide open: `ok` is the rule alone
    d_h, d_s = H.to_dev(h), H.to_dev(st)
    d_stats = torch.zeros(n * 4, dtype=torch.float32, device=H.DEV)
    d_bits = torch.zeros(n * 8, dtype=torch.int32, device=H.DEV)
    d_ok = torch.full((n,), 9, dtype=torch.uint8, device=H.DEV)
    ctx.vl_op_compare_bits(d_h.data_ptr(), d_s.data_ptr(), H.hidden_dtype_code(dtype), n, tol, rule, d_stats.data_ptr(),
                           d_bits.data_ptr(), d_ok.data_ptr())
    got = bits_from_dev(d_bits, n)
    ref = O.bit_compare(h, st, 1e-2, e_m, step_log2, 1e-5, 0.1)
    for k in BIT_KEYS:
        np.testing.assert_array_equal(got[k], ref[k], err_msg=k)
    cmp_ref = O.compare_hidden(h, st, math.inf, math.inf)
    want = O.bit_rule(ref, cmp_ref["mean_signed"], 0.05, 0.75, 0.80, 0.01, 0.0, 0.3)
    # the mean is summed in another order on the GPU: leave out rows whose |mean| sits within rounding of the bound
    with np.errstate(invalid="ignore"):
        clear = ~(np.abs(np.abs(cmp_ref["mean_signed"]) - 0.01) < 1e-5)
    np.testing.assert_array_equal(got["ok"][clear], want[clear])
    nanrow = np.isnan(cmp_ref["mean_signed"])               # NaN never passes a <= / > test, so such rows fail
    np.testing.assert_array_equal(d_ok.cpu().numpy().astype(bool)[clear & ~nanrow], want[clear & ~nanrow])
    assert not d_ok.cpu().numpy()[nanrow].any()
    if n > 100:
        assert want.any() and (~want).any()                 # the mix really exercises both verdicts
    with pytest.raises(P.VerilLMError) as e:
        ctx.vl_op_compare_bits(d_h.data_ptr(), d_s.data_ptr(), H.hidden_dtype_code(dtype), n, tol,
                               P.BitRule(1e-2, 7, 24, 1e-5, 0.1, 0.05, 0.75, 0.8, 0.01, 0.0, 1.0), 0, d_bits.data_ptr(), 0)
    assert e.value.code == -1


# ------------------------------------------------------------------ argmax + TokenMatch
@pytest.mark.parametrize("vocab,n", [(1000, 37), (4096, 5), (128256, 9), (1001, 6)])
def test_argmax_and_token_check_match_oracle(vocab, n):
    say(f"argmax vocab={vocab} n={n}")
    m = synth.small_model("f32", vocab=vocab, n_layers=1)
    ctx = P.Context(H.c_cfg(m, 64, 4, 64), 0, 0)          # op calls need no weights
    try:
        rng = np.random.default_rng(vocab + n)
        z = rng.standard_normal((n, vocab)).astype(np.float32)
        z[0, 17] = z[0, 400] = z[0].max() + 1.0           # exact tie: lowest index wins
        z[1, vocab - 1] = 50.0                            # maximum in the very last column
        z[2, 0] = 60.0
        a_true = np.argmax(z, axis=1)
        cam = a_true.astype(np.int32).copy()
        cam[0] = 400                                      # tied token: gap 0 passes at margin 0
        cam[1] = 3                                        # wrong token
        cam[2] = -1                                       # skipped
        cam[3] = vocab                                    # out of range
        margin = 0.0
        d_z, d_c = H.to_dev(z), H.to_dev(cam)
        d_a = torch.zeros(n, dtype=torch.int32, device=H.DEV)
        d_g = torch.zeros(n, dtype=torch.float32, device=H.DEV)
        d_ok = torch.zeros(n, dtype=torch.uint8, device=H.DEV)
        ctx.vl_op_argmax(d_z.data_ptr(), n, d_c.data_ptr(), margin, d_a.data_ptr(), d_g.data_ptr(), d_ok.data_ptr())
        a, gap, ok = O.token_check(z, cam, margin)
        np.testing.assert_array_equal(d_a.cpu().numpy(), a)
        np.testing.assert_array_equal(d_ok.cpu().numpy().astype(bool), ok)
        np.testing.assert_allclose(d_g.cpu().numpy().astype(np.float64), gap, rtol=1e-6, atol=1e-6)   # one fp32 subtraction
        assert d_a.cpu().numpy()[0] == 17
        # a positive margin lets a near-tie through
        cam2 = a_true.astype(np.int32).copy()
        z2 = z.copy()
        z2[4, (a_true[4] + 1) % vocab] = z2[4, a_true[4]] - 0.01
        cam2[4] = (a_true[4] + 1) % vocab
        d_z2, d_c2 = H.to_dev(z2), H.to_dev(cam2)
        ctx.vl_op_argmax(d_z2.data_ptr(), n, d_c2.data_ptr(), 0.05, d_a.data_ptr(), d_g.data_ptr(), d_ok.data_ptr())
        _, _, ok2 = O.token_check(z2, cam2, 0.05)
        np.testing.assert_array_equal(d_ok.cpu().numpy().astype(bool), ok2)
        assert ok2[4]
    finally:
        ctx.close()


# ------------------------------------------------------------------ bf16 matrix-core GEMM
@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (300, 200, 128), (1, 1, 64), (1000, 520, 192), (513, 257, 4096),
                                   (2048, 1536, 512), (65, 520, 192),
                                   # M <= 64: the weight-streaming kernel of the token-by-token path
                                   (8, 6144, 4096), (16, 4096, 14336), (17, 1000, 256), (33, 130, 192), (64, 4096, 4096),
                                   (3, 31, 64), (48, 33, 320)])
@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_gemm_bf16_matches_float64_product(ctx_small_bf16, M, N, K, out_dtype):
    ctx, _ = ctx_small_bf16
    say(f"gemm M={M} N={N} K={K} out={out_dtype}")
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    a_bits = synth.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    w_bits = synth.f32_to_bf16_bits((rng.standard_normal((N, K)) * 0.05).astype(np.float32))
    ref = O.upcast(a_bits) @ O.upcast(w_bits).T
    d_a, d_w = H.to_dev(a_bits), H.to_dev(w_bits)
    if out_dtype == "f32":
        d_o = torch.full((M, N), 7.0, dtype=torch.float32, device=H.DEV)
        ctx.vl_op_gemm_bf16(d_a.data_ptr(), d_w.data_ptr(), d_o.data_ptr(), P.VL_F32, M, N, K)
        got = d_o.cpu().numpy().astype(np.float64)
        # fp32 accumulation of K products of O(0.05) magnitude: error ~ sqrt(K) * 2^-24 * |terms|
        tol = 1e-5 * math.sqrt(K) * 0.05 * 4
    else:
        d_o = torch.zeros((M, N), dtype=torch.int16, device=H.DEV)
        ctx.vl_op_gemm_bf16(d_a.data_ptr(), d_w.data_ptr(), d_o.data_ptr(), P.VL_BF16, M, N, K)
        got = O.upcast(H.bits_from_dev(d_o))
        tol = None
    if tol is not None:
        np.testing.assert_allclose(got, ref, rtol=0, atol=max(tol, 1e-5))
    else:
        np.testing.assert_allclose(got, ref, rtol=2 ** -8, atol=1e-5)       # one bf16 rounding of the fp32 sum


# ------------------------------------------------------------------ matrix-core causal GQA attention
def _attention_case(ctx, m, lengths, seed, late_key_gain=1.0):
    hq, hkv, hd = m.n_q_heads, m.n_kv_heads, m.head_dim
    n = sum(lengths)
    rng = np.random.default_rng(seed)
    qkv = (rng.standard_normal((n, (hq + 2 * hkv) * hd)) * 1.5).astype(np.float32)
    if late_key_gain != 1.0:
        # keys from position 40 on are much larger than the first ones: scores far above those of the first key block
        lo = 0
        for t in lengths:
            qkv[lo + 40:lo + t, hq * hd:(hq + hkv) * hd] *= late_key_gain
            lo += t
    bits = synth.f32_to_bf16_bits(qkv)
    vals = O.upcast(bits)
    d_qkv = H.to_dev(bits)
    d_out = torch.zeros((n, hq * hd), dtype=torch.int16, device=H.DEV)
    ctx.vl_op_attention_bf16(d_qkv.data_ptr(), lengths, d_out.data_ptr())
    got = O.upcast(H.bits_from_dev(d_out)).reshape(n, hq, hd)
    lo = 0
    worst = 0.0
    for t in lengths:
        if t == 0:
            continue
        blk = vals[lo:lo + t]
        q = blk[:, : hq * hd].reshape(t, hq, hd)
        k = blk[:, hq * hd:(hq + hkv) * hd].reshape(t, hkv, hd)
        v = blk[:, (hq + hkv) * hd:].reshape(t, hkv, hd)
        ref = O.causal_attention(q, k, v, np.arange(t))
        err = np.abs(got[lo:lo + t] - ref).max()
        worst = max(worst, err)
        lo += t
    return worst


@pytest.mark.parametrize("lengths", [[1], [5, 64, 1, 130], [128], [129, 255, 256, 63], [700], [0, 33, 0, 200]])
def test_attention_hd64_matches_oracle(ctx_small_bf16, lengths):
    ctx, m = ctx_small_bf16
    say(f"attention hd64 lengths={lengths}")
    # probabilities and outputs are rounded to bf16 (2^-9 relative); values are O(1.5)
    assert _attention_case(ctx, m, lengths, 1) < 3e-2


@pytest.mark.parametrize("lengths", [[3], [200, 77], [1024], [65, 1, 127, 128, 192]])
def test_attention_hd128_gqa4_matches_oracle(ctx_hd128, lengths):
    ctx, m = ctx_hd128
    say(f"attention hd128 lengths={lengths}")
    assert _attention_case(ctx, m, lengths, 2) < 3e-2


@pytest.mark.parametrize("hq,hkv,hd", [(4, 2, 128), (8, 1, 128), (6, 2, 64), (16, 2, 64), (2, 2, 128)])
def test_attention_head_groupings_match_oracle(hq, hkv, hd):
    """A workgroup of the prefill attention kernel serves 4, 2 or 1 query heads of one KV head (group sizes that are
    multiples of 4, even, odd), with query tiles of 64, 128 or 256 rows; every such mapping against the oracle, on
    lengths that leave ragged last tiles."""
    say(f"attention hq={hq} hkv={hkv} hd={hd}")
    m = synth.small_model("bf16", n_layers=1, n_q_heads=hq, n_kv_heads=hkv, head_dim=hd, d_model=256)
    lengths = [300, 64, 1, 257, 129]
    ctx = P.Context(H.c_cfg(m, sum(lengths), len(lengths), max(lengths)), 0, 0)        # op calls need no weights
    try:
        assert _attention_case(ctx, m, lengths, hq * 100 + hkv * 10 + hd) < 3e-2
    finally:
        ctx.close()


@pytest.mark.parametrize("gain", [6.0, 40.0])
def test_attention_scores_far_above_the_first_block(ctx_hd128, ctx_small_bf16, gain):
    """The kernel fixes a query's exponent reference on its first 32 keys and repeats a workgroup with exact row maxima
    when later scores outgrow it (gain 6: by dozens of binary orders; gain 40: beyond the range of float32 exponentials)."""
    for (ctx, m), lengths in ((ctx_hd128, [300, 129, 64]), (ctx_small_bf16, [520, 70])):
        say(f"attention with late keys x{gain}, head_dim {m.head_dim}, lengths={lengths}")
        assert _attention_case(ctx, m, lengths, 5, late_key_gain=gain) < 3e-2


# ------------------------------------------------------------------ attention of the token-by-token path
@pytest.mark.parametrize("hq,hkv,hd", [(4, 4, 64), (4, 2, 64), (8, 2, 128), (32, 8, 128), (8, 1, 128), (16, 2, 64)])
def test_decode_attention_matches_oracle(hq, hkv, hd):
    say(f"decode attention hq={hq} hkv={hkv} hd={hd}")
    m = synth.small_model("bf16", n_layers=1, n_q_heads=hq, n_kv_heads=hkv, head_dim=hd, d_model=256)
    ctx = P.Context(H.c_cfg(m, 256, 16, 256), 0, 0)        # op calls need no weights
    try:
        rng = np.random.default_rng(hq * 100 + hkv * 10 + hd)
        n_keys = [1, 2, 63, 64, 65, 129, 512, 513, 1000, 3000]          # one query row per entry, caches back to back
        first = np.concatenate([[0], np.cumsum(n_keys)[:-1]]).astype(np.int64) + 7          # and not at row 0
        cache_rows = int(first[-1] + n_keys[-1] + 5)
        kvd = hkv * hd
        k_bits = synth.f32_to_bf16_bits((rng.standard_normal((cache_rows, kvd)) * 1.5).astype(np.float32))
        v_bits = synth.f32_to_bf16_bits(rng.standard_normal((cache_rows, kvd)).astype(np.float32))
        q_bits = synth.f32_to_bf16_bits((rng.standard_normal((len(n_keys), hq * hd)) * 1.5).astype(np.float32))
        d_q, d_k, d_v = H.to_dev(q_bits), H.to_dev(k_bits), H.to_dev(v_bits)
        d_o = torch.zeros((len(n_keys), hq * hd), dtype=torch.int16, device=H.DEV)
        ctx.vl_op_attention_decode_bf16(d_q.data_ptr(), d_k.data_ptr(), d_v.data_ptr(), cache_rows, first.tolist(), n_keys, d_o.data_ptr())
        got = O.upcast(H.bits_from_dev(d_o)).reshape(len(n_keys), hq, hd)
        kf, vf, qf = O.upcast(k_bits), O.upcast(v_bits), O.upcast(q_bits)
        worst = 0.0
        for r, (f0, t) in enumerate(zip(first.tolist(), n_keys)):
            ref = O.causal_attention(qf[r].reshape(1, hq, hd), kf[f0:f0 + t].reshape(t, hkv, hd), vf[f0:f0 + t].reshape(t, hkv, hd),
                                     np.array([t - 1]))[0]
            worst = max(worst, np.abs(got[r] - ref).max())
            # fp32 scores and sums; the only roundings of size are the output's bf16 (2^-9 relative of |o| <~ 4)
            np.testing.assert_allclose(got[r], ref, rtol=2 ** -8, atol=2e-3)
        print("  max abs err", worst, flush=True)
        with pytest.raises(P.VerilLMError) as e:
            ctx.vl_op_attention_decode_bf16(d_q.data_ptr(), d_k.data_ptr(), d_v.data_ptr(), cache_rows, [cache_rows - 3], [4], d_o.data_ptr())
        assert e.value.code == -1
    finally:
        ctx.close()


@pytest.mark.parametrize("hq,hkv,hd,rows", [(32, 8, 128, 64), (8, 1, 128, 256), (4, 2, 64, 128), (8, 2, 128, 70)])
def test_decode_attention_many_rows(hq, hkv, hd, rows):
    """With enough query rows one workgroup serves all (or half of) the query heads of a KV head; with few rows, as in the
    test above, every query head has a workgroup of its own.  Rows read overlapping windows of one cache."""
    say(f"decode attention hq={hq} hkv={hkv} hd={hd} rows={rows}")
    m = synth.small_model("bf16", n_layers=1, n_q_heads=hq, n_kv_heads=hkv, head_dim=hd, d_model=256)
    ctx = P.Context(H.c_cfg(m, 1024, 512, 256), 0, 0)
    try:
        rng = np.random.default_rng(rows * 1000 + hq * 100 + hkv * 10 + hd)
        cache_rows, kvd = 450, hkv * hd
        n_keys = rng.integers(1, 260, size=rows)
        n_keys[:4] = [1, 64, 65, 259]
        first = rng.integers(0, cache_rows - n_keys + 1)
        k_bits = synth.f32_to_bf16_bits((rng.standard_normal((cache_rows, kvd)) * 1.5).astype(np.float32))
        v_bits = synth.f32_to_bf16_bits(rng.standard_normal((cache_rows, kvd)).astype(np.float32))
        q_bits = synth.f32_to_bf16_bits((rng.standard_normal((rows, hq * hd)) * 1.5).astype(np.float32))
        d_q, d_k, d_v = H.to_dev(q_bits), H.to_dev(k_bits), H.to_dev(v_bits)
        d_o = torch.zeros((rows, hq * hd), dtype=torch.int16, device=H.DEV)
        ctx.vl_op_attention_decode_bf16(d_q.data_ptr(), d_k.data_ptr(), d_v.data_ptr(), cache_rows, first.tolist(), n_keys.tolist(),
                                        d_o.data_ptr())
        got = O.upcast(H.bits_from_dev(d_o)).reshape(rows, hq, hd)
        kf, vf, qf = O.upcast(k_bits), O.upcast(v_bits), O.upcast(q_bits)
        for r, (f0, t) in enumerate(zip(first.tolist(), n_keys.tolist())):
            ref = O.causal_attention(qf[r].reshape(1, hq, hd), kf[f0:f0 + t].reshape(t, hkv, hd), vf[f0:f0 + t].reshape(t, hkv, hd),
                                     np.array([t - 1]))[0]
            np.testing.assert_allclose(got[r], ref, rtol=2 ** -8, atol=2e-3)
    finally:
        ctx.close()


# ------------------------------------------------------------------ Merkle commitment (Section 5.6 / 5.7)
@pytest.mark.parametrize("d,dtype", [(256, "f32"), (256, "bf16"), (64, "f32"), (200, "bf16"), (4096, "bf16"), (8192, "f32"),
                                     (1000, "f32"), (16384, "bf16"), (264, "f32"), (72, "bf16"), (8200, "f32"), (8, "f32")])
def test_merkle_roots_and_openings_match_oracle(d, dtype):
    say(f"merkle d={d} dtype={dtype}")
    # the context only fixes d_model here (an fp32 model allows any multiple of 8); the state dtype is an argument
    m = synth.small_model("f32", n_layers=1, d_model=d, n_q_heads=1, n_kv_heads=1, head_dim=64, d_ffn=64)
    ctx = P.Context(H.c_cfg(m, 64, 4, 64), 0, 0)          # op calls need no weights
    try:
        rng = np.random.default_rng(d)
        rows = 5 if d >= 4096 else 19
        x = (rng.standard_normal((rows, d)) * 3).astype(np.float32)
        x[0, 0], x[0, 1], x[1, d - 1] = 0.0, -0.0, np.inf
        st = H.stored(x, dtype)
        d_s = H.to_dev(st)
        d_roots = torch.zeros((rows, 32), dtype=torch.uint8, device=H.DEV)
        ctx.vl_op_merkle_roots(d_s.data_ptr(), H.hidden_dtype_code(dtype), rows, d_roots.data_ptr())
        got = d_roots.cpu().numpy()
        ref = O.merkle_roots(st)
        np.testing.assert_array_equal(got, ref)                                    # bytes: bit-exact
        # openings: first, last, a middle element and the ragged edge
        sel_row = [0, rows - 1, rows // 2, 1, 2]
        sel_idx = [0, d - 1, d // 2, d - 2 if d > 1 else 0, (d // 3) | 1 if d > 3 else 0]
        depth = max(d - 1, 0).bit_length()
        d_paths = torch.full((len(sel_row), depth, 32), 7, dtype=torch.uint8, device=H.DEV)
        d_vals = torch.zeros(len(sel_row), dtype=torch.float32, device=H.DEV)
        lens = ctx.vl_op_merkle_open(d_s.data_ptr(), H.hidden_dtype_code(dtype), rows, sel_row, sel_idx, d_vals.data_ptr(), d_paths.data_ptr())
        paths, vals = d_paths.cpu().numpy(), d_vals.cpu().numpy()
        vals_ref = O.upcast(st).astype(np.float32)
        for q, (r, j) in enumerate(zip(sel_row, sel_idx)):
            want = O.merkle_open(st[r], j)
            assert lens[q] == len(want)
            assert [bytes(paths[q, k]) for k in range(lens[q])] == want
            assert not paths[q, lens[q]:].any()
            assert vals[q].tobytes() == vals_ref[r, j].tobytes()
            assert O.merkle_verify(bytes(got[r]), vals[q], j, d, [bytes(paths[q, k]) for k in range(lens[q])])
        with pytest.raises(P.VerilLMError) as e:
            ctx.vl_op_merkle_open(d_s.data_ptr(), H.hidden_dtype_code(dtype), rows, [rows], [0], 0, d_paths.data_ptr())
        assert e.value.code == -1
        with pytest.raises(P.VerilLMError) as e:
            ctx.vl_op_merkle_open(d_s.data_ptr(), H.hidden_dtype_code(dtype), rows, [0] * 65, [0] * 65, 0, d_paths.data_ptr())
        assert e.value.code == -3
    finally:
        ctx.close()
