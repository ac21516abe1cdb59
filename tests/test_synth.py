"""The seeded input generators: determinism, formats, and the recipe of the five workloads."""
import numpy as np
import torch

import synth


def test_bf16_rounding_is_nearest_even_like_torch():
    x = (np.random.default_rng(1).standard_normal(200000) * 3).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]      # exact ties: round to even mantissa
    mine = synth.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(mine, ref)
    np.testing.assert_array_equal(synth.bf16_bits_to_f32(mine[:4]), [1.0, 1.015625, -1.0, 0.0])


def test_weights_are_reproducible_and_thread_independent():
    m = synth.small_model("bf16")
    a = synth.weight(m, synth.W_UP, 1, threads=1)
    b = synth.weight(m, synth.W_UP, 1, threads=4)
    np.testing.assert_array_equal(a, b)
    assert a.dtype == np.uint16 and a.shape == (512, 256)
    assert not np.array_equal(a, synth.weight(m, synth.W_UP, 2, threads=1))
    assert not np.array_equal(a, synth.weight(m, synth.W_GATE, 1, threads=1))
    v = synth.bf16_bits_to_f32(synth.weight(synth.ModelCfg("x", 1, 512, 4, 4, 128, 1024, 64, dtype="bf16", sigma=0.02),
                                            synth.W_GATE, 0))
    assert abs(v.std() - 0.02) < 2e-4 and abs(v.mean()) < 2e-4
    f = synth.weight(synth.TINY_F32, synth.WQ, 0)
    assert f.dtype == np.float32 and abs(f.std() - 0.02) < 5e-4
    assert (synth.weight(synth.TINY_F32, synth.ATTN_NORM, 0) == 1.0).all()


def test_workload_recipes():
    w0, w1, w2, w3, w4 = (synth.workload(i) for i in range(5))
    assert w0.n_tokens == 128 and w0.model.dtype == "f32" and w0.commit_layers == (1, 2) and w0.tamper_count == 4
    assert w1.n_tokens == 8192 and w1.commit_layers == (8, 16, 24, 32) and w1.tamper_count == 82
    assert len(w2.lengths) == 64 and min(w2.lengths) >= 64 and max(w2.lengths) <= 256 and not w2.check_argmax
    assert w2.commit_layers == (32,) and w2.tamper_count == round(0.001 * w2.n_tokens)
    assert w3.lengths == (9216, 9216) and w3.commit_layers == (4, 8, 12, 16, 20, 24, 28, 32)
    assert w4.model.n_layers == 80 and w4.n_tokens == 8192 and w4.model.sigma == 0.01
    assert abs(w1.model.gemm_flops_per_token() / 1e9 - 15.01) < 0.01
    assert abs(w4.model.gemm_flops_per_token() / 1e9 - 139.0) < 0.05
    t = synth.tokens(w1)
    assert t.dtype == np.int32 and t.min() >= 0 and t.max() < 128256 and len(t) == 8192
    p = synth.tamper_positions(w1)
    assert len(np.unique(p)) == 82 and p.max() < 8192


def test_tamper_is_large_against_tolerance():
    m = synth.small_model("bf16")
    wl = synth.small_workload(m, [40, 24], [3], tamper_count=5)
    h = (np.random.default_rng(0).standard_normal((1, 64, 256)) * 4).astype(np.float32)
    pos = synth.tamper_positions(wl)
    t = synth.tamper_hidden(wl, h, pos)
    untouched = np.setdiff1d(np.arange(64), pos)
    np.testing.assert_array_equal(t[0, untouched], h[0, untouched])
    rel = np.linalg.norm(t[0, pos] - h[0, pos], axis=1) / np.linalg.norm(h[0, pos], axis=1)
    assert (rel > 0.8).all()          # kappa = 1: about 10x the 0.1 tolerance
    a = np.arange(64, dtype=np.int32)
    b, changed = synth.tamper_argmax(wl, a, pos)
    assert (b[changed] != a[changed]).all() and len(changed) == 3
