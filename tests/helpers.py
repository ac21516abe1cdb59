"""Shared plumbing for the GPU tests: contexts fed from the seeded generators, oracle models, device buffers.

PyTorch appears here only to hold device memory; every computation under test happens inside libverillm.so,
every expected value comes from oracle/.
"""
from __future__ import annotations

import ctypes as C
import math

import numpy as np
import torch

import paper_2509_24257_amd as P
import synth
from oracle import verillm_oracle as O

DEV = "cuda:0"


CAPTURE_MANAGER = None      # set by conftest.py


def progress(msg: str):
    """One line that names the step about to run, written past pytest's output capture: a long GPU test must show
    what it is doing while it runs (a faulting kernel can take the captured text with it, and a quiet run looks hung)."""
    cm = CAPTURE_MANAGER
    if cm is not None:
        with cm.global_and_fixture_disabled():
            print(msg, flush=True)
    else:
        print(msg, flush=True)


def c_cfg(m: synth.ModelCfg, max_tokens: int, max_seqs: int, max_seq_len: int) -> P.ModelCfg:
    return P.ModelCfg(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn, m.vocab, m.rms_eps,
                      m.rope_base, P.VL_BF16 if m.dtype == "bf16" else P.VL_F32, max_tokens, max_seqs, max_seq_len)


def load_all_weights(ctx: P.Context, m: synth.ModelCfg, threads: int = 16, override=None):
    override = override or {}

    def put(kind, layer):
        w = override.get((kind, layer))
        if w is None:
            w = synth.weight(m, kind, layer, threads)
        w = np.ascontiguousarray(w)
        ctx.vl_load_weights(kind, layer, w.ctypes.data, w.nbytes)

    for k in synth.GLOBAL_KINDS:
        put(k, 0)
    for l in range(m.n_layers):
        for k in synth.PER_LAYER_KINDS:
            put(k, l)


def make_ctx(m: synth.ModelCfg, max_tokens: int, max_seqs: int, max_seq_len: int, override=None) -> P.Context:
    ctx = P.Context(c_cfg(m, max_tokens, max_seqs, max_seq_len), 0, 0)
    load_all_weights(ctx, m, override=override)
    return ctx


def oracle_model(m: synth.ModelCfg, override=None, progress: str = "", operand_dtype=None) -> O.Model:
    override = override or {}

    def w(kind, layer):
        if progress and kind == synth.ATTN_NORM and layer % 8 == 0:
            globals()["progress"]("[oracle %s] layer %d/%d" % (progress, layer, m.n_layers))
        if (kind, layer) in override:
            return override[(kind, layer)]
        return synth.weight(m, kind, layer, 16)

    return O.Model(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn, m.vocab, m.rms_eps,
                   m.rope_base, w, operand_dtype=operand_dtype)


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy -> device tensor; uint16 arrays (bf16 bit patterns) travel as int16."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def bits_from_dev(t: torch.Tensor) -> np.ndarray:
    """device int16 tensor holding bf16 bit patterns -> numpy uint16."""
    return t.cpu().numpy().view(np.uint16)


def hidden_dtype_code(name: str) -> int:
    return P.VL_BF16 if name == "bf16" else P.VL_F32


def stored(committed_f32: np.ndarray, hidden_dtype: str) -> np.ndarray:
    """Commitments in their stored dtype: float32 as is, bf16 as bit patterns (round to nearest even)."""
    if hidden_dtype == "bf16":
        return synth.f32_to_bf16_bits(committed_f32)
    return np.ascontiguousarray(committed_f32, dtype=np.float32)


def stats_from_dev(t: torch.Tensor) -> dict:
    a = t.cpu().numpy().reshape(-1, 4)
    return {"rel_l2": a[:, 0], "max_abs": a[:, 1], "mean_abs": a[:, 2], "mean_signed": a[:, 3]}


def run_verify(ctx: P.Context, wl: synth.Workload, tokens: np.ndarray, committed_stored: np.ndarray,
               committed_argmax, tol=None):
    """Calls vl_verify_prefill; returns (flags uint8 [N], stats list over C of dicts, summary dict)."""
    n = int(sum(wl.lengths))
    c = len(wl.commit_layers)
    d_tok = to_dev(tokens.astype(np.int32))
    d_com = to_dev(committed_stored)
    d_cam = to_dev(np.asarray(committed_argmax, dtype=np.int32)) if committed_argmax is not None else None
    d_flags = torch.zeros(max(n, 1), dtype=torch.uint8, device=DEV)
    d_stats = torch.zeros(max(c * n, 1) * 4, dtype=torch.float32, device=DEV)
    tol = tol or P.Tol(wl.tol_rel_l2, wl.tol_max_abs, wl.tol_logit_margin)
    sm = ctx.vl_verify_prefill(d_tok.data_ptr(), wl.lengths, wl.commit_layers, d_com.data_ptr(),
                               hidden_dtype_code(wl.hidden_dtype), d_cam.data_ptr() if d_cam is not None else 0, tol,
                               d_flags.data_ptr(), d_stats.data_ptr())
    st = d_stats.cpu().numpy()[: c * n * 4].reshape(c, n, 4)
    stats = [{"rel_l2": st[i, :, 0], "max_abs": st[i, :, 1], "mean_abs": st[i, :, 2], "mean_signed": st[i, :, 3]}
             for i in range(c)]
    return d_flags.cpu().numpy()[:n], stats, sm.as_dict()


def run_verify_segment(ctx: P.Context, wl: synth.Workload, tokens, start_layer: int, end_layer: int, upstream_stored,
                       commit_layers, committed_stored: np.ndarray, committed_argmax, tol=None):
    """Calls vl_verify_segment; upstream/committed arrays are in the workload's stored dtype.  Same returns as run_verify."""
    n = int(sum(wl.lengths))
    c = len(commit_layers)
    d_tok = to_dev(np.asarray(tokens).astype(np.int32)) if tokens is not None else None
    d_up = to_dev(upstream_stored) if upstream_stored is not None else None
    d_com = to_dev(committed_stored)
    d_cam = to_dev(np.asarray(committed_argmax, dtype=np.int32)) if committed_argmax is not None else None
    d_flags = torch.zeros(max(n, 1), dtype=torch.uint8, device=DEV)
    d_stats = torch.zeros(max(c * n, 1) * 4, dtype=torch.float32, device=DEV)
    tol = tol or P.Tol(wl.tol_rel_l2, wl.tol_max_abs, wl.tol_logit_margin)
    code = hidden_dtype_code(wl.hidden_dtype)
    sm = ctx.vl_verify_segment(start_layer, end_layer, d_up.data_ptr() if d_up is not None else 0, code,
                               d_tok.data_ptr() if d_tok is not None else 0, wl.lengths, list(commit_layers), d_com.data_ptr(), code,
                               d_cam.data_ptr() if d_cam is not None else 0, tol, d_flags.data_ptr(), d_stats.data_ptr())
    st = d_stats.cpu().numpy()[: c * n * 4].reshape(c, n, 4)
    stats = [{"rel_l2": st[i, :, 0], "max_abs": st[i, :, 1], "mean_abs": st[i, :, 2], "mean_signed": st[i, :, 3]}
             for i in range(c)]
    return d_flags.cpu().numpy()[:n], stats, sm.as_dict()


def run_commit(ctx: P.Context, wl: synth.Workload, tokens: np.ndarray, mode: str, prompt_lens=None,
               want_argmax: bool = True):
    """vl_prefill_commit (mode 'prefill') or vl_decode_commit (mode 'decode').
    Returns (hidden float32 [C, N, d] upcast from the stored dtype, stored array, argmax int32 [N] or None)."""
    n = int(sum(wl.lengths))
    c = len(wl.commit_layers)
    d = wl.model.d_model
    d_tok = to_dev(tokens.astype(np.int32))
    bf = wl.hidden_dtype == "bf16"
    d_hid = torch.zeros((c, n, d), dtype=torch.int16 if bf else torch.float32, device=DEV)
    d_arg = torch.full((n,), -7, dtype=torch.int32, device=DEV) if want_argmax else None
    if mode == "prefill":
        ctx.vl_prefill_commit(d_tok.data_ptr(), wl.lengths, wl.commit_layers, d_hid.data_ptr(),
                              hidden_dtype_code(wl.hidden_dtype), d_arg.data_ptr() if want_argmax else 0)
    else:
        ctx.vl_decode_commit(d_tok.data_ptr(), wl.lengths, prompt_lens, wl.commit_layers, d_hid.data_ptr(),
                             hidden_dtype_code(wl.hidden_dtype), d_arg.data_ptr() if want_argmax else 0)
    if bf:
        st = bits_from_dev(d_hid)
        val = synth.bf16_bits_to_f32(st)
    else:
        st = d_hid.cpu().numpy()
        val = st
    return val, st, (d_arg.cpu().numpy() if want_argmax else None)


def get_logits(ctx: P.Context, lo: int, hi: int, vocab: int) -> np.ndarray:
    out = torch.empty((hi - lo, vocab), dtype=torch.float32, device=DEV)
    ctx.vl_get_logits(lo, hi, out.data_ptr())
    return out.cpu().numpy()


def get_argmax(ctx: P.Context, lo: int, hi: int):
    a = torch.empty(hi - lo, dtype=torch.int32, device=DEV)
    g = torch.empty(hi - lo, dtype=torch.float32, device=DEV)
    ctx.vl_get_argmax(lo, hi, a.data_ptr(), g.data_ptr())
    return a.cpu().numpy(), g.cpu().numpy()


def rel_l2_rows(a: np.ndarray, ref: np.ndarray) -> np.ndarray:
    a = np.asarray(a, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return np.linalg.norm(a - ref, axis=-1) / np.maximum(np.linalg.norm(ref, axis=-1), 1e-30)
