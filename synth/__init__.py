"""Seeded synthetic inputs for the verification hot path.

This module only *draws inputs*: model shapes, random weights, token ids,
sequence lengths, tamper positions and tamper noise.  It holds none of the
method's arithmetic (no norm, no attention, no GEMM, no comparison), so that the
CPU oracle and the HIP library can both be fed from it without sharing any code
of the method itself.

Random streams are numpy PCG64 generators seeded by (seed, stream ids), so any
tensor can be drawn on demand, in any order, without holding the rest of the
model in memory (a 70B-shape layer is 1.7 GB in bf16).

Weight matrices are returned in [out_features, in_features] row-major order,
i.e. y = x @ W.T.  For bf16 models the returned array holds the bf16 bit patterns
(uint16) of N(0, sigma) draws rounded to nearest-even; both consumers upcast
those bits exactly, so both see identical weight *values*.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

# Tensor kinds (the numeric values are the ones the C header uses).
EMBED, ATTN_NORM, WQ, WK, WV, WO, FFN_NORM, W_GATE, W_UP, W_DOWN, FINAL_NORM, LM_HEAD = range(12)
KIND_NAMES = ["EMBED", "ATTN_NORM", "WQ", "WK", "WV", "WO", "FFN_NORM", "W_GATE", "W_UP",
              "W_DOWN", "FINAL_NORM", "LM_HEAD"]
PER_LAYER_KINDS = (ATTN_NORM, WQ, WK, WV, WO, FFN_NORM, W_GATE, W_UP, W_DOWN)
GLOBAL_KINDS = (EMBED, FINAL_NORM, LM_HEAD)
NORM_KINDS = (ATTN_NORM, FFN_NORM, FINAL_NORM)


@dataclasses.dataclass(frozen=True)
class ModelCfg:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    dtype: str = "f32"          # "f32" | "bf16": weights and GEMM operands
    sigma: float = 0.02         # std of every matrix (embedding and LM head included)
    seed: int = 1000
    random_gains: bool = False  # norm gains 1.0 exactly unless set (then 1 + 0.1 N(0,1))

    def shape(self, kind: int) -> Tuple[int, ...]:
        d, hq, hkv, hd, f, v = (self.d_model, self.n_q_heads, self.n_kv_heads, self.head_dim,
                                self.d_ffn, self.vocab)
        return {
            EMBED: (v, d), ATTN_NORM: (d,), WQ: (hq * hd, d), WK: (hkv * hd, d), WV: (hkv * hd, d),
            WO: (d, hq * hd), FFN_NORM: (d,), W_GATE: (f, d), W_UP: (f, d), W_DOWN: (d, f),
            FINAL_NORM: (d,), LM_HEAD: (v, d),
        }[kind]

    def n_params(self) -> int:
        per = sum(int(np.prod(self.shape(k))) for k in PER_LAYER_KINDS)
        glob = sum(int(np.prod(self.shape(k))) for k in GLOBAL_KINDS)
        return per * self.n_layers + glob

    def gemm_flops_per_token(self) -> float:
        mats = sum(int(np.prod(self.shape(k))) for k in (WQ, WK, WV, WO, W_GATE, W_UP, W_DOWN))
        return 2.0 * (mats * self.n_layers + int(np.prod(self.shape(LM_HEAD))))


@dataclasses.dataclass(frozen=True)
class Workload:
    """One verification job: a model shape, a batch of packed sequences, what was committed."""
    name: str
    model: ModelCfg
    lengths: Tuple[int, ...]            # total length of each sequence (prompt + generated)
    prompt_lens: Tuple[int, ...]
    commit_layers: Tuple[int, ...]      # 1-based, ascending
    check_argmax: bool
    hidden_dtype: str                   # dtype commitments are stored in: "f32" | "bf16"
    tamper_count: int
    tamper_mode: str                    # "abs": h += 0.5 N(0,1); "rel": h += kappa rms(h) N(0,1)
    tol_rel_l2: float
    tol_max_abs: float
    tol_logit_margin: float
    token_seed: int = 2000
    tamper_seed: int = 3000

    @property
    def n_tokens(self) -> int:
        return int(sum(self.lengths))


# ----------------------------------------------------------------------------------------------
# bf16 bit patterns (storage format only)
# ----------------------------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact upcast of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------------------------
# random streams
# ----------------------------------------------------------------------------------------------

_ROW_CHUNK = 1024  # rows drawn per random stream; fixes the values independently of threading
_LUT_CACHE: Dict[Tuple[float, bool], np.ndarray] = {}


def _rng(seed: int, *stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed)] + [int(s) for s in stream])))


def _normal_lut(sigma: float, as_bf16: bool) -> np.ndarray:
    """65536 equiprobable quantile midpoints of N(0, sigma): a uniform 16-bit draw indexes a normal draw.

    Drawing through a table is an order of magnitude faster than a float normal sampler, which matters
    for the 8e9- and 70e9-parameter shapes.  The tails stop at about 4.2 sigma.
    """
    key = (float(sigma), bool(as_bf16))
    if key not in _LUT_CACHE:
        from scipy.special import ndtri
        q = (float(sigma) * ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)).astype(np.float32)
        _LUT_CACHE[key] = f32_to_bf16_bits(q) if as_bf16 else q
    return _LUT_CACHE[key]


def weight(model: ModelCfg, kind: int, layer: int = 0, threads: int = 8) -> np.ndarray:
    """Tensor `kind` of `layer` (0-based; ignored for the global tensors).

    f32 model: float32 values.  bf16 model: uint16 bf16 bit patterns.
    Norm gains are float32 for both.
    """
    shape = model.shape(kind)
    if kind in NORM_KINDS:
        if not model.random_gains:
            return np.ones(shape, dtype=np.float32)
        g = _rng(model.seed, kind, layer + 1, 0)
        return (1.0 + 0.1 * g.standard_normal(shape)).astype(np.float32)
    rows, cols = shape
    chunks = [(c, min(_ROW_CHUNK, rows - c * _ROW_CHUNK)) for c in range((rows + _ROW_CHUNK - 1) // _ROW_CHUNK)]
    as_bf16 = model.dtype == "bf16"
    lut = _normal_lut(model.sigma, as_bf16)
    out = np.empty(shape, dtype=lut.dtype)

    def fill(item):
        c, n = item
        bg = np.random.PCG64(np.random.SeedSequence([int(model.seed), int(kind), int(layer) + 1, int(c)]))
        cnt = n * cols
        raw = bg.random_raw((cnt + 3) // 4).view(np.uint16)[:cnt]
        r0 = c * _ROW_CHUNK
        np.take(lut, raw, out=out[r0:r0 + n].reshape(-1), mode="wrap")

    if threads > 1 and len(chunks) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, chunks))
    else:
        for it in chunks:
            fill(it)
    return out


def weight_values_f32(model: ModelCfg, kind: int, layer: int = 0, threads: int = 8) -> np.ndarray:
    """The weight *values* as float32 (exact for both storage types)."""
    w = weight(model, kind, layer, threads)
    return bf16_bits_to_f32(w) if w.dtype == np.uint16 else w


def tokens(wl: Workload) -> np.ndarray:
    """Packed token ids, uniform in [0, vocab), int32 [N]."""
    g = _rng(wl.token_seed, 1)
    return g.integers(0, wl.model.vocab, size=wl.n_tokens, dtype=np.int32)


def draw_lengths(seed: int, n_seqs: int, lo: int, hi: int) -> Tuple[int, ...]:
    """Sequence lengths uniform in [lo, hi] (inclusive)."""
    g = _rng(seed, 2)
    return tuple(int(v) for v in g.integers(lo, hi + 1, size=n_seqs))


def cu_seqlens(lengths: Sequence[int]) -> np.ndarray:
    return np.concatenate([[0], np.cumsum(np.asarray(lengths, dtype=np.int64))]).astype(np.int64)


def tamper_positions(wl: Workload, n_tokens: Optional[int] = None, count: Optional[int] = None) -> np.ndarray:
    """Sorted distinct packed positions to tamper (int64)."""
    n = wl.n_tokens if n_tokens is None else n_tokens
    k = wl.tamper_count if count is None else count
    k = min(k, n)
    g = _rng(wl.tamper_seed, 3)
    return np.sort(g.choice(n, size=k, replace=False)).astype(np.int64)


def tamper_hidden(wl: Workload, committed: np.ndarray, positions: np.ndarray, kappa: float = 1.0) -> np.ndarray:
    """Return a float32 copy of `committed` [C, N, d] with noise added at `positions` (every layer).

    mode "abs": + 0.5 * N(0,1) per element.
    mode "rel": + kappa * rms(row) * N(0,1) per element, rms taken over the row being perturbed.
    """
    out = np.array(committed, dtype=np.float32, copy=True)
    c, _, d = out.shape
    g = _rng(wl.tamper_seed, 4)
    noise = g.standard_normal((c, len(positions), d), dtype=np.float32)
    for ci in range(c):
        rows = out[ci, positions, :]
        if wl.tamper_mode == "abs":
            scale = np.float32(0.5)
            out[ci, positions, :] = rows + scale * noise[ci]
        else:
            rms = np.sqrt(np.mean(rows.astype(np.float64) ** 2, axis=1, keepdims=True)).astype(np.float32)
            out[ci, positions, :] = rows + np.float32(kappa) * rms * noise[ci]
    return out


def tamper_argmax(wl: Workload, committed_argmax: np.ndarray, positions: np.ndarray,
                  wrong_tokens: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Replace the committed argmax at every second tampered position.

    Returns (new int32 array, the positions that were changed).  `wrong_tokens[n]`, if given, is the
    token to write at position n; otherwise a different token is drawn at random.
    """
    out = np.array(committed_argmax, dtype=np.int32, copy=True)
    chosen = positions[::2]
    g = _rng(wl.tamper_seed, 5)
    shift = g.integers(1, wl.model.vocab, size=len(chosen), dtype=np.int64)
    for i, p in enumerate(chosen):
        if wrong_tokens is not None:
            out[p] = np.int32(wrong_tokens[p])
        else:
            out[p] = np.int32((int(out[p]) + int(shift[i])) % wl.model.vocab)
    return out, np.asarray(chosen, dtype=np.int64)


# ----------------------------------------------------------------------------------------------
# model shapes and workloads
# ----------------------------------------------------------------------------------------------

TINY_F32 = ModelCfg("tiny-f32", 2, 256, 4, 4, 64, 688, 4096, 1e-5, 10000.0, "f32", 0.02, seed=1001)
LLAMA8B = ModelCfg("8b-shape", 32, 4096, 32, 8, 128, 14336, 128256, 1e-5, 500000.0, "bf16", 0.02, seed=1002)
LLAMA70B = ModelCfg("70b-shape", 80, 8192, 64, 8, 128, 28672, 128256, 1e-5, 500000.0, "bf16", 0.01, seed=1005)

INF = float("inf")


def _count(frac: float, n: int) -> int:
    return max(1, int(round(frac * n))) if frac > 0 else 0


def workload(idx: int) -> Workload:
    """The five evaluation workloads (idx 0..4)."""
    if idx == 0:
        return Workload("cfg0-tiny-f32", TINY_F32, (128,), (64,), (1, 2), True, "f32", 4, "abs",
                        1e-3, INF, 1e-3, 2001, 3001)
    if idx == 1:
        n = 8 * 1024
        return Workload("cfg1-8b-b8x1024", LLAMA8B, (1024,) * 8, (512,) * 8, (8, 16, 24, 32), True, "bf16",
                        _count(0.01, n), "rel", 1e-1, INF, 0.25, 2002, 3002)
    if idx == 2:
        lens = draw_lengths(4003, 64, 64, 256)
        n = sum(lens)
        return Workload("cfg2-8b-varlen64", LLAMA8B, lens, tuple(t // 2 for t in lens), (32,), False, "bf16",
                        _count(0.001, n), "rel", 1e-1, INF, 0.25, 2003, 3003)
    if idx == 3:
        n = 2 * 9216
        return Workload("cfg3-8b-long9216", LLAMA8B, (9216,) * 2, (8192,) * 2, tuple(range(4, 33, 4)), True,
                        "bf16", _count(0.01, n), "rel", 1e-1, INF, 0.25, 2004, 3004)
    if idx == 4:
        n = 4 * 2048
        return Workload("cfg4-70b-b4x2048", LLAMA70B, (2048,) * 4, (1024,) * 4, (20, 40, 60, 80), True, "bf16",
                        _count(0.01, n), "rel", 1e-1, INF, 0.25, 2005, 3005)
    raise IndexError(idx)


def small_model(dtype: str = "bf16", **kw) -> ModelCfg:
    """A small GQA model for tests (dims are multiples of 64 so every GPU tile path is legal)."""
    base = dict(name="small-" + dtype, n_layers=3, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64,
                d_ffn=512, vocab=1000, rms_eps=1e-5, rope_base=10000.0, dtype=dtype, sigma=0.05, seed=77)
    base.update(kw)
    return ModelCfg(**base)


def small_workload(model: ModelCfg, lengths: Sequence[int], commit_layers: Sequence[int],
                   check_argmax: bool = True, tamper_count: int = 3, seed: int = 0,
                   hidden_dtype: Optional[str] = None) -> Workload:
    bf = model.dtype == "bf16"
    return Workload("small", model, tuple(int(t) for t in lengths), tuple(int(t) // 2 for t in lengths),
                    tuple(commit_layers), check_argmax, hidden_dtype or ("bf16" if bf else "f32"),
                    tamper_count, "rel" if bf else "abs",
                    1e-1 if bf else 1e-3, INF, 0.25 if bf else 1e-3, 2100 + seed, 3100 + seed)


class WeightStream:
    """Draws tensors on demand; keeps at most the most recent layer's tensors alive."""

    def __init__(self, model: ModelCfg, threads: int = 8):
        self.model = model
        self.threads = threads

    def raw(self, kind: int, layer: int = 0) -> np.ndarray:
        return weight(self.model, kind, layer, self.threads)

    def values(self, kind: int, layer: int = 0) -> np.ndarray:
        return weight_values_f32(self.model, kind, layer, self.threads)
