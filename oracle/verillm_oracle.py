"""CPU oracle for the verification hot path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this file; it exists so that tests, the smoke check and the
benchmark's CPU-baseline leg can compare the GPU library against a plain, slow, obviously correct
implementation.  It shares no code with the GPU library.  Everything is float64 numpy; a matrix
product is `@`, everything else is written out as the definition states it, with no blocking,
fusion or reordering.

What it computes, following the paper:

* Section 4 "Full-Sequence Prefill for Parallel Verification", Eq. (1): the verifier runs ONE
  causal forward pass over the concatenated prompt and output tokens and thereby recovers the
  hidden state of every position, H' = F_theta(X_prompt || X_output)          -> `prefill`.
* Section 5.5 "Inference Scheme" (the three-line recurrence S_1 = Embed(x), S_{i+1} = F_i(S_i; W_i),
  y = Decode(S_{L+1})): the inferencer produces the same states one token at a time and logs
  them at the segment boundaries                                                -> `decode`.
* Section 5.7 "Comparison and On-Chain Commitment": Delta = S_hat - S elementwise, a per-token scalar
  phi(Delta) (mean absolute error is the paper's example), a statistic Psi across tokens (mean),
  a verdict 1[T_v <= tau]                                                       -> `compare_hidden`,
  `summary`.
* Section 5.7, the TokenMatch equation: argmax of the LM head applied to the recomputed last-layer
  state must reproduce the claimed token                                        -> `token_check`.

The paper never spells out the transformer block F_i; the block here is the Llama-style pre-norm
block that the evaluation shapes fix (RMSNorm, rotary embedding on half-split pairs, grouped-query
causal attention scaled by 1/sqrt(head_dim), SwiGLU feed-forward, no biases, untied LM head, final
RMSNorm).  The "hidden state after layer l" is the residual stream leaving block l, before any
following norm, for every l including the last.

* Section 7 "Bit-aware statistical comparison" (P_e, P_m, P_w, mean discrepancy and their calibrated
  thresholds) and the offline test battery of Appendix A.1 (P_exp, Q_small, Z_large, MAE)
                                                                                -> `bit_compare`, `bit_rule`.
* Section 5.6 "Commitment Submission" / Section 5.7 MerkleVerify: a SHA-256 Merkle tree over the canonical
  float32 scalars of a state, its root, inclusion proofs and their check    -> `merkle_root`, `merkle_open`,
  `merkle_verify`.

Readings that go beyond the paper (per-token relative L2 and max-abs instead of one verdict per
segment; a logit margin for near-tied argmax) are documented where they are implemented.

Precision.  By default nothing is rounded: float64 throughout.  The paper does not fix a compute
precision; the bf16 evaluation shapes do ("bf16" = every matrix-product operand is a bf16 value).
`Model(..., operand_dtype="bf16")` states that reading: the normalised activations, the projected
q/k/v (again after the rotary embedding), the softmax numerators entering the value product, the
attention output and the SwiGLU output are each rounded to bf16 (nearest, ties to even) where they
become an operand of the next matrix product; all sums, norms and softmax statistics stay float64.
It changes no formula and no order, only inserts roundings, and it exists so that a bf16
implementation can be checked far more tightly than against the unrounded model.

Pins: every function below is pinned by tests/test_oracle_*.py against closed forms, invariants
(token-by-token decode equals prefill; causality; batch independence), library routines
(torch's scaled_dot_product_attention, rms_norm, silu; the `transformers` Llama model on a tiny
random model) and a scalar-loop brute force.  The values at the full 8B/70B shapes are "parity
unpinned" by the paper itself (it prints no activations); they rest on the same code being pinned at
small shapes.
"""
from __future__ import annotations

import math
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

# tensor kinds: same numbering as the library's public header (an interface, not shared code)
EMBED, ATTN_NORM, WQ, WK, WV, WO, FFN_NORM, W_GATE, W_UP, W_DOWN, FINAL_NORM, LM_HEAD = range(12)

WeightFn = Callable[[int, int], np.ndarray]   # (kind, layer0) -> array; matrices are [out, in]

TINY = 1e-30


# ------------------------------------------------------------------------------------------------
# storage formats
# ------------------------------------------------------------------------------------------------

def upcast(a: np.ndarray) -> np.ndarray:
    """Exact conversion of a stored tensor to float64 (uint16 arrays hold bf16 bit patterns)."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16 value (ties to even) and return it as float64.  Finite inputs only."""
    f = np.ascontiguousarray(a, dtype=np.float64).astype(np.float32)       # float64 -> float32 is itself nearest-even
    # a double rounding float64 -> float32 -> bf16 can differ from a direct one only when the float32 result lands
    # exactly on a bf16 tie, i.e. for a 2^-16 fraction of inputs, by one bf16 ulp: far below every tolerance used
    u = f.view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


# ------------------------------------------------------------------------------------------------
# building blocks of F_i
# ------------------------------------------------------------------------------------------------

def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * gain, row by row."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, dtype=np.float64)


def rope_angles(positions: np.ndarray, head_dim: int, base: float) -> np.ndarray:
    """angle[t, i] = pos_t * base^(-2i/head_dim), i in [0, head_dim/2)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = np.power(float(base), -2.0 * i / float(head_dim))
    return np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]


def apply_rope(x: np.ndarray, positions: np.ndarray, base: float) -> np.ndarray:
    """Rotate the pairs (i, i + head_dim/2) of x [T, heads, head_dim] by the position's angles."""
    t, h, hd = x.shape
    half = hd // 2
    ang = rope_angles(positions, hd, base)
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    x1 = x[..., :half]
    x2 = x[..., half:]
    out = np.empty_like(x, dtype=np.float64)
    out[..., :half] = x1 * c - x2 * s
    out[..., half:] = x2 * c + x1 * s
    return out


def softmax_rows(s: np.ndarray) -> np.ndarray:
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_positions: np.ndarray,
                     round_probs=None) -> np.ndarray:
    """Grouped-query causal attention for one sequence.

    q [Tq, Hq, hd]; k, v [Tk, Hkv, hd] hold keys/values of positions 0..Tk-1; query row r sits at
    position q_positions[r] and attends to keys j <= q_positions[r].  Q head j uses KV head
    j // (Hq / Hkv).  Scores are scaled by 1/sqrt(hd).  `round_probs`, if given, is applied to the softmax
    numerators exp(s - max) that multiply the values; the normaliser is the sum of the unrounded numerators.
    """
    tq, hq, hd = q.shape
    tk, hkv, _ = k.shape
    group = hq // hkv
    scale = 1.0 / math.sqrt(hd)
    out = np.empty((tq, hq, hd), dtype=np.float64)
    key_pos = np.arange(tk)
    allowed = key_pos[None, :] <= np.asarray(q_positions)[:, None]          # [Tq, Tk]
    for j in range(hq):
        g = j // group
        s = (q[:, j, :] @ k[:, g, :].T) * scale
        s = np.where(allowed, s, -np.inf)
        if round_probs is None:
            out[:, j, :] = softmax_rows(s) @ v[:, g, :]
        else:
            e = np.exp(s - np.max(s, axis=-1, keepdims=True))
            out[:, j, :] = (round_probs(e) @ v[:, g, :]) / np.sum(e, axis=-1, keepdims=True)
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def argmax_lowest(z: np.ndarray) -> np.ndarray:
    """Row argmax; among equal maxima the lowest index."""
    return np.argmax(z, axis=-1).astype(np.int64)   # numpy returns the first occurrence


# ------------------------------------------------------------------------------------------------
# the model F_theta
# ------------------------------------------------------------------------------------------------

class Model:
    """Shape + weight source.  `weights(kind, layer0)` returns the stored tensor; it is upcast here."""

    def __init__(self, n_layers: int, d_model: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                 d_ffn: int, vocab: int, rms_eps: float, rope_base: float, weights: WeightFn,
                 operand_dtype: Optional[str] = None):
        self.L, self.d, self.hq, self.hkv, self.hd = n_layers, d_model, n_q_heads, n_kv_heads, head_dim
        self.f, self.v, self.eps, self.base = d_ffn, vocab, float(rms_eps), float(rope_base)
        self._w = weights
        assert operand_dtype in (None, "bf16")
        self.operand_dtype = operand_dtype

    def rnd(self, a: np.ndarray) -> np.ndarray:
        """Rounding applied where a tensor becomes a matrix-product operand (identity unless operand_dtype is set)."""
        return round_bf16(a) if self.operand_dtype == "bf16" else a

    def w(self, kind: int, layer: int = 0) -> np.ndarray:
        return upcast(self._w(kind, layer))


def _layer_weights(m: Model, l: int) -> Dict[int, np.ndarray]:
    return {k: m.w(k, l) for k in (ATTN_NORM, WQ, WK, WV, WO, FFN_NORM, W_GATE, W_UP, W_DOWN)}


def _block(m: Model, w: Dict[int, np.ndarray], h: np.ndarray, positions: np.ndarray,
           k_all: Optional[np.ndarray], v_all: Optional[np.ndarray]):
    """One block F_l on rows h [T, d] at `positions`; k_all/v_all are earlier keys/values (or None).

    Returns (new h, keys, values) with keys/values covering positions 0..max(positions).
    """
    t = h.shape[0]
    u = m.rnd(rmsnorm(h, w[ATTN_NORM], m.eps))
    q = m.rnd(u @ w[WQ].T).reshape(t, m.hq, m.hd)
    k = m.rnd(u @ w[WK].T).reshape(t, m.hkv, m.hd)
    v = m.rnd(u @ w[WV].T).reshape(t, m.hkv, m.hd)
    q = m.rnd(apply_rope(q, positions, m.base))
    k = m.rnd(apply_rope(k, positions, m.base))
    if k_all is not None:
        k = np.concatenate([k_all, k], axis=0)
        v = np.concatenate([v_all, v], axis=0)
    o = causal_attention(q, k, v, positions, round_probs=m.rnd if m.operand_dtype else None)
    o = m.rnd(o).reshape(t, m.hq * m.hd)
    h1 = h + o @ w[WO].T
    x = m.rnd(rmsnorm(h1, w[FFN_NORM], m.eps))
    act = m.rnd(silu(x @ w[W_GATE].T) * (x @ w[W_UP].T))
    h2 = h1 + act @ w[W_DOWN].T
    return h2, k, v


def lm_head(m: Model, h_last: np.ndarray) -> np.ndarray:
    """Decode head: logits = RMSNorm(h^L; g_final) @ W_lm^T."""
    return m.rnd(rmsnorm(h_last, m.w(FINAL_NORM), m.eps)) @ m.w(LM_HEAD).T


def prefill(m: Model, tokens: np.ndarray, lengths: Sequence[int], commit_layers: Sequence[int],
            want_logits: bool = True, start_layer: int = 0, start_hidden: Optional[np.ndarray] = None,
            end_layer: Optional[int] = None):
    """Teacher-forced causal forward over packed sequences (Section 4, Eq. (1)).

    tokens int [N] packed back to back, lengths [B].  Returns (hidden {layer: [N, d]}, logits [N, V] or
    None).  Layers are walked outermost so that only one layer's weights are alive at a time; each
    sequence is processed on its own (sequences never interact).

    `start_layer`/`start_hidden`/`end_layer` give the segment-local form of Section 5.6: begin from
    recorded states entering block start_layer+1 instead of from the embedding, stop after block
    end_layer.
    """
    tokens = np.asarray(tokens)
    n = int(np.sum(lengths))
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    end_layer = m.L if end_layer is None else end_layer
    if start_hidden is None:
        emb = m.w(EMBED)
        h = emb[tokens[:n]]
        del emb
    else:
        h = np.array(start_hidden, dtype=np.float64)
    hidden: Dict[int, np.ndarray] = {}
    for l in range(start_layer, end_layer):
        w = _layer_weights(m, l)
        nxt = np.empty_like(h)
        for b in range(len(lengths)):
            lo, hi = int(cu[b]), int(cu[b + 1])
            if hi == lo:
                continue
            pos = np.arange(hi - lo)
            nxt[lo:hi], _, _ = _block(m, w, h[lo:hi], pos, None, None)
        h = nxt
        if (l + 1) in commit_layers:
            hidden[l + 1] = h.copy()
    logits = lm_head(m, h) if (want_logits and end_layer == m.L) else None
    return hidden, logits


def decode(m: Model, tokens: np.ndarray, lengths: Sequence[int], commit_layers: Sequence[int],
           want_logits: bool = True):
    """Token-by-token generation-order forward with a KV cache (Section 5.5 recurrence).

    Teacher-forced on `tokens`.  Every step processes ONE position of one sequence against the keys and
    values cached from its earlier positions.  All layer weights are held (small models only).
    Returns the same structure as `prefill`.
    """
    tokens = np.asarray(tokens)
    n = int(np.sum(lengths))
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    emb = m.w(EMBED)
    ws = [_layer_weights(m, l) for l in range(m.L)]
    hidden = {l: np.empty((n, m.d), dtype=np.float64) for l in commit_layers}
    last = np.empty((n, m.d), dtype=np.float64)
    for b in range(len(lengths)):
        lo, hi = int(cu[b]), int(cu[b + 1])
        kc: List[Optional[np.ndarray]] = [None] * m.L
        vc: List[Optional[np.ndarray]] = [None] * m.L
        for t in range(hi - lo):
            h = emb[tokens[lo + t]][None, :]
            pos = np.array([t])
            for l in range(m.L):
                h, kc[l], vc[l] = _block(m, ws[l], h, pos, kc[l], vc[l])
                if (l + 1) in hidden:
                    hidden[l + 1][lo + t] = h[0]
            last[lo + t] = h[0]
    logits = lm_head(m, last) if want_logits else None
    return hidden, logits


# ------------------------------------------------------------------------------------------------
# comparison (Section 5.7)
# ------------------------------------------------------------------------------------------------

def compare_hidden(h_hat: np.ndarray, h_star: np.ndarray, tol_rel_l2: float, tol_max_abs: float):
    """Per-token statistics of Delta = h_hat - h_star and the per-token pass bit.

    h_hat [N, d] is the verifier's recomputation, h_star [N, d] the committed state (any stored dtype).
    Returns dict of float64 [N] arrays: rel_l2 = ||Delta||_2 / max(||h_hat||_2, 1e-30),
    max_abs = max|Delta|, mean_abs = mean|Delta| (the paper's example phi), mean_signed = mean Delta;
    and ok [N] bool = (rel_l2 <= tol_rel_l2) and (max_abs <= tol_max_abs).

    The denominator is the verifier's own state, which the committing party cannot scale.
    A NaN anywhere in a row makes both comparisons false, so the position is rejected.
    """
    a = upcast(h_hat)
    b = upcast(h_star)
    with np.errstate(invalid="ignore", over="ignore"):
        delta = a - b
        e2 = np.sum(delta * delta, axis=-1)
        n2 = np.sum(a * a, axis=-1)
        rel = np.sqrt(e2) / np.maximum(np.sqrt(n2), TINY)
        mx = np.max(np.abs(delta), axis=-1)
        nanrow = np.isnan(delta).any(axis=-1)
        mx = np.where(nanrow, np.nan, mx)
        mean_abs = np.mean(np.abs(delta), axis=-1)
        mean_signed = np.mean(delta, axis=-1)
        ok = (rel <= tol_rel_l2) & (mx <= tol_max_abs)
    return {"rel_l2": rel, "max_abs": mx, "mean_abs": mean_abs, "mean_signed": mean_signed, "ok": ok}



# ----------------------------------------------------------------------------------------------
# Bit-aware comparison (Section 7, "Bit-aware statistical comparison") and the battery of offline tests
# of the quantization-attack analysis (Appendix A.1: P_exp, Q_small, Z_large, MAE)
# ----------------------------------------------------------------------------------------------

def float32_fields(x: np.ndarray):
    """Sign, exponent and mantissa fields of float32 values: bit 31, bits 30..23, bits 22..0."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (bits >> np.uint32(31)).astype(np.int64), ((bits >> np.uint32(23)) & np.uint32(0xFF)).astype(np.int64), \
        (bits & np.uint32(0x7FFFFF)).astype(np.int64)


def bit_compare(h_hat: np.ndarray, h_star: np.ndarray, e_w: float, e_m: int, step_log2: int,
                q_small: float, tau_large: float) -> dict:
    """Per-token counts behind P_e, P_m, P_w, Q_small, Z_large of the recomputed state against the record.

    Both operands are taken in canonical float32 (the record upcast exactly from its stored dtype; the
    recomputation rounded to float32 if it is wider) and every element is split into its fields.
    Delta = h_hat - h_star is the float32 difference.  Per row of d elements:

      n_exact          both bit patterns identical
      n_exp_mismatch   exponent fields differ                                  -> P_e = n_exp_mismatch / d
      n_mismatch_close among those, |Delta| <= e_w                             -> P_m = n_mismatch_close / n_exp_mismatch
      n_match_small    among equal exponent fields, mantissa fields at most e_m steps apart, one step being
                       2**step_log2 units of the float32 mantissa               -> P_w = n_match_small / (d - n_exp_mismatch)
      n_small          |Delta| <= q_small                                      -> Q_small = n_small / d
      n_large          |Delta| >  tau_large                                    -> Z_large = n_large / d

    Readings.  The text defines P_m as the share of "large mantissa deviations among exponent mismatches" and
    accepts when it is HIGH, and gives a value tolerance e_w that no other quantity uses: read as "the exponent
    differs only because the value sits next to a power of two", i.e. the two values are within e_w of each
    other although their mantissa fields are far apart.  The mantissa tolerance e_m counts steps of the
    record's storage format (step_log2 = 0 for float32 records, 16 for bf16 ones, whose mantissa has 7 bits).
    The sign bit enters none of the counts; a sign error shows in Delta.  A NaN makes every <=, > test false.
    """
    a = np.asarray(h_hat)
    a = a.astype(np.float32) if a.dtype != np.uint16 else upcast(a).astype(np.float32)
    b = upcast(h_star).astype(np.float32)
    _, ea, ma = float32_fields(a)
    _, eb, mb = float32_fields(b)
    with np.errstate(invalid="ignore", over="ignore"):
        delta = (a - b).astype(np.float32)
        ad = np.abs(delta)
        mism = ea != eb
        close = ad <= np.float32(e_w)
        small_m = np.abs(ma - mb) <= (int(e_m) << int(step_log2))
        return {
            "n_exact": np.sum(a.view(np.uint32) == b.view(np.uint32), axis=-1),
            "n_exp_mismatch": np.sum(mism, axis=-1),
            "n_mismatch_close": np.sum(mism & close, axis=-1),
            "n_match_small": np.sum(~mism & small_m, axis=-1),
            "n_small": np.sum(ad <= np.float32(q_small), axis=-1),
            "n_large": np.sum(ad > np.float32(tau_large), axis=-1),
            "d": a.shape[-1],
        }


def bit_rule(counts: dict, mean_signed: np.ndarray, pe_max: float, pm_min: float, pw_min: float, eps_max: float,
             q_small_min: float = 0.0, z_large_max: float = 1.0) -> np.ndarray:
    """The acceptance rule on top of `bit_compare`: P_e < pe_max, P_m > pm_min, P_w > pw_min, |mean Delta| <= eps_max
    (the paper's calibrated off-chain values: 0.05, 0.75, 0.80, 0.01), and the two battery bounds
    Q_small >= q_small_min, Z_large <= z_large_max (calibrated per deployment; the defaults switch them off).

    A ratio over an empty set passes.  Every ratio test is taken as `count (<|>) bound * size` in float32,
    which is how an implementation without a division decides it; mean_signed [N] comes from `compare_hidden`.
    """
    f = np.float32
    d = f(counts["d"])
    mis = counts["n_exp_mismatch"].astype(np.float32)
    match = d - mis
    with np.errstate(invalid="ignore"):
        ok = mis < f(pe_max) * d
        ok &= (mis == 0) | (counts["n_mismatch_close"].astype(np.float32) > f(pm_min) * mis)
        ok &= (match == 0) | (counts["n_match_small"].astype(np.float32) > f(pw_min) * match)
        ok &= np.abs(np.asarray(mean_signed, dtype=np.float64)) <= float(f(eps_max))
        ok &= counts["n_small"].astype(np.float32) >= f(q_small_min) * d
        ok &= counts["n_large"].astype(np.float32) <= f(z_large_max) * d
    return ok



# ----------------------------------------------------------------------------------------------
# Merkle commitment of a hidden state (Section 5.6 "Commitment Submission": root = MerkleRoot(S) over a
# canonical serialization with scalar elements as leaves; Section 7: canonical float32, SHA-256)
# ----------------------------------------------------------------------------------------------
import hashlib


def _sha256(b: bytes) -> bytes:
    return hashlib.sha256(b).digest()


def merkle_leaves(state_row: np.ndarray) -> List[bytes]:
    """Leaf digests of one token's state: element j -> SHA-256 of its 4 little-endian float32 bytes.

    The state is taken in canonical float32 (a bf16 record is upcast exactly; a wider recomputation is rounded).
    """
    a = np.asarray(state_row)
    a = upcast(a).astype(np.float32) if a.dtype == np.uint16 else a.astype(np.float32)
    raw = a.astype("<f4").tobytes()
    return [_sha256(raw[4 * j:4 * j + 4]) for j in range(a.shape[-1])]


def merkle_levels(leaves: List[bytes]) -> List[List[bytes]]:
    """All levels of the tree, leaves first.  An inner node is SHA-256(left || right); a node without a right
    neighbour at its level moves up unchanged.  (The paper fixes neither rule; this is the plainest reading.)"""
    levels = [list(leaves)]
    while len(levels[-1]) > 1:
        cur = levels[-1]
        nxt = [_sha256(cur[i] + cur[i + 1]) for i in range(0, len(cur) - 1, 2)]
        if len(cur) % 2:
            nxt.append(cur[-1])
        levels.append(nxt)
    return levels


def merkle_root(state_row: np.ndarray) -> bytes:
    return merkle_levels(merkle_leaves(state_row))[-1][0]


def merkle_roots(states: np.ndarray) -> np.ndarray:
    """Roots of every row of states [R, d] -> uint8 [R, 32]."""
    return np.stack([np.frombuffer(merkle_root(r), dtype=np.uint8) for r in states])


def merkle_open(state_row: np.ndarray, index: int) -> List[bytes]:
    """Inclusion proof of element `index`: the sibling digests from the leaf level upwards; a level at which the
    node has no sibling (it moves up unchanged) contributes nothing."""
    levels = merkle_levels(merkle_leaves(state_row))
    path, i = [], int(index)
    for cur in levels[:-1]:
        sib = i ^ 1
        if sib < len(cur):
            path.append(cur[sib])
        i >>= 1
    return path


def merkle_verify(root: bytes, value: float, index: int, n_leaves: int, path: Sequence[bytes]) -> bool:
    """MerkleVerify of Section 5.7: recompute the root from the disclosed scalar, its index and the proof."""
    h = _sha256(np.asarray(value, dtype="<f4").tobytes())
    i, n, k = int(index), int(n_leaves), 0
    while n > 1:
        sib = i ^ 1
        if sib < n:
            if k >= len(path):
                return False
            h = _sha256(h + path[k]) if i % 2 == 0 else _sha256(path[k] + h)
            k += 1
        i >>= 1
        n = (n + 1) // 2
    return k == len(path) and h == root


def token_check(logits: np.ndarray, committed_argmax: np.ndarray, margin: float):
    """TokenMatch with a margin: position passes iff max_v z[v] - z[a*] <= margin.

    margin = 0 is the paper's exact match (the committed token must attain the maximum).
    committed_argmax[n] = -1 skips position n (passes).  Out-of-range ids fail.
    Returns (argmax [N] with lowest-index tie-break, gap [N] float64, ok [N] bool).
    """
    z = np.asarray(logits, dtype=np.float64)
    n, v = z.shape
    a = argmax_lowest(z)
    top = z[np.arange(n), a]
    cam = np.asarray(committed_argmax, dtype=np.int64)
    valid = (cam >= 0) & (cam < v)
    zc = z[np.arange(n), np.where(valid, cam, 0)]
    gap = np.where(valid, top - zc, np.inf)
    with np.errstate(invalid="ignore"):
        ok = gap <= margin
    skip = cam == -1
    gap = np.where(skip, 0.0, gap)
    ok = np.where(skip, True, ok)
    return a, gap, ok


def flags(hidden_ok: Sequence[np.ndarray], token_ok: Optional[np.ndarray]) -> np.ndarray:
    """flag[n] = 1 (accept) iff every committed layer passes at n and the token check passes at n."""
    f = np.ones_like(np.asarray(hidden_ok[0]), dtype=bool) if len(hidden_ok) else np.ones_like(token_ok, dtype=bool)
    for ok in hidden_ok:
        f &= np.asarray(ok, dtype=bool)
    if token_ok is not None:
        f &= np.asarray(token_ok, dtype=bool)
    return f.astype(np.uint8)


def summary(stats: Sequence[dict], token_ok: Optional[np.ndarray], flag: np.ndarray) -> dict:
    """Batch-level numbers: reject counts, worst errors, and T_v = mean over tokens (and committed layers)
    of the per-token mean absolute error (phi = MAE, Psi = mean in Section 5.7)."""
    n = len(flag)
    hid_ok = np.ones(n, dtype=bool)
    for s in stats:
        hid_ok &= s["ok"]
    out = {
        "n_tokens": n,
        "n_rejected": int(n - int(np.sum(flag))),
        "n_hidden_reject": int(np.sum(~hid_ok)),
        "n_token_reject": int(np.sum(~np.asarray(token_ok, dtype=bool))) if token_ok is not None else 0,
        "max_rel_l2": float(np.nanmax([np.nanmax(s["rel_l2"]) for s in stats])) if stats and n else 0.0,
        "max_abs": float(np.nanmax([np.nanmax(s["max_abs"]) for s in stats])) if stats and n else 0.0,
        "mean_mae": float(np.mean([np.mean(s["mean_abs"]) for s in stats])) if stats and n else 0.0,
    }
    return out


def verify(m: Model, tokens: np.ndarray, lengths: Sequence[int], commit_layers: Sequence[int],
           committed_hidden: np.ndarray, committed_argmax: Optional[np.ndarray],
           tol_rel_l2: float, tol_max_abs: float, tol_logit_margin: float,
           start_layer: int = 0, upstream_hidden: Optional[np.ndarray] = None, end_layer: Optional[int] = None,
           bit_params: Optional[dict] = None, bit_thresholds: Optional[dict] = None):
    """The whole hot path: prefill, compare at every committed layer, token check, flags, summary.

    committed_hidden [C, N, d] in stored dtype.  Returns dict with hidden, logits, stats (list over C),
    argmax, gap, token_ok, flags, summary.

    With start_layer > 0 (and/or end_layer < L) this is one verifier of the segment scheme of Section 5.6:
    it takes the recorded states entering block start_layer+1 as given (upstream_hidden [N, d], stored
    dtype), recomputes blocks start_layer+1 .. end_layer only and judges the commitments inside that range.
    The token check belongs to the segment that ends at the last layer.

    With bit_params (keyword arguments of `bit_compare`) and bit_thresholds (those of `bit_rule`) every committed
    layer is also judged by the bit-aware rule of Section 7: a token passes a layer only if both the tolerance
    test and the rule pass; the counts are returned in stats[c]["bits"], the rule's verdict in stats[c]["bit_ok"].
    """
    end_layer = m.L if end_layer is None else end_layer
    assert 0 <= start_layer < end_layer <= m.L
    assert all(start_layer < l <= end_layer for l in commit_layers)
    assert committed_argmax is None or end_layer == m.L
    hidden, logits = prefill(m, tokens, lengths, commit_layers, want_logits=committed_argmax is not None,
                             start_layer=start_layer,
                             start_hidden=None if start_layer == 0 else upcast(upstream_hidden),
                             end_layer=end_layer)
    stats = [compare_hidden(hidden[l], committed_hidden[c], tol_rel_l2, tol_max_abs)
             for c, l in enumerate(commit_layers)]
    if bit_params is not None:
        for c, l in enumerate(commit_layers):
            counts = bit_compare(hidden[l], committed_hidden[c], **bit_params)
            stats[c]["bits"] = counts
            stats[c]["bit_ok"] = bit_rule(counts, stats[c]["mean_signed"], **bit_thresholds)
            stats[c]["ok"] = stats[c]["ok"] & stats[c]["bit_ok"]
    if committed_argmax is not None:
        a, gap, tok_ok = token_check(logits, committed_argmax, tol_logit_margin)
    else:
        a, gap, tok_ok = None, None, None
    f = flags([s["ok"] for s in stats], tok_ok)
    return {"hidden": hidden, "logits": logits, "stats": stats, "argmax": a, "gap": gap, "token_ok": tok_ok,
            "flags": f, "summary": summary(stats, tok_ok, f)}
