"""ctypes binding of libverillm.so (include/verillm.h).  Argument marshalling only.

PyTorch is used by callers for device memory and streams; this module itself only needs raw device
pointers (ints).  There is no fallback: if the shared library is missing or a call fails, an exception
is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

VL_F32, VL_BF16 = 0, 1
VL_OK, VL_E_ARG, VL_E_WEIGHTS, VL_E_CAPACITY, VL_E_HIP, VL_E_NOMEM = 0, -1, -2, -3, -4, -5
_STATUS = {0: "VL_OK", -1: "VL_E_ARG", -2: "VL_E_WEIGHTS", -3: "VL_E_CAPACITY", -4: "VL_E_HIP", -5: "VL_E_NOMEM"}

EXPORTS = ["vl_plan_memory", "vl_create", "vl_load_weights", "vl_destroy", "vl_last_error", "vl_verify_prefill",
           "vl_verify_segment", "vl_prefill_commit", "vl_decode_commit", "vl_get_logits", "vl_get_argmax",
           "vl_set_bit_rule", "vl_get_bit_stats", "vl_profile_enable", "vl_profile_read", "vl_op_gemm_bf16",
           "vl_op_attention_bf16", "vl_op_attention_decode_bf16", "vl_op_compare", "vl_op_compare_bits", "vl_op_argmax", "vl_op_merkle_roots",
           "vl_op_merkle_open"]


STAGES = ["embed", "norm", "qkv_gemm", "rope", "attention", "o_gemm", "gateup_gemm", "down_gemm", "compare", "lm_gemm",
          "argmax", "finalize"]


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("rms_eps", C.c_float),
                ("rope_base", C.c_float), ("dtype", C.c_int32), ("max_tokens", C.c_int32), ("max_seqs", C.c_int32),
                ("max_seq_len", C.c_int32)]


class Tol(C.Structure):
    _fields_ = [("rel_l2", C.c_float), ("max_abs", C.c_float), ("logit_margin", C.c_float)]


class TokStats(C.Structure):
    _fields_ = [("rel_l2", C.c_float), ("max_abs", C.c_float), ("mean_abs", C.c_float), ("mean_signed", C.c_float)]


class BitRule(C.Structure):
    _fields_ = [("e_w", C.c_float), ("e_m", C.c_int32), ("step_log2", C.c_int32), ("q_small", C.c_float), ("tau_large", C.c_float),
                ("pe_max", C.c_float), ("pm_min", C.c_float), ("pw_min", C.c_float), ("eps_max", C.c_float),
                ("q_small_min", C.c_float), ("z_large_max", C.c_float)]


class BitStats(C.Structure):
    _fields_ = [("n_exact", C.c_int32), ("n_exp_mismatch", C.c_int32), ("n_mismatch_close", C.c_int32),
                ("n_match_small", C.c_int32), ("n_small", C.c_int32), ("n_large", C.c_int32), ("mean_signed", C.c_float),
                ("ok", C.c_uint32)]


class Summary(C.Structure):
    _fields_ = [("n_tokens", C.c_int64), ("n_rejected", C.c_int64), ("n_hidden_reject", C.c_int64),
                ("n_token_reject", C.c_int64), ("max_rel_l2", C.c_float), ("max_abs", C.c_float),
                ("mean_mae", C.c_float), ("ms_forward", C.c_float), ("ms_compare", C.c_float)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class VerilLMError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("%s: %s" % (_STATUS.get(code, str(code)), msg))
        self.code = code


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libverillm.so")


_lib = None


def load_library():
    """Load libverillm.so (building it first only if it has never been built)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build(verbose=False)
    lib = C.CDLL(path)
    vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
    lib.vl_plan_memory.argtypes = [C.POINTER(ModelCfg), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
    lib.vl_create.argtypes = [C.POINTER(ModelCfg), C.c_int, vp, C.POINTER(vp)]
    lib.vl_load_weights.argtypes = [vp, C.c_int, C.c_int, vp, C.c_size_t]
    lib.vl_destroy.argtypes = [vp]
    lib.vl_destroy.restype = None
    lib.vl_last_error.argtypes = [vp]
    lib.vl_last_error.restype = C.c_char_p
    lib.vl_verify_prefill.argtypes = [vp, vp, i32p, C.c_int32, i32p, C.c_int32, vp, C.c_int32, vp, C.POINTER(Tol), vp, vp,
                                      C.POINTER(Summary)]
    lib.vl_verify_segment.argtypes = [vp, C.c_int32, C.c_int32, vp, C.c_int32, vp, i32p, C.c_int32, i32p, C.c_int32, vp, C.c_int32,
                                      vp, C.POINTER(Tol), vp, vp, C.POINTER(Summary)]
    lib.vl_prefill_commit.argtypes = [vp, vp, i32p, C.c_int32, i32p, C.c_int32, vp, C.c_int32, vp]
    lib.vl_decode_commit.argtypes = [vp, vp, i32p, i32p, C.c_int32, i32p, C.c_int32, vp, C.c_int32, vp]
    lib.vl_get_logits.argtypes = [vp, C.c_int64, C.c_int64, vp]
    lib.vl_get_argmax.argtypes = [vp, C.c_int64, C.c_int64, vp, vp]
    lib.vl_set_bit_rule.argtypes = [vp, C.POINTER(BitRule)]
    lib.vl_get_bit_stats.argtypes = [vp, C.c_int32, C.c_int64, C.c_int64, vp]
    lib.vl_op_compare_bits.argtypes = [vp, vp, vp, C.c_int32, C.c_int64, C.POINTER(Tol), C.POINTER(BitRule), vp, vp, vp]
    lib.vl_profile_enable.argtypes = [vp, C.c_int]
    lib.vl_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.vl_op_gemm_bf16.argtypes = [vp, vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.vl_op_attention_bf16.argtypes = [vp, vp, i32p, C.c_int32, vp]
    lib.vl_op_attention_decode_bf16.argtypes = [vp, vp, vp, vp, C.c_int64, i32p, i32p, C.c_int32, vp]
    lib.vl_op_compare.argtypes = [vp, vp, vp, C.c_int32, C.c_int64, C.POINTER(Tol), vp, vp]
    lib.vl_op_merkle_roots.argtypes = [vp, vp, C.c_int32, C.c_int64, vp]
    lib.vl_op_merkle_open.argtypes = [vp, vp, C.c_int32, C.c_int64, C.POINTER(C.c_int64), i32p, C.c_int32, vp, vp, i32p]
    lib.vl_op_argmax.argtypes = [vp, vp, C.c_int64, vp, C.c_float, vp, vp, vp]
    for name in EXPORTS:
        if name not in ("vl_destroy", "vl_last_error"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def lib():
    return load_library()


def _i32(seq: Optional[Sequence[int]]):
    if seq is None:
        return None, 0
    arr = (C.c_int32 * len(seq))(*[int(v) for v in seq])
    return arr, len(seq)


def vl_plan_memory(cfg: ModelCfg):
    w, s = C.c_uint64(0), C.c_uint64(0)
    rc = lib().vl_plan_memory(C.byref(cfg), C.byref(w), C.byref(s))
    if rc:
        raise VerilLMError(rc, (lib().vl_last_error(None) or b"").decode())
    return int(w.value), int(s.value)


class Context:
    """Owns one vl_ctx.  Methods mirror the C entry points; device buffers are passed as integer addresses."""

    def __init__(self, cfg: ModelCfg, device: int = 0, stream: int = 0):
        self.cfg = cfg
        self._h = C.c_void_p(None)
        rc = lib().vl_create(C.byref(cfg), int(device), C.c_void_p(stream or None), C.byref(self._h))
        if rc:
            raise VerilLMError(rc, (lib().vl_last_error(None) or b"").decode())

    def _check(self, rc: int):
        if rc:
            raise VerilLMError(rc, (lib().vl_last_error(self._h) or b"").decode())

    def close(self):
        if self._h:
            lib().vl_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def vl_load_weights(self, kind: int, layer: int, ptr: int, nbytes: int):
        self._check(lib().vl_load_weights(self._h, int(kind), int(layer), C.c_void_p(ptr), C.c_size_t(nbytes)))

    def vl_verify_prefill(self, tokens: int, lengths: Sequence[int], commit_layers: Sequence[int], committed_hidden: int,
                          hidden_dtype: int, committed_argmax: int, tol: Tol, flags: int, stats: int = 0) -> Summary:
        la, b = _i32(lengths)
        ca, c = _i32(commit_layers)
        sm = Summary()
        self._check(lib().vl_verify_prefill(self._h, C.c_void_p(tokens or None), la, b, ca, c,
                                            C.c_void_p(committed_hidden or None), int(hidden_dtype),
                                            C.c_void_p(committed_argmax or None), C.byref(tol), C.c_void_p(flags or None),
                                            C.c_void_p(stats or None), C.byref(sm)))
        return sm

    def vl_verify_segment(self, start_layer: int, end_layer: int, upstream_hidden: int, upstream_dtype: int, tokens: int,
                          lengths: Sequence[int], commit_layers: Sequence[int], committed_hidden: int, hidden_dtype: int,
                          committed_argmax: int, tol: Tol, flags: int, stats: int = 0) -> Summary:
        la, b = _i32(lengths)
        ca, c = _i32(commit_layers)
        sm = Summary()
        self._check(lib().vl_verify_segment(self._h, int(start_layer), int(end_layer), C.c_void_p(upstream_hidden or None),
                                            int(upstream_dtype), C.c_void_p(tokens or None), la, b, ca, c,
                                            C.c_void_p(committed_hidden or None), int(hidden_dtype),
                                            C.c_void_p(committed_argmax or None), C.byref(tol), C.c_void_p(flags or None),
                                            C.c_void_p(stats or None), C.byref(sm)))
        return sm

    def vl_prefill_commit(self, tokens: int, lengths: Sequence[int], commit_layers: Sequence[int], out_hidden: int,
                          hidden_dtype: int, out_argmax: int):
        la, b = _i32(lengths)
        ca, c = _i32(commit_layers)
        self._check(lib().vl_prefill_commit(self._h, C.c_void_p(tokens or None), la, b, ca, c, C.c_void_p(out_hidden or None),
                                            int(hidden_dtype), C.c_void_p(out_argmax or None)))

    def vl_decode_commit(self, tokens: int, lengths: Sequence[int], prompt_lens: Optional[Sequence[int]],
                         commit_layers: Sequence[int], out_hidden: int, hidden_dtype: int, out_argmax: int):
        la, b = _i32(lengths)
        pa, _ = _i32(prompt_lens)
        ca, c = _i32(commit_layers)
        self._check(lib().vl_decode_commit(self._h, C.c_void_p(tokens or None), la, pa, b, ca, c,
                                           C.c_void_p(out_hidden or None), int(hidden_dtype), C.c_void_p(out_argmax or None)))

    def vl_get_logits(self, tok_begin: int, tok_end: int, out: int):
        self._check(lib().vl_get_logits(self._h, int(tok_begin), int(tok_end), C.c_void_p(out or None)))

    def vl_get_argmax(self, tok_begin: int, tok_end: int, out_argmax: int = 0, out_gap: int = 0):
        self._check(lib().vl_get_argmax(self._h, int(tok_begin), int(tok_end), C.c_void_p(out_argmax or None),
                                        C.c_void_p(out_gap or None)))

    def vl_set_bit_rule(self, rule: Optional[BitRule]):
        self._check(lib().vl_set_bit_rule(self._h, C.byref(rule) if rule is not None else None))

    def vl_get_bit_stats(self, c: int, tok_begin: int, tok_end: int, out: int):
        self._check(lib().vl_get_bit_stats(self._h, int(c), int(tok_begin), int(tok_end), C.c_void_p(out or None)))

    def vl_op_compare_bits(self, h_hat: int, committed: int, hidden_dtype: int, n: int, tol: Tol, rule: BitRule, stats: int,
                           bits: int, ok: int):
        self._check(lib().vl_op_compare_bits(self._h, C.c_void_p(h_hat or None), C.c_void_p(committed or None), int(hidden_dtype),
                                             int(n), C.byref(tol), C.byref(rule), C.c_void_p(stats or None),
                                             C.c_void_p(bits or None), C.c_void_p(ok or None)))

    def vl_profile_enable(self, mode: int):
        self._check(lib().vl_profile_enable(self._h, int(mode)))

    def vl_profile_read(self):
        ms = (C.c_double * len(STAGES))()
        cnt = (C.c_int64 * len(STAGES))()
        self._check(lib().vl_profile_read(self._h, ms, cnt))
        return {name: (float(ms[i]), int(cnt[i])) for i, name in enumerate(STAGES)}

    def vl_op_gemm_bf16(self, a: int, w: int, out: int, out_dtype: int, m: int, n: int, k: int):
        self._check(lib().vl_op_gemm_bf16(self._h, C.c_void_p(a), C.c_void_p(w), C.c_void_p(out), int(out_dtype), m, n, k))

    def vl_op_attention_bf16(self, qkv: int, lengths: Sequence[int], out: int):
        la, b = _i32(lengths)
        self._check(lib().vl_op_attention_bf16(self._h, C.c_void_p(qkv), la, b, C.c_void_p(out)))

    def vl_op_attention_decode_bf16(self, q: int, k_cache: int, v_cache: int, cache_rows: int, first_row: Sequence[int],
                                    n_keys: Sequence[int], out: int):
        fa, rows = _i32(first_row)
        na, _ = _i32(n_keys)
        self._check(lib().vl_op_attention_decode_bf16(self._h, C.c_void_p(q or None), C.c_void_p(k_cache or None),
                                                      C.c_void_p(v_cache or None), int(cache_rows), fa, na, rows,
                                                      C.c_void_p(out or None)))

    def vl_op_merkle_roots(self, states: int, dtype: int, rows: int, roots: int):
        self._check(lib().vl_op_merkle_roots(self._h, C.c_void_p(states or None), int(dtype), int(rows), C.c_void_p(roots or None)))

    def vl_op_merkle_open(self, states: int, dtype: int, rows: int, sel_row: Sequence[int], sel_index: Sequence[int], values: int,
                          paths: int):
        """Returns the list of proof lengths."""
        k = len(sel_row)
        ra = (C.c_int64 * max(k, 1))(*[int(v) for v in sel_row])
        ia, _ = _i32(sel_index)
        lens = (C.c_int32 * max(k, 1))()
        self._check(lib().vl_op_merkle_open(self._h, C.c_void_p(states or None), int(dtype), int(rows), ra, ia, k,
                                            C.c_void_p(values or None), C.c_void_p(paths or None), lens))
        return [int(v) for v in lens[:k]]

    def vl_op_compare(self, h_hat: int, committed: int, hidden_dtype: int, n: int, tol: Tol, stats: int, ok: int):
        self._check(lib().vl_op_compare(self._h, C.c_void_p(h_hat or None), C.c_void_p(committed or None), int(hidden_dtype),
                                        int(n), C.byref(tol), C.c_void_p(stats or None), C.c_void_p(ok or None)))

    def vl_op_argmax(self, logits: int, n: int, committed_argmax: int, margin: float, out_argmax: int, out_gap: int,
                     out_ok: int):
        self._check(lib().vl_op_argmax(self._h, C.c_void_p(logits or None), int(n), C.c_void_p(committed_argmax or None),
                                       C.c_float(margin), C.c_void_p(out_argmax or None), C.c_void_p(out_gap or None),
                                       C.c_void_p(out_ok or None)))
