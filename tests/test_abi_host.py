"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header
declares, validates configurations, plans memory, and fails loudly instead of falling back."""
import ctypes as C
import os
import re

import pytest

import paper_2509_24257_amd as P
from paper_2509_24257_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "verillm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vl_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = P.load_library()
    names = declared_functions()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), "libverillm.so does not export " + n
    assert sorted(binding.EXPORTS) == names


def test_struct_layouts_match_the_header():
    assert C.sizeof(P.ModelCfg) == 13 * 4
    assert C.sizeof(P.Tol) == 12 and C.sizeof(P.TokStats) == 16
    assert C.sizeof(P.BitRule) == 11 * 4 and C.sizeof(P.BitStats) == 8 * 4
    assert C.sizeof(P.Summary) == 4 * 8 + 5 * 4 + 4          # 4 bytes of tail padding to the int64 alignment


def cfg(**kw):
    base = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=688, vocab=4096, rms_eps=1e-5,
                rope_base=10000.0, dtype=P.VL_F32, max_tokens=128, max_seqs=1, max_seq_len=128)
    base.update(kw)
    return P.ModelCfg(*[base[k] for k, _ in P.ModelCfg._fields_])


def test_plan_memory_matches_the_parameter_count():
    w, s = P.vl_plan_memory(cfg())
    params = 4096 * 256 * 2 + 2 * (4 * 256 * 256 + 3 * 688 * 256 + 2 * 256) + 256
    assert params * 4 <= w <= params * 4 + 64 * 256
    assert s > 128 * 4096 * 4
    w8, _ = P.vl_plan_memory(cfg(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, d_ffn=14336,
                                 vocab=128256, rope_base=500000.0, dtype=P.VL_BF16, max_tokens=8192, max_seqs=8,
                                 max_seq_len=1024))
    assert abs(w8 / 2 - 8.03e9) < 0.01e9
    w70, s70 = P.vl_plan_memory(cfg(n_layers=80, d_model=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, d_ffn=28672,
                                    vocab=128256, rope_base=500000.0, dtype=P.VL_BF16, max_tokens=8192, max_seqs=4,
                                    max_seq_len=2048))
    assert 140e9 < w70 < 142e9 and w70 + s70 < 288e9          # the 70B shape fits one 288 GB device


@pytest.mark.parametrize("bad", [
    dict(dtype=7), dict(n_layers=0), dict(n_q_heads=6, n_kv_heads=4), dict(rms_eps=0.0), dict(max_tokens=0),
    dict(dtype=P.VL_BF16, d_ffn=688), dict(dtype=P.VL_BF16, d_ffn=704, head_dim=32, n_q_heads=8, n_kv_heads=8),
    dict(d_ffn=690), dict(head_dim=258, n_q_heads=1, n_kv_heads=1), dict(rope_base=1.0)])
def test_invalid_configurations_are_rejected(bad):
    with pytest.raises(P.VerilLMError) as e:
        P.vl_plan_memory(cfg(**bad))
    assert e.value.code == binding.VL_E_ARG
    lib = P.load_library()
    h = C.c_void_p(None)
    assert lib.vl_create(C.byref(cfg(**bad)), 0, None, C.byref(h)) == binding.VL_E_ARG and not h.value


def test_null_arguments_return_error_codes_not_crashes():
    lib = P.load_library()
    assert lib.vl_plan_memory(None, None, None) == binding.VL_E_ARG
    assert lib.vl_create(None, 0, None, None) == binding.VL_E_ARG
    assert lib.vl_load_weights(None, 0, 0, None, 0) == binding.VL_E_ARG
    assert lib.vl_verify_prefill(None, None, None, 0, None, 0, None, 0, None, None, None, None, None) == binding.VL_E_ARG
    assert lib.vl_prefill_commit(None, None, None, 0, None, 0, None, 0, None) == binding.VL_E_ARG
    assert lib.vl_decode_commit(None, None, None, None, 0, None, 0, None, 0, None) == binding.VL_E_ARG
    assert lib.vl_get_logits(None, 0, 0, None) == binding.VL_E_ARG
    assert lib.vl_get_argmax(None, 0, 0, None, None) == binding.VL_E_ARG
    assert lib.vl_op_gemm_bf16(None, None, None, None, 0, 1, 1, 64) == binding.VL_E_ARG
    assert lib.vl_op_attention_bf16(None, None, None, 0, None) == binding.VL_E_ARG
    assert lib.vl_op_compare(None, None, None, 0, 0, None, None, None) == binding.VL_E_ARG
    assert lib.vl_op_argmax(None, None, 0, None, 0.0, None, None, None) == binding.VL_E_ARG
    lib.vl_destroy(None)
    assert isinstance(lib.vl_last_error(None), bytes)


def test_no_device_means_an_error_not_a_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(P.VerilLMError) as e:
        P.Context(cfg())
    assert e.value.code == binding.VL_E_HIP


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2509_24257_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "binding.py" and False, f + " mentions the oracle"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2509_24257_amd" not in text and "ctypes" not in text
