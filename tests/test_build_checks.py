"""Host logic of the build: the check that reads the attention kernel's generated assembly (no GPU needed)."""
import os
import sys
import textwrap

sys.path.insert(0, os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2509_24257_amd"))
import check_mfma_asm  # noqa: E402

HEAD = "_ZN2vl16attn_mfma_kernelILi128ELi4EEEvTest:\n"


def _write(tmp_path, body):
    p = tmp_path / "k.s"
    p.write_text(HEAD + textwrap.dedent(body) + "\ts_endpgm\n")
    return str(p)


def test_operand_copy_next_to_a_hand_issued_mfma_is_flagged(tmp_path):
    bad = _write(tmp_path, """\
        \tv_accvgpr_write_b32 a0, v90
        \tv_accvgpr_write_b32 a1, v91
        \t;;#ASMSTART
        \tv_mfma_f32_32x32x16_bf16 v[2:17], v[34:37], a[0:3], v[2:17]
        \t;;#ASMEND
        """)
    problems = check_mfma_asm.check(bad)
    assert len(problems) == 2 and all("a" in p for p in problems)


def test_padding_inside_the_statement_counts_as_distance(tmp_path):
    ok = _write(tmp_path, """\
        \tv_accvgpr_write_b32 a3, v93
        \t;;#ASMSTART
        \ts_nop 3
        \tv_mfma_f32_32x32x16_bf16 v[2:17], v[34:37], a[0:3], 0
        \t;;#ASMEND
        \tv_accvgpr_write_b32 a8, v1
        """)
    assert check_mfma_asm.check(ok) == []


def test_early_read_of_a_result_is_flagged_and_compiler_issued_mfma_is_not_checked(tmp_path):
    bad = _write(tmp_path, """\
        \t;;#ASMSTART
        \tv_mfma_f32_32x32x16_bf16 v[2:17], v[34:37], a[0:3], 0
        \t;;#ASMEND
        \tv_add_f32_e32 v40, v41, v42
        \tv_max_f32_e32 v50, v5, v50
        """)
    assert len(check_mfma_asm.check(bad)) == 1
    overwritten = _write(tmp_path, """\
        \t;;#ASMSTART
        \tv_mfma_f32_32x32x16_bf16 v[2:17], v[34:37], a[0:3], 0
        \t;;#ASMEND
        \tv_mov_b32_e32 v9, 0xff800000
        """)
    assert len(check_mfma_asm.check(overwritten)) == 1
    fine = _write(tmp_path, """\
        \tv_accvgpr_write_b32 a0, v90
        \tv_mfma_f32_32x32x16_bf16 a[4:19], v[34:37], a[0:3], a[4:19]
        \tv_accvgpr_read_b32 v1, a4
        """)
    assert check_mfma_asm.check(fine) == []        # the compiler pads its own instructions


def test_the_built_kernel_passes():
    asm = os.path.join(os.path.dirname(check_mfma_asm.__file__), "_build", "kernels_attn_mfma.s")
    if not os.path.exists(asm):
        import pytest
        pytest.skip("library not built in this tree")
    assert check_mfma_asm.check(asm) == []
