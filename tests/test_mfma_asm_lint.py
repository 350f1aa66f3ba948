"""The build-time hazard check of the hand-written MFMA statements (paper_2510_08431_amd/csrc/lint_mfma_asm.py):
it must accept a correct sequence, catch each kind of planted violation, and pass on the assembly of the built
library when that is at hand (build() keeps it under _build/)."""
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.join(ROOT, "paper_2510_08431_amd", "csrc"))
import lint_mfma_asm as lint  # noqa: E402

GOOD = """
	ds_read_b128 v[4:7], v100
	s_waitcnt lgkmcnt(0)
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[32:47], v[4:7], a[0:3], 0
	;;#ASMEND
	v_add_f32_e32 v1, v2, v3
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[32:47], v[8:11], a[4:7], v[32:47]
	;;#ASMEND
	;;#ASMSTART
	s_nop 7
	s_nop 3
	;;#ASMEND
	v_fma_f32 v1, v32, s2, -v3
"""


def test_accepts_a_correct_sequence():
    assert lint.lint(GOOD) == []
    assert lint.count_asm_mfma(GOOD) == 2


def test_catches_a_result_read_too_early():
    bad = GOOD.replace("\ts_nop 7\n", "")
    assert any("v_fma_f32 touches" in p for p in lint.lint(bad))


def test_catches_a_register_of_the_result_reused_too_early():
    bad = GOOD.replace("\tv_add_f32_e32 v1, v2, v3\n", "\tds_read_b64_tr_b16 v[40:41], v9\n")
    assert any("ds_read_b64_tr_b16 touches" in p for p in lint.lint(bad))


def test_catches_an_operand_written_right_before():
    bad = GOOD.replace("\ts_waitcnt lgkmcnt(0)\n", "\tv_mov_b32_e32 v5, v9\n")
    assert any("written by v_mov_b32_e32" in p for p in lint.lint(bad))
    far = GOOD.replace("\ts_waitcnt lgkmcnt(0)\n", "\tv_mov_b32_e32 v5, v9\n\ts_nop 1\n")
    assert lint.lint(far) == []


def test_a_compiler_mfma_reading_the_result_is_caught_but_a_chain_is_not():
    bad = GOOD.replace("\tv_add_f32_e32 v1, v2, v3\n", "\tv_mfma_f32_32x32x16_f16 a[0:15], v[32:35], v[60:63], a[0:15]\n")
    assert any("v_mfma_f32_32x32x16_f16 touches" in p for p in lint.lint(bad))


def test_built_library_passes():
    asm = os.path.join(ROOT, "_build", "attn_jvp_mfma-hip-amdgcn-amd-amdhsa-gfx950.s")
    if not os.path.exists(asm):
        pytest.skip("no compiled assembly under _build/ (run __graft_entry__.build())")
    with open(asm) as f:
        text = f.read()
    assert lint.count_asm_mfma(text) > 0
    assert lint.lint(text, asm) == []
