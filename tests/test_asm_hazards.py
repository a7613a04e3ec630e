"""The compiled matrix-core decode kernels hold no asm-block write into the destination of a
matrix instruction that may still be in flight, and no asm block of the decode kernels or of the
encoder reads a DPP operand inside two issue slots of its write -- hazards the compiler cannot
guard (paper_2605_19660_amd/check_asm_hazards.py).  Needs hipcc, no GPU."""
import shutil

import pytest

from paper_2605_19660_amd import check_asm_hazards as chk


def test_scanner_flags_a_planted_case_and_accepts_a_guarded_one():
    bad = """
_Zkernel:
	v_mfma_f32_16x16x32_f16 v[110:113], v[110:113], v[118:121], v[114:117]
	v_fma_f32 v18, v18, v163, -v212
	;;#ASMSTART
	v_fma_mix_f32 v112, v18, v20, 0 op_sel_hi:[0,1,0]
	;;#ASMEND
"""
    found = chk.scan(bad)
    assert len(found) == 1 and found[0][5] == 1
    # the same write after a compiler-scheduled read of the result: the result has landed
    ok = bad.replace("\tv_fma_f32 v18, v18, v163, -v212\n", "\ts_nop 6\n\tv_add_f32_e32 v19, v112, v113\n")
    assert chk.scan(ok) == []
    # a write by an instruction the compiler schedules itself is the compiler's business
    ok2 = bad.replace(";;#ASMSTART\n", "").replace("\t;;#ASMEND\n", "")
    assert chk.scan(ok2) == []
    # far enough behind the matrix instruction
    far = bad.replace("\tv_fma_f32 v18, v18, v163, -v212\n", "\tv_fma_f32 v18, v18, v163, -v212\n" * (chk.WINDOW + 1))
    assert chk.scan(far) == []


def test_dpp_scanner_wants_two_slots_between_a_write_and_its_dpp_read():
    dpp = "\tv_max_f32_dpp v5, v5, v5 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
    def block(between):
        return "_Zkernel:\n\tv_add_f32_e32 v5, v1, v2\n" + between + "\t;;#ASMSTART\n" + dpp + "\t;;#ASMEND\n"
    assert len(chk.scan_dpp(block(""))) == 1
    assert len(chk.scan_dpp(block("\tv_mov_b32_e32 v9, v8\n"))) == 1
    assert chk.scan_dpp(block("\tv_mov_b32_e32 v9, v8\n\tv_mov_b32_e32 v10, v8\n")) == []
    assert chk.scan_dpp(block("\ts_nop 1\n")) == []
    assert len(chk.scan_dpp(block("\ts_nop 0\n"))) == 1
    # the wait may sit inside the block, and another register's write does not matter
    inside = "_Zkernel:\n\tv_add_f32_e32 v5, v1, v2\n\t;;#ASMSTART\n\ts_nop 1\n" + dpp + "\t;;#ASMEND\n"
    assert chk.scan_dpp(inside) == []
    assert chk.scan_dpp(block("").replace("v_add_f32_e32 v5,", "v_add_f32_e32 v6,")) == []
    # back to back inside a block: the second reads what the first wrote
    twice = "_Zkernel:\n\t;;#ASMSTART\n\ts_nop 1\n" + dpp + dpp + "\t;;#ASMEND\n"
    assert len(chk.scan_dpp(twice)) == 1
    # the compiler's own DPP instructions are its business
    assert chk.scan_dpp(block("").replace("\t;;#ASMSTART\n", "").replace("\t;;#ASMEND\n", "")) == []


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_compiled_kernels_are_clean():
    assert chk.main() == 0
