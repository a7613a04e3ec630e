"""The compiled matrix-core decode kernels hold no asm-block write into the destination of a
matrix instruction that may still be in flight (a hazard the compiler cannot guard, see
paper_2605_19660_amd/check_asm_hazards.py).  Needs hipcc, no GPU."""
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


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_compiled_decode_kernels_are_clean():
    assert chk.main() == 0
