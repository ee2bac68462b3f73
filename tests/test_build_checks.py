"""The build's own checks, on hand-written snippets: a check that never fires is no check."""
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from paper_2510_08874_amd import build  # noqa: E402

GOOD = """
	v_readlane_b32 s6, v152, 36
	v_readlane_b32 s7, v152, 37
	;;#ASMSTART
	s_nop 4
	global_store_dword v5, a[0], s[6:7] offset:0 nt
	;;#ASMEND
	v_readfirstlane_b32 s2, v1
	v_add_u32_e32 v5, s18, v5
	v_add_u32_e32 v5, s18, v5
	v_add_u32_e32 v5, s18, v5
	v_add_u32_e32 v5, s18, v5
	v_add_u32_e32 v5, s18, v5
	;;#ASMSTART
	global_load_lds_dwordx4 v3, s[2:3]
	;;#ASMEND
	v_readlane_b32 s8, v152, 1
	global_load_dword v9, v4, s[8:9]
"""

# the pair that sent a store to a wild address: base fetched from a spill lane right in front of the statement
BAD_STORE = """
	v_readlane_b32 s0, v152, 36
	;;#ASMSTART
	;;#ASMEND
	v_readlane_b32 s1, v152, 37
	;;#ASMSTART
	global_store_dword v5, a[0], s[0:1] offset:0 nt
	;;#ASMEND
"""

BAD_LOAD = """
	v_readfirstlane_b32 s2, v1
	s_add_u32 s4, s4, 64
	s_nop 1
	;;#ASMSTART
	s_add_u32 m0, m0, 0x400
	global_load_lds_dwordx4 v3, s[2:3]
	;;#ASMEND
"""

BAD_COMPARE = """
	v_cmp_gt_i32_e64 s[10:11], s2, v54
	;;#ASMSTART
	buffer_load_dword v1, v2, s[8:11], 0 offen
	;;#ASMEND
"""


def _check(tmp_path, text):
    p = tmp_path / "unit.s"
    p.write_text(text)
    build.check_wait_states(str(p))


def test_spaced_instructions_pass(tmp_path):
    # five idle cycles inside the statement; five instructions in between; the compiler's own
    # instructions (outside assembly statements) are its business
    _check(tmp_path, GOOD)


@pytest.mark.parametrize("text,line", [(BAD_STORE, 7), (BAD_LOAD, 7), (BAD_COMPARE, 4)])
def test_missing_wait_states_fail_the_build(tmp_path, text, line):
    with pytest.raises(RuntimeError) as e:
        _check(tmp_path, text)
    assert f"unit.s:{line}:" in str(e.value)


def test_compiler_use_of_m0_fails_the_build(tmp_path):
    ok = tmp_path / "ok.s"
    ok.write_text("\t;;#ASMSTART\n\ts_mov_b32 m0, s5\n\tglobal_load_lds_dwordx4 v3, s[2:3]\n\t;;#ASMEND\n\tv_add_u32_e32 v5, s18, v5\n")
    build.check_m0_private(str(ok))
    for text in ("\ts_mov_b32 m0, s7\n", "\ts_set_gpr_idx_on s3, gpr_idx(SRC0)\n", "\tv_movrels_b32_e32 v1, v0\n"):
        bad = tmp_path / "bad.s"
        bad.write_text("\t;;#ASMSTART\n\ts_mov_b32 m0, s5\n\t;;#ASMEND\n" + text)
        with pytest.raises(RuntimeError):
            build.check_m0_private(str(bad))


def test_resource_check_rejects_scratch_and_lost_accumulators():
    ok = ("remark: k.hpp:1:0: Function Name: _ZN3dmm19grouped_gemm_kernelILi2ELb0EEEv [-Rpass]\n"
          "remark: k.hpp:1:0:     VGPRs: 152 [-Rpass]\nremark: k.hpp:1:0:     AGPRs: 256 [-Rpass]\n"
          "remark: k.hpp:1:0:     ScratchSize [bytes/lane]: 0 [-Rpass]\nremark: k.hpp:1:0:     SGPRs Spill: 243 [-Rpass]\n"
          "remark: k.hpp:1:0:     VGPRs Spill: 0 [-Rpass]\n")
    build.check_resources(ok, want_kernel=True)
    for bad in (ok.replace("ScratchSize [bytes/lane]: 0", "ScratchSize [bytes/lane]: 36"),
                ok.replace("VGPRs Spill: 0", "VGPRs Spill: 3"), ok.replace("AGPRs: 256", "AGPRs: 240")):
        with pytest.raises(RuntimeError):
            build.check_resources(bad, want_kernel=True)
    with pytest.raises(RuntimeError):
        build.check_resources("remark: nothing here\n", want_kernel=True)
    build.check_resources("remark: nothing here\n", want_kernel=False)
