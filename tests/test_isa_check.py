"""The check of the generated code for matrix-core instructions under a lane mask (they ignore the mask, so a guard
whose branch the compiler dropped lets them run on registers that were never loaded)."""
import shutil

import pytest

from paper_2509_08721_amd import isa_check

MASKED_NO_BRANCH = """
_Z6kernelPv:
	s_and_saveexec_b64 s[2:3], vcc
	global_load_dwordx4 v[0:3], v[4:5], off
	s_waitcnt vmcnt(0)
	v_mfma_f32_16x16x32_f16 v[8:11], v[0:3], v[0:3], v[8:11]
	s_or_b64 exec, exec, s[2:3]
	s_endpgm
"""

MASKED_WITH_BRANCH = MASKED_NO_BRANCH.replace(
    "\tglobal_load_dwordx4", "\ts_cbranch_execz .LBB0_2\n\tglobal_load_dwordx4").replace(
    "\ts_or_b64 exec", ".LBB0_2:\n\ts_or_b64 exec")

AFTER_RESTORE = """
_Z6kernelPv:
	s_and_saveexec_b64 s[2:3], vcc
	v_mov_b32_e32 v0, 0
	s_or_b64 exec, exec, s[2:3]
	v_mfma_f32_32x32x16_f16 v[8:23], v[0:3], v[0:3], v[8:23]
	s_endpgm
"""


def test_flags_an_mfma_under_a_mask_without_a_branch():
    found = isa_check.unguarded_mfmas(MASKED_NO_BRANCH)
    assert len(found) == 1 and found[0][0] == "_Z6kernelPv" and found[0][2].startswith("v_mfma_f32_16x16x32_f16")


def test_accepts_a_branch_on_the_mask_and_code_after_the_restore():
    assert isa_check.unguarded_mfmas(MASKED_WITH_BRANCH) == []
    assert isa_check.unguarded_mfmas(AFTER_RESTORE) == []


@pytest.mark.skipif(shutil.which("hipcc") is None and not shutil.os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_every_source_of_the_library_is_clean():
    assert isa_check.check_sources(verbose=False) == []


STORE_THEN_LOAD = """
_Z6kernelPv:
	global_load_dwordx4 v[0:3], v[4:5], off
	s_waitcnt vmcnt(0)
	global_store_dwordx4 v[4:5], v[0:3], off
	global_load_dwordx4 v[8:11], v[6:7], off
	s_waitcnt vmcnt(0)
	global_store_dwordx4 v[6:7], v[8:11], off
	s_endpgm
"""

LOADS_AHEAD = """
_Z6kernelPv:
	global_load_dwordx4 v[0:3], v[4:5], off
	global_load_dwordx4 v[8:11], v[6:7], off
	s_waitcnt vmcnt(1)
	global_store_dwordx4 v[4:5], v[0:3], off
	s_waitcnt vmcnt(1)
	global_store_dwordx4 v[6:7], v[8:11], off
	s_endpgm
"""


def test_reports_a_wait_that_covers_a_store():
    found = isa_check.waits_behind_stores(STORE_THEN_LOAD)
    assert list(found) == ["_Z6kernelPv"] and found["_Z6kernelPv"] == [(7, 0, 1)]
    # the second load requested before the first store: the wait for it leaves the store outstanding
    assert isa_check.waits_behind_stores(LOADS_AHEAD) == {}


@pytest.mark.skipif(shutil.which("hipcc") is None and not shutil.os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_residual_epilogues_of_the_decode_gemms_do_not_wait_behind_their_stores(tmp_path):
    found = isa_check.waits_behind_stores(isa_check.assemble("kernels_decode.hip", str(tmp_path)))
    resid = [fn for fn in found if "k_skinny16" in fn and fn.endswith("ELi1EEEvNS_10SkinnyArgsEi")]
    assert resid == [], resid
