"""The scanner for hand-placed scalar loads, and the code-generation checks of the build.

A scalar load written as inline asm is invisible to the compiler between its issue and the
s_waitcnt that follows: nothing scheduled there may touch its destination SGPRs.  The kernels
use compiler-tracked constant-address-space loads instead; the scanner guards against a
hand-placed load coming back.  It is first shown to catch a planted violation in a small
listing, then run over the real device code of every source (where it must find nothing).
"""
import os
import shutil

import pytest

from paper_1705_09864_amd import build as hip_build
from paper_1705_09864_amd import isa_check

GOOD = """
_Z4kernv:
	s_load_dwordx2 s[4:5], s[0:1], 0x0
	s_waitcnt lgkmcnt(0)
	;;#ASMSTART
	s_load_dwordx16 s[36:51], s[4:5], 0x0
	;;#ASMEND
	v_xor_b32_e32 v1, s8, v2
	s_add_u32 s6, s6, s7
	;;#ASMSTART
	s_waitcnt lgkmcnt(0)
	;;#ASMEND
	v_xor_b32_e32 v1, s36, v2
	s_endpgm
"""

# the compiler reloads a kernel argument into s[48:51] on the loop exit path while the
# inline-asm load of s[36:51] may still be in flight
BAD_WRITE = GOOD.replace("s_add_u32 s6, s6, s7", "s_cbranch_scc1 .LBB0_9").replace(
    "s_endpgm", "s_endpgm\n.LBB0_9:\n\ts_load_dwordx4 s[48:51], s[0:1], 0x78\n\ts_waitcnt lgkmcnt(0)\n\ts_endpgm")
BAD_READ = GOOD.replace("v_xor_b32_e32 v1, s8, v2", "v_xor_b32_e32 v1, s40, v2")


def _scan_text(tmp_path, text):
    f = tmp_path / "k.s"
    f.write_text(text)
    return isa_check.scan(str(f))


def test_scanner_accepts_clean_listing(tmp_path):
    assert _scan_text(tmp_path, GOOD) == []


def test_scanner_flags_write_on_branch_target(tmp_path):
    bad = _scan_text(tmp_path, BAD_WRITE)
    assert len(bad) == 1 and bad[0][3] == "writes" and bad[0][4] == (48, 49, 50, 51)


def test_scanner_flags_early_read(tmp_path):
    bad = _scan_text(tmp_path, BAD_READ)
    assert len(bad) == 1 and bad[0][3] == "reads" and bad[0][4] == (40,)


@pytest.mark.skipif(shutil.which(hip_build.HIPCC) is None and not os.path.exists(hip_build.HIPCC),
                    reason="hipcc not available")
def test_compiled_kernels_have_no_inflight_hazard():
    hip_build.check_scalar_loads()   # raises with the offending lines


@pytest.mark.skipif(shutil.which(hip_build.HIPCC) is None and not os.path.exists(hip_build.HIPCC),
                    reason="hipcc not available")
def test_compiled_kernels_keep_registers_and_wide_lds_reads():
    """No vector-register spills, no scratch memory, and one 16-byte LDS read per MFMA filter operand in the
    short-K convolution kernel (see build.check_codegen)."""
    hip_build.check_scalar_loads()   # makes sure the device listings exist
    hip_build.check_codegen()
    stats = isa_check.kernel_stats(hip_build.device_asm("conv_mfma.hip"))
    assert any("conv_mfma_ws_kernelILi9ELi1E" in k for k in stats)
