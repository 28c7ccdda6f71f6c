"""The build's static check of the GEMM's hand-pipelined loads (paper_2510_25590_amd/isa_check.py): it must accept
code that waits before it touches a load's registers and reject a copy, a read or an overwrite made too early."""
import os

import pytest

from paper_2510_25590_amd import isa_check as ic


def _fn(body: str):
    return [l for l in body.strip().splitlines()]


CLEAN = """
	s_load_dwordx2 s[0:1], s[4:5], 0x0
	;;#ASMSTART
	global_load_dwordx4 v[10:13], v[2:3], off
	;;#ASMEND
	;;#ASMSTART
	global_load_dwordx4 v[14:17], v[2:3], off offset:1024
	;;#ASMEND
.LBB0_1:
	;;#ASMSTART
	global_load_dwordx4 v[18:21], v[2:3], off offset:2048
	;;#ASMEND
	;;#ASMSTART
	s_waitcnt vmcnt(2)
	;;#ASMEND
	ds_write_b128 v1, v[10:13]
	;;#ASMSTART
	s_waitcnt vmcnt(0)
	;;#ASMEND
	v_mfma_f32_32x32x16_bf16 a[0:15], v[30:33], v[14:17], a[0:15]
	v_mov_b32_e32 v40, v18
	s_endpgm
"""


def test_accepts_uses_behind_the_wait():
    assert ic.check_function("clean", _fn(CLEAN)) == []


@pytest.mark.parametrize("early", [
    "v_accvgpr_write_b32 a40, v12",                       # spill of a register whose load is in flight
    "v_mov_b32_e32 v50, v13",                             # copy
    "ds_write_b128 v1, v[10:13]",                         # use in front of the wait
    "ds_read_b128 v[10:13], v1",                          # overwrite
    "v_lshl_add_u64 v[2:3], v[10:11], 0, s[0:1]",         # address arithmetic on it
])
def test_rejects_early_touch(early):
    body = CLEAN.replace(".LBB0_1:", "\t" + early + "\n.LBB0_1:")
    errs = ic.check_function("early", _fn(body))
    assert errs and "still in flight" in errs[0]


def test_rejects_wait_that_is_too_weak():
    errs = ic.check_function("weak", _fn(CLEAN.replace("vmcnt(2)", "vmcnt(3)")))
    assert errs and "ds_write_b128" in errs[0]


def test_rejects_load_in_flight_at_the_end():
    errs = ic.check_function("tail", _fn(CLEAN.replace("\ts_waitcnt vmcnt(0)\n", "").replace(
        "\tv_mfma_f32_32x32x16_bf16 a[0:15], v[30:33], v[14:17], a[0:15]\n\tv_mov_b32_e32 v40, v18\n", "")))
    assert errs and "s_endpgm" in errs[-1]


def test_loop_carried_state_is_followed():
    # the load issued at the bottom of the loop body is still in flight when the top of the body touches its register
    body = """
.LBB0_1:
	v_add_u32_e32 v5, v10, v6
	;;#ASMSTART
	global_load_dwordx4 v[10:13], v[2:3], off
	;;#ASMEND
	s_cbranch_scc1 .LBB0_1
	;;#ASMSTART
	s_waitcnt vmcnt(0)
	;;#ASMEND
	s_endpgm
"""
    errs = ic.check_function("loop", _fn(body))
    assert errs and "v_add_u32_e32" in errs[0]


@pytest.mark.skipif(not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_gemm_source_passes():
    from paper_2510_25590_amd import build as b
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument", "-I", os.path.join(b.ROOT, "include"), "-I", b.CSRC]
    ic.check_gemm("/opt/rocm/bin/hipcc", flags, os.path.join(b.CSRC, "gemm.hip"))
