"""Build-time safety net for the hand-scheduled kernels (no GPU needed): see paper_2203_04071_amd/isa_check.py."""
import os
import shutil

import pytest

from paper_2203_04071_amd import isa_check


@pytest.mark.skipif(not (shutil.which("hipcc") or os.path.exists("/opt/rocm/bin/hipcc")), reason="hipcc not available")
def test_no_compiler_access_to_registers_with_loads_in_flight(capsys):
    bad = isa_check.check_build()
    out = capsys.readouterr().out
    assert "checked 0 functions" not in out, "no kernel matched: the check would be vacuous"
    assert bad == 0, out[-4000:]


def test_checker_flags_a_planted_copy(tmp_path):
    """The checker itself: a copy of a register whose LDS read has not been waited for must be reported."""
    good = """_Z6kernelv:
\t;;#ASMSTART
\tds_read_b128 v[4:7], v1 offset:0
\t;;#ASMEND
\tv_mov_b32_e32 v9, v2
\t;;#ASMSTART
\ts_waitcnt lgkmcnt(0)
\tv_add_u32 v8, v8, v4
\t;;#ASMEND
\tv_mov_b32_e32 v10, v4
\ts_endpgm
"""
    bad = good.replace("v_mov_b32_e32 v9, v2", "v_mov_b32_e32 v9, v5")
    p = tmp_path / "k.s"
    p.write_text(good)
    assert isa_check.check(str(p), "kernel") == 0
    p.write_text(bad)
    assert isa_check.check(str(p), "kernel") == 1


def test_checker_flags_a_touched_matrix_accumulator(tmp_path):
    """A compiler-generated instruction that reads the destination of a matrix instruction issued from asm, before the
    kernel has drained the matrix pipe, must be reported; after the drain it is fine."""
    good = """_Z6kernelv:
\t;;#ASMSTART
\tv_mfma_i32_16x16x64_i8 v[4:7], v[8:11], v[12:15], v[4:7]
\t;;#ASMEND
\tv_mov_b32_e32 v20, v8
\t;;#ASMSTART
\ts_nop 15
\ts_nop 15
\t;;#ASMEND
\tv_mov_b32_e32 v21, v5
\ts_endpgm
"""
    bad = good.replace("v_mov_b32_e32 v20, v8", "v_mov_b32_e32 v20, v6")
    p = tmp_path / "k.s"
    p.write_text(good)
    assert isa_check.check(str(p), "kernel") == 0
    p.write_text(bad)
    assert isa_check.check(str(p), "kernel") == 1


def test_checker_follows_branches(tmp_path):
    """The walk follows the control-flow graph: a load issued in a block that the text puts AFTER its consumer is still
    seen in flight when a branch leads from one to the other."""
    text = """_Z6kernelv:
\ts_branch .LBB0_2
.LBB0_1:
\tv_mov_b32_e32 v9, v5
\t;;#ASMSTART
\ts_waitcnt vmcnt(0)
\t;;#ASMEND
\ts_endpgm
.LBB0_2:
\t;;#ASMSTART
\tglobal_load_dwordx4 v[4:7], v1, s[2:3]
\t;;#ASMEND
\ts_branch .LBB0_1
"""
    p = tmp_path / "k.s"
    p.write_text(text)
    assert isa_check.check(str(p), "kernel") == 1
    p.write_text(text.replace("v_mov_b32_e32 v9, v5", "v_mov_b32_e32 v9, v3"))
    assert isa_check.check(str(p), "kernel") == 0
