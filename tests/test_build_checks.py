"""Checks of the compiler's output for the hand-scheduled kernels (no GPU needed: hipcc cross-compiles).

The large-tile kernels issue their MFMAs as volatile assembly statements, which hides from the
compiler that the result registers are written late.  Two things can then go wrong without any
error: an instruction placed right behind such a statement reads the accumulators before they
are written (it happened with a register spill placed at a loop exit), and spills inside a main
loop cost 10-25 % unnoticed.  Both are looked for in the generated assembly."""
import shutil

import pytest

from paper_2006_03031_amd import build

STMT_MFMA = ";;#ASMSTART\n\tv_mfma_f32_16x16x32_bf16 a[124:127], v[0:3], v[4:7], a[124:127]\n{extra}\t;;#ASMEND\n"


def _kernel(extra_in_stmt: str, after: str) -> str:
    return ("_Z4testv:\n\ts_load_dword s0, s[4:5], 0x0\n.LBB0_1:\n" + STMT_MFMA.format(extra=extra_in_stmt) +
            "\ts_cbranch_scc1 .LBB0_1\n.LBB0_2:\n" + after + "\ts_endpgm\n")


def test_checker_flags_a_spill_store_right_behind_a_statement_mfma():
    hazards, _ = build.asm_mfma_findings(_kernel("", "\tscratch_store_dwordx4 off, a[124:127], off\n"))
    assert len(hazards) == 1 and hazards[0][0] == "_Z4testv" and "scratch_store" in hazards[0][2]
    hazards, _ = build.asm_mfma_findings(_kernel("", "\tv_accvgpr_read_b32 v9, a125\n"))
    assert len(hazards) == 1
    hazards, _ = build.asm_mfma_findings(_kernel("", "\tv_accvgpr_write_b32 a127, 0\n"))
    assert len(hazards) == 1


def test_checker_accepts_wait_states_in_the_statement_or_other_registers():
    nops = "\ts_nop 15\n\ts_nop 15\n"
    hazards, spills = build.asm_mfma_findings(_kernel(nops, "\tscratch_store_dwordx4 off, a[124:127], off\n"))
    assert hazards == [] and spills == []
    hazards, _ = build.asm_mfma_findings(_kernel("", "\tv_accvgpr_read_b32 v9, a3\n"))
    assert hazards == []
    # a short wait is not enough; 18 single-slot instructions are
    hazards, _ = build.asm_mfma_findings(_kernel("\ts_nop 7\n", "\tv_accvgpr_read_b32 v9, a124\n"))
    assert len(hazards) == 1
    filler = "".join("\tv_mov_b32_e32 v1, v2\n" for _ in range(18))
    hazards, _ = build.asm_mfma_findings(_kernel("", filler + "\tv_accvgpr_read_b32 v9, a124\n"))
    assert hazards == []


def test_checker_ignores_compiler_issued_mfmas():
    asm = ("_Z4testv:\n\tv_mfma_f32_16x16x32_bf16 a[0:3], v[0:3], v[4:7], a[0:3]\n"
           "\tv_accvgpr_read_b32 v9, a0\n\ts_endpgm\n")
    hazards, spills = build.asm_mfma_findings(asm)
    assert hazards == [] and spills == []


def test_checker_reports_scratch_traffic_in_a_block_with_statement_mfmas():
    asm = ("_Z4testv:\n.LBB0_1:\n\tscratch_load_dword v1, off, off\n" + STMT_MFMA.format(extra="") +
           "\ts_cbranch_scc1 .LBB0_1\n.LBB0_2:\n\tscratch_load_dword v2, off, off\n\ts_endpgm\n")
    _, spills = build.asm_mfma_findings(asm)
    assert spills == [("_Z4testv", ".LBB0_1", 1)]


def test_checker_counts_spills_only_at_the_deepest_loop_level_that_holds_statement_mfmas():
    mf = STMT_MFMA.format(extra="")
    # a stage peeled off in front of the K loop (level 1: once per tile) may spill; the K loop (level 2) may not
    peeled = (".LBB0_1:                                ;   in Loop: Header=BB0_0 Depth=1\n"
              "\tscratch_load_dword v1, off, off\n" + mf)
    inner = (".LBB0_2:                                ;   Parent Loop BB0_0 Depth=1\n"
             "                                        ; =>  This Inner Loop Header: Depth=2\n" + mf +
             "\ts_cbranch_scc1 .LBB0_2\n")
    # a block entered by falling through is a block of its own: its spill is not the loop's
    after = ("; %bb.3:                                ;   in Loop: Header=BB0_0 Depth=1\n"
             "\tscratch_store_dword off, v1, off\n\ts_endpgm\n")
    _, spills = build.asm_mfma_findings("_Z4testv:\n" + peeled + inner + after)
    assert spills == []
    inner_spilling = inner.replace(mf, "\tscratch_load_dword v2, off, off\n" + mf)
    _, spills = build.asm_mfma_findings("_Z4testv:\n" + peeled + inner_spilling + after)
    assert spills == [("_Z4testv", ".LBB0_2", 1)]


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_generated_kernels_keep_clear_of_statement_mfma_results_and_do_not_spill_in_main_loops():
    asm = build.device_assembly()
    assert asm.count("v_mfma_f32_16x16x32_bf16") > 1000  # the ring kernels are in there
    hazards, spills = build.asm_mfma_findings(asm)
    assert hazards == [], hazards[:5]
    assert spills == [], spills[:5]
