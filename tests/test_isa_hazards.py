"""The compiler's output for the fp16 kernels holds no read of an accumulator register right
behind the inline-assembly matrix instruction that writes it (paper_1611_07819_amd/check_isa.py
explains the hazard).  Compiling both sources to assembly takes about five minutes, so the
check runs only when DMATH_CHECK_ISA=1 is set; the scanner itself is always tested on
hand-written snippets."""
import os

import pytest

from paper_1611_07819_amd import check_isa


def _lines(text):
    return [l.strip() for l in text.strip().split("\n")]


def test_scanner_flags_an_early_copy_and_accepts_a_drained_one():
    early = _lines("""
        s_nop 0
        v_mfma_f32_16x16x32_f16 a[60:63], v[2:5], v[38:41], a[60:63]
        ds_read_b64_tr_b16 v[38:39], v2
        v_accvgpr_mov_b32 a127, a63
    """)
    assert [l for _, l, _ in check_isa.scan_function(early)] == ["v_accvgpr_mov_b32 a127, a63"]
    drained = early[:3] + ["s_nop 15", "s_nop 15"] + early[3:]
    assert check_isa.scan_function(drained) == []
    other_register = early[:3] + ["v_accvgpr_mov_b32 a127, a59"]
    assert check_isa.scan_function(other_register) == []
    store = early[:3] + ["global_store_dwordx4 v[0:1], a[60:63], off"]
    assert len(check_isa.scan_function(store)) == 1


def test_scanner_flags_a_copy_directly_in_front_of_a_matrix_instruction():
    bare = _lines("""
        v_accvgpr_mov_b32 a3, a67
        v_mfma_f32_16x16x32_f16 a[0:3], v[2:5], v[38:41], a[0:3]
    """)
    assert len(check_isa.scan_function(bare)) == 1
    waited = [bare[0], "s_nop 0", bare[1]]
    assert check_isa.scan_function(waited) == []
    elsewhere = ["v_accvgpr_mov_b32 a9, a67", bare[1]]
    assert check_isa.scan_function(elsewhere) == []


def test_scanner_follows_a_backward_branch():
    loop = _lines("""
        .LBB0_1:
        v_accvgpr_read_b32 v7, a3
        s_nop 0
        v_mfma_f32_16x16x32_f16 a[0:3], v[2:5], v[38:41], a[0:3]
        s_cbranch_scc1 .LBB0_1
    """)
    assert [l for _, l, _ in check_isa.scan_function(loop)] == ["v_accvgpr_read_b32 v7, a3"]


@pytest.mark.skipif(os.environ.get("DMATH_CHECK_ISA") != "1", reason="takes five minutes of compilation: set DMATH_CHECK_ISA=1")
def test_fp16_kernels_have_no_early_accumulator_reads():
    report, looked = check_isa.check()
    assert looked >= 36
    assert report == {}


def test_scanner_knows_the_longer_fp64_instruction():
    early = _lines("""
        s_nop 0
        v_mfma_f64_16x16x4_f64 a[16:23], v[122:123], v[126:127], a[16:23]
        s_nop 15
        s_nop 15
        v_accvgpr_read_b32 v7, a23
    """)
    assert len(check_isa.scan_function(early)) == 1      # 32 cycles of drain are enough for fp16 only
    drained = early[:2] + ["s_nop 15"] * 5 + early[-1:]
    assert check_isa.scan_function(drained) == []


def test_scanner_accepts_only_the_pipelines_own_forms_on_fixed_accumulators():
    own = _lines("""
        v_accvgpr_write_b32 a5, 0
        s_nop 0
        v_mfma_f32_16x16x32_f16 a[4:7], v[2:5], v[38:41], a[4:7]
        s_nop 15
        s_nop 15
        v_accvgpr_read_b32 v9, a5
    """)
    assert check_isa.scan_function(own, fixed=True) == []
    # a register the compiler parks in the accumulation file: fine in an ordinary kernel, not here
    parked = own + ["v_accvgpr_write_b32 a200, v17"]
    assert check_isa.scan_function(parked) == []
    assert [l for _, l, _ in check_isa.scan_function(parked, fixed=True)] == \
        ["v_accvgpr_write_b32 a200, v17   (accumulation register used by the compiler)"]
