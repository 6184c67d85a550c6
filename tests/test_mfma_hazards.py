"""The build's static check of the inline-MFMA kernels' assembly: the checker itself on hand-written
snippets, and the assembly the last build kept."""
import glob
import os

import pytest

from paper_2511_07423_amd import mfma_hazards as mh

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MFMA32 = "\tv_mfma_f32_32x32x16_bf16 a[0:15], v[0:3], v[4:7], a[0:15]"
MFMA16 = "\tv_mfma_f32_16x16x32_bf16 v[8:11], v[0:3], v[4:7], v[8:11]"


def test_copy_right_behind_an_mfma_is_reported():
    rep = mh.check_kernel("k", [MFMA32, "\tv_accvgpr_mov_b32 a20, a3"])
    assert len(rep) == 1 and "a20, a3" in rep[0]
    rep = mh.check_kernel("k", [MFMA16, "\tv_add_f32_e32 v20, v9, v9"])
    assert len(rep) == 1


def test_wait_states_settle_it():
    # 8 passes + 3 = 11 wait states: s_nop 10 is exactly enough, s_nop 9 is one short
    assert mh.check_kernel("k", [MFMA32, "\ts_nop 10", "\tv_accvgpr_read_b32 v9, a3"]) == []
    assert len(mh.check_kernel("k", [MFMA32, "\ts_nop 9", "\tv_accvgpr_read_b32 v9, a3"])) == 1
    # 4 passes + 3 = 7: seven unrelated instructions in between are enough, six are not
    other = ["\ts_add_i32 s0, s0, 1"] * 7
    assert mh.check_kernel("k", [MFMA16] + other + ["\tv_mov_b32_e32 v20, v8"]) == []
    assert len(mh.check_kernel("k", [MFMA16] + other[:6] + ["\tv_mov_b32_e32 v20, v8"])) == 1


def test_accumulating_onto_the_same_registers_is_allowed_but_using_them_as_an_operand_is_not():
    assert mh.check_kernel("k", [MFMA32, MFMA32]) == []
    assert len(mh.check_kernel("k", [MFMA32, "\tv_mfma_f32_32x32x16_bf16 a[16:31], a[0:3], v[4:7], a[16:31]"])) == 1
    assert len(mh.check_kernel("k", [MFMA32, "\tv_mfma_f32_32x32x16_bf16 a[8:23], v[0:3], v[4:7], a[8:23]"])) == 1


def test_unrelated_registers_and_memory_stores():
    assert mh.check_kernel("k", [MFMA32, "\tv_accvgpr_mov_b32 a20, a16", "\tds_read_b128 v[0:3], v40"]) == []
    assert len(mh.check_kernel("k", [MFMA32, "\tscratch_store_dwordx4 off, a[12:15], off"])) == 1


def test_branch_targets_are_followed():
    body = [".LBB0_1:", "\tv_accvgpr_read_b32 v9, a3", MFMA32, "\ts_cbranch_scc1 .LBB0_1"]
    rep = mh.check_kernel("k", body)           # the back edge lands on a read of the MFMA's result
    assert len(rep) == 1
    body = [".LBB0_1:", "\tv_accvgpr_read_b32 v9, a3", MFMA32, "\ts_nop 15", "\ts_cbranch_scc1 .LBB0_1"]
    assert mh.check_kernel("k", body) == []


MFMA_F16 = "\tv_mfma_f32_16x16x32_f16 a[8:11], v[0:3], v[4:7], a[8:11]"


def test_mfma_source_written_by_a_vector_instruction_just_before_is_reported():
    cvt = "\tv_cvt_pkrtz_f16_f32 v3, v20, v21"
    assert len(mh.check_kernel("k", [cvt, MFMA_F16])) == 1
    assert len(mh.check_kernel("k", [cvt, "\ts_nop 0", MFMA_F16])) == 1
    assert mh.check_kernel("k", [cvt, "\ts_nop 1", MFMA_F16]) == []
    assert mh.check_kernel("k", [cvt, "\tv_add_u32 v30, s1, v30", "\tv_add_u32 v31, s1, v31", MFMA_F16]) == []
    # an LDS read into a source is the compiler's to wait for, and unrelated writes do not matter
    assert mh.check_kernel("k", ["\tds_read_b128 v[0:3], v40", MFMA_F16]) == []
    assert mh.check_kernel("k", ["\tv_cvt_pkrtz_f16_f32 v12, v20, v21", MFMA_F16]) == []


def test_assembly_of_the_last_build_is_clean():
    asm = glob.glob(os.path.join(ROOT, "paper_2511_07423_amd", "_build", "gemm_nf*-hip-amdgcn-amd-amdhsa-gfx950*.s")) + \
        glob.glob(os.path.join(ROOT, "paper_2511_07423_amd", "_build", "gemm_k64-hip-amdgcn-amd-amdhsa-gfx950*.s"))
    if not asm:
        pytest.skip("no build in this tree yet (build() keeps the assembly it checked)")
    assert len(asm) == 4
    kernels = mfmas = 0
    for f in asm:
        n_kernels, n_mfma, rep = mh.check_file(f, "proj_kernel")
        assert rep == []
        kernels += n_kernels
        mfmas += n_mfma
    # 116 with one MFMA K step per stage, 87 of them again for the paired activation array, 56 with two steps
    assert kernels == 259 and mfmas > 15000
