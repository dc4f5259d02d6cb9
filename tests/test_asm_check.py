"""The checker of the emitted device assembly (paper_2502_02581_amd/asm_check.py): unit cases, and
the assembly of the current build when the build step has left it in place.  CPU only."""
from __future__ import annotations

import os

import pytest

from paper_2502_02581_amd import asm_check, build

LOAD = "\tbuffer_load_dwordx4 v4, s[4:7], 0 offen lds"


def _asm(*body):
    return ["_ZN3moe15row_gemm_kernelIxEEv:", *body, "\ts_endpgm", "; ScratchSize: 0"]


def test_descriptor_written_by_vector_instruction_is_flagged():
    bad = _asm("\tv_readlane_b32 s6, v106, 55", "\tv_add_u32_e32 v13, s3, v12", "\ts_add_i32 s3, s68, 0xc000",
               "\ts_mov_b32 m0, s3", "\ts_nop 0", LOAD)
    found = asm_check.check_descriptor_hazards(bad)
    assert len(found) == 1 and "s[6]" in found[0] and "4 wait states" in found[0]
    # v_readfirstlane and a carry-out count as well
    assert asm_check.check_descriptor_hazards(_asm("\tv_readfirstlane_b32 s4, v1", "\ts_mov_b32 m0, s3", "\ts_nop 0", LOAD))
    assert asm_check.check_descriptor_hazards(_asm("\tv_add_co_u32_e64 v1, s[4:5], v2, v3", "\ts_nop 0", LOAD))


def test_enough_wait_states_or_other_registers_pass():
    ok = _asm("\tv_readlane_b32 s6, v106, 55", "\ts_mov_b32 m0, s3", "\ts_nop 4", LOAD)       # 1 + 5 wait states
    assert asm_check.check_descriptor_hazards(ok) == []
    ok = _asm("\tv_readlane_b32 s8, v106, 55", "\ts_mov_b32 m0, s3", "\ts_nop 0", LOAD)       # not a descriptor word
    assert asm_check.check_descriptor_hazards(ok) == []
    ok = _asm("\ts_add_u32 s4, s4, s20", "\ts_addc_u32 s5, s5, s21", "\ts_mov_b32 m0, s3", "\ts_nop 0", LOAD)  # scalar writes
    assert asm_check.check_descriptor_hazards(ok) == []
    ok = _asm("\tv_readlane_b32 s6, v106, 55", "\tbuffer_load_dwordx4 v[0:3], v4, s[4:7], 0 offen")   # not an LDS-DMA load
    assert asm_check.check_descriptor_hazards(ok) == []


def test_writers_on_other_paths_are_found():
    # the writer sits at the tail of the loop, below the load in the file: it precedes the load through the back edge
    loop = _asm(".LBB0_1:", "\ts_mov_b32 m0, s3", "\ts_nop 0", LOAD, "\tv_mfma_f32_32x32x16_bf16 a[0:15], v[0:3], v[4:7], a[0:15]",
                "\tv_readfirstlane_b32 s5, v9", "\ts_cbranch_scc1 .LBB0_1")
    found = asm_check.check_descriptor_hazards(loop)
    assert len(found) == 1 and "s[5]" in found[0] and "3 wait states" in found[0]
    # the writer sits in the arm of an `if` that jumps over the other arm to the load
    arm = _asm("\ts_cbranch_scc0 .LBB0_2", "\tv_readfirstlane_b32 s7, v9", "\ts_branch .LBB0_3", ".LBB0_2:",
               "\ts_mov_b32 s7, 0", "\ts_nop 7", ".LBB0_3:", "\ts_mov_b32 m0, s3", "\ts_nop 0", LOAD)
    found = asm_check.check_descriptor_hazards(arm)
    assert len(found) == 1 and "s[7]" in found[0]
    # the same with enough wait states behind the writer on that path
    arm[2:3] = ["\tv_readfirstlane_b32 s7, v9", "\ts_nop 4"]
    assert asm_check.check_descriptor_hazards(arm) == []
    # a path that ends before the load: what stands right above the load in the file but never runs into it is no writer
    dead = _asm("\ts_cbranch_scc1 .LBB0_5", "\tv_readfirstlane_b32 s4, v1", "\ts_endpgm", ".LBB0_5:", "\ts_mov_b32 m0, s3",
                "\ts_nop 0", LOAD)
    assert asm_check.check_descriptor_hazards(dead) == []


def test_scratch_in_a_gemm_kernel_is_flagged():
    lines = ["_ZN3moe15row_gemm_kernelIxEEv:", "\ts_endpgm", "; ScratchSize: 1088",
             "_ZN3moe12route_kernelIxEEv:", "\ts_endpgm", "; ScratchSize: 16"]
    found = asm_check.check_no_scratch(lines)
    assert len(found) == 1 and "row_gemm_kernel" in found[0] and "1088" in found[0]


def test_packed_fp32_is_flagged():
    assert asm_check.check_no_packed_fp32(_asm("\tv_pk_fma_f32 v[0:1], v[2:3], v[4:5], v[6:7]"))
    assert asm_check.check_no_packed_fp32(_asm("\tv_fma_f32 v0, v1, v2, v3", "\tv_pk_add_f16 v0, v1, v2")) == []


def test_current_build_passes():
    for src in build.CHECKED:
        path = build.device_asm(src)
        if not os.path.exists(path):
            pytest.skip("the build step has not left its device assembly here")
        assert asm_check.check(path) == []
