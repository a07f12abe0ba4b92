"""The checker of hand-placed wait states: does it flag what it must, and does the attention
kernel's assembly pass it?  (CPU only: hipcc cross-compiles.)"""
import os
import shutil

import pytest

from paper_2603_06274_amd import build, wait_states

HEAD = "_Z1kv:                                  ; @_Z1kv\n"
TAIL = "\ts_endpgm\n.Lfunc_end0:\n"
S_TILE = "\tv_mfma_f32_32x32x16_bf16 v[0:15], v[20:23], a[0:3], v[0:15]\n"
ROW_SUM = "\tv_mfma_f32_4x4x4_16b_bf16 v[40:43], v[36:37], v[44:45], v[40:43]\n"
FILLER = "\ts_add_i32 s1, s1, 1\n"


def broken(body):
    return wait_states.check_kernel(HEAD + body + TAIL, "_Z1kv")


def test_vector_read_of_a_matrix_result():
    read = "\tv_mul_f32_e32 v30, v31, v7\n"
    assert broken(S_TILE + FILLER * 11 + read)
    assert not broken(S_TILE + FILLER * 12 + read)
    assert broken(S_TILE + "\ts_nop 10\n" + read)
    assert not broken(S_TILE + "\ts_nop 11\n" + read)
    assert not broken(S_TILE + "\tv_mul_f32_e32 v30, v31, v16\n")      # another register


def test_accumulation_follows_at_once_but_a_shifted_result_does_not():
    assert not broken(S_TILE + S_TILE)
    shifted = "\tv_mfma_f32_32x32x16_bf16 v[8:23], v[24:27], a[0:3], v[8:23]\n"
    assert broken(S_TILE + FILLER * 9 + shifted)
    assert not broken(S_TILE + FILLER * 10 + shifted)
    # results that overlap without a read in between are ordered by the pipe itself
    assert not broken(S_TILE + "\tv_mfma_f32_32x32x16_bf16 v[8:23], v[24:27], a[0:3], 0\n")
    as_operand = "\tv_mfma_f32_32x32x16_bf16 v[48:63], v[0:3], a[0:3], v[48:63]\n"
    assert broken(S_TILE + FILLER * 11 + as_operand)
    assert not broken(S_TILE + FILLER * 12 + as_operand)


def test_accumulator_registers_are_tracked_too():
    o_tile = "\tv_mfma_f32_32x32x16_bf16 a[16:31], v[20:23], v[24:27], a[16:31]\n"
    read = "\tv_accvgpr_read_b32 v1, a17\n"
    assert broken(o_tile + FILLER * 3 + read)
    assert not broken(o_tile + "\ts_nop 15\n" + read)


def test_row_sum_instruction():
    read = "\tv_add_f32_e32 v1, v2, v40\n"
    assert broken(ROW_SUM + FILLER * 4 + read)
    assert not broken(ROW_SUM + FILLER * 5 + read)
    assert broken(ROW_SUM + FILLER + ROW_SUM)
    assert not broken(ROW_SUM + FILLER * 2 + ROW_SUM)


def test_matrix_read_after_vector_write():
    write = "\tv_accvgpr_write_b32 a2, v9\n"
    assert broken(write + FILLER + S_TILE)
    assert not broken(write + "\ts_nop 1\n" + S_TILE)
    assert broken("\tv_cvt_pk_bf16_f32 v45, v1, v2\n" + ROW_SUM)
    assert broken("\tv_permlane32_swap_b32_e32 v9, v21\n" + S_TILE)


def test_branch_targets_are_followed():
    read = "\tv_mul_f32_e32 v30, v31, v7\n"
    body = S_TILE + "\ts_cbranch_scc0 .LBB0_2\n" + FILLER * 12 + "\ts_branch .LBB0_3\n.LBB0_2:\n" + read + ".LBB0_3:\n"
    assert broken(body)
    # a second branch on the way
    body = (S_TILE + "\ts_cbranch_scc0 .LBB0_2\n" + FILLER * 12 + "\ts_branch .LBB0_4\n.LBB0_2:\n" + FILLER * 2 +
            "\ts_cbranch_scc1 .LBB0_3\n" + FILLER * 12 + "\ts_branch .LBB0_4\n.LBB0_3:\n" + read + ".LBB0_4:\n")
    assert broken(body)
    # after an unconditional branch nothing falls through
    assert not broken(S_TILE + "\ts_branch .LBB0_3\n.LBB0_2:\n" + read + ".LBB0_3:\n" + FILLER * 12)


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="needs hipcc to produce the kernel's assembly")
def test_attention_kernel_assembly_passes():
    os.makedirs(build.OBJ, exist_ok=True)
    build.check_wait_states()                      # raises with the offending lines
    with open(os.path.join(build.OBJ, "stem_attn.s")) as f:
        asm = f.read()
    hand_placed = [k for k in wait_states.kernels(asm, "sparse_attn_kernel") if "ELi256E" in k]
    assert len(hand_placed) == 2
    for k in hand_placed:                          # the check did look at hand-placed instructions
        body = asm[asm.index(k + ":"):]
        assert "v_mfma_f32_32x32x16_bf16 v[" in body[:body.index(".Lfunc_end")]
