"""The build-time scan of the generated device assembly (host logic, no GPU): a value that the register
allocator brings back from the accumulation registers right in front of an asm matrix instruction that reads
it must fail the build; the same move far enough away, or feeding another register, must not."""
import os

from paper_2303_02191_amd.build import check_matrix_hazards

MFMA = "\t;;#ASMSTART\n\tv_smfmac_f32_16x16x64_bf16 a[0:3], v[10:13], v[20:27], v5 cbsz:0 abid:0\n\t;;#ASMEND\n"


def _scan(tmp_path, text):
    p = os.path.join(str(tmp_path), "k.s")
    with open(p, "w") as f:
        f.write(text)
    return check_matrix_hazards(p)


def test_parked_value_restored_in_front_of_matrix_instruction_is_flagged(tmp_path):
    found = _scan(tmp_path, "kernel:\n\tv_accvgpr_read_b32 v22, a200\n\tv_add_u32_e32 v1, v2, v3\n" + MFMA)
    assert len(found) == 1 and "v_accvgpr_read_b32 v22" in found[0][0] and "v_smfmac" in found[0][1]
    # the index register and the A operand count as sources too
    assert len(_scan(tmp_path, "\tv_accvgpr_read_b32 v5, a7\n" + MFMA)) == 1
    assert len(_scan(tmp_path, "\tv_accvgpr_mov_b32 v11, a7\n" + MFMA)) == 1


def test_distance_other_registers_and_compiler_emitted_instructions_pass(tmp_path):
    far = "\tv_accvgpr_read_b32 v22, a200\n" + "\tv_add_u32_e32 v1, v2, v3\n" * 4 + MFMA
    assert _scan(tmp_path, far) == []
    # s_nop N idles N + 1 cycles: s_nop 3 alone is distance enough
    assert _scan(tmp_path, "\tv_accvgpr_read_b32 v22, a200\n\ts_nop 3\n" + MFMA) == []
    assert len(_scan(tmp_path, "\tv_accvgpr_read_b32 v22, a200\n\ts_nop 1\n" + MFMA)) == 1
    # a restored value the matrix instruction does not read
    assert _scan(tmp_path, "\tv_accvgpr_read_b32 v40, a200\n" + MFMA) == []
    # an ordinary vector-ALU producer is interlocked by the hardware
    assert _scan(tmp_path, "\tv_perm_b32 v22, v1, v2, v3\n" + MFMA) == []
    # a matrix instruction the compiler emitted itself (no asm markers) gets its wait states from the compiler
    plain = "\tv_accvgpr_read_b32 v22, a200\n\tv_mfma_f32_16x16x32_bf16 a[0:3], v[10:13], v[20:23], a[0:3]\n"
    assert _scan(tmp_path, plain) == []
    # the destination of the matrix instruction is not a source
    assert _scan(tmp_path, "\tv_accvgpr_read_b32 v0, a200\n" + MFMA) == []


def test_accumulator_moves_right_behind_an_asm_matrix_instruction_are_flagged(tmp_path):
    # the compiler copying an accumulator that the asm instruction in front is still writing
    assert len(_scan(tmp_path, MFMA + "\ts_nop 0\n\tv_accvgpr_read_b32 v9, a2\n")) == 1
    assert len(_scan(tmp_path, MFMA + "\tv_accvgpr_mov_b32 a200, a3\n")) == 1
    assert len(_scan(tmp_path, MFMA + "\tv_accvgpr_write_b32 a0, v9\n")) == 1
    assert len(_scan(tmp_path, MFMA + "\tscratch_load_dwordx4 a[0:3], off, off offset:660\n")) == 1
    # other accumulators, or the same ones after the instruction has drained (two s_nop 15, as in front of the epilogues)
    assert _scan(tmp_path, MFMA + "\tv_accvgpr_read_b32 v9, a8\n") == []
    assert _scan(tmp_path, MFMA + "\ts_nop 15\n\ts_nop 15\n\tv_accvgpr_read_b32 v9, a2\n") == []
    # the next matrix instruction on the same accumulator is the hardware's business
    assert _scan(tmp_path, MFMA + MFMA) == []
