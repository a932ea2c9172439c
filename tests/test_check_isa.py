"""The static check of the generated code (check_isa.py) must itself report the hazards it
guards against: hand-written gfx950 snippets, each with one planted mistake."""
from paper_2511_22481_amd.check_isa import check

HEAD = "_ZN8omniattn13decode_kernelILi4ELb0EEEvNS_12DecodeParamsE:\n"
TAIL = "\ts_endpgm\n"
MFMA = "\tv_mfma_f32_32x32x16_bf16 v[2:17], v[190:193], v[26:29], v[2:17]\n"
MFMA_ACC = "\tv_mfma_f32_32x32x16_bf16 a[0:15], v[190:193], v[26:29], a[0:15]\n"


def test_clean_stream_passes():
    asm = HEAD + MFMA * 4 + "\ts_nop 11\n\tv_mul_f32_e32 v40, v2, v3\n" + TAIL
    assert check(asm) == []


def test_early_valu_read_is_reported():
    asm = HEAD + MFMA + "\ts_nop 3\n\tv_mul_f32_e32 v40, v2, v3\n" + TAIL
    probs = check(asm)
    assert probs and "wait states after MFMA write of v2" in probs[0]


def test_early_overwrite_is_reported():
    asm = HEAD + MFMA + "\tv_mov_b32_e32 v5, 0\n" + TAIL
    probs = check(asm)
    assert probs and "overwrite" in probs[0] and "v5" in probs[0]


def test_early_memory_read_needs_more_states():
    # 13 wait states are enough for the vector ALU but not for a store of the result
    asm = HEAD + MFMA + "\ts_nop 12\n\tglobal_store_dwordx4 v[60:61], v[2:5], off\n" + TAIL
    probs = check(asm)
    assert probs and "global_store" in probs[0]
    asm = HEAD + MFMA + "\ts_nop 15\n\ts_nop 3\n\tglobal_store_dwordx4 v[60:61], v[2:5], off\n" + TAIL
    assert check(asm) == []


def test_accumulator_read_through_accvgpr_is_reported():
    asm = HEAD + MFMA_ACC + "\tv_accvgpr_read_b32 v40, a3\n" + TAIL
    assert any("a3" in p for p in check(asm))


def test_mfma_operand_written_by_mfma_is_reported():
    asm = HEAD + MFMA + "\tv_mfma_f32_32x32x16_bf16 v[60:75], v[2:5], v[26:29], 0\n" + TAIL
    assert any("MFMA reads" in p for p in check(asm))


def test_spill_in_front_of_mfmas_is_reported():
    asm = HEAD + ".LBB0_1:\n\tscratch_load_dwordx4 v[238:241], off, off\n" + MFMA * 8 + TAIL
    assert any("spill" in p for p in check(asm))
    # behind a block's last MFMAs a spill access is harmless
    asm = HEAD + ".LBB0_1:\n" + MFMA * 8 + "\ts_nop 15\n\tscratch_store_dwordx4 off, v[238:241], off\n" + TAIL
    assert check(asm) == []


def test_other_kernels_are_not_checked():
    asm = "_ZN8omniattn14combine_kernelILb0EEEvNS_13CombineParamsE:\n" + MFMA + "\tv_mov_b32_e32 v5, 0\n" + TAIL
    assert check(asm) == []
