"""The two checks the build runs over the generated code of the hot kernels (paper_2309_14509_amd/build.py),
on hand-made snippets: each must flag the mistake it is there for and accept the safe form."""
from paper_2309_14509_amd import build

HEAD = "_Z6kernelv:\n"
ASM_MFMA = ";;#ASMSTART\n\tv_mfma_f32_32x32x16_bf16 v[0:15], v[20:23], a[0:3], v[0:15]\n;;#ASMEND\n"


def test_result_of_a_hand_written_mfma_touched_at_once_is_flagged():
    bad = HEAD + ASM_MFMA + "\tv_add_f32_e32 v40, v41, v42\n\tv_min3_i32 v0, s4, v50, v51\n\ts_endpgm\n"
    found = build.early_touches_of_asm_mfma_results(bad)
    assert len(found) == 1 and "v_min3_i32" in found[0][2]


def test_result_left_alone_long_enough_is_accepted():
    nops = "\ts_nop 15\n" * 4
    assert build.early_touches_of_asm_mfma_results(HEAD + ASM_MFMA + nops + "\tv_min3_i32 v0, s4, v50, v51\n\ts_endpgm\n") == []
    two_mfmas = "\tv_mfma_f32_32x32x16_bf16 a[0:15], v[30:33], v[34:37], a[0:15]\n" * 2
    assert build.early_touches_of_asm_mfma_results(HEAD + ASM_MFMA + two_mfmas + "\tv_max_f32_e32 v60, v1, v2\n\ts_endpgm\n") == []


def test_an_accumulation_chain_in_place_is_accepted_and_the_compilers_own_mfmas_are_not_checked():
    chain = HEAD + ASM_MFMA + ASM_MFMA + "\ts_nop 15\n" * 4 + "\ts_endpgm\n"
    assert build.early_touches_of_asm_mfma_results(chain) == []
    own = HEAD + "\tv_mfma_f32_32x32x16_bf16 v[0:15], v[20:23], v[24:27], v[0:15]\n\tv_mov_b32_e32 v0, v1\n\ts_endpgm\n"
    assert build.early_touches_of_asm_mfma_results(own) == []


def test_the_other_side_of_a_branch_is_followed():
    text = (HEAD + ASM_MFMA + "\ts_cbranch_scc1 .LBB0_2\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_endpgm\n"
            ".LBB0_2:\n\tv_mov_b32_e32 v3, v70\n\ts_endpgm\n")
    found = build.early_touches_of_asm_mfma_results(text)
    assert len(found) == 1 and "v_mov_b32" in found[0][2]


KERNEL = "_ZN3uly4bf1619attn_fwd_q64_kernelILb1EEEvv:\n"


def test_register_of_an_lds_read_in_flight_copied_is_flagged():
    bad = KERNEL + "\tds_read_b128 v[8:11], v2 offset:64\n\tv_mov_b64_e32 v[30:31], v[10:11]\n\ts_waitcnt lgkmcnt(0)\n\ts_endpgm\n"
    found = build.touches_of_lds_reads_in_flight(bad)
    assert len(found) == 1 and "v_mov_b64" in found[0][2]


def test_partial_waits_retire_the_oldest_reads_only():
    text = (KERNEL + "\tds_read_b128 v[8:11], v2\n\tds_read_b128 v[12:15], v2 offset:16\n\ts_waitcnt lgkmcnt(1)\n"
            "\tv_mov_b32_e32 v40, v8\n\tv_mov_b32_e32 v41, v12\n\ts_waitcnt lgkmcnt(0)\n\tv_mov_b32_e32 v42, v13\n\ts_endpgm\n")
    found = build.touches_of_lds_reads_in_flight(text)
    assert [f[2] for f in found] == ["v_mov_b32_e32 v41, v12"]


def test_kernels_that_manage_their_reads_through_the_compiler_are_not_checked():
    other = "_Z5otherv:\n\tds_read_b128 v[8:11], v2\n\tv_mov_b32_e32 v40, v8\n\ts_endpgm\n"
    assert build.touches_of_lds_reads_in_flight(other) == []


def test_a_read_in_flight_is_followed_into_both_sides_of_a_branch():
    text = (KERNEL + "\tds_read_b128 v[8:11], v2\n\ts_cbranch_scc1 .LBB0_2\n\ts_waitcnt lgkmcnt(0)\n\tv_mov_b32_e32 v40, v8\n\ts_endpgm\n"
            ".LBB0_2:\n\tv_mov_b64_e32 v[50:51], v[8:9]\n\ts_waitcnt lgkmcnt(0)\n\ts_endpgm\n")
    found = build.touches_of_lds_reads_in_flight(text)
    assert [f[2] for f in found] == ["v_mov_b64_e32 v[50:51], v[8:9]"]


def test_lds_writes_count_in_the_same_counter():
    text = (KERNEL + "\tds_read_b128 v[8:11], v2\n\tds_write_b32 v3, v4\n\ts_waitcnt lgkmcnt(1)\n\tv_mov_b32_e32 v40, v8\n\ts_endpgm\n")
    assert build.touches_of_lds_reads_in_flight(text) == []
