"""Host-side checks of the build's assembly verifier (no GPU, no compiler)."""
from paper_2605_29157_amd import asm_check

MFMA = "\tv_mfma_f32_32x32x16_bf16 v[34:49], v[70:73], a[160:163], v[34:49] ; unguarded\n"


def test_clean_sequence_passes():
    asm = "\tds_read_b128 v[2:5], v1 offset:32\n\ts_waitcnt lgkmcnt(2)\n" + MFMA
    assert asm_check.find_violations(asm) == []


def test_late_vector_write_of_a_source_is_flagged():
    asm = "\ts_waitcnt lgkmcnt(2)\n\tv_accvgpr_read_b32 v71, a9\n" + MFMA
    bad = asm_check.find_violations(asm)
    assert len(bad) == 1 and "v_accvgpr_read_b32" in bad[0]
    # two instructions earlier is still inside the window
    asm = "\tv_mov_b32_e32 v36, 0\n\ts_add_i32 s1, s1, 1\n" + MFMA
    assert len(asm_check.find_violations(asm)) == 1


def test_write_outside_the_window_or_of_other_registers_passes():
    asm = "\tv_mov_b32_e32 v36, 0\n\ts_add_i32 s1, s1, 1\n\ts_add_i32 s2, s2, 1\n" + MFMA
    assert asm_check.find_violations(asm) == []
    asm = "\tv_mov_b32_e32 v36, 0\n\ts_nop 1\n" + MFMA          # s_nop 1 = two wait states
    assert asm_check.find_violations(asm) == []
    asm = "\tv_mov_b32_e32 v100, 0\n\tv_mov_b32_e32 v74, 0\n" + MFMA
    assert asm_check.find_violations(asm) == []


def test_branch_target_just_before_is_flagged_and_marker_is_required():
    asm = "\ts_add_i32 s1, s1, 1\n.LBB0_3:\n" + MFMA
    assert any("branch target" in b for b in asm_check.find_violations(asm))
    guarded = "\ts_nop 1\n\tv_mfma_f32_32x32x16_bf16 v[34:49], v[70:73], a[160:163], v[34:49]\n"
    assert any("no unguarded MFMA" in b for b in asm_check.find_violations(guarded))


def test_m0_must_only_be_touched_by_the_inline_assembly():
    ok = "\t;;#ASMSTART\n\ts_mov_b32 m0, s4\n\tglobal_load_lds_dwordx4 v1, s[2:3]\n\t;;#ASMEND\n\ts_add_i32 s1, s1, 1\n"
    assert asm_check.find_m0_uses_outside_inline_asm(ok) == []
    bad = ok + "\ts_mov_b32 m0, -1\n\tds_read_b32 v1, v2\n"
    found = asm_check.find_m0_uses_outside_inline_asm(bad)
    assert len(found) == 1 and "s_mov_b32 m0, -1" in found[0]
