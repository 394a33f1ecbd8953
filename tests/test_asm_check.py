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


ASM_MFMA = ("\t;;#ASMSTART\n\ts_nop 1\n\tv_mfma_f32_32x32x16_bf16 v[34:49], v[70:73], a[160:163], v[34:49]\n"
            "\t;;#ASMEND\n")
OTHER_MFMA = "\tv_mfma_f32_32x32x16_bf16 a[0:15], v[80:83], v[90:93], a[0:15]\n"


def test_early_read_of_an_assembly_mfma_result_is_flagged():
    # a register-allocator copy straight behind the MFMA, a spill, a vector op after one more MFMA
    for reader in ("\tv_accvgpr_write_b32 a200, v40\n", "\tscratch_store_dword off, v34, off offset:16\n",
                   "\tv_fma_f32 v1, v49, v2, v3\n"):
        bad = asm_check.find_early_reads_of_asm_mfma_results(ASM_MFMA + reader)
        assert len(bad) == 1 and "0 wait states" in bad[0], reader
    bad = asm_check.find_early_reads_of_asm_mfma_results(ASM_MFMA + OTHER_MFMA + "\tv_add_f32 v1, v34, v2\n")
    assert len(bad) == 1 and "8 wait states" in bad[0]


def test_late_reads_chained_mfmas_and_writes_pass():
    check = asm_check.find_early_reads_of_asm_mfma_results
    # two further MFMAs, or one and a few instructions, or twelve plain instructions
    assert check(ASM_MFMA + OTHER_MFMA + OTHER_MFMA + "\tv_add_f32 v1, v34, v2\n") == []
    assert check(ASM_MFMA + OTHER_MFMA + "\ts_nop 3\n" + "\tv_add_f32 v1, v34, v2\n") == []
    assert check(ASM_MFMA + "\ts_add_i32 s1, s1, 1\n" * 12 + "\tv_add_f32 v1, v34, v2\n") == []
    # the next MFMA of the same chain reads the block as its accumulator input
    assert check(ASM_MFMA + ASM_MFMA + ASM_MFMA) == []
    # other registers; an MFMA the compiler knows about is its own business
    assert check(ASM_MFMA + "\tv_add_f32 v1, v50, v2\n\tv_mov_b32_e32 v60, v33\n") == []
    assert check(OTHER_MFMA + "\tv_accvgpr_read_b32 v1, a0\n") == []


def test_foreign_use_of_an_assembly_loaded_register_is_reported():
    """Registers written by inline-assembly global loads may only be touched by inline assembly
    until the last inline-assembly LDS store: a compiler-made copy in between is reported."""
    ok = """
kernel_a:
	;;#ASMSTART
	global_load_dwordx4 a[0:3], v1, s[2:3]
	;;#ASMEND
	v_add_u32_e32 v9, v8, v7
	;;#ASMSTART
	s_waitcnt vmcnt(0)
	;;#ASMEND
	;;#ASMSTART
	ds_write_b128 v5, a[0:3]
	;;#ASMEND
	v_accvgpr_read_b32 v2, a1
	s_endpgm
"""
    assert asm_check.find_foreign_uses_of_asm_loaded_registers(ok) == []
    bad = ok.replace("v_add_u32_e32 v9, v8, v7", "v_accvgpr_read_b32 v9, a2")
    found = asm_check.find_foreign_uses_of_asm_loaded_registers(bad)
    assert len(found) == 1 and "a2" in found[0].replace("('a', 2)", "a2")


def _asm_dot(dst, src):
    return "\t;;#ASMSTART\n\tv_dot2c_f32_bf16_e32 %s, %s, %s\n\t;;#ASMEND\n" % (dst, src, src)


def test_early_read_of_an_assembly_dot_product_result_is_flagged():
    check = asm_check.find_early_reads_of_asm_dot_results
    dpp = "\tv_add_f32_dpp v9, v9, v9 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
    other = "\tv_mul_f32_e32 v20, v21, v22\n"
    for gap in (0, 1, 2):
        bad = check(_asm_dot("v9", "v3") + other * gap + dpp)
        assert len(bad) == 1 and "%d wait states" % gap in bad[0]
    assert check(_asm_dot("v9", "v3") + other * 3 + dpp) == []
    assert check(_asm_dot("v9", "v3") + "\ts_nop 2\n" + dpp) == []
    # a chain of dot products into one accumulator is fine; its END is what gets checked
    chain = _asm_dot("v9", "v3") + _asm_dot("v9", "v4") + _asm_dot("v9", "v5")
    assert check(chain + other * 3 + dpp) == []
    assert len(check(chain + other + dpp)) == 1
    # a dot product that takes the fresh result as a FACTOR is not the chain
    assert len(check(_asm_dot("v9", "v3") + _asm_dot("v10", "v9"))) == 1
    # overwriting the result early is reported too; other registers are nobody's business
    assert len(check(_asm_dot("v9", "v3") + "\tv_mov_b32_e32 v9, 0\n")) == 1
    assert check(_asm_dot("v9", "v3") + "\tv_mov_b32_e32 v8, v10\n" + dpp.replace("v9", "v7")) == []
