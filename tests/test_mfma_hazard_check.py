"""The build-time scan of the generated assembly (paper_2506_20675_amd/mfma_hazard_check.py) on hand-written snippets:
it must flag a matrix-core result that is read too soon on ANY path (in particular behind a taken branch, where the
compiler's own padding has been seen to fall short) and accept padded code and MFMA-to-MFMA accumulation."""
from paper_2506_20675_amd import mfma_hazard_check as chk

HEAD = "kern:\n"
MFMA = "\tv_mfma_f32_16x16x32_bf16 a[4:7], v[10:13], v[14:17], a[4:7]\n"
END = "\ts_endpgm\n"


def test_reader_behind_a_taken_branch_is_flagged_and_the_fall_through_alone_is_not_enough():
    asm = (HEAD + MFMA + "\ts_cbranch_scc1 .LBB0_2\n"
           + "".join(f"\tglobal_load_dwordx4 v[{20 + 4 * i}:{23 + 4 * i}], v4, s[16:17]\n" for i in range(6))
           + ".LBB0_2:\n\ts_add_i32 s1, s4, 6\n\ts_nop 0\n\tv_accvgpr_read_b32 v105, a7\n" + END)
    bad = chk.check(asm, 8)
    assert len(bad) == 1 and bad[0][0] == "kern" and bad[0][3] == 3 and "v_accvgpr_read_b32" in bad[0][2]
    assert chk.check(asm, 3) == []                       # the short path has exactly 3 slots


def test_padding_counts_n_plus_one_slots_and_clears_the_reader():
    asm = HEAD + MFMA + "\ts_nop 7\n\ts_cbranch_scc1 .LBB0_2\n.LBB0_2:\n\tv_accvgpr_read_b32 v105, a7\n" + END
    assert chk.check(asm, 8) == []
    asm = HEAD + MFMA + "\ts_nop 5\n\tv_accvgpr_read_b32 v105, a7\n" + END
    assert [b[3] for b in chk.check(asm, 8)] == [6]


def test_accumulating_mfma_and_unrelated_registers_are_not_readers():
    asm = (HEAD + MFMA + MFMA + "\tv_add_f32_e32 v1, v2, v3\n\tglobal_store_dwordx4 v[0:1], v[20:23], off\n"
           + "\ts_nop 7\n\tv_accvgpr_read_b32 v9, a4\n" + END)
    assert chk.check(asm, 8) == []


def test_stores_and_vector_alu_reads_of_the_result_are_readers():
    for reader in ("\tds_write_b128 v3, a[4:7]\n", "\tscratch_store_dwordx4 off, a[4:7], off offset:16\n",
                   "\tv_add_f32_e32 v8, v8, a5\n"):
        asm = HEAD + MFMA + "\ts_nop 1\n" + reader + END
        assert [b[3] for b in chk.check(asm, 8)] == [2], reader


def test_loop_back_edge_is_followed():
    asm = (HEAD + ".LBB0_1:\n\tv_accvgpr_read_b32 v111, a7\n" + MFMA + "\ts_add_i32 s19, s19, 4\n\ts_cmp_lt_i32 s21, s19\n"
           + "\ts_cbranch_scc1 .LBB0_1\n" + END)
    assert [b[3] for b in chk.check(asm, 8)] == [3]
