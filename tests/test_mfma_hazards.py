"""The build-time check for MFMA results touched before write-back (paper_2604_26881_amd/mfma_hazards.py), on
hand-written assembly: the control-flow case the compiler's own padding misses, the padded forms, and a result
in ordinary vector registers."""
import textwrap

from paper_2604_26881_amd import mfma_hazards as H


def kernel(body: str) -> str:
    return "kern:\n" + textwrap.dedent(body) + "\ts_endpgm\n"


def flagged(tmp_path, body: str):
    p = tmp_path / "k.s"
    p.write_text(kernel(body))
    return H.check_file(str(p))


FILLER = "\ts_add_u32 s0, s0, 1\n"


def test_read_behind_a_branch_is_found(tmp_path):
    # the last MFMA of a loop, a conditional branch over a block, and the accumulator read at the branch target:
    # 11 instructions lie between them in straight-line order, 2 along the taken branch
    body = ("\tv_mfma_f32_32x32x16_bf16 a[0:15], v[2:5], v[6:9], a[0:15]\n"
            "\ts_cbranch_vccnz .LBB0_2\n" + FILLER * 10 + ".LBB0_2:\n" + FILLER +
            "\tv_accvgpr_read_b32 v17, a15\n")
    out = flagged(tmp_path, body)
    assert len(out) == 1 and "a15" in out[0] and "needs 11" in out[0]


def test_padding_on_every_path_passes(tmp_path):
    body = ("\tv_mfma_f32_32x32x16_bf16 a[0:15], v[2:5], v[6:9], a[0:15]\n"
            "\ts_cbranch_vccnz .LBB0_2\n" + FILLER * 10 + ".LBB0_2:\n\ts_nop 9\n"
            "\tv_accvgpr_read_b32 v17, a15\n")
    assert flagged(tmp_path, body) == []
    straight = ("\tv_mfma_f32_32x32x16_bf16 a[0:15], v[2:5], v[6:9], a[0:15]\n" + FILLER * 11 +
                "\tv_accvgpr_read_b32 v17, a15\n")
    assert flagged(tmp_path, straight) == []
    one_short = straight.replace(FILLER * 11, FILLER * 10)
    assert len(flagged(tmp_path, one_short)) == 1


def test_other_registers_and_back_to_back_mfmas_are_not_flagged(tmp_path):
    body = ("\tv_mfma_f32_32x32x16_bf16 a[0:15], v[2:5], v[6:9], a[0:15]\n"
            "\tv_mfma_f32_32x32x16_bf16 a[0:15], v[2:5], v[6:9], a[0:15]\n"      # accumulating on: the pipe's own business
            "\tv_accvgpr_read_b32 v17, a16\n"                                    # another accumulator
            "\tv_add_u32_e32 v2, v3, v4\n" + FILLER * 11 +
            "\tv_accvgpr_read_b32 v18, a0\n")
    assert flagged(tmp_path, body) == []


def test_results_in_ordinary_registers_and_the_shorter_mfma(tmp_path):
    # 16x16x32 (4 passes) writing v[10:13]: 7 wait states before anything else reads or overwrites them
    body = ("\tv_mfma_f32_16x16x32_bf16 v[10:13], v[2:5], v[6:9], v[10:13]\n" + FILLER * 6 +
            "\tv_add_f32_e32 v20, v12, v14\n")
    out = flagged(tmp_path, body)
    assert len(out) == 1 and "needs 7" in out[0]
    assert flagged(tmp_path, body.replace(FILLER * 6, FILLER * 7)) == []
    # through a loop back-edge: the read at the loop head follows the MFMA at the loop's end
    loop = (".LBB0_1:\n\tv_mov_b32_e32 v30, v10\n" + FILLER * 3 +
            "\tv_mfma_f32_16x16x32_bf16 v[10:13], v[2:5], v[6:9], v[10:13]\n"
            "\ts_cbranch_scc1 .LBB0_1\n")
    assert len(flagged(tmp_path, loop)) == 1


def test_lds_writing_load_directly_behind_the_write_of_m0(tmp_path):
    bad = "\ts_mov_b32 m0, s5\n\tglobal_load_lds_dwordx4 v2, s[4:5]\n"
    out = flagged(tmp_path, bad)
    assert len(out) == 1 and "m0" in out[0]
    assert flagged(tmp_path, "\ts_mov_b32 m0, s5\n\ts_nop 0\n\tglobal_load_lds_dwordx4 v2, s[4:5]\n") == []
    assert flagged(tmp_path, "\ts_add_i32 m0, s0, 0x400\n\tglobal_load_lds_dwordx4 v[2:3], off\n") != []
    assert flagged(tmp_path, "\ts_mov_b32 m0, s5\n\tv_mov_b32_e32 v1, v2\n\tglobal_load_lds_dwordx4 v2, s[4:5] nt\n") == []
