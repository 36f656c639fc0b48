"""The wait-state checker that guards the hand-written matrix instructions: each rule fires on a listing that breaks
it and stays quiet on one that keeps it (text only, no GPU and no compiler involved)."""
from paper_2605_26266_amd import mfma_hazard_check as hc

MFMA = "v_mfma_scale_f32_32x32x64_f8f6f4 v[0:15], v[20:23], a[0:5], v[0:15], v30, v31 op_sel:[0,0,0] cbsz:4 blgp:2"


def test_result_read_too_early_is_reported():
    n, problems = hc.check("\n".join([MFMA, "s_nop 9", "v_add_f32 v40, v3, v41", "s_endpgm"]))
    assert n == 1 and len(problems) == 1 and "after 10 wait states" in problems[0]


def test_result_read_after_twelve_wait_states_passes():
    assert hc.check("\n".join([MFMA, "s_nop 11", "v_add_f32 v40, v3, v41", "s_endpgm"])) == (1, [])
    filler = ["v_mov_b32 v%d, v%d" % (50 + i, 70 + i) for i in range(12)]
    assert hc.check("\n".join([MFMA, *filler, "v_add_f32 v40, v15, v41", "s_endpgm"])) == (1, [])


def test_overwriting_the_destination_counts_like_a_read():
    _, problems = hc.check("\n".join([MFMA, "s_nop 3", "v_mov_b32 v7, 0", "s_endpgm"]))
    assert len(problems) == 1


def test_dependent_mfma_may_follow_at_once():
    second = MFMA.replace("v[20:23]", "v[24:27]")
    assert hc.check("\n".join([MFMA, second, "s_nop 11", "v_add_f32 v40, v3, v41", "s_endpgm"])) == (2, [])


def test_window_that_reaches_a_branch_is_open():
    _, problems = hc.check("\n".join([MFMA, "s_nop 4", "s_cbranch_scc1 .LBB0_3", "v_add_f32 v40, v3, v41"]))
    assert len(problems) == 1 and problems[0].startswith("open window")


def test_operand_written_right_before_the_mfma_is_reported():
    _, problems = hc.check("\n".join(["v_and_b32 v21, 0x33333333, v60", MFMA, "s_nop 11", "s_endpgm"]))
    assert len(problems) == 1 and "writes an operand" in problems[0]
    _, problems = hc.check("\n".join(["v_mov_b32 v30, 0x7f7f7f7f", "v_mov_b32 v90, v91", MFMA, "s_nop 11", "s_endpgm"]))
    assert len(problems) == 1                                 # the scale operand, one wait state earlier
    assert hc.check("\n".join(["v_and_b32 v21, 0x33333333, v60", "s_nop 1", MFMA, "s_nop 11", "s_endpgm"])) == (1, [])


def test_accumulation_register_destinations_are_the_compilers_business():
    ins = "v_mfma_f32_32x32x16_bf16 a[0:15], v[2:5], v[6:9], a[0:15]"
    assert hc.check("\n".join([ins, "v_accvgpr_read_b32 v1, a0", "s_endpgm"])) == (1, [])
