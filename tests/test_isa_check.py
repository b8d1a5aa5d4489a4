"""The build-time check of the device assembly (an MFMA result must not be read by another unit sooner than
eight issue slots after the MFMA): the checker itself, on fabricated assembly text."""
from paper_2302_06646_amd import isa_check

GOOD = """
_Zkernel_good:
	v_mfma_f32_16x16x32_f16 v[10:13], v[2:5], v[6:9], 0
	v_mfma_f32_16x16x32_f16 v[14:17], v[2:5], v[6:9], 0
	s_nop 7
	v_cvt_pk_f16_f32 v20, v10, v14
	s_endpgm
.Lfunc_end0:
"""

BAD = """
_Zkernel_bad:
	v_mfma_f32_16x16x32_f16 v[10:13], v[2:5], v[6:9], 0
	v_mfma_f32_16x16x32_f16 v[14:17], v[2:5], v[6:9], 0
	s_cbranch_scc1 .LBB0_9
.LBB0_1:
	v_mov_b64_e32 v[30:31], v[12:13]
	s_nop 4
	v_mov_b64_e32 v[32:33], v[16:17]
	s_endpgm
.Lfunc_end1:
"""

CHAIN = """
_Zkernel_chain:
	v_mfma_f32_16x16x32_f16 v[10:13], v[2:5], v[6:9], 0
	v_mfma_f32_16x16x32_f16 v[10:13], v[2:5], v[6:9], v[10:13]
	s_nop 7
	ds_write_b128 v40, v[10:13]
	s_endpgm
.Lfunc_end2:
"""


def test_enough_slots_pass():
    assert isa_check.check_text(GOOD) == []
    (name, body), = list(isa_check.kernels(GOOD))
    assert name == "_Zkernel_good"
    assert isa_check.min_mfma_read_distance(body)[0] == 8      # s_nop 7 behind the second MFMA


def test_copy_right_behind_an_mfma_at_a_branch_is_flagged():
    bad = isa_check.check_text(BAD)
    assert len(bad) == 1 and bad[0][0] == "_Zkernel_bad" and bad[0][1] == 2
    assert "v_mov_b64" in bad[0][3]


def test_accumulator_chains_are_not_readers_and_stores_count_their_data():
    assert isa_check.check_text(CHAIN) == []
    (_, body), = list(isa_check.kernels(CHAIN))
    assert isa_check.min_mfma_read_distance(body)[0] == 8

TAKEN = """
_Zkernel_taken:
	v_mfma_f32_16x16x32_f16 v[10:13], v[2:5], v[6:9], 0
	s_cbranch_scc1 .LBB3_5
	s_nop 7
	v_cvt_pk_f16_f32 v20, v10, v11
	s_endpgm
.LBB3_5:
	v_ldexp_f32 v21, v12, s4
	s_endpgm
.Lfunc_end3:
"""


def test_the_taken_side_of_a_branch_is_followed_too():
    bad = isa_check.check_text(TAKEN)
    assert len(bad) == 1 and bad[0][1] == 1 and "v_ldexp_f32" in bad[0][3]
