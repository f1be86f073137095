"""The compiled matrix-core kernels are scanned for results of matrix instructions that are read
too early on the far side of a branch (a case the compiler's own padding has missed; see
tests/isa_check.py).  CPU only: hipcc cross-compiles to assembly."""
from tests import isa_check

PLANTED = """
.LBB0_1:
	v_mfma_f32_32x32x16_bf16 a[64:79], v[72:75], v[112:115], a[64:79]
	s_cbranch_vccnz .LBB0_3
	v_add_u32_e32 v68, s57, v162
	v_ashrrev_i32_e32 v69, 31, v68
	v_and_b32_e32 v69, s16, v69
	v_add_u32_e32 v68, v68, v69
	v_cmp_ge_i32_e64 s[6:7], s21, v68
	v_mov_b32_e32 v1, 0
	v_mov_b32_e32 v2, 0
	v_mov_b32_e32 v3, 0
	v_mov_b32_e32 v4, 0
.LBB0_3:
	s_nop 1
	v_accvgpr_read_b32 v83, a79
	s_endpgm
"""

STRAIGHT = """
	v_mfma_f32_32x32x16_bf16 a[64:79], v[72:75], v[112:115], a[64:79]
	s_nop 11
	v_accvgpr_read_b32 v83, a79
	v_mfma_f32_32x32x16_bf16 a[0:15], v[72:75], v[112:115], a[0:15]
	v_mfma_f32_32x32x16_bf16 a[0:15], v[76:79], v[116:119], a[0:15]
	s_cbranch_scc1 .LBB0_9
	s_nop 15
.LBB0_9:
	s_nop 15
	v_accvgpr_read_b32 v1, a0
	s_endpgm
"""


def test_scanner_finds_a_result_read_too_early_across_a_branch():
    hits = isa_check.scan(PLANTED)
    assert len(hits) == 1
    mfma, reader, wait_states = hits[0]
    assert reader.startswith("v_accvgpr_read_b32 v83, a79") and wait_states == 3


INLINE_ASM = """
	v_mfma_f32_32x32x16_bf16 v[210:225], v[14:17], v[226:229], 0
	v_fma_f32 v16, s3, v210, v0
	s_endpgm
"""


def test_scanner_checks_vgpr_results_on_straight_paths_too():
    """A result tile in VGPRs comes from the kernels' inline assembly, which the compiler never pads."""
    hits = isa_check.scan(INLINE_ASM)
    assert len(hits) == 1 and hits[0][2] == 0


SRC_C = """
	v_mfma_f32_32x32x16_bf16 v[210:225], v[14:17], v[226:229], 0
	v_mfma_f32_32x32x16_bf16 v[100:115], v[14:17], v[226:229], v[210:225]
	s_endpgm
"""

RESTART = """
	v_mfma_f32_32x32x16_bf16 v[210:225], v[14:17], v[226:229], 0
	v_mfma_f32_32x32x16_bf16 v[210:225], v[18:21], v[230:233], 0
	s_endpgm
"""

DEEP = "\n\tv_mfma_f32_32x32x16_bf16 v[210:225], v[14:17], v[226:229], 0\n" + "".join(
    f"\ts_cbranch_scc1 .LBB0_{i}\n.LBB0_{i}:\n" for i in range(1, 9)) + "\tv_mov_b32_e32 v1, v210\n\ts_endpgm\n"


def test_scanner_counts_srcc_and_overlapping_destinations_of_other_matrix_instructions():
    """Another matrix instruction reads the tile as SrcC into a different destination, or restarts the
    same destination from zero: neither is the interlocked accumulation form."""
    assert len(isa_check.scan(SRC_C)) == 1
    assert len(isa_check.scan(RESTART)) == 1


def test_scanner_reports_the_branch_depth_limit():
    """Eight nested branches inside the hazard window: the walk gives up at depth 6 and must say so."""
    hits = isa_check.scan(DEEP)
    assert len(hits) == 1 and hits[0][1] == isa_check.DEPTH_LIMIT and hits[0][2] < isa_check.WAIT_STATES


def test_scanner_accepts_padded_code_and_accumulation_chains():
    assert isa_check.scan(STRAIGHT) == []


def test_compiled_kernels_are_clean():
    for src, hits in isa_check.check_all().items():
        assert not hits, (src, hits)
