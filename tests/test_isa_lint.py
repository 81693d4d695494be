"""The compiled kernels hold no matrix instruction inside an execution-mask region that the compiler left
without a skip branch (MFMA ignores EXEC: such an instruction runs although its source-level condition is
false).  This is the cause of a wrong result the streaming GEMM once gave for one launch shape: the MFMAs of
register slots past a wavefront's K share ran with an empty mask and added the last weight tile again."""
from paper_2603_25702_amd import isa_lint

BAD = """
_Z6kernelv:
	v_cmp_lt_i32_e32 vcc, v18, v66
	s_and_saveexec_b64 s[20:21], vcc
; %bb.12:
	v_mfma_f32_16x16x32_bf16 v[54:57], v[6:9], v[46:49], v[54:57]
	s_or_b64 exec, exec, s[20:21]
	v_mfma_f32_16x16x32_bf16 v[54:57], v[6:9], v[46:49], v[54:57]
	s_endpgm
"""
GOOD = """
_Z6kernelv:
	v_cmp_lt_i32_e32 vcc, v18, v66
	s_and_saveexec_b64 s[20:21], vcc
	s_cbranch_execz .LBB0_2
; %bb.12:
	v_mfma_f32_16x16x32_bf16 v[54:57], v[6:9], v[46:49], v[54:57]
.LBB0_2:
	s_or_b64 exec, exec, s[20:21]
	s_cmp_ge_i32 s14, s12
	s_cbranch_scc1 .LBB0_3
	v_mfma_f32_16x16x32_bf16 v[54:57], v[6:9], v[46:49], v[54:57]
.LBB0_3:
	s_endpgm
"""


def test_scanner_flags_an_mfma_in_a_mask_region_without_a_skip_branch():
    found = isa_lint.scan_asm(BAD)
    assert [(k, no) for k, no, _ in found] == [("_Z6kernelv", 6)]
    assert isa_lint.scan_asm(GOOD) == []


def test_compiled_kernels_have_no_mfma_under_a_narrowed_execution_mask():
    found = isa_lint.lint_sources()
    assert not found, "\n".join(f"{s}: {k}: line {no}: {ins}" for s, k, no, ins in found[:20])
