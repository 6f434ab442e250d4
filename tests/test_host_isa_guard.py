"""The build's scan for matrix instructions that could run under an empty execution mask."""
from paper_2504_00030_amd import isa_guard

BAD = """
_ZN2sd1kEv:
\ts_and_saveexec_b64 s[40:41], vcc
; %bb.63:
\tv_mfma_f32_16x16x32_bf16 a[0:3], v[104:107], v[48:51], a[0:3]
\ts_or_b64 exec, exec, s[40:41]
\ts_endpgm
"""

GOOD_SKIPPED = """
_ZN2sd1kEv:
\ts_and_saveexec_b64 s[40:41], vcc
\ts_cbranch_execz .LBB0_2
\tv_mfma_f32_16x16x32_bf16 a[0:3], v[104:107], v[48:51], a[0:3]
.LBB0_2:
\ts_or_b64 exec, exec, s[40:41]
\tv_mfma_f32_16x16x32_bf16 a[0:3], v[104:107], v[48:51], a[0:3]
\ts_endpgm
"""

GOOD_RESTORED = """
_ZN2sd1kEv:
\ts_and_saveexec_b64 s[0:1], vcc
\tglobal_load_dword v1, v[2:3], off
\ts_or_b64 exec, exec, s[0:1]
\tv_mfma_f32_16x16x32_bf16 a[0:3], v[104:107], v[48:51], a[0:3]
\ts_endpgm
"""


def test_flags_matrix_instruction_in_unskipped_masked_block():
    msgs = isa_guard.scan(BAD)
    assert len(msgs) == 1 and "_ZN2sd1kEv" in msgs[0]


def test_accepts_skipped_or_restored_blocks():
    assert isa_guard.scan(GOOD_SKIPPED) == []
    assert isa_guard.scan(GOOD_RESTORED) == []
