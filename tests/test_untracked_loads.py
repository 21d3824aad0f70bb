"""Host-side check of the build's guard for loads issued as uninterpreted inline assembly
(build.untracked_load_violations): it accepts the kernel as compiled and catches a planted early use."""
import os
import shutil

import pytest

from paper_2511_21699_amd import build

LISTING = """
\ts_mov_b32 s0, 0
\t;;#ASMSTART
\tglobal_load_dwordx4 v[6:9], v[2:3], off
\t;;#ASMEND
\tv_or_b32_e32 v2, 0x200, v0
%s
\ts_waitcnt vmcnt(8)
\ts_barrier
\tv_mfma_f32_16x16x32_bf16 v[56:59], v[56:59], v[6:9], 0
"""


def test_checker_accepts_a_wait_before_the_first_use():
    assert build.untracked_load_violations(LISTING % "\tv_add_u32_e32 v10, v11, v12") == []


@pytest.mark.parametrize("early", ["\tv_mov_b32_e32 v40, v7", "\tv_mov_b64_e32 v[40:41], v[8:9]",
                                   "\tbuffer_store_dword v6, off, s[0:3], 0 offset:4",
                                   "\tv_accvgpr_write_b32 a0, v9"])
def test_checker_reports_a_use_before_the_wait(early):
    bad = build.untracked_load_violations(LISTING % early)
    assert len(bad) == 1 and "global_load_dwordx4 v[6:9]" in bad[0][1]


def test_checker_ignores_loads_the_compiler_tracks():
    text = "\tglobal_load_dwordx4 v[6:9], v[2:3], off\n\tv_mov_b32_e32 v40, v7\n"
    assert build.untracked_load_violations(text) == []


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_compiled_attention_kernel_passes():
    asm = build.device_asm(os.path.join(build.CSRC, "cb_attn_mfma.hip"))
    assert asm.count("global_load_lds_dwordx4") > 50          # the ring's requests are there, as inline assembly
    assert build.untracked_load_violations(asm) == []
    res = build.kernel_resources(asm)
    attn = {k: v for k, v in res.items() if "k_attn_mfma" in k or "k_verify_mfma" in k}
    assert len(attn) == 8                                      # four variants, each with and without the timeline stamps
    assert build.scratch_violations(asm) == []
    assert all(v[0] <= 256 for v in attn.values())             # two waves per SIMD


def test_scratch_checker_reports_spills():
    meta = """
  - .name:           k_good
    .private_segment_fixed_size: 0
    .vgpr_count:     200
    .vgpr_spill_count: 0
  - .name:           k_spills
    .private_segment_fixed_size: 864
    .vgpr_count:     256
    .vgpr_spill_count: 216
"""
    assert build.kernel_resources(meta) == {"k_good": (200, 0, 0), "k_spills": (256, 216, 864)}
    assert [k for k, _ in build.scratch_violations(meta)] == ["k_spills"]
