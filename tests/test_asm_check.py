"""The kernels with hand-placed LDS waits are only correct for compiler output in which nothing touches the
destination registers of an LDS read before the wait that covers it.  These CPU tests pin the compiler version
that was validated, run the static check on what this compiler generates, and show on small planted mistakes
that the check sees what it is meant to see."""
import os
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2407_12075_amd import asm_check, build as hip_build


def test_hipcc_is_the_validated_version():
    text = hip_build.hipcc_version()
    assert hip_build.VALIDATED_HIP_VERSION in text and hip_build.VALIDATED_CLANG in text, (
        "hipcc differs from the version the inline-assembly LDS reads were validated with "
        f"({hip_build.VALIDATED_HIP_VERSION}, {hip_build.VALIDATED_CLANG}); run `python -m paper_2407_12075_amd.asm_check` "
        "and the GPU tests with the new compiler, then update paper_2407_12075_amd/build.py.\n" + text)


def test_generated_assembly_has_no_early_use_of_pending_reads():
    srcs = [os.path.join(hip_build.CSRC, s) for s in asm_check.CHECKED_SOURCES]
    with ThreadPoolExecutor(max_workers=4) as ex:
        texts = list(ex.map(asm_check.compile_to_asm, srcs))
    for src, text in zip(srcs, texts):
        names, findings = asm_check.check_asm_text(text)
        assert names, f"no kernel found in the assembly of {src}"
        assert not findings, f"{src}:\n" + "\n".join(findings[:20])


_GOOD = """
kernel_a:
    s_load_dwordx2 s[0:1], s[4:5], 0x0
    s_waitcnt lgkmcnt(0)
    ds_read_b128 v[4:7], v1
    ds_read_b128 v[8:11], v1 offset:16
    v_add_u32_e32 v2, v2, v3
    s_waitcnt lgkmcnt(1)
    v_mfma_f32_32x32x16_bf16 a[0:15], v[4:7], v[12:15], a[0:15]
    s_waitcnt lgkmcnt(0)
    v_mfma_f32_32x32x16_bf16 a[0:15], v[8:11], v[12:15], a[0:15]
    s_endpgm
    .end_amdhsa_kernel
"""


def _check(text):
    names, findings = asm_check.check_asm_text(text)
    assert names == ["kernel_a"]
    return findings


def test_checker_accepts_correct_waits():
    assert _check(_GOOD) == []


@pytest.mark.parametrize("old,new,what", [
    # the wait that covers the first read lets one more read stay pending: the MFMA reads v[4:7] too early
    ("s_waitcnt lgkmcnt(1)", "s_waitcnt lgkmcnt(2)", "touches registers of a pending LDS read"),
    # a register copy out of a pending read (what a compiler-inserted move would look like)
    ("v_add_u32_e32 v2, v2, v3", "v_mov_b32_e32 v20, v9", "touches registers of a pending LDS read"),
    # an LDS read whose address register is the destination of a read that is still pending
    ("ds_read_b128 v[8:11], v1 offset:16", "ds_read_b128 v[8:11], v5 offset:16", "uses registers of a pending LDS read"),
    # a scalar load shares the counter but returns out of order
    ("v_add_u32_e32 v2, v2, v3", "s_load_dword s6, s[0:1], 0x0", "scalar load"),
    # reads still in flight at the end of the program
    ("    s_waitcnt lgkmcnt(0)\n    v_mfma_f32_32x32x16_bf16 a[0:15], v[8:11], v[12:15], a[0:15]\n", "", "pending at s_endpgm"),
])
def test_checker_sees_planted_mistakes(old, new, what):
    assert old in _GOOD
    findings = _check(_GOOD.replace(old, new))
    assert any(what in f for f in findings), findings


def test_checker_follows_branches():
    # the read is pending on the path that skips the wait
    text = """
kernel_a:
    ds_read_b128 v[4:7], v1
    s_cbranch_scc1 .LBB0_2
    s_waitcnt lgkmcnt(0)
.LBB0_2:
    v_add_f32_e32 v8, v4, v4
    s_waitcnt lgkmcnt(0)
    s_endpgm
    .end_amdhsa_kernel
"""
    assert any("touches registers" in f for f in _check(text))
