"""Static checks on the compiled MFMA kernels (CPU only: hipcc cross-compiles gfx950).

The dK/dV kernel keeps dK, dV and its K/V fragments in the accumulation registers
a[0:191] and addresses them by name from inline assembly.  That is only sound while the
compiler itself never touches an accumulation register in that kernel and spills nothing,
which is what these tests pin down, together with the absence of spills in the other two
kernels (a spill there costs scratch traffic in the hot loop).
"""
import os
import re

import pytest

from paper_2410_20305_amd import build


def _asm(tmp_path, src):
    return build.device_asm(src, str(tmp_path / (src + ".s")))


def _kernel_meta(text, kernel):
    """amdhsa.kernels metadata entry whose .name contains `kernel`, as a dict of scalars."""
    blocks = re.split(r"\n  - \.agpr_count:", text)
    for b in blocks[1:]:
        b = ".agpr_count:" + b
        if re.search(r"\.name:\s+\S*" + kernel, b):
            return {k: v for k, v in re.findall(r"\.([a-z_]+):\s+(\S+)", b)}
    raise AssertionError("no metadata for " + kernel)


def test_dkdv_accumulation_registers_belong_to_the_assembly(tmp_path):
    text = _asm(tmp_path, "psattn_mfma_dkdv.hip")
    body = text.split(".amdhsa_kernel")[0]
    inside = False
    offenders = []
    for ln in body.splitlines():
        if "#ASMSTART" in ln:
            inside = True
        elif "#ASMEND" in ln:
            inside = False
        elif not inside:
            code = ln.split(";")[0]
            if re.search(r"accvgpr|\ba\[|[ ,\[]a\d+\b", code):
                offenders.append(ln.strip())
    assert not offenders, offenders[:5]
    meta = _kernel_meta(text, "psattn_dkdv_bf16_mfma")
    assert int(meta["agpr_count"]) == 192
    assert int(meta["vgpr_spill_count"]) == 0 and int(meta["sgpr_spill_count"]) == 0
    assert int(meta["private_segment_fixed_size"]) == 0
    # one wave per SIMD: ordinary + accumulation registers of one lane
    assert int(meta["vgpr_count"]) <= 512


@pytest.mark.parametrize("src,kernel", [("psattn_mfma_fwd.hip", "psattn_fwd_bf16_mfma"),
                                        ("psattn_mfma_bwd.hip", "psattn_dq_bf16_mfma")])
def test_two_workgroups_per_cu_without_spills(tmp_path, src, kernel):
    meta = _kernel_meta(_asm(tmp_path, src), kernel)
    assert int(meta["vgpr_count"]) <= 256          # two waves per SIMD
    assert int(meta["agpr_count"]) == 0
    assert int(meta["vgpr_spill_count"]) == 0 and int(meta["sgpr_spill_count"]) == 0
    assert int(meta["private_segment_fixed_size"]) == 0
    assert int(meta["group_segment_fixed_size"]) <= 80 * 1024  # two workgroups in 160 KB of LDS


def _outside_asm(text):
    """Instruction lines of the device code that the compiler itself emitted."""
    body = text.split(".amdhsa_kernel")[0]
    inside = False
    for ln in body.splitlines():
        if "#ASMSTART" in ln:
            inside = True
        elif "#ASMEND" in ln:
            inside = False
        elif not inside:
            code = ln.split(";")[0].strip()
            if code and not code.startswith(".") and not code.endswith(":"):
                yield code


@pytest.mark.parametrize("src", ["psattn_mfma_fwd.hip", "psattn_mfma_bwd.hip", "psattn_mfma_dkdv.hip"])
def test_compiler_keeps_m0_and_the_copy_counter_free(tmp_path, src):
    """The asynchronous global -> LDS copies are issued from inline assembly that writes M0
    and counts its own outstanding copies (vmcnt).  Sound only while compiled code never
    keeps a value in M0, and while the only vector-memory loads the compiler issues between
    the first and the last copy are the one-dword tile-list refills."""
    text = _asm(tmp_path, src)
    for code in _outside_asm(text):
        assert not re.search(r"\bm0\b", code), code
    body = text.split(".amdhsa_kernel")[0]
    first, last = body.index("global_load_lds_dwordx4"), body.rindex("global_load_lds_dwordx4")
    loop = body[first:last]
    inside = True  # the slice starts in the middle of an assembly statement
    for ln in loop.splitlines():
        if "#ASMSTART" in ln:
            inside = True
        elif "#ASMEND" in ln:
            inside = False
        elif not inside:
            code = ln.split(";")[0].strip()
            m = re.match(r"(global_load|buffer_load|flat_load|scratch_load)\w*", code)
            if m:
                assert m.group(0) == "global_load_dword", code
