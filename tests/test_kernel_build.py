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
