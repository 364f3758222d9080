"""The generated device code: no packed-fp32 VALU instructions (the build switches the feature
off for the device pass; this checks that the switch is honoured), and no kernel spills registers
to scratch memory (spill traffic would show up as HBM bytes beyond the algorithmic ones)."""
import os
import re
import tempfile

import pytest

from paper_2503_08154_amd import build


@pytest.fixture(scope="module")
def device_asm():
    with tempfile.TemporaryDirectory() as d:
        path = build.device_assembly(os.path.join(d, "s2a_device.s"))
        text = open(path).read()
    assert "s2a" in text and "fwd_kernel" in text          # it is the library's device code
    return text


def test_device_code_has_no_packed_fp32_arithmetic(device_asm):
    found = sorted(set(re.findall(r"\bv_pk_(?:add|mul|fma)_f32\b", device_asm)))
    assert not found, f"packed fp32 instructions in the device code: {found}"


def test_no_kernel_uses_scratch_memory(device_asm):
    kernels = re.findall(r"\.amdhsa_kernel (\S+)(.*?)\.end_amdhsa_kernel", device_asm, re.S)
    assert len(kernels) > 50
    spilling = {}
    for name, body in kernels:
        size = int(re.search(r"\.amdhsa_private_segment_fixed_size\s+(\d+)", body).group(1))
        if size:
            spilling[name] = size
    assert not spilling, f"kernels with per-lane scratch (register spills), bytes per lane: {spilling}"
