"""The generated device code: no packed-fp32 VALU instructions (the build switches the feature
off for the device pass; this checks that the switch is honoured)."""
import os
import re
import tempfile

from paper_2503_08154_amd import build


def test_device_code_has_no_packed_fp32_arithmetic():
    with tempfile.TemporaryDirectory() as d:
        path = build.device_assembly(os.path.join(d, "s2a_device.s"))
        text = open(path).read()
    assert "s2a" in text and "fwd_kernel" in text          # it is the library's device code
    found = sorted(set(re.findall(r"\bv_pk_(?:add|mul|fma)_f32\b", text)))
    assert not found, f"packed fp32 instructions in the device code: {found}"
