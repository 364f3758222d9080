"""Host-side checks of the C ABI: the library loads without a GPU, exports every
symbol include/*.h declares, and rejects bad arguments before touching a
device.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2503_08154_amd import s2a

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(s2a_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert _declared_symbols() == sorted(s2a.EXPORTS)


def test_library_exports_every_declared_symbol():
    lib = s2a.lib()
    for name in _declared_symbols():
        assert getattr(lib, name) is not None


def test_error_paths_need_no_gpu():
    lib = ctypes.CDLL(s2a.LIB_PATH)  # same handle; state is process-global
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every call below fails validation first
    odd_q = ctypes.c_void_p(0x1002)
    if lib.s2a_qtable_get(None, None, None) == s2a.ERR_NOT_INIT:
        assert s2a.act_fwd(fake, fake, fake, 8, s2a.F32, check=False) == s2a.ERR_NOT_INIT
        assert s2a.act_bwd(fake, fake, fake, 8, s2a.F32, check=False) == s2a.ERR_NOT_INIT
    for bad in (0, 1, 2, 8, 15, 17, 256, -16):
        assert s2a.qtable_init(bad, check=False) == s2a.ERR_LEVELS
    assert s2a.qtable_init(16) == s2a.OK
    assert s2a.qtable_init(16) == s2a.OK  # idempotent
    for fn in (s2a.act_fwd, s2a.act_bwd):
        assert fn(fake, fake, fake, 8, 2, check=False) == s2a.ERR_DTYPE
        assert fn(fake, fake, fake, 8, -1, check=False) == s2a.ERR_DTYPE
        assert fn(fake, fake, fake, -1, s2a.BF16, check=False) == s2a.ERR_SIZE
        assert fn(None, fake, fake, 8, s2a.BF16, check=False) == s2a.ERR_NULL
        assert fn(fake, None, fake, 8, s2a.F32, check=False) == s2a.ERR_NULL
        assert fn(fake, fake, None, 8, s2a.F32, check=False) == s2a.ERR_NULL
        assert fn(None, None, None, 0, s2a.F32, check=False) == s2a.OK  # n == 0: nothing to do
    with pytest.raises(s2a.S2AError):
        s2a.act_fwd(None, fake, fake, 8, s2a.BF16)
    # softmax entry points: checked before any device work, no table needed
    assert s2a.softmax_fwd(fake, fake, fake, fake, 4, 0, s2a.F32, check=False) == s2a.ERR_SIZE
    assert s2a.softmax_fwd(fake, fake, fake, fake, 4, s2a.SOFTMAX_MAX_L + 1, s2a.F32, check=False) == s2a.ERR_SIZE
    assert s2a.softmax_bwd(fake, fake, fake, None, 4, 8, s2a.BF16, check=False) == s2a.ERR_NULL
    assert s2a.softmax_bwd(fake, fake, odd_q, fake, 4, 8, s2a.BF16, check=False) == s2a.ERR_ALIGN
    assert s2a.softmax_fwd(None, None, None, None, 0, 197, s2a.BF16, check=False) == s2a.OK
    # ReLU entry points need no table
    for fn in (s2a.relu_fwd, s2a.relu_bwd):
        assert fn(fake, fake, fake, 8, 3, check=False) == s2a.ERR_DTYPE
        assert fn(fake, fake, fake, -2, s2a.F32, check=False) == s2a.ERR_SIZE
        assert fn(fake, None, fake, 8, s2a.F32, check=False) == s2a.ERR_NULL
        assert fn(None, None, None, 0, s2a.BF16, check=False) == s2a.OK
    # measured-range entry points: same checks, plus the state buffer
    odd = ctypes.c_void_p(0x1002)
    assert s2a.act_fwd_dyn(fake, fake, fake, fake, 8, 7, check=False) == s2a.ERR_DTYPE
    assert s2a.act_fwd_dyn(fake, fake, fake, fake, -5, s2a.F32, check=False) == s2a.ERR_SIZE
    assert s2a.act_fwd_dyn(fake, None, fake, fake, 8, s2a.F32, check=False) == s2a.ERR_NULL
    assert s2a.act_fwd_dyn(fake, fake, fake, None, 8, s2a.F32, check=False) == s2a.ERR_NULL
    assert s2a.act_fwd_dyn(fake, fake, fake, odd, 8, s2a.F32, check=False) == s2a.ERR_ALIGN
    assert s2a.act_bwd_dyn(fake, fake, fake, fake, 8, 7, check=False) == s2a.ERR_DTYPE
    assert s2a.act_bwd_dyn(fake, fake, None, fake, 8, s2a.BF16, check=False) == s2a.ERR_NULL
    assert s2a.act_bwd_dyn(fake, fake, odd, fake, 8, s2a.BF16, check=False) == s2a.ERR_ALIGN
    assert s2a.act_bwd_dyn(None, None, fake, None, 0, s2a.BF16, check=False) == s2a.OK
    # the measurement aid
    assert s2a.stream_copy(fake, fake, -16, check=False) == s2a.ERR_SIZE
    assert s2a.stream_copy(fake, fake, 24, check=False) == s2a.ERR_SIZE
    assert s2a.stream_copy(None, fake, 32, check=False) == s2a.ERR_NULL
    assert s2a.stream_copy(fake, odd, 32, check=False) == s2a.ERR_ALIGN
    assert s2a.stream_copy(None, None, 0, check=False) == s2a.OK
    assert s2a.stream_copy_shaped(fake, fake, fake, 32, 3, 0, check=False) == s2a.ERR_SIZE
    assert s2a.stream_copy_shaped(fake, fake, fake, 24, 4, 0, check=False) == s2a.ERR_SIZE
    assert s2a.stream_copy_shaped(fake, fake, None, 32, 4, 1, check=False) == s2a.ERR_NULL
    assert s2a.stream_copy_shaped(fake, fake, odd, 32, 2, 1, check=False) == s2a.ERR_ALIGN
    assert s2a.stream_copy_shaped(None, None, None, 0, 4, 0, check=False) == s2a.OK
    # Low-Rank Prompt: rank and shape limits come before any pointer is looked at
    assert s2a.lrp_bwd(fake, fake, fake, fake, fake, fake, 2, 3, 16, 129, s2a.F32, check=False) == s2a.ERR_SIZE
    assert s2a.lrp_bwd_noalloc(fake, fake, fake, fake, fake, 2, 3, 16, 0, s2a.F32, check=False) == s2a.ERR_SIZE


def test_strerror_is_total():
    seen = set()
    for code in range(-9, 2):
        msg = s2a.strerror(code)
        assert isinstance(msg, str) and msg
        seen.add(msg)
    assert len(seen) >= 9  # 8 known codes + "unknown"


def test_table_matches_oracle_to_fp32_rounding():
    """The library's host-built table is the oracle's, rounded once to fp32."""
    s2a.qtable_init(16)
    xhat, deriv, bounds = s2a.qtable_get()
    oxhat, oderiv, obounds = oracle.table()
    np.testing.assert_array_equal(np.array(xhat, np.float32), oxhat.astype(np.float32))
    np.testing.assert_array_equal(np.array(deriv, np.float32), oderiv.astype(np.float32))
    np.testing.assert_array_equal(np.array(bounds, np.float32), obounds.astype(np.float32))
