"""ctypes binding of libs2a.so -- argument marshalling only.

Function names and argument order follow include/s2a.h.  Device pointers are
plain integers (e.g. ``tensor.data_ptr()``), the stream is a ``hipStream_t``
as an integer (e.g. ``torch.cuda.current_stream().cuda_stream``).  Every step
of the activation path runs inside the library's kernels; there is no Python
or CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

F32 = 0
BF16 = 1

OK = 0
ERR_NULL = -1
ERR_SIZE = -2
ERR_DTYPE = -3
ERR_LEVELS = -4
ERR_NOT_INIT = -5
ERR_LAUNCH = -6
ERR_ALIGN = -7
QSTATE_FLOATS = 544
SOFTMAX_MAX_L = 1 << 20
LRP_NOALLOC_MAX_FLOATS = 1 << 20

EXPORTS = ("s2a_qtable_init", "s2a_qtable_get", "s2a_act_fwd", "s2a_act_bwd",
           "s2a_act_fwd_dyn", "s2a_act_bwd_dyn", "s2a_silu_fwd", "s2a_silu_bwd", "s2a_relu_fwd", "s2a_relu_bwd",
           "s2a_softmax_fwd", "s2a_softmax_bwd", "s2a_cap_fwd", "s2a_cap_bwd",
           "s2a_lrp_fwd", "s2a_lrp_bwd", "s2a_lrp_bwd_noalloc", "s2a_stream_copy", "s2a_stream_copy_shaped",
           "s2a_strerror")

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libs2a.so")
_lib = None


class S2AError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


def lib() -> ctypes.CDLL:
    """Load libs2a.so (built by ``python -m paper_2503_08154_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2503_08154_amd.build`; "
                "there is no fallback path")
        l = ctypes.CDLL(LIB_PATH)
        vp, i, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        l.s2a_qtable_init.restype = i
        l.s2a_qtable_init.argtypes = [i]
        l.s2a_qtable_get.restype = i
        l.s2a_qtable_get.argtypes = [vp, vp, vp]
        l.s2a_act_fwd.restype = i
        l.s2a_act_fwd.argtypes = [vp, vp, vp, i64, i, vp]
        l.s2a_act_bwd.restype = i
        l.s2a_act_bwd.argtypes = [vp, vp, vp, i64, i, vp]
        l.s2a_act_fwd_dyn.restype = i
        l.s2a_act_fwd_dyn.argtypes = [vp, vp, vp, vp, i64, i, vp]
        l.s2a_act_bwd_dyn.restype = i
        l.s2a_act_bwd_dyn.argtypes = [vp, vp, vp, vp, i64, i, vp]
        l.s2a_silu_fwd.restype = i
        l.s2a_silu_fwd.argtypes = [vp, vp, vp, i64, i, vp]
        l.s2a_silu_bwd.restype = i
        l.s2a_silu_bwd.argtypes = [vp, vp, vp, i64, i, vp]
        l.s2a_relu_fwd.restype = i
        l.s2a_relu_fwd.argtypes = [vp, vp, vp, i64, i, vp]
        l.s2a_relu_bwd.restype = i
        l.s2a_relu_bwd.argtypes = [vp, vp, vp, i64, i, vp]
        l.s2a_softmax_fwd.restype = i
        l.s2a_softmax_fwd.argtypes = [vp, vp, vp, vp, i64, i64, i, vp]
        l.s2a_softmax_bwd.restype = i
        l.s2a_softmax_bwd.argtypes = [vp, vp, vp, vp, i64, i64, i, vp]
        l.s2a_cap_fwd.restype = i
        l.s2a_cap_fwd.argtypes = [vp, vp, i64, i, i, vp]
        l.s2a_cap_bwd.restype = i
        l.s2a_cap_bwd.argtypes = [vp, vp, i64, i, i, vp]
        l.s2a_lrp_fwd.restype = i
        l.s2a_lrp_fwd.argtypes = [vp, vp, vp, vp, i64, i64, i64, i, i, vp]
        l.s2a_lrp_bwd.restype = i
        l.s2a_lrp_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i, i, vp]
        l.s2a_lrp_bwd_noalloc.restype = i
        l.s2a_lrp_bwd_noalloc.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i, i, vp]
        l.s2a_stream_copy.restype = i
        l.s2a_stream_copy.argtypes = [vp, vp, i64, vp]
        l.s2a_stream_copy_shaped.restype = i
        l.s2a_stream_copy_shaped.argtypes = [vp, vp, vp, i64, i, i, vp]
        l.s2a_strerror.restype = ctypes.c_char_p
        l.s2a_strerror.argtypes = [i]
        _lib = l
    return _lib


def strerror(code: int) -> str:
    return lib().s2a_strerror(int(code)).decode()


def qtable_init(levels: int = 16, check: bool = True) -> int:
    rc = lib().s2a_qtable_init(int(levels))
    if check and rc != OK:
        raise S2AError(rc, "s2a_qtable_init")
    return rc


def qtable_get():
    """(xhat[16], deriv[16], bounds[15]) as Python lists of fp32 values."""
    xh = (ctypes.c_float * 16)()
    dv = (ctypes.c_float * 16)()
    bd = (ctypes.c_float * 15)()
    rc = lib().s2a_qtable_get(xh, dv, bd)
    if rc != OK:
        raise S2AError(rc, "s2a_qtable_get")
    return list(xh), list(dv), list(bd)


def act_fwd(x: int, y: int, codes: int, n: int, dtype: int, stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_act_fwd(x, y, codes, int(n), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_act_fwd")
    return rc


def act_bwd(dy: int, codes: int, dx: int, n: int, dtype: int, stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_act_bwd(dy, codes, dx, int(n), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_act_bwd")
    return rc


def act_fwd_dyn(x: int, y: int, codes: int, qstate: int, n: int, dtype: int, stream: int = 0,
                check: bool = True) -> int:
    rc = lib().s2a_act_fwd_dyn(x, y, codes, qstate, int(n), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_act_fwd_dyn")
    return rc


def act_bwd_dyn(dy: int, codes: int, qstate: int, dx: int, n: int, dtype: int, stream: int = 0,
                check: bool = True) -> int:
    rc = lib().s2a_act_bwd_dyn(dy, codes, qstate, dx, int(n), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_act_bwd_dyn")
    return rc


def relu_fwd(x: int, y: int, mask: int, n: int, dtype: int, stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_relu_fwd(x, y, mask, int(n), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_relu_fwd")
    return rc


def relu_bwd(dy: int, mask: int, dx: int, n: int, dtype: int, stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_relu_bwd(dy, mask, dx, int(n), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_relu_bwd")
    return rc


def softmax_fwd(x: int, y: int, codes: int, qparams: int, rows: int, L: int, dtype: int, stream: int = 0,
                check: bool = True) -> int:
    rc = lib().s2a_softmax_fwd(x, y, codes, qparams, int(rows), int(L), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_softmax_fwd")
    return rc


def softmax_bwd(dy: int, codes: int, qparams: int, dx: int, rows: int, L: int, dtype: int, stream: int = 0,
                check: bool = True) -> int:
    rc = lib().s2a_softmax_bwd(dy, codes, qparams, dx, int(rows), int(L), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_softmax_bwd")
    return rc


def silu_fwd(x: int, y: int, codes: int, n: int, dtype: int, stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_silu_fwd(x, y, codes, int(n), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_silu_fwd")
    return rc


def silu_bwd(dy: int, codes: int, dx: int, n: int, dtype: int, stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_silu_bwd(dy, codes, dx, int(n), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_silu_bwd")
    return rc


def cap_fwd(x: int, y: int, n_out: int, r: int, dtype: int, stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_cap_fwd(x, y, int(n_out), int(r), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_cap_fwd")
    return rc


def cap_bwd(dy: int, dx: int, n_out: int, r: int, dtype: int, stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_cap_bwd(dy, dx, int(n_out), int(r), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_cap_bwd")
    return rc


def lrp_fwd(x: int, y: int, A: int, B: int, batch: int, N: int, C: int, r: int, dtype: int, stream: int = 0,
            check: bool = True) -> int:
    rc = lib().s2a_lrp_fwd(x, y, A, B, int(batch), int(N), int(C), int(r), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_lrp_fwd")
    return rc


def lrp_bwd(dy: int, A: int, B: int, dA: int, dB: int, work: int, batch: int, N: int, C: int, r: int,
            dtype: int, stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_lrp_bwd(dy, A, B, dA, dB, work, int(batch), int(N), int(C), int(r), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_lrp_bwd")
    return rc


def lrp_bwd_noalloc(dy: int, A: int, B: int, dA: int, dB: int, batch: int, N: int, C: int, r: int,
                    dtype: int, stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_lrp_bwd_noalloc(dy, A, B, dA, dB, int(batch), int(N), int(C), int(r), int(dtype), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_lrp_bwd_noalloc")
    return rc


def stream_copy(src: int, dst: int, nbytes: int, stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_stream_copy(src, dst, int(nbytes), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_stream_copy")
    return rc


def stream_copy_shaped(src: int, dst: int, side: int, nbytes: int, side_bytes: int, side_is_input: int,
                       stream: int = 0, check: bool = True) -> int:
    rc = lib().s2a_stream_copy_shaped(src, dst, side, int(nbytes), int(side_bytes), int(side_is_input), stream)
    if check and rc != OK:
        raise S2AError(rc, "s2a_stream_copy_shaped")
    return rc
