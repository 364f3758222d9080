"""CPU oracle for the S2A 4-bit GELU activation step -- TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around ``s2a_oracle.c`` (plain C, IEEE double, scalar
loops; S2A paper Sec. 3.2, GeLU paragraph, Eq. 8-12).  Only the tests, the
smoke check and the benchmark's ``cpu_baseline`` leg may import this package;
the GPU library and its Python binding never do, and nothing here imports
them.  All arithmetic of the method lives in the C file; this module only
marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

F32 = 0
BF16 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "s2a_oracle.c")
_LIB = os.path.join(_HERE, "libs2a_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no vectorisation hints)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math",
             "-ffp-contract=off", "-o", tmp, _SRC, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        d, i, i64, vp = ctypes.c_double, ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
        for name in ("s2a_oracle_gelu", "s2a_oracle_gelu_deriv_exact",
                     "s2a_oracle_gelu_deriv_approx"):
            getattr(lib, name).restype = d
            getattr(lib, name).argtypes = [d]
        lib.s2a_oracle_quantize.restype = i
        lib.s2a_oracle_quantize.argtypes = [d]
        lib.s2a_oracle_dequantize.restype = d
        lib.s2a_oracle_dequantize.argtypes = [i]
        lib.s2a_oracle_table.restype = None
        lib.s2a_oracle_table.argtypes = [vp, vp, vp]
        lib.s2a_oracle_fwd.restype = i
        lib.s2a_oracle_fwd.argtypes = [vp, i, i64, vp, vp, vp, vp, d]
        lib.s2a_oracle_bwd.restype = i
        lib.s2a_oracle_bwd.argtypes = [vp, i, vp, i64, vp]
        lib.s2a_oracle_relu_fwd.restype = i
        lib.s2a_oracle_relu_fwd.argtypes = [vp, i, i64, vp, vp, vp]
        lib.s2a_oracle_relu_bwd.restype = i
        lib.s2a_oracle_relu_bwd.argtypes = [vp, i, vp, i64, vp]
        lib.s2a_oracle_softmax_fwd.restype = i
        lib.s2a_oracle_softmax_fwd.argtypes = [vp, i, i64, i64, vp, vp, vp, vp, vp, vp, d]
        lib.s2a_oracle_softmax_bwd.restype = i
        lib.s2a_oracle_softmax_bwd.argtypes = [vp, i, vp, vp, vp, i64, i64, vp]
        for name in ("s2a_oracle_silu", "s2a_oracle_silu_deriv_approx"):
            getattr(lib, name).restype = d
            getattr(lib, name).argtypes = [d]
        lib.s2a_oracle_silu_quantize.restype = i
        lib.s2a_oracle_silu_quantize.argtypes = [d]
        lib.s2a_oracle_silu_dequantize.restype = d
        lib.s2a_oracle_silu_dequantize.argtypes = [i]
        lib.s2a_oracle_silu_fwd.restype = i
        lib.s2a_oracle_silu_fwd.argtypes = [vp, i, i64, vp, vp, vp, vp, d]
        lib.s2a_oracle_silu_bwd.restype = i
        lib.s2a_oracle_silu_bwd.argtypes = [vp, i, vp, i64, vp]
        lib.s2a_oracle_cap_fwd.restype = i
        lib.s2a_oracle_cap_fwd.argtypes = [vp, i, i64, i, vp]
        lib.s2a_oracle_cap_bwd.restype = i
        lib.s2a_oracle_cap_bwd.argtypes = [vp, i, i64, i, vp]
        lib.s2a_oracle_lrp_fwd.restype = i
        lib.s2a_oracle_lrp_fwd.argtypes = [vp, i, vp, vp, i64, i64, i64, i, vp]
        lib.s2a_oracle_lrp_bwd.restype = i
        lib.s2a_oracle_lrp_bwd.argtypes = [vp, i, vp, vp, i64, i64, i64, i, vp, vp]
        lib.s2a_oracle_range.restype = i
        lib.s2a_oracle_range.argtypes = [vp, i, i64, vp, vp]
        lib.s2a_oracle_quantize_dyn.restype = i
        lib.s2a_oracle_quantize_dyn.argtypes = [d, d, d]
        lib.s2a_oracle_dequantize_dyn.restype = d
        lib.s2a_oracle_dequantize_dyn.argtypes = [i, d, d]
        lib.s2a_oracle_fwd_dyn.restype = i
        lib.s2a_oracle_fwd_dyn.argtypes = [vp, i, i64, vp, vp, vp, vp, vp, vp, d]
        lib.s2a_oracle_bwd_dyn.restype = i
        lib.s2a_oracle_bwd_dyn.argtypes = [vp, i, vp, i64, d, d, vp]
        _lib = lib
    return _lib


def gelu(x: float) -> float:
    """Eq. 10 at one point."""
    return _load().s2a_oracle_gelu(float(x))


def gelu_deriv_exact(x: float) -> float:
    """Eq. 11 at one point (cross-checks only)."""
    return _load().s2a_oracle_gelu_deriv_exact(float(x))


def gelu_deriv_approx(x: float) -> float:
    """Eq. 12 at one point."""
    return _load().s2a_oracle_gelu_deriv_approx(float(x))


def quantize(x: float) -> int:
    """Clip to [-2, 2] then Eq. 8 on x with N = 4."""
    return _load().s2a_oracle_quantize(float(x))


def dequantize(q: int) -> float:
    """Eq. 9 on a code."""
    return _load().s2a_oracle_dequantize(int(q))


def table():
    """(xhat[16], deriv[16], bounds[15]) as float64 arrays."""
    xhat = np.empty(16, np.float64)
    deriv = np.empty(16, np.float64)
    bounds = np.empty(15, np.float64)
    _load().s2a_oracle_table(xhat.ctypes.data, deriv.ctypes.data, bounds.ctypes.data)
    return xhat, deriv, bounds


def _storage(a: np.ndarray, dtype: int) -> np.ndarray:
    """Check that `a` is the raw storage for `dtype`: float32, or uint16 bf16 bit patterns."""
    want = np.float32 if dtype == F32 else np.uint16
    if a.dtype != want or a.ndim != 1 or not a.flags.c_contiguous:
        raise TypeError(f"oracle input must be a contiguous 1-D {np.dtype(want)} array")
    return a


def fwd(x: np.ndarray, dtype: int, band: float = 1e-6, want_near: bool = True):
    """Forward pass.  Returns (y float64[n], code uint8[n], packed uint8[(n+1)//2], near uint8[n]).

    `near` flags inputs within `band` of a decision point (test bookkeeping, not part
    of the method); with want_near=False it is skipped and returned as None.
    """
    x = _storage(x, dtype)
    n = x.shape[0]
    y = np.empty(n, np.float64)
    code = np.empty(n, np.uint8)
    packed = np.empty((n + 1) // 2, np.uint8)
    near = np.empty(n, np.uint8) if want_near else None
    rc = _load().s2a_oracle_fwd(x.ctypes.data, dtype, n, y.ctypes.data, code.ctypes.data,
                                packed.ctypes.data, near.ctypes.data if want_near else None,
                                float(band))
    if rc != 0:
        raise ValueError("s2a_oracle_fwd rejected its arguments")
    return y, code, packed, near


def bwd(dy: np.ndarray, dtype: int, packed: np.ndarray) -> np.ndarray:
    """Backward pass from packed codes.  Returns dx float64[n]."""
    dy = _storage(dy, dtype)
    n = dy.shape[0]
    if packed.dtype != np.uint8 or packed.shape != ((n + 1) // 2,) or not packed.flags.c_contiguous:
        raise TypeError("packed must be contiguous uint8 of length ceil(n/2)")
    dx = np.empty(n, np.float64)
    rc = _load().s2a_oracle_bwd(dy.ctypes.data, dtype, packed.ctypes.data, n, dx.ctypes.data)
    if rc != 0:
        raise ValueError("s2a_oracle_bwd rejected its arguments")
    return dx


# ---- measured-range variant (Eq. 8 with the tensor's own min and max) ----

def quantize_dyn(x: float, qmin: float, qscale: float) -> int:
    return _load().s2a_oracle_quantize_dyn(float(x), float(qmin), float(qscale))


def dequantize_dyn(q: int, qmin: float, qscale: float) -> float:
    return _load().s2a_oracle_dequantize_dyn(int(q), float(qmin), float(qscale))


def fwd_dyn(x: np.ndarray, dtype: int, band: float = 1e-6, want_near: bool = True):
    """Forward pass with the measured range.
    Returns (y, code, packed, near, qmin, qscale); qmin/qscale are Python floats."""
    x = _storage(x, dtype)
    n = x.shape[0]
    y = np.empty(n, np.float64)
    code = np.empty(n, np.uint8)
    packed = np.empty((n + 1) // 2, np.uint8)
    near = np.empty(n, np.uint8) if want_near else None
    qmin = ctypes.c_double()
    qscale = ctypes.c_double()
    rc = _load().s2a_oracle_fwd_dyn(x.ctypes.data, dtype, n, y.ctypes.data, code.ctypes.data,
                                    packed.ctypes.data, ctypes.addressof(qmin), ctypes.addressof(qscale),
                                    near.ctypes.data if want_near else None, float(band))
    if rc != 0:
        raise ValueError("s2a_oracle_fwd_dyn rejected its arguments")
    return y, code, packed, near, qmin.value, qscale.value


def bwd_dyn(dy: np.ndarray, dtype: int, packed: np.ndarray, qmin: float, qscale: float) -> np.ndarray:
    dy = _storage(dy, dtype)
    n = dy.shape[0]
    if packed.dtype != np.uint8 or packed.shape != ((n + 1) // 2,) or not packed.flags.c_contiguous:
        raise TypeError("packed must be contiguous uint8 of length ceil(n/2)")
    dx = np.empty(n, np.float64)
    rc = _load().s2a_oracle_bwd_dyn(dy.ctypes.data, dtype, packed.ctypes.data, n, float(qmin),
                                    float(qscale), dx.ctypes.data)
    if rc != 0:
        raise ValueError("s2a_oracle_bwd_dyn rejected its arguments")
    return dx


# ---- ReLU 1-bit mask ----

def relu_fwd(x: np.ndarray, dtype: int):
    """Returns (y float64[n], bit uint8[n], packed uint8[(n+7)//8])."""
    x = _storage(x, dtype)
    n = x.shape[0]
    y = np.empty(n, np.float64)
    bit = np.empty(n, np.uint8)
    packed = np.empty((n + 7) // 8, np.uint8)
    if _load().s2a_oracle_relu_fwd(x.ctypes.data, dtype, n, y.ctypes.data, bit.ctypes.data, packed.ctypes.data) != 0:
        raise ValueError("s2a_oracle_relu_fwd rejected its arguments")
    return y, bit, packed


def relu_bwd(dy: np.ndarray, dtype: int, packed: np.ndarray) -> np.ndarray:
    dy = _storage(dy, dtype)
    n = dy.shape[0]
    if packed.dtype != np.uint8 or packed.shape != ((n + 7) // 8,) or not packed.flags.c_contiguous:
        raise TypeError("packed must be contiguous uint8 of length ceil(n/8)")
    dx = np.empty(n, np.float64)
    if _load().s2a_oracle_relu_bwd(dy.ctypes.data, dtype, packed.ctypes.data, n, dx.ctypes.data) != 0:
        raise ValueError("s2a_oracle_relu_bwd rejected its arguments")
    return dx


# ---- Softmax with 4-bit y (Eq. 7-9) ----

def softmax_fwd(x: np.ndarray, dtype: int, rows: int, L: int, band_t: float = 1e-4):
    """x: storage array of rows*L elements.  Returns (y[rows*L], code[rows*L],
    packed[rows*ceil(L/2)], qmin[rows], qscale[rows], near[rows*L])."""
    x = _storage(x, dtype)
    if x.shape[0] != rows * L:
        raise ValueError("x must hold rows*L elements")
    y = np.empty(rows * L, np.float64)
    code = np.empty(rows * L, np.uint8)
    packed = np.empty(rows * ((L + 1) // 2), np.uint8)
    qmin = np.empty(rows, np.float64)
    qscale = np.empty(rows, np.float64)
    near = np.empty(rows * L, np.uint8)
    rc = _load().s2a_oracle_softmax_fwd(x.ctypes.data, dtype, rows, L, y.ctypes.data, code.ctypes.data,
                                        packed.ctypes.data, qmin.ctypes.data, qscale.ctypes.data,
                                        near.ctypes.data, float(band_t))
    if rc != 0:
        raise ValueError("s2a_oracle_softmax_fwd rejected its arguments")
    return y, code, packed, qmin, qscale, near


def softmax_bwd(dy: np.ndarray, dtype: int, packed: np.ndarray, qmin: np.ndarray, qscale: np.ndarray,
                rows: int, L: int) -> np.ndarray:
    dy = _storage(dy, dtype)
    if dy.shape[0] != rows * L or packed.shape != (rows * ((L + 1) // 2),) or packed.dtype != np.uint8:
        raise ValueError("shape mismatch")
    qmin = np.ascontiguousarray(qmin, np.float64)
    qscale = np.ascontiguousarray(qscale, np.float64)
    if qmin.shape != (rows,) or qscale.shape != (rows,):
        raise ValueError("one (min, scale) pair per row")
    dx = np.empty(rows * L, np.float64)
    rc = _load().s2a_oracle_softmax_bwd(dy.ctypes.data, dtype, packed.ctypes.data, qmin.ctypes.data,
                                        qscale.ctypes.data, rows, L, dx.ctypes.data)
    if rc != 0:
        raise ValueError("s2a_oracle_softmax_bwd rejected its arguments")
    return dx


# ---- SiLU / Swish (the GELU scheme under x -> x / 1.702) ----

def silu(x: float) -> float:
    return _load().s2a_oracle_silu(float(x))


def silu_deriv_approx(x: float) -> float:
    return _load().s2a_oracle_silu_deriv_approx(float(x))


def silu_quantize(x: float) -> int:
    return _load().s2a_oracle_silu_quantize(float(x))


def silu_dequantize(q: int) -> float:
    return _load().s2a_oracle_silu_dequantize(int(q))


def silu_fwd(x: np.ndarray, dtype: int, band: float = 1e-6):
    """Returns (y, code, packed, near) as fwd() does, for SiLU."""
    x = _storage(x, dtype)
    n = x.shape[0]
    y = np.empty(n, np.float64)
    code = np.empty(n, np.uint8)
    packed = np.empty((n + 1) // 2, np.uint8)
    near = np.empty(n, np.uint8)
    if _load().s2a_oracle_silu_fwd(x.ctypes.data, dtype, n, y.ctypes.data, code.ctypes.data,
                                   packed.ctypes.data, near.ctypes.data, float(band)) != 0:
        raise ValueError("s2a_oracle_silu_fwd rejected its arguments")
    return y, code, packed, near


def silu_bwd(dy: np.ndarray, dtype: int, packed: np.ndarray) -> np.ndarray:
    dy = _storage(dy, dtype)
    n = dy.shape[0]
    if packed.dtype != np.uint8 or packed.shape != ((n + 1) // 2,) or not packed.flags.c_contiguous:
        raise TypeError("packed must be contiguous uint8 of length ceil(n/2)")
    dx = np.empty(n, np.float64)
    if _load().s2a_oracle_silu_bwd(dy.ctypes.data, dtype, packed.ctypes.data, n, dx.ctypes.data) != 0:
        raise ValueError("s2a_oracle_silu_bwd rejected its arguments")
    return dx


# ---- Channel Average Pooling (Eq. 5) and Low-Rank Prompt (Eq. 3-4) ----

def cap_fwd(x: np.ndarray, dtype: int, r: int) -> np.ndarray:
    x = _storage(x, dtype)
    if x.shape[0] % r:
        raise ValueError("length must be a multiple of r")
    y = np.empty(x.shape[0] // r, np.float64)
    if _load().s2a_oracle_cap_fwd(x.ctypes.data, dtype, y.shape[0], int(r), y.ctypes.data) != 0:
        raise ValueError("s2a_oracle_cap_fwd rejected its arguments")
    return y


def cap_bwd(dy: np.ndarray, dtype: int, r: int) -> np.ndarray:
    dy = _storage(dy, dtype)
    dx = np.empty(dy.shape[0] * r, np.float64)
    if _load().s2a_oracle_cap_bwd(dy.ctypes.data, dtype, dy.shape[0], int(r), dx.ctypes.data) != 0:
        raise ValueError("s2a_oracle_cap_bwd rejected its arguments")
    return dx


def _f32(a, shape):
    a = np.ascontiguousarray(a, np.float32)
    if a.shape != shape:
        raise ValueError(f"expected shape {shape}")
    return a


def lrp_fwd(x: np.ndarray, dtype: int, A: np.ndarray, B: np.ndarray, batch: int, N: int, C: int) -> np.ndarray:
    x = _storage(x, dtype)
    r = A.shape[1]
    A, B = _f32(A, (N, r)), _f32(B, (r, C))
    if x.shape[0] != batch * N * C:
        raise ValueError("x must hold batch*N*C elements")
    y = np.empty(batch * N * C, np.float64)
    if _load().s2a_oracle_lrp_fwd(x.ctypes.data, dtype, A.ctypes.data, B.ctypes.data, batch, N, C, r, y.ctypes.data) != 0:
        raise ValueError("s2a_oracle_lrp_fwd rejected its arguments")
    return y


def lrp_bwd(dy: np.ndarray, dtype: int, A: np.ndarray, B: np.ndarray, batch: int, N: int, C: int):
    dy = _storage(dy, dtype)
    r = A.shape[1]
    A, B = _f32(A, (N, r)), _f32(B, (r, C))
    dA = np.empty((N, r), np.float64)
    dB = np.empty((r, C), np.float64)
    if _load().s2a_oracle_lrp_bwd(dy.ctypes.data, dtype, A.ctypes.data, B.ctypes.data, batch, N, C, r,
                                  dA.ctypes.data, dB.ctypes.data) != 0:
        raise ValueError("s2a_oracle_lrp_bwd rejected its arguments")
    return dA, dB
