"""Device plumbing for the GPU tests: numpy storage arrays <-> torch device
buffers, and calls into the C ABI through the ctypes binding.  torch is used
only for memory and streams."""
from __future__ import annotations

import numpy as np
import torch

from paper_2503_08154_amd import s2a
from paper_2503_08154_amd import workloads as wl

GUARD = 64  # bytes of canary kept either side of every output buffer


def esize(dtype: int) -> int:
    return 4 if dtype == wl.F32 else 2


class Buf:
    """A byte buffer on the device with canaries before and after the payload.

    `offset` shifts the payload start by that many bytes from a 256-byte
    aligned address, to exercise the element-aligned (non-vector) kernels.
    """

    def __init__(self, nbytes: int, offset: int = 0, fill: int = 0xA5):
        self.nbytes, self.fill = nbytes, fill
        self.off = 256 + offset
        self.raw = torch.full((self.off + nbytes + GUARD + 256,), fill, dtype=torch.uint8, device="cuda")
        base = self.raw.data_ptr()
        assert base % 256 == 0
        self.ptr = base + self.off

    def upload(self, a: np.ndarray):
        b = np.ascontiguousarray(a).view(np.uint8).reshape(-1)
        assert b.shape[0] == self.nbytes
        self.raw[self.off:self.off + self.nbytes] = torch.from_numpy(b.copy()).cuda()
        return self

    def download(self, np_dtype) -> np.ndarray:
        torch.cuda.synchronize()
        return self.raw[self.off:self.off + self.nbytes].cpu().numpy().view(np_dtype).copy()

    def canaries_intact(self) -> bool:
        torch.cuda.synchronize()
        head = self.raw[self.off - GUARD:self.off].cpu().numpy()
        tail = self.raw[self.off + self.nbytes:self.off + self.nbytes + GUARD].cpu().numpy()
        return bool((head == self.fill).all() and (tail == self.fill).all())


def storage_np(dtype: int):
    return np.float32 if dtype == wl.F32 else np.uint16


def run_fwd(x: np.ndarray, dtype: int, offset_elems: int = 0, code_offset: int = 0,
            inplace: bool = False, stream=None):
    """x storage array -> (y storage array, packed codes) computed by the library."""
    n = x.shape[0]
    es = esize(dtype)
    bx = Buf(n * es, offset_elems * es).upload(x)
    by = bx if inplace else Buf(n * es, offset_elems * es)
    bc = Buf((n + 1) // 2, code_offset)
    st = torch.cuda.current_stream() if stream is None else stream
    if stream is not None:
        stream.wait_stream(torch.cuda.current_stream())
    s2a.act_fwd(bx.ptr, by.ptr, bc.ptr, n, dtype, st.cuda_stream)
    st.synchronize()
    assert bx.canaries_intact() and by.canaries_intact() and bc.canaries_intact(), "write outside a buffer"
    if not inplace:
        assert np.array_equal(bx.download(storage_np(dtype)).view(np.uint8), x.view(np.uint8)), "x was modified"
    return by.download(storage_np(dtype)), bc.download(np.uint8)


def run_bwd(dy: np.ndarray, packed: np.ndarray, dtype: int, offset_elems: int = 0,
            code_offset: int = 0, inplace: bool = False, stream=None):
    n = dy.shape[0]
    es = esize(dtype)
    bdy = Buf(n * es, offset_elems * es).upload(dy)
    bdx = bdy if inplace else Buf(n * es, offset_elems * es)
    bc = Buf((n + 1) // 2, code_offset).upload(packed)
    st = torch.cuda.current_stream() if stream is None else stream
    if stream is not None:
        stream.wait_stream(torch.cuda.current_stream())
    s2a.act_bwd(bdy.ptr, bc.ptr, bdx.ptr, n, dtype, st.cuda_stream)
    st.synchronize()
    assert bdy.canaries_intact() and bdx.canaries_intact() and bc.canaries_intact(), "write outside a buffer"
    assert np.array_equal(bc.download(np.uint8), packed), "codes were modified"
    return bdx.download(storage_np(dtype))
