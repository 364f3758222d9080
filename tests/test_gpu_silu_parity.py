"""GPU parity of the SiLU entry points (s2a_silu_fwd / s2a_silu_bwd) against the
oracle, with the activation path's comparison rules."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_08154_amd import s2a
from paper_2503_08154_amd import workloads as wl

import gpu_util as gu
import parity

pytestmark = pytest.mark.gpu
DTYPES = [wl.F32, wl.BF16]


@pytest.fixture(scope="module", autouse=True)
def _init():
    assert torch.cuda.is_available()
    s2a.qtable_init(16)


def _run(x, dy, packed_in, dtype, offset=0, code_offset=0):
    n = x.shape[0]
    es = gu.esize(dtype)
    st = torch.cuda.current_stream().cuda_stream
    bx = gu.Buf(n * es, offset * es).upload(x)
    by = gu.Buf(n * es, offset * es, fill=0xFF)
    bc = gu.Buf((n + 1) // 2, code_offset, fill=0xFF)
    s2a.silu_fwd(bx.ptr, by.ptr, bc.ptr, n, dtype, st)
    torch.cuda.synchronize()
    assert bx.canaries_intact() and by.canaries_intact() and bc.canaries_intact()
    y, packed = by.download(gu.storage_np(dtype)), bc.download(np.uint8)
    bdy = gu.Buf(n * es, offset * es).upload(dy)
    bdx = gu.Buf(n * es, offset * es, fill=0xFF)
    bc2 = gu.Buf((n + 1) // 2, code_offset).upload(packed_in)
    s2a.silu_bwd(bdy.ptr, bc2.ptr, bdx.ptr, n, dtype, st)
    torch.cuda.synchronize()
    assert bdx.canaries_intact()
    return y, packed, bdx.download(gu.storage_np(dtype))


def _check(x, dy, dtype, **kw):
    n = x.shape[0]
    y_ref, code_ref, packed_ref, near = oracle.silu_fwd(x, dtype, band=parity.BAND)
    dx_ref = oracle.silu_bwd(dy, dtype, packed_ref)
    y, packed, dx = _run(x, dy, packed_ref, dtype, **kw)
    finite = np.isfinite(wl.storage_to_f64(x, dtype))
    rep = parity.check_codes(packed, code_ref, near, n, parity.band_mask(wl.storage_to_f64(x, dtype), parity.SILU_POINTS))
    wy = parity.check_values(y, y_ref, dtype, "y", finite_in=finite)
    wdx = parity.check_values(dx, dx_ref, dtype, "dx", finite_in=np.isfinite(wl.storage_to_f64(dy, dtype)))
    return rep, wy, wdx


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("n", [0, 1, 2, 3, 7, 8, 9, 63, 64, 65, 511, 513, 4097, 8192 * 3 + 5, 302592])
def test_sizes(dtype, n):
    x = wl.draw_x(n, "student_t", 3.0, dtype, seed=600 + n)
    dy = wl.draw_dy(n, 1.0, dtype, seed=700 + n)
    _check(x, dy, dtype)


@pytest.mark.parametrize("dtype", DTYPES)
def test_unaligned(dtype):
    n = 8192 * 2 + 3
    x = wl.draw_x(n, "normal", 2.5, dtype, seed=1)
    dy = wl.draw_dy(n, 1.0, dtype, seed=2)
    _check(x, dy, dtype, offset=1, code_offset=1)


def test_exhaustive_bf16_domain():
    bits = np.arange(65536, dtype=np.uint16)
    rep, wy, wdx = _check(bits, bits[::-1].copy(), wl.BF16)
    print(f"\n[silu exhaustive bf16] {rep} worst y {wy:.3f} worst dx {wdx:.3f}")


def test_levels_through_the_kernel():
    levels = np.array([oracle.silu_deriv_approx(oracle.silu_dequantize(k)) for k in range(16)])
    x = np.array([oracle.silu_dequantize(k) for k in range(16)], np.float32)
    y, packed, dx = _run(x, np.ones(16, np.float32), np.array([0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE], np.uint8), wl.F32)
    np.testing.assert_array_equal(dx, levels.astype(np.float32))
    assert packed.tolist() == [0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE]


@pytest.mark.parametrize("name", ["vit_l16", "vit_g14_f32"])
def test_workload_full_size(name):
    w = wl.WORKLOADS[name]
    x, dy = wl.layer_inputs(w, 0, 0)
    n = x.shape[0]
    st = torch.cuda.current_stream().cuda_stream
    tx = torch.from_numpy(x.view(np.uint8)).cuda()
    ty = torch.empty_like(tx)
    tc = torch.empty((n + 1) // 2, dtype=torch.uint8, device="cuda")
    tdy = torch.from_numpy(dy.view(np.uint8)).cuda()
    tdx = torch.empty_like(tdy)
    s2a.silu_fwd(tx.data_ptr(), ty.data_ptr(), tc.data_ptr(), n, w.dtype, st)
    s2a.silu_bwd(tdy.data_ptr(), tc.data_ptr(), tdx.data_ptr(), n, w.dtype, st)
    torch.cuda.synchronize()
    y_ref, code_ref, packed_ref, near = oracle.silu_fwd(x, w.dtype, band=parity.BAND)
    packed = tc.cpu().numpy()
    rep = parity.check_codes(packed, code_ref, near, n, parity.band_mask(wl.storage_to_f64(x, w.dtype), parity.SILU_POINTS))
    wy = parity.check_values(ty.cpu().numpy().view(gu.storage_np(w.dtype)), y_ref, w.dtype, "y")
    differs = parity.unpack(packed, n) != code_ref
    wdx = parity.check_values(tdx.cpu().numpy().view(gu.storage_np(w.dtype)), oracle.silu_bwd(dy, w.dtype, packed_ref),
                              w.dtype, "dx", skip=differs)
    print(f"\n[silu {name}] n={n} {rep} worst y {wy:.3f} worst dx {wdx:.3f}")
