"""GPU parity of the ReLU 1-bit-mask kernels against the oracle.  Everything is
bit-exact here: y is x or 0, the mask is a comparison, dx is dy or 0."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_08154_amd import s2a
from paper_2503_08154_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DTYPES = [wl.F32, wl.BF16]
SIZES = [0, 1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 33, 63, 64, 65, 255, 256, 257, 259, 261, 511, 512, 513, 517,
         1023, 4097, 8192 * 3 + 5, 65536 + 3, 302592, 2_000_003]


def _run(x, dy, dtype, offset=0, mask_offset=0, inplace=False):
    n = x.shape[0]
    es = gu.esize(dtype)
    st = torch.cuda.current_stream().cuda_stream
    bx = gu.Buf(n * es, offset * es).upload(x)
    by = bx if inplace else gu.Buf(n * es, offset * es, fill=0xFF)
    bm = gu.Buf((n + 7) // 8, mask_offset, fill=0xFF)
    s2a.relu_fwd(bx.ptr, by.ptr, bm.ptr, n, dtype, st)
    torch.cuda.synchronize()
    assert bx.canaries_intact() and by.canaries_intact() and bm.canaries_intact()
    y = by.download(gu.storage_np(dtype))
    mask = bm.download(np.uint8)
    bdy = gu.Buf(n * es, offset * es).upload(dy)
    bdx = bdy if inplace else gu.Buf(n * es, offset * es, fill=0xFF)
    s2a.relu_bwd(bdy.ptr, bm.ptr, bdx.ptr, n, dtype, st)
    torch.cuda.synchronize()
    assert bdy.canaries_intact() and bdx.canaries_intact() and bm.canaries_intact()
    return y, mask, bdx.download(gu.storage_np(dtype))


def _check(x, dy, dtype, **kw):
    y_ref, bit, packed = oracle.relu_fwd(x, dtype)
    dx_ref = oracle.relu_bwd(dy, dtype, packed)
    y, mask, dx = _run(x, dy, dtype, **kw)
    np.testing.assert_array_equal(mask, packed)
    np.testing.assert_array_equal(wl.storage_to_f64(y, dtype), y_ref)
    got_dx = wl.storage_to_f64(dx, dtype)
    same = (got_dx == dx_ref) | (np.isnan(got_dx) & np.isnan(dx_ref))
    assert same.all()


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("n", SIZES)
def test_sizes(dtype, n):
    x = wl.draw_x(n, "normal", 1.0, dtype, seed=300 + n)
    if n > 8:
        x[:6] = wl.to_storage(np.array([0.0, -0.0, np.nan, np.inf, -np.inf, 1e-40]), dtype)
    dy = wl.draw_dy(n, 1.0, dtype, seed=400 + n)
    _check(x, dy, dtype)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("n", [9, 4097, 100001])
@pytest.mark.parametrize("off", [(1, 0), (0, 1), (3, 3)])
def test_unaligned(dtype, n, off):
    x = wl.draw_x(n, "normal", 1.0, dtype, seed=31 + n)
    dy = wl.draw_dy(n, 1.0, dtype, seed=32 + n)
    _check(x, dy, dtype, offset=off[0], mask_offset=off[1])


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("off", [0, 1])
def test_in_place(dtype, off):
    n = 8192 * 5 + 3
    x = wl.draw_x(n, "normal", 1.0, dtype, seed=5)
    dy = wl.draw_dy(n, 1.0, dtype, seed=6)
    _check(x, dy, dtype, inplace=True, offset=off)


def test_exhaustive_bf16_domain():
    bits = np.arange(65536, dtype=np.uint16)
    _check(bits, bits[::-1].copy(), wl.BF16)


@pytest.mark.parametrize("name", ["vit_l16", "vit_g14_f32"])
def test_workload_full_size(name):
    w = wl.WORKLOADS[name]
    x, dy = wl.layer_inputs(w, 0, 0)
    n = x.shape[0]
    st = torch.cuda.current_stream().cuda_stream
    tx = torch.from_numpy(x.view(np.uint8)).cuda()
    ty = torch.empty_like(tx)
    tm = torch.empty((n + 7) // 8, dtype=torch.uint8, device="cuda")
    tdy = torch.from_numpy(dy.view(np.uint8)).cuda()
    tdx = torch.empty_like(tdy)
    s2a.relu_fwd(tx.data_ptr(), ty.data_ptr(), tm.data_ptr(), n, w.dtype, st)
    s2a.relu_bwd(tdy.data_ptr(), tm.data_ptr(), tdx.data_ptr(), n, w.dtype, st)
    torch.cuda.synchronize()
    y_ref, _, packed = oracle.relu_fwd(x, w.dtype)
    np.testing.assert_array_equal(tm.cpu().numpy(), packed)
    np.testing.assert_array_equal(wl.storage_to_f64(ty.cpu().numpy().view(gu.storage_np(w.dtype)), w.dtype), y_ref)
    np.testing.assert_array_equal(wl.storage_to_f64(tdx.cpu().numpy().view(gu.storage_np(w.dtype)), w.dtype),
                                  oracle.relu_bwd(dy, w.dtype, packed))


def test_more_than_2_31_elements():
    """bf16, n just above 2^31 with a ragged tail: a seeded tile repeated on the device; spans at both
    ends, across the 2^31 mark and at random places are compared bit for bit with the oracle."""
    dtype = wl.BF16
    tile_n = (1 << 22) + 8                      # a multiple of 8: spans that start on a tile boundary own whole mask bytes
    n = (1 << 31) + 8 * 64 * 3 + 5
    tile_x = wl.draw_x(tile_n, "normal", 1.0, dtype, seed=515)
    tile_dy = wl.draw_dy(tile_n, 1.0, dtype, seed=516)
    reps = -(-n // tile_n)
    tx = torch.from_numpy(tile_x.view(np.int16)).cuda().repeat(reps)[:n]
    ty = torch.empty_like(tx)
    tm = torch.empty((n + 7) // 8, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    s2a.relu_fwd(tx.data_ptr(), ty.data_ptr(), tm.data_ptr(), n, dtype, st)
    torch.cuda.synchronize()
    del tx
    tdy = torch.from_numpy(tile_dy.view(np.int16)).cuda().repeat(reps)[:n]
    tdx = torch.empty_like(tdy)
    s2a.relu_bwd(tdy.data_ptr(), tm.data_ptr(), tdx.data_ptr(), n, dtype, st)
    torch.cuda.synchronize()
    g = np.random.default_rng(5)
    spans = [(0, 4096), ((n - 5000) & ~7, n - ((n - 5000) & ~7)), ((1 << 31) - 2048, 3072)]
    spans += [(int(a) & ~7, 4096) for a in g.integers(0, n - 4096, 61)]
    for a, m in spans:
        pos = np.arange(a, a + m, dtype=np.int64) % tile_n
        y_ref, _, packed = oracle.relu_fwd(tile_x[pos].copy(), dtype)
        dx_ref = oracle.relu_bwd(tile_dy[pos].copy(), dtype, packed)
        np.testing.assert_array_equal(tm[a // 8:(a + m + 7) // 8].cpu().numpy(), packed)
        np.testing.assert_array_equal(wl.storage_to_f64(ty[a:a + m].cpu().numpy().view(np.uint16), dtype), y_ref)
        np.testing.assert_array_equal(wl.storage_to_f64(tdx[a:a + m].cpu().numpy().view(np.uint16), dtype), dx_ref)
