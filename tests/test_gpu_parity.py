"""GPU parity: the HIP library, called through its C ABI, against the CPU
oracle on identical seeded inputs -- element by element at sizes that span
several tiles and ragged tails, exhaustively over the bf16 domain, on special
values, on unaligned and in-place buffers, and at every workload's full size."""
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
# lane-vector = 16 B (4 fp32 / 8 bf16); one block = one wave of 64 vectors (256 fp32 / 512 bf16 elements)
SIZES = [0, 1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 255, 256, 257, 259, 511, 512, 513, 519,
         767, 1023, 1535, 4095, 4096, 4097, 8191, 8192, 8193, 8192 * 3 + 5, 65536 + 1, 3 * 8192 * 4 + 8191, 302592]


@pytest.fixture(scope="module", autouse=True)
def _init():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    s2a.qtable_init(16)


def _fwd_bwd_check(x, dy, dtype, report=None, **kw):
    n = x.shape[0]
    y_ref, code_ref, packed_ref, near = oracle.fwd(x, dtype, band=parity.BAND)
    y, packed = gu.run_fwd(x, dtype, **kw)
    finite = np.isfinite(wl.storage_to_f64(x, dtype))
    rep = parity.check_codes(packed, code_ref, near, n, parity.band_mask(wl.storage_to_f64(x, dtype), parity.GELU_POINTS))
    wy = parity.check_values(y, y_ref, dtype, "y", finite_in=finite)
    # backward in isolation: the oracle's codes in, every element checked
    dx_ref = oracle.bwd(dy, dtype, packed_ref)
    dx = gu.run_bwd(dy, packed_ref, dtype, **kw)
    fin_dy = np.isfinite(wl.storage_to_f64(dy, dtype))
    wdx = parity.check_values(dx, dx_ref, dtype, "dx", finite_in=fin_dy)
    # backward on the GPU's own codes: elements whose code legitimately differs are skipped
    if rep.differing:
        dx2 = gu.run_bwd(dy, packed, dtype, **kw)
        differs = parity.unpack(packed, n) != code_ref
        parity.check_values(dx2, dx_ref, dtype, "dx", finite_in=fin_dy, skip=differs)
    if report is not None:
        report.append((n, rep.flagged, rep.differing, wy, wdx))
    return rep, wy, wdx


def test_table_through_the_kernel():
    """dy = 1 and codes 0..15 recover the derivative table exactly (fp32)."""
    _, deriv, _ = oracle.table()
    packed = np.array([0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE], np.uint8)
    dx = gu.run_bwd(np.ones(16, np.float32), packed, wl.F32)
    np.testing.assert_array_equal(dx, deriv.astype(np.float32))
    xhat = oracle.table()[0].astype(np.float32)
    y, codes = gu.run_fwd(xhat, wl.F32)
    np.testing.assert_array_equal(codes, packed)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("n", SIZES)
def test_sizes(dtype, n):
    x = wl.draw_x(n, "student_t", 2.0, dtype, seed=1000 + n)
    dy = wl.draw_dy(n, 1.0, dtype, seed=2000 + n)
    _fwd_bwd_check(x, dy, dtype)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("n", [1, 9, 33, 4097, 8192 * 2 + 3, 100001])
@pytest.mark.parametrize("off", [(1, 0), (0, 1), (1, 1), (3, 3)])
def test_unaligned_pointers(dtype, n, off):
    x = wl.draw_x(n, "normal", 1.5, dtype, seed=31 + n)
    dy = wl.draw_dy(n, 1e-2, dtype, seed=32 + n)
    _fwd_bwd_check(x, dy, dtype, offset_elems=off[0], code_offset=off[1])


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("n", [17, 8192 * 5 + 1, 302592])
@pytest.mark.parametrize("off", [0, 1])
def test_in_place(dtype, n, off):
    x = wl.draw_x(n, "normal_outliers", 1.5, dtype, seed=41 + n)
    dy = wl.draw_dy(n, 1e-2, dtype, seed=42 + n)
    _fwd_bwd_check(x, dy, dtype, inplace=True, offset_elems=off)


def test_exhaustive_bf16_domain():
    """All 65,536 bf16 bit patterns as x (NaNs and infinities included), and as dy
    against every code."""
    bits = np.arange(65536, dtype=np.uint16)
    y_ref, code_ref, packed_ref, near = oracle.fwd(bits, wl.BF16, band=parity.BAND)
    y, packed = gu.run_fwd(bits, wl.BF16)
    finite = np.isfinite(wl.bf16_bits_to_f32(bits))
    rep = parity.check_codes(packed, code_ref, near, 65536, parity.band_mask(wl.storage_to_f64(bits, wl.BF16), parity.GELU_POINTS))
    parity.check_values(y, y_ref, wl.BF16, "y", finite_in=finite)
    print(f"\n[exhaustive bf16] {rep}")
    # non-finite x: NaN -> code 0, +inf -> 15, -inf -> 0 (checked above through the oracle's codes)
    assert parity.unpack(packed, 65536)[0x7FC0] == 0 and parity.unpack(packed, 65536)[0x7F80] == 15
    for shift in range(16):
        codes = ((np.arange(65536) + shift) % 16).astype(np.uint8)
        pk = (codes[0::2] | (codes[1::2] << 4)).astype(np.uint8)
        dx_ref = oracle.bwd(bits, wl.BF16, pk)
        dx = gu.run_bwd(bits, pk, wl.BF16)
        parity.check_values(dx, dx_ref, wl.BF16, "dx", finite_in=finite)


def test_fp32_special_values():
    _, _, bounds = oracle.table()
    b32 = bounds.astype(np.float32)
    near_bounds = np.concatenate([np.nextafter(b32, np.float32(-9), dtype=np.float32),
                                  b32, np.nextafter(b32, np.float32(9), dtype=np.float32),
                                  b32 + np.float32(3e-6), b32 - np.float32(3e-6)])
    tiny = np.array([0.0, -0.0, 1e-45, -1e-45, 1e-38, -1e-38, 1.17549435e-38, -1.17549435e-38,
                     1e-30, -1e-30, 1e-10, -1e-10, 2.0 ** -24, -2.0 ** -24, 2.0 ** -60, -2.0 ** -60], np.float32)
    huge = np.array([3.4028235e38, -3.4028235e38, 1e30, -1e30, 129.0, -129.0, 128.0, -128.0, 127.99, -127.99,
                     np.inf, -np.inf, np.nan], np.float32)
    # the range where y leaves the normal fp32 numbers and then underflows
    under = -np.linspace(20.0, 70.0, 5001).astype(np.float32)
    grid = np.linspace(-30.0, 30.0, 60001).astype(np.float32)
    levels = np.array([-2.0, 2.0, np.nextafter(np.float32(2), np.float32(3)), np.nextafter(np.float32(-2), np.float32(-3)),
                       -1.0, 1.0, 0.5, -0.5], np.float32)
    x = np.concatenate([near_bounds, tiny, huge, under, grid, levels]).astype(np.float32)
    dy = wl.draw_dy(x.shape[0], 1.0, wl.F32, seed=5)
    dy[:8] = np.array([0.0, -0.0, 1e-45, 3.4028235e38, -3.4028235e38, np.inf, -np.inf, np.nan], np.float32)
    rep, wy, wdx = _fwd_bwd_check(x, dy, wl.F32)
    print(f"\n[fp32 special] {rep} worst y {wy:.3f} worst dx {wdx:.3f} (fractions of the tolerance)")
    # expected by construction: the 15 decision points and their fp32 neighbours are in the band
    assert rep.flagged >= 45


def test_fp32_dense_sweep_accuracy():
    """2^22 fp32 values log-spaced in magnitude over both signs: y within 1e-6 relative."""
    m = 1 << 21
    mag = np.exp2(np.linspace(-30.0, 7.0, m)).astype(np.float32)
    x = np.concatenate([mag, -mag])
    dy = wl.draw_dy(x.shape[0], 1e-2, wl.F32, seed=6)
    rep, wy, wdx = _fwd_bwd_check(x, dy, wl.F32)
    print(f"\n[fp32 sweep] {rep} worst y {wy:.3f} worst dx {wdx:.3f} (fractions of the tolerance)")


def test_side_stream():
    s = torch.cuda.Stream()
    n = 8192 * 7 + 13
    x = wl.draw_x(n, "normal", 1.0, wl.BF16, seed=77)
    dy = wl.draw_dy(n, 1e-2, wl.BF16, seed=78)
    _fwd_bwd_check(x, dy, wl.BF16, stream=s)


def test_two_streams_in_flight_together():
    """Launches of every kind interleaved on two streams with no synchronisation in between (the
    library keeps no per-call device state, the measured-range variant only its caller's qstate):
    each stream's results match the oracle."""
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    jobs = []
    for k, (dtype, n) in enumerate([(wl.BF16, 3_000_003), (wl.F32, 2_500_001)]):
        es = gu.esize(dtype)
        x = wl.draw_x(n, "normal", 1.2, dtype, seed=900 + k)
        dy = wl.draw_dy(n, 1e-2, dtype, seed=910 + k)
        b = {"x": gu.Buf(n * es).upload(x), "dy": gu.Buf(n * es).upload(dy)}
        for name in ("y", "dx", "yd", "dxd"):
            b[name] = gu.Buf(n * es)
        b["c"], b["cd"], b["q"] = gu.Buf((n + 1) // 2), gu.Buf((n + 1) // 2), gu.Buf(4 * s2a.QSTATE_FLOATS)
        jobs.append((dtype, n, x, dy, b))
    torch.cuda.synchronize()
    for rep in range(3):  # several rounds so that the two streams really overlap
        for (dtype, n, x, dy, b), st in zip(jobs, streams):
            s2a.act_fwd(b["x"].ptr, b["y"].ptr, b["c"].ptr, n, dtype, st.cuda_stream)
            s2a.act_fwd_dyn(b["x"].ptr, b["yd"].ptr, b["cd"].ptr, b["q"].ptr, n, dtype, st.cuda_stream)
        for (dtype, n, x, dy, b), st in zip(jobs, streams):
            s2a.act_bwd(b["dy"].ptr, b["c"].ptr, b["dx"].ptr, n, dtype, st.cuda_stream)
            s2a.act_bwd_dyn(b["dy"].ptr, b["cd"].ptr, b["q"].ptr, b["dxd"].ptr, n, dtype, st.cuda_stream)
    torch.cuda.synchronize()
    for dtype, n, x, dy, b in jobs:
        y_ref, code_ref, packed_ref, near = oracle.fwd(x, dtype, band=parity.BAND)
        packed = b["c"].download(np.uint8)
        parity.check_codes(packed, code_ref, near, n, parity.band_mask(wl.storage_to_f64(x, dtype), parity.GELU_POINTS))
        parity.check_values(b["y"].download(gu.storage_np(dtype)), y_ref, dtype, "y")
        differs = parity.unpack(packed, n) != code_ref
        parity.check_values(b["dx"].download(gu.storage_np(dtype)), oracle.bwd(dy, dtype, packed_ref), dtype, "dx", skip=differs)
        yd_ref, coded_ref, packedd_ref, neard, qmin, qscale = oracle.fwd_dyn(x, dtype, band=parity.BAND)
        qs = b["q"].download(np.float32)
        assert qs[2] == np.float32(qmin) and qs[3] == np.float32(qscale)
        packedd = b["cd"].download(np.uint8)
        parity.check_codes(packedd, coded_ref, neard, n,
                           parity.band_mask(wl.storage_to_f64(x, dtype), parity.range_points(qmin, qscale), clip=True))
        differs = parity.unpack(packedd, n) != coded_ref
        parity.check_values(b["dxd"].download(gu.storage_np(dtype)), oracle.bwd_dyn(dy, dtype, packedd_ref, qmin, qscale),
                            dtype, "dx", skip=differs)
        assert all(v.canaries_intact() for v in b.values())


def test_outputs_are_fully_overwritten():
    """Stale 0xFF bytes in y / codes / dx never survive, including the pad nibble."""
    for dtype in DTYPES:
        for n in (1, 7, 8193, 40001):
            x = wl.draw_x(n, "normal", 1.0, dtype, seed=n)
            es = gu.esize(dtype)
            bx = gu.Buf(n * es).upload(x)
            by = gu.Buf(n * es, fill=0xFF)
            bc = gu.Buf((n + 1) // 2, fill=0xFF)
            s2a.act_fwd(bx.ptr, by.ptr, bc.ptr, n, dtype, torch.cuda.current_stream().cuda_stream)
            y_ref, code_ref, packed_ref, near = oracle.fwd(x, dtype, band=parity.BAND)
            parity.check_codes(bc.download(np.uint8), code_ref, near, n, parity.band_mask(wl.storage_to_f64(x, dtype), parity.GELU_POINTS))
            parity.check_values(by.download(gu.storage_np(dtype)), y_ref, dtype, "y")


WORKLOAD_CASES = [("tiny", 0, 0), ("vit_b16", 0, 0), ("vit_b16", 11, 0), ("vit_l16", 0, 0), ("vit_l16", 23, 0),
                  ("swin_b", 0, 0), ("swin_b", 0, 1), ("swin_b", 0, 2), ("swin_b", 0, 3),
                  ("vit_g14", 0, 0), ("vit_g14_f32", 0, 0)]


@pytest.mark.parametrize("name,layer,stage", WORKLOAD_CASES)
def test_workload_full_size(name, layer, stage):
    """Every configuration at its full size, in the launch configuration the benchmark
    times (256-byte aligned buffers, the caller's stream), every element checked."""
    w = wl.WORKLOADS[name]
    x, dy = wl.layer_inputs(w, layer, stage)
    n = x.shape[0]
    es = gu.esize(w.dtype)
    st = torch.cuda.current_stream().cuda_stream
    tx = torch.from_numpy(x.view(np.uint8)).cuda()
    ty = torch.empty_like(tx)
    tc = torch.empty((n + 1) // 2, dtype=torch.uint8, device="cuda")
    s2a.act_fwd(tx.data_ptr(), ty.data_ptr(), tc.data_ptr(), n, w.dtype, st)
    torch.cuda.synchronize()
    y = ty.cpu().numpy().view(gu.storage_np(w.dtype))
    packed = tc.cpu().numpy()
    del ty
    y_ref, code_ref, packed_ref, near = oracle.fwd(x, w.dtype, band=parity.BAND)
    rep = parity.check_codes(packed, code_ref, near, n, parity.band_mask(wl.storage_to_f64(x, w.dtype), parity.GELU_POINTS))
    wy = parity.check_values(y, y_ref, w.dtype, "y")
    del y, y_ref
    tdy = torch.from_numpy(dy.view(np.uint8)).cuda()
    tdx = torch.empty_like(tdy)
    s2a.act_bwd(tdy.data_ptr(), tc.data_ptr(), tdx.data_ptr(), n, w.dtype, st)
    torch.cuda.synchronize()
    dx = tdx.cpu().numpy().view(gu.storage_np(w.dtype))
    dx_ref = oracle.bwd(dy, w.dtype, packed_ref)
    differs = parity.unpack(packed, n) != code_ref
    wdx = parity.check_values(dx, dx_ref, w.dtype, "dx", skip=differs if rep.differing else None)
    print(f"\n[{name} layer {layer} stage {stage}] n={n} {rep} worst y {wy:.3f} worst dx {wdx:.3f} "
          f"(fractions of the tolerance)")
    assert es * n == x.nbytes


@pytest.mark.parametrize("dtype", DTYPES)
def test_more_than_2_31_elements(dtype):
    """n just above 2^31 (64-bit indexing everywhere, ragged tail): a seeded tile is
    repeated on the device, and 256 sampled spans of ~4096 outputs (both ends and the
    2^31 crossing included) are checked one by one against the oracle."""
    tile_n = (1 << 22) + 3                      # odd: every repetition has a different alignment
    n = (1 << 31) + 8 * 64 * 3 + 5              # odd: pad nibble, leftover elements
    tile_x = wl.draw_x(tile_n, "student_t", 2.0, dtype, seed=4242)
    tile_dy = wl.draw_dy(tile_n, 1e-2, dtype, seed=4243)
    reps = -(-n // tile_n)

    def tiled(tile):
        t = torch.from_numpy(tile.view(np.int16) if dtype == wl.BF16 else tile).cuda()
        return t.repeat(reps)[:n]

    tx = tiled(tile_x)
    ty = torch.empty_like(tx)
    tc = torch.empty((n + 1) // 2, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    s2a.act_fwd(tx.data_ptr(), ty.data_ptr(), tc.data_ptr(), n, dtype, st)
    torch.cuda.synchronize()

    # Spans are copied back slice by slice (plain device-to-host copies): advanced
    # indexing of a tensor this large faults inside torch's own index kernel here.
    g = np.random.default_rng(99)
    spans = [(0, 4096), (n - 5001, 5001), ((1 << 31) - 2048, 3072)]   # the tensor ends 1541 past 2^31
    spans += [(int(a) & ~1, 4096) for a in g.integers(0, n - 4096, 253)]   # even starts own whole code bytes

    def fetch(t):
        return np.concatenate([t[a:a + m].cpu().numpy() for a, m in spans]).view(gu.storage_np(dtype))

    pos = np.concatenate([np.arange(a, a + m, dtype=np.int64) for a, m in spans])
    x_s = tile_x[pos % tile_n].copy()
    dy_s = tile_dy[pos % tile_n].copy()
    y_ref, code_ref, _, near = oracle.fwd(x_s, dtype, band=parity.BAND)
    parity.check_values(fetch(ty), y_ref, dtype, "y")
    code_s = np.concatenate([parity.unpack(tc[a // 2:(a + m + 1) // 2].cpu().numpy(), m) for a, m in spans])
    diff = code_s != code_ref
    parity.check_flags(near, parity.band_mask(wl.storage_to_f64(x_s, dtype), parity.GELU_POINTS))
    assert not (diff & (near == 0)).any()
    assert (tc[-1:].cpu().numpy()[0] >> 4) == 0  # pad nibble of the odd-length tensor
    del ty
    tdy = tiled(tile_dy)
    tdx = torch.empty_like(tdy)
    s2a.act_bwd(tdy.data_ptr(), tc.data_ptr(), tdx.data_ptr(), n, dtype, st)
    torch.cuda.synchronize()
    # the oracle's backward reads packed codes: pack each span's oracle codes with the oracle itself
    dx_ref = np.concatenate([oracle.bwd(dy_s[o:o + m].copy(), dtype, oracle.fwd(x_s[o:o + m].copy(), dtype)[2])
                             for o, m in zip(np.cumsum([0] + [m for _, m in spans[:-1]]), [m for _, m in spans])])
    parity.check_values(fetch(tdx), dx_ref, dtype, "dx", skip=diff)
    print(f"\n[n={n} dtype={dtype}] checked {pos.shape[0]} sampled elements, in-band {int(near.sum())}, "
          f"differing {int(diff.sum())}")


@pytest.mark.parametrize("nbytes", [16, 1024, 1040, 16 * 64 * 37 + 16, 1 << 24])
def test_stream_copy_is_a_copy(nbytes):
    """The measurement aid moves the bytes it is given and nothing else."""
    g = np.random.Generator(np.random.Philox(nbytes))
    src = g.integers(0, 256, nbytes, dtype=np.uint8)
    bs = gu.Buf(nbytes).upload(src)
    bd = gu.Buf(nbytes, fill=0x11)
    s2a.stream_copy(bs.ptr, bd.ptr, nbytes, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert bd.canaries_intact() and bs.canaries_intact()
    np.testing.assert_array_equal(bd.download(np.uint8), src)
