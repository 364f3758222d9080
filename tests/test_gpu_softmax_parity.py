"""GPU parity of the softmax-with-4-bit-y kernels (s2a_softmax_fwd / _bwd)
against the oracle.

Tolerances, each from the arithmetic of the kernels (eps = 2^-24):
- y as for the activation path (1e-6 relative in fp32, 1 bf16 ulp).
- (min, scale) per row: min is one of the y, so QP_RTOL = 1e-6 relative (1e-5 for bf16
  storage, whose exponentials carry no compensated argument: the rounding of x * log2(e)
  at |x - max| up to 100 is 100 * 1.44 * eps ~ 9e-6); scale = (hi - lo)/15 adds the
  errors of both ends and a division: 4 * QP_RTOL.
- codes: the kernel rounds t = (y - lo) * (15/(hi - lo)) + 1/2 in fp32 from its own y, lo
  and scale, the oracle in fp64 from exact ones.  With relative errors e of y and lo and
  e_s of the scale, |dt| <= 15 * (2e * hi/(hi - lo) + e_s).  Softmax rows of random logits
  have lo << hi, so hi/(hi - lo) ~ 1 and with e = e_s = 1e-6 the bound is 4.5e-5: BAND_T =
  5e-5 (fp32).  bf16 storage: e, e_s ~ 4e-6 (fast exp2 and rcp) give 1.8e-4: 2e-4.  A code
  may differ only where t is within BAND_T of k + 1/2 (counted; a differing code is off by
  one).  Rows of nearly equal values have hi/(hi - lo) = R >> 1 and the band grows with R
  (test_nearly_flat_rows).
- dx_i = yh_i * (dy_i - sum_j yh_j dy_j) is a difference of two terms, so its error is
  measured against their magnitudes, S_i = yh_i * (|dy_i| + sum_j yh_j |dy_j|).  Backward
  alone on the oracle's codes and parameters: one rounding per yh, a sum of L <= 1024
  terms taken as <= 32 sequential adds per lane and 6 tree steps (38 * eps = 2.3e-6), a
  subtraction and a product: |err| <= 1e-5 * S_i has a factor 4 in hand (+ 2 bf16 ulps of
  the result for bf16 storage).
- dx end to end (the GPU's own codes and parameters against the oracle's): a relative
  perturbation rho of every yh moves dx_i by at most 2 * rho * S_i (once through yh_i, once
  through the sum).  yh = lo + k * scale with k * scale <= yh: rho <= QP_RTOL + 4 * QP_RTOL.
  fp32: 2 * 5e-6 = 1e-5 on top of the arithmetic's 1e-5: factor 2.  bf16: the tested
  factor is 10 (rho <= 4.5e-5), a little tighter than the 11 that QP_RTOL alone allows.
"""
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
BAND_T = {wl.F32: 5e-5, wl.BF16: 2e-4}
QP_RTOL = {wl.F32: 1e-6, wl.BF16: 1e-5}


def _logits(rows, L, dtype, seed, scale=2.0, masked=False):
    g = np.random.Generator(np.random.Philox(seed))
    a = g.standard_normal(rows * L) * scale
    if masked and L > 2:
        m = g.random(rows * L) < 0.15
        m.reshape(rows, L)[:, 0] = False          # keep at least one finite entry per row
        a[m] = -np.inf
    return wl.to_storage(a, dtype)


def _dx_scale(yh, dy, rows, L):
    yh, dy = np.abs(yh.reshape(rows, L)), np.abs(dy.reshape(rows, L))
    return (yh * (dy + (yh * dy).sum(axis=1, keepdims=True))).reshape(-1)


def _check_dx(got_storage, ref, dtype, scale, factor=1.0, skip_rows=None, rows=0, L=0):
    got = wl.storage_to_f64(got_storage, dtype)
    tol = 1e-5 * factor * scale + 1e-300
    if dtype == wl.BF16:
        tol = tol + 2.0 * parity.bf16_ulp(ref)
    bad = np.abs(got - ref) > tol
    if skip_rows is not None:
        bad.reshape(rows, L)[skip_rows] = False
    assert not bad.any(), f"{int(bad.sum())} dx out of tolerance, first at {int(np.argmax(bad))}: " \
                          f"{got[np.argmax(bad)]!r} vs {ref[np.argmax(bad)]!r}"


def _run_and_check(x, dy, dtype, rows, L, offset=0, spread=1.0):
    """`spread` >= 1 widens what depends on hi - lo (the band of the codes, the tolerance of the scale and
    of the end-to-end dx) for rows whose values are nearly equal: R = hi / (hi - lo) of the flattest row."""
    n = rows * L
    band_t = BAND_T[dtype] * spread
    es = gu.esize(dtype)
    rb = (L + 1) // 2
    st = torch.cuda.current_stream().cuda_stream
    y_ref, code_ref, packed_ref, qmin, qscale, near = oracle.softmax_fwd(x, dtype, rows, L, band_t=band_t)
    bx = gu.Buf(n * es, offset * es).upload(x)
    by = gu.Buf(n * es, offset * es, fill=0xFF)
    bc = gu.Buf(rows * rb, offset, fill=0xFF)
    bq = gu.Buf(8 * rows, fill=0xFF)
    s2a.softmax_fwd(bx.ptr, by.ptr, bc.ptr, bq.ptr, rows, L, dtype, st)
    torch.cuda.synchronize()
    assert bx.canaries_intact() and by.canaries_intact() and bc.canaries_intact() and bq.canaries_intact()
    y = by.download(gu.storage_np(dtype))
    packed = bc.download(np.uint8)
    qp = bq.download(np.float32).reshape(rows, 2)
    finite_rows = np.isfinite(y_ref.reshape(rows, L)).all(axis=1)
    parity.check_values(y, y_ref, dtype, "y", finite_in=np.repeat(finite_rows, L))
    np.testing.assert_allclose(qp[finite_rows, 0], qmin[finite_rows], rtol=QP_RTOL[dtype], atol=1e-37)
    np.testing.assert_allclose(qp[finite_rows, 1], qscale[finite_rows], rtol=QP_RTOL[dtype] * 4 * spread, atol=1e-37)
    # codes, row by row (each row starts on a byte)
    got = np.stack([parity.unpack(packed[r * rb:(r + 1) * rb], L) for r in range(rows)]).reshape(-1) if rows else np.empty(0, np.uint8)
    diff = (got != code_ref) & np.repeat(finite_rows, L)
    parity.check_flags(near, parity.level_band_mask(y_ref, qmin, qscale, L, band_t))
    assert not (diff & (near == 0)).any(), "a code differs outside the band"
    if diff.any():
        assert (np.abs(got[diff].astype(int) - code_ref[diff].astype(int)) == 1).all()
    if L % 2 and rows:
        assert (packed.reshape(rows, rb)[:, -1] >> 4 == 0).all(), "pad nibble not zero"
    # backward alone: the oracle's codes and its (min, scale) rounded to fp32 go in
    qp32 = np.stack([qmin, qscale], axis=1).astype(np.float32)
    dx_ref = oracle.softmax_bwd(dy, dtype, packed_ref, qp32[:, 0].astype(np.float64), qp32[:, 1].astype(np.float64), rows, L)
    yh = code_ref * np.repeat(qp32[:, 1].astype(np.float64), L) + np.repeat(qp32[:, 0].astype(np.float64), L)
    scale = _dx_scale(yh, wl.storage_to_f64(dy, dtype), rows, L)
    bdy = gu.Buf(n * es, offset * es).upload(dy)
    bdx = gu.Buf(n * es, offset * es, fill=0xFF)
    bc2 = gu.Buf(rows * rb, offset).upload(packed_ref)
    bq2 = gu.Buf(8 * rows).upload(qp32.reshape(-1))
    s2a.softmax_bwd(bdy.ptr, bc2.ptr, bq2.ptr, bdx.ptr, rows, L, dtype, st)
    torch.cuda.synchronize()
    assert bdx.canaries_intact() and bdy.canaries_intact()
    bad_rows = ~finite_rows
    _check_dx(bdx.download(gu.storage_np(dtype)), dx_ref, dtype, scale, skip_rows=bad_rows, rows=rows, L=L)
    # end to end: the GPU's own codes and parameters; rows with a legitimately differing code are skipped
    s2a.softmax_bwd(bdy.ptr, bc.ptr, bq.ptr, bdx.ptr, rows, L, dtype, st)
    torch.cuda.synchronize()
    dx_ref2 = oracle.softmax_bwd(dy, dtype, packed_ref, qmin, qscale, rows, L)
    skip = bad_rows | diff.reshape(rows, L).any(axis=1) if rows else None
    _check_dx(bdx.download(gu.storage_np(dtype)), dx_ref2, dtype, scale, factor=1.0 + (9.0 if dtype == wl.BF16 else 1.0) * spread,
              skip_rows=skip, rows=rows, L=L)
    return int(near.sum()), int(diff.sum())


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("L", [1, 2, 3, 7, 8, 9, 16, 17, 49, 64, 65, 127, 128, 129, 196, 197, 256, 257,
                               511, 512, 513, 1023, 1024])
def test_row_lengths(dtype, L):
    for rows in (1, 5, 67):
        x = _logits(rows, L, dtype, seed=L * 10 + rows)
        dy = wl.draw_dy(rows * L, 1.0, dtype, seed=L * 10 + rows + 1)
        _run_and_check(x, dy, dtype, rows, L)


@pytest.mark.parametrize("dtype", DTYPES)
def test_every_row_length(dtype):
    """All L in 1..1024: every (lanes per row, pair slots) instantiation of the staged kernels,
    with a row count that leaves the last block ragged; every seventh length over several blocks."""
    for L in range(1, 1025):
        rows = 131 if L % 7 == 0 else 3 + L % 5
        x = _logits(rows, L, dtype, seed=40000 + L)
        dy = wl.draw_dy(rows * L, 1.0, dtype, seed=50000 + L)
        _run_and_check(x, dy, dtype, rows, L)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("L", [1025, 1026, 2048, 4097, 20001])
def test_rows_longer_than_the_register_kernels_hold(dtype, L):
    """L above 1024: one block per row, the row read three times (forward) or twice (backward).  Buffers
    aligned and one element off; a few rows, with masked entries in the second case."""
    for rows, masked, offset in ((1, False, 0), (5, True, 1)):
        x = _logits(rows, L, dtype, seed=L + rows, scale=3.0, masked=masked)
        dy = wl.draw_dy(rows * L, 1.0, dtype, seed=L + rows + 1)
        _run_and_check(x, dy, dtype, rows, L, offset=offset)


def test_longest_row():
    """One row of S2A_SOFTMAX_MAX_L elements."""
    L = s2a.SOFTMAX_MAX_L
    x = _logits(1, L, wl.BF16, seed=77, scale=4.0)
    dy = wl.draw_dy(L, 1.0, wl.BF16, seed=78)
    _run_and_check(x, dy, wl.BF16, 1, L)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("L", [49, 197, 257])
def test_masked_and_peaked_rows(dtype, L):
    rows = 333
    x = _logits(rows, L, dtype, seed=5 + L, scale=6.0, masked=True)
    dy = wl.draw_dy(rows * L, 1e-2, dtype, seed=6 + L)
    _run_and_check(x, dy, dtype, rows, L)


@pytest.mark.parametrize("dtype", DTYPES)
def test_constant_and_two_valued_rows(dtype):
    L, rows = 197, 4
    a = np.zeros((rows, L))
    a[1] = 0.75                      # constant rows: scale 0, codes 0
    a[2, ::2] = 1.0                  # two values: codes 0 and 15 only
    a[3, 5] = 30.0                   # one dominant entry
    x = wl.to_storage(a.reshape(-1), dtype)
    dy = wl.draw_dy(rows * L, 1.0, dtype, seed=3)
    _run_and_check(x, dy, dtype, rows, L)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("sigma", [0.05, 0.005])
def test_nearly_flat_rows(dtype, sigma):
    """Logits that differ little: y_max / (y_max - y_min) = R is 4 ... 40 instead of about 1, and the
    rounding of each y (relative to y) is R times larger relative to the step of Eq. 8.  The band of the
    codes and the tolerances that hang on hi - lo scale with R; everything else is as for other rows."""
    rows, L = 300, 197
    x = _logits(rows, L, dtype, seed=900, scale=sigma)
    dy = wl.draw_dy(rows * L, 1.0, dtype, seed=901)
    _, _, _, qmin, qscale, _ = oracle.softmax_fwd(x, dtype, rows, L, band_t=BAND_T[dtype])
    live = qscale > 0
    R = float(((qmin[live] + 15.0 * qscale[live]) / (15.0 * qscale[live])).max())
    assert 2.0 < R < 200.0
    near, differing = _run_and_check(x, dy, dtype, rows, L, spread=R)
    print(f"\n[softmax flat rows sigma={sigma} dtype={dtype}] R={R:.1f} flagged {near} differing {differing}")


@pytest.mark.parametrize("dtype", DTYPES)
def test_unaligned_buffers(dtype):
    rows, L = 50, 197
    x = _logits(rows, L, dtype, seed=77)
    dy = wl.draw_dy(rows * L, 1.0, dtype, seed=78)
    _run_and_check(x, dy, dtype, rows, L, offset=1)


def test_argument_errors():
    fake = 0x1000
    assert s2a.softmax_fwd(fake, fake, fake, fake, 4, 0, s2a.F32, check=False) == s2a.ERR_SIZE
    assert s2a.softmax_fwd(fake, fake, fake, fake, 4, s2a.SOFTMAX_MAX_L + 1, s2a.F32, check=False) == s2a.ERR_SIZE
    assert s2a.softmax_fwd(fake, fake, fake, fake, -1, 8, s2a.F32, check=False) == s2a.ERR_SIZE
    assert s2a.softmax_fwd(fake, fake, fake, fake, 4, 8, 9, check=False) == s2a.ERR_DTYPE
    assert s2a.softmax_fwd(fake, None, fake, fake, 4, 8, s2a.F32, check=False) == s2a.ERR_NULL
    assert s2a.softmax_bwd(fake, fake, 0x1002, fake, 4, 8, s2a.F32, check=False) == s2a.ERR_ALIGN
    assert s2a.softmax_fwd(None, None, None, None, 0, 8, s2a.F32, check=False) == s2a.OK


@pytest.mark.parametrize("dtype", DTYPES)
def test_vit_b16_attention_full_size(dtype):
    """ViT-B/16 attention probabilities of one layer: [64, 12, 197, 197] -> 151,296 rows of 197."""
    rows, L = 64 * 12 * 197, 197
    x = _logits(rows, L, dtype, seed=2024)
    dy = wl.draw_dy(rows * L, 1e-2, dtype, seed=2025)
    near, differing = _run_and_check(x, dy, dtype, rows, L)
    print(f"\n[softmax vit_b16 attention dtype={dtype}] n={rows * L} in-band={near} differing={differing}")


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("L", [49, 128, 197, 513])
@pytest.mark.parametrize("offset", [0, 1])
def test_in_place(dtype, L, offset):
    """y written over x and dx over dy (several blocks; the staged and the element-wise kernels)."""
    rows = 301
    n, rb, es = rows * L, (L + 1) // 2, gu.esize(dtype)
    x = _logits(rows, L, dtype, seed=900 + L)
    dy = wl.draw_dy(n, 1.0, dtype, seed=901 + L)
    st = torch.cuda.current_stream().cuda_stream
    y_ref, code_ref, packed_ref, qmin, qscale, near = oracle.softmax_fwd(x, dtype, rows, L, band_t=BAND_T[dtype])
    bx = gu.Buf(n * es, offset * es).upload(x)
    bc = gu.Buf(rows * rb, offset, fill=0xFF)
    bq = gu.Buf(8 * rows, fill=0xFF)
    s2a.softmax_fwd(bx.ptr, bx.ptr, bc.ptr, bq.ptr, rows, L, dtype, st)
    torch.cuda.synchronize()
    assert bx.canaries_intact() and bc.canaries_intact()
    parity.check_values(bx.download(gu.storage_np(dtype)), y_ref, dtype, "y")
    got = np.stack([parity.unpack(bc.download(np.uint8)[r * rb:(r + 1) * rb], L) for r in range(rows)]).reshape(-1)
    parity.check_flags(near, parity.level_band_mask(y_ref, qmin, qscale, L, BAND_T[dtype]))
    assert not ((got != code_ref) & (near == 0)).any()
    qp32 = np.stack([qmin, qscale], axis=1).astype(np.float32)
    dx_ref = oracle.softmax_bwd(dy, dtype, packed_ref, qp32[:, 0].astype(np.float64), qp32[:, 1].astype(np.float64), rows, L)
    yh = code_ref * np.repeat(qp32[:, 1].astype(np.float64), L) + np.repeat(qp32[:, 0].astype(np.float64), L)
    bdy = gu.Buf(n * es, offset * es).upload(dy)
    bc2 = gu.Buf(rows * rb, offset).upload(packed_ref)
    bq2 = gu.Buf(8 * rows).upload(qp32.reshape(-1))
    s2a.softmax_bwd(bdy.ptr, bc2.ptr, bq2.ptr, bdy.ptr, rows, L, dtype, st)
    torch.cuda.synchronize()
    assert bdy.canaries_intact()
    _check_dx(bdy.download(gu.storage_np(dtype)), dx_ref, dtype, _dx_scale(yh, wl.storage_to_f64(dy, dtype), rows, L))


def test_more_than_2_31_bytes():
    """A bf16 tensor whose byte offsets pass 2^31 (5.45 M rows of 197): row groups at the start, across
    the 2^31-byte mark and at the end are compared with the oracle; forward and backward."""
    L, dtype = 197, wl.BF16
    rb = (L + 1) // 2
    block_rows = 1 << 16
    block = _logits(block_rows, L, dtype, seed=31)
    rows = (1 << 31) // (L * 2) + 1534
    reps = -(-rows // block_rows)
    x = np.tile(block, reps)[:rows * L]
    dyb = wl.draw_dy(block_rows * L, 1e-2, dtype, seed=32)
    tx = torch.from_numpy(x.view(np.uint8)).cuda()
    ty = torch.empty_like(tx)
    tc = torch.empty(rows * rb, dtype=torch.uint8, device="cuda")
    tq = torch.empty(2 * rows, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    s2a.softmax_fwd(tx.data_ptr(), ty.data_ptr(), tc.data_ptr(), tq.data_ptr(), rows, L, dtype, st)
    tdy = torch.from_numpy(np.tile(dyb, reps)[:rows * L].view(np.uint8)).cuda()
    del tx
    tdx = torch.empty_like(tdy)
    s2a.softmax_bwd(tdy.data_ptr(), tc.data_ptr(), tq.data_ptr(), tdx.data_ptr(), rows, L, dtype, st)
    torch.cuda.synchronize()
    mark = (1 << 31) // (L * 2)
    for r0 in (0, mark - 700, rows - 1400):
        nr = 1400
        xs = x[r0 * L:(r0 + nr) * L]
        y_ref, code_ref, packed_ref, qmin, qscale, near = oracle.softmax_fwd(xs, dtype, nr, L, band_t=BAND_T[dtype])
        y = ty[r0 * L * 2:(r0 + nr) * L * 2].cpu().numpy().view(np.uint16)
        parity.check_values(y, y_ref, dtype, "y")
        packed = tc[r0 * rb:(r0 + nr) * rb].cpu().numpy()
        got = np.stack([parity.unpack(packed[r * rb:(r + 1) * rb], L) for r in range(nr)]).reshape(-1)
        diff = got != code_ref
        parity.check_flags(near, parity.level_band_mask(y_ref, qmin, qscale, L, BAND_T[dtype]))
        assert not (diff & (near == 0)).any(), f"rows from {r0}: a code differs outside the band"
        qp = tq[2 * r0:2 * (r0 + nr)].cpu().numpy().reshape(nr, 2)
        np.testing.assert_allclose(qp[:, 0], qmin, rtol=QP_RTOL[dtype], atol=1e-37)
        # backward on the GPU's own codes and parameters; rows with a legitimately differing code are skipped
        k0 = (r0 * L) % (block_rows * L)            # the gradients repeat with the block, like x
        dys = np.concatenate([dyb, dyb])[k0:k0 + nr * L]
        dx_ref = oracle.softmax_bwd(dys, dtype, packed_ref, qmin, qscale, nr, L)
        yh = code_ref * np.repeat(qscale, L) + np.repeat(qmin, L)
        dx = tdx[r0 * L * 2:(r0 + nr) * L * 2].cpu().numpy().view(np.uint16)
        _check_dx(dx, dx_ref, dtype, _dx_scale(yh, wl.storage_to_f64(dys, dtype), nr, L), factor=10.0,
                  skip_rows=diff.reshape(nr, L).any(axis=1), rows=nr, L=L)
