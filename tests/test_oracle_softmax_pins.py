"""Pins for the softmax part of the oracle (Sec. 3.2 "Softmax layer", Eq. 7-9):
library softmax and its autograd, exact rationals, closed forms."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2503_08154_amd import workloads as wl


def _rows(rows, L, scale, seed, dtype=wl.F32):
    return wl.draw_x(rows * L, "normal", scale, dtype, seed=seed)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("L", [1, 2, 3, 16, 49, 197])
def test_y_is_library_softmax(dtype, L):
    rows = 37
    x = _rows(rows, L, 3.0, 7 + L, dtype)
    y, *_ = oracle.softmax_fwd(x, dtype, rows, L)
    xt = torch.from_numpy(wl.storage_to_f64(x, dtype)).reshape(rows, L)
    np.testing.assert_allclose(y.reshape(rows, L), torch.softmax(xt, dim=-1).numpy(), rtol=1e-13, atol=0)
    np.testing.assert_allclose(y.reshape(rows, L).sum(axis=1), 1.0, rtol=1e-14)


def test_literal_quotient_of_eq7_and_shift_invariance():
    rows, L = 5, 33
    x = (np.round(_rows(rows, L, 2.0, 3) * 1024) / 1024).astype(np.float32)   # multiples of 2^-10: +8 is exact
    xv = x.astype(np.float64).reshape(rows, L)
    y = oracle.softmax_fwd(x, wl.F32, rows, L)[0].reshape(rows, L)
    np.testing.assert_allclose(y, np.exp(xv) / np.exp(xv).sum(axis=1, keepdims=True), rtol=1e-13)
    shifted = (xv + 8.0).astype(np.float32)               # exact shift for these magnitudes
    assert np.array_equal(shifted.astype(np.float64), xv + 8.0)
    y2 = oracle.softmax_fwd(shifted.reshape(-1), wl.F32, rows, L)[0].reshape(rows, L)
    np.testing.assert_allclose(y2, y, rtol=1e-13)


def test_masked_and_large_logits():
    x = np.array([1000.0, 999.0, -np.inf, -1000.0], np.float32)
    y = oracle.softmax_fwd(x, wl.F32, 1, 4)[0]
    e = np.exp(-1.0)
    np.testing.assert_allclose(y, [1 / (1 + e), e / (1 + e), 0.0, 0.0], rtol=1e-15)


def _exact_codes(yrow):
    ys = [Fraction(float(v)) for v in yrow]
    lo, hi = min(ys), max(ys)
    if hi == lo:
        return [0] * len(ys)
    out = []
    for v in ys:
        t = (v - lo) * 15 / (hi - lo)
        fl = t.numerator // t.denominator
        fr = t - fl
        if fr > Fraction(1, 2) or (fr == Fraction(1, 2) and fl % 2 == 1):
            fl += 1
        out.append(int(fl))
    return out


@pytest.mark.parametrize("L", [2, 5, 16, 49, 197])
def test_codes_against_exact_rationals_and_invariants(L):
    rows = 9
    x = _rows(rows, L, 2.5, 11 + L)
    y, code, packed, qmin, qscale, near = oracle.softmax_fwd(x, wl.F32, rows, L, band_t=1e-9)
    y, code, near = y.reshape(rows, L), code.reshape(rows, L), near.reshape(rows, L)
    for r in range(rows):
        want = _exact_codes(y[r])
        for i in range(L):
            if not near[r, i]:
                assert code[r, i] == want[i]
        assert qmin[r] == y[r].min() and qscale[r] == pytest.approx((y[r].max() - y[r].min()) / 15, rel=1e-15)
        assert code[r, y[r].argmin()] == 0 and code[r, y[r].argmax()] == 15
        order = np.argsort(y[r], kind="stable")
        assert np.all(np.diff(code[r, order].astype(int)) >= 0)
        recon = code[r] * qscale[r] + qmin[r]
        assert np.all(np.abs(recon - y[r]) <= qscale[r] / 2 * (1 + 1e-9))
    # row-aligned packing, low nibble first, pad nibble zero
    rb = (L + 1) // 2
    pk = packed.reshape(rows, rb)
    for r in range(rows):
        bits = np.unpackbits(pk[r], bitorder="little").reshape(-1, 4)
        nib = (bits * np.array([1, 2, 4, 8], np.uint8)).sum(axis=1)
        np.testing.assert_array_equal(nib[:L], code[r])
        if L % 2:
            assert nib[L] == 0


def test_backward_is_autograd_when_y_sits_on_the_levels():
    """Rows whose y are exactly min + k*scale: Eq. 9 reconstructs y, so the oracle's
    backward must equal automatic differentiation of a library softmax."""
    L = 16
    k = np.arange(L, dtype=np.float64)
    g = np.random.default_rng(0)
    for base, step in ((0.01, 0.0065), (0.03, 0.00433)):
        target = base + step * k
        target /= target.sum()                                   # still affine in k
        x64 = np.log(target)
        x = g.permutation(x64).astype(np.float64)
        # use float64-exact inputs by feeding float32 that round-trips: scale so values are coarse
        x32 = x.astype(np.float32)
        y, code, packed, qmin, qscale, near = oracle.softmax_fwd(x32, wl.F32, 1, L, band_t=0.05)
        assert not near.any()                                     # float32 rounding of x keeps y near the levels
        dy = wl.draw_dy(L, 1.0, wl.F32, seed=9)
        dx = oracle.softmax_bwd(dy, wl.F32, packed, qmin, qscale, 1, L)
        xt = torch.from_numpy(x32.astype(np.float64)).requires_grad_(True)
        torch.softmax(xt, dim=-1).backward(torch.from_numpy(dy.astype(np.float64)))
        # y is within float32 rounding of the levels, so y-hat = y to ~1e-7 relative
        np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=0, atol=5e-8)


def test_closed_forms():
    # constant row: y = 1/L, scale 0, codes 0, dx_i = (dy_i - mean(dy)) / L
    L = 7
    x = np.full(L, 0.3, np.float32)
    dy = wl.draw_dy(L, 1.0, wl.F32, seed=4)
    y, code, packed, qmin, qscale, _ = oracle.softmax_fwd(x, wl.F32, 1, L)
    assert not code.any() and qscale[0] == 0.0 and qmin[0] == pytest.approx(1 / L, rel=1e-15)
    dx = oracle.softmax_bwd(dy, wl.F32, packed, qmin, qscale, 1, L)
    np.testing.assert_allclose(dx, (dy.astype(np.float64) - dy.astype(np.float64).mean()) / L, rtol=1e-13, atol=1e-17)
    # L = 2: the two values are min and max, codes {0, 15}, y-hat = y, dx_0 = y0 y1 (dy_0 - dy_1)
    x = np.array([0.75, -0.5], np.float32)
    dy = np.array([2.0, -1.0], np.float32)
    y, code, packed, qmin, qscale, _ = oracle.softmax_fwd(x, wl.F32, 1, 2)
    assert code.tolist() == [15, 0] and packed.tolist() == [0x0F]
    dx = oracle.softmax_bwd(dy, wl.F32, packed, qmin, qscale, 1, 2)
    s = 1 / (1 + np.exp(-1.25))
    np.testing.assert_allclose(dx, [s * (1 - s) * 3.0, -s * (1 - s) * 3.0], rtol=1e-14)
    # gradients of a softmax row sum to zero when y-hat sums to one (here exactly reconstructed)
    assert abs(dx.sum()) < 1e-15


def test_quantization_error_bound_on_the_gradient():
    """|y-hat - y| <= scale/2 bounds the deviation from the exact softmax gradient."""
    rows, L = 20, 197
    x = _rows(rows, L, 2.0, 21)
    dy = wl.draw_dy(rows * L, 1.0, wl.F32, seed=22)
    y, code, packed, qmin, qscale, _ = oracle.softmax_fwd(x, wl.F32, rows, L)
    dx = oracle.softmax_bwd(dy, wl.F32, packed, qmin, qscale, rows, L).reshape(rows, L)
    xt = torch.from_numpy(x.astype(np.float64)).reshape(rows, L).requires_grad_(True)
    torch.softmax(xt, dim=-1).backward(torch.from_numpy(dy.astype(np.float64)).reshape(rows, L))
    dyv = np.abs(dy.astype(np.float64)).reshape(rows, L)
    half = qscale[:, None] / 2
    yv = y.reshape(rows, L)
    bound = half * (dyv + (yv * dyv).sum(axis=1, keepdims=True)) + (yv + half) * (half * dyv).sum(axis=1, keepdims=True)
    assert np.all(np.abs(dx - xt.grad.numpy()) <= bound * (1 + 1e-9) + 1e-18)


@pytest.mark.parametrize("band_t", [0.2, 0.05, 1e-3])
def test_near_flag_marks_exactly_the_band_of_the_level_index(band_t):
    """The softmax flag is on the real-valued level index t = (y - min y) / scale (Eq. 8): an
    element is flagged when t is within band_t of k + 1/2.  Recomputed in exact rationals from the
    oracle's own y (the flag is bookkeeping on y, not part of the method)."""
    rows, L = 40, 197
    x = _rows(rows, L, 2.0, 77)
    y, code, _, qmin, qscale, near = oracle.softmax_fwd(x, wl.F32, rows, L, band_t=band_t)
    y, near = y.reshape(rows, L), near.reshape(rows, L)
    flagged = 0
    for r in range(rows):
        ys = [Fraction(float(v)) for v in y[r]]
        lo, hi = min(ys), max(ys)
        for i, v in enumerate(ys):
            t = (v - lo) * 15 / (hi - lo)
            d = abs(t - (t.numerator // t.denominator) - Fraction(1, 2))
            if abs(float(d) - band_t) < 1e-9:      # the oracle forms t in doubles: skip the edge of the band
                continue
            assert near[r, i] == int(d <= Fraction(band_t)), (r, i, float(t))
            flagged += int(near[r, i])
    # most y of a row crowd near its minimum (t close to 0), so fewer than the uniform share
    # 2 * band_t are flagged -- but some are, and far from all
    assert 0.1 * 2 * band_t * rows * L < flagged < 2 * band_t * rows * L + 10


def test_near_flag_hand_placed_row():
    """A row of two extremes and probes whose y sit at known level indices: y proportional to
    (1, 16) spans 15 steps of size 1 (in units of y_0), so an element with weight 1 + k + 1/2 + d has t = k + 1/2 + d."""
    offs = [(0.0, 1), (4e-5, 1), (-4e-5, 1), (3e-4, 0), (-3e-4, 0), (0.25, 0)]
    weights = [1.0, 16.0] + [1.0 + 6 + 0.5 + d for d, _ in offs]
    x = np.log(np.array(weights)).astype(np.float32)
    y, _, _, qmin, qscale, near = oracle.softmax_fwd(x, wl.F32, 1, len(weights), band_t=1e-4)
    # fp32 rounding of log(w) moves t by at most ~16 * 2^-24 * |log w| * w ~ 3e-6: far inside the placements
    assert near.tolist() == [0, 0] + [f for _, f in offs]
