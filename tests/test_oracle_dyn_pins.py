"""Pins for the measured-range variant of the oracle (Eq. 8 taken literally:
min and max of the clipped tensor).  Independent of the oracle's own code:
reduction to the already pinned fixed-range oracle, exact rational arithmetic,
invariances and the degenerate cases."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2503_08154_amd import workloads as wl


def _exact_codes(vals):
    """Clip to [-2,2], Eq. 8 with the tensor's own extremes, exact rationals, ties to even."""
    xc = [min(max(Fraction(float(v)), Fraction(-2)), Fraction(2)) for v in vals]
    lo, hi = min(xc), max(xc)
    if hi == lo:
        return [0] * len(xc), lo, Fraction(0)
    s = (hi - lo) / 15
    out = []
    for v in xc:
        t = (v - lo) / s
        fl = t.numerator // t.denominator
        fr = t - fl
        if fr > Fraction(1, 2) or (fr == Fraction(1, 2) and fl % 2 == 1):
            fl += 1
        out.append(int(fl))
    return out, lo, s


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_reduces_to_the_fixed_range_when_both_clip_limits_are_reached(dtype):
    x = wl.draw_x(50_000, "normal", 1.5, dtype, seed=5)          # certainly has |x| > 2 on both sides
    dy = wl.draw_dy(50_000, 1.0, dtype, seed=6)
    y0, c0, p0, _ = oracle.fwd(x, dtype)
    y1, c1, p1, _, qmin, qscale = oracle.fwd_dyn(x, dtype)
    assert qmin == -2.0 and qscale == 4.0 / 15.0
    np.testing.assert_array_equal(c0, c1)
    np.testing.assert_array_equal(p0, p1)
    np.testing.assert_array_equal(y0, y1)
    np.testing.assert_array_equal(oracle.bwd(dy, dtype, p0), oracle.bwd_dyn(dy, dtype, p1, qmin, qscale))


@pytest.mark.parametrize("seed", range(6))
def test_exact_rational_arithmetic_on_small_tensors(seed):
    g = np.random.default_rng(seed)
    lo, hi = sorted(g.uniform(-2.5, 2.5, 2))
    x = g.uniform(lo, hi, 400).astype(np.float32)
    _, code, _, near, qmin, qscale = oracle.fwd_dyn(x, wl.F32, band=1e-9)
    want, elo, es = _exact_codes(x)
    assert Fraction(qmin) == elo
    assert abs(Fraction(qscale) - es) < Fraction(1, 10 ** 15)
    for i in range(x.shape[0]):
        if not near[i]:
            assert code[i] == want[i]
        else:
            assert abs(int(code[i]) - want[i]) <= 1


def test_extremes_levels_and_reconstruction():
    g = np.random.default_rng(3)
    x = g.uniform(-1.3, 0.9, 10_000).astype(np.float32)
    _, code, _, _, qmin, qscale = oracle.fwd_dyn(x, wl.F32)
    assert qmin == float(x.min()) and qscale == pytest.approx((float(x.max()) - float(x.min())) / 15, rel=1e-15)
    assert code[x.argmin()] == 0 and code[x.argmax()] == 15
    assert sorted(set(code.tolist())) == list(range(16))
    order = np.argsort(x, kind="stable")
    assert np.all(np.diff(code[order].astype(int)) >= 0)                         # monotone
    recon = np.array([oracle.dequantize_dyn(int(c), qmin, qscale) for c in code])
    assert np.all(np.abs(recon - x.astype(np.float64)) <= qscale / 2 + 1e-12)   # half a step
    for k in range(16):                                                          # levels reproduce themselves
        assert oracle.quantize_dyn(oracle.dequantize_dyn(k, qmin, qscale), qmin, qscale) == k


def test_codes_are_invariant_under_a_shift_inside_the_clip_range():
    """Shifting the whole tensor (without touching the clip limits) moves min and max
    with it, so every code stays put; the scale is unchanged."""
    base = np.linspace(-0.75, 0.5, 321)                      # multiples of 2^-8: shifts below are exact
    base = (np.round(base * 256) / 256).astype(np.float32)
    _, c0, _, near0, m0, s0 = oracle.fwd_dyn(base, wl.F32, band=1e-9)
    for shift in (0.25, -0.5, 1.0):
        shifted = (base + np.float32(shift)).astype(np.float32)
        _, c1, _, near1, m1, s1 = oracle.fwd_dyn(shifted, wl.F32, band=1e-9)
        assert m1 == m0 + shift and s1 == s0
        keep = (near0 == 0) & (near1 == 0)
        np.testing.assert_array_equal(c0[keep], c1[keep])


def test_backward_uses_the_measured_levels():
    x = np.linspace(-1.0, 0.5, 16).astype(np.float32)        # exactly the 16 levels of its own range
    _, code, packed, _, qmin, qscale = oracle.fwd_dyn(x, wl.F32)
    assert code.tolist() == list(range(16))
    dx = oracle.bwd_dyn(np.ones(16, np.float32), wl.F32, packed, qmin, qscale)
    want = [oracle.gelu_deriv_approx(oracle.dequantize_dyn(k, qmin, qscale)) for k in range(16)]
    np.testing.assert_array_equal(dx, np.array(want))
    # the representatives are within rounding of the inputs themselves
    np.testing.assert_allclose([oracle.dequantize_dyn(k, qmin, qscale) for k in range(16)], x.astype(np.float64), atol=1e-7)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_degenerate_tensors(dtype):
    # all equal: scale 0, codes 0, Eq. 9 returns the value itself
    x = wl.to_storage(np.full(7, 0.75), dtype)
    _, code, packed, _, qmin, qscale = oracle.fwd_dyn(x, dtype)
    assert qmin == 0.75 and qscale == 0.0 and not code.any() and not packed.any()
    dx = oracle.bwd_dyn(wl.to_storage(np.full(7, 2.0), dtype), dtype, packed, qmin, qscale)
    np.testing.assert_array_equal(dx, np.full(7, 2.0 * oracle.gelu_deriv_approx(0.75)))
    # everything beyond one clip limit: also a single value after the clip
    x = wl.to_storage(np.array([5.0, 7.0, 1e30, np.inf]), dtype)
    _, code, _, _, qmin, qscale = oracle.fwd_dyn(x, dtype)
    assert qmin == 2.0 and qscale == 0.0 and not code.any()
    # empty
    y, code, packed, near, qmin, qscale = oracle.fwd_dyn(np.empty(0, x.dtype), dtype)
    assert y.shape == (0,) and packed.shape == (0,) and qscale == 0.0
    # a NaN clips to -2 and therefore sets the minimum
    x = wl.to_storage(np.array([0.5, np.nan, 1.0]), dtype)
    _, code, _, _, qmin, qscale = oracle.fwd_dyn(x, dtype)
    assert qmin == -2.0 and code[1] == 0 and code[2] == 15


def _in_band_exact(x32, lo: Fraction, scale: Fraction, band: Fraction):
    """Which elements lie within `band` of a decision point lo + (j + 1/2) * scale, j = 0..14,
    after the clip to [-2, 2]: exact rational arithmetic on the stored values."""
    pts = [lo + (Fraction(2 * j + 1, 2)) * scale for j in range(15)]
    out = []
    for v in x32:
        xc = min(max(Fraction(float(v)), Fraction(-2)), Fraction(2))
        out.append(int(min(abs(xc - p) for p in pts) <= band))
    return out


def test_near_flag_marks_exactly_the_band_of_the_measured_range():
    """Sec. 3.2, GeLU paragraph read literally: the decision points of Eq. 8 are
    min + (j + 1/2) * scale of the clipped tensor.  Range [-1, 0.875] has scale 1/8, so every
    decision point is a binary fraction and the hand-placed offsets are what they say."""
    lo, hi = -1.0, 0.875
    pts = [lo + (j + 0.5) * 0.125 for j in range(15)]
    vals, want = [lo, hi], [0, 0]
    for j in (0, 3, 7, 11, 14):
        for off, flag in ((5e-7, 1), (-5e-7, 1), (2e-6, 0), (-2e-6, 0), (0.0, 1), (0.03, 0)):
            vals.append(pts[j] + off)
            want.append(flag)
    x = np.array(vals, np.float32)
    _, _, _, near, qmin, qscale = oracle.fwd_dyn(x, wl.F32, band=1e-6)
    assert qmin == lo and qscale == 0.125
    assert near.tolist() == want
    assert near.tolist() == _in_band_exact(x, Fraction(lo), Fraction(1, 8), Fraction(1, 10 ** 6))
    # a wider band takes in the +-2e-6 points as well, and nothing else
    _, _, _, near3, _, _ = oracle.fwd_dyn(x, wl.F32, band=3e-6)
    assert near3.tolist() == _in_band_exact(x, Fraction(lo), Fraction(1, 8), Fraction(3, 10 ** 6))
    assert sum(near3.tolist()) == sum(want) + 10


def test_near_flag_uses_the_clipped_value_and_the_measured_points():
    """Values beyond a clip limit are judged where the clip puts them (the end of the range, half a
    step from the nearest decision point), and the points move with the measured range: the same x
    is in the band for one tensor and outside it for another."""
    probe = np.float32(-0.9375)                                   # = -1 + 0.5 * 0.125
    a = np.array([-1.0, 0.875, probe, 7.0, -9.0], np.float32)     # clips to [-2, 2]: range [-2, 2]
    _, _, _, near_a, qmin, qscale = oracle.fwd_dyn(a, wl.F32, band=1e-6)
    assert qmin == -2.0 and qscale == 4.0 / 15.0
    assert near_a.tolist() == _in_band_exact(a, Fraction(-2), Fraction(4, 15), Fraction(1, 10 ** 6)) == [0, 0, 0, 0, 0]
    b = np.array([-1.0, 0.875, probe], np.float32)                # range [-1, 0.875]
    _, _, _, near_b, _, _ = oracle.fwd_dyn(b, wl.F32, band=1e-6)
    assert near_b.tolist() == [0, 0, 1]
    # a range so narrow that its upper end is within the band of the last decision point: a value
    # far beyond the clip limit is flagged, because it is the clipped value 2 that is judged
    c = np.array([2.0 - 3e-5, 7.0], np.float32)
    _, _, _, near_c, qmin, qscale = oracle.fwd_dyn(c, wl.F32, band=1.5e-6)
    lo = Fraction(float(c[0]))
    assert near_c.tolist() == _in_band_exact(c, lo, (2 - lo) / 15, Fraction(15, 10 ** 7)) == [1, 1]


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_near_flag_on_random_tensors_against_exact_rationals(dtype):
    g = np.random.default_rng(12)
    x = wl.to_storage(g.uniform(-1.25, 0.75, 3000), dtype)
    band = 2e-3                                                   # wide enough to catch a few dozen draws
    _, _, _, near, qmin, qscale = oracle.fwd_dyn(x, dtype, band=band)
    xv = wl.storage_to_f64(x, dtype)
    lo, hi = Fraction(float(xv.min())), Fraction(float(xv.max()))
    want = np.array(_in_band_exact(xv, lo, (hi - lo) / 15, Fraction(band)))
    # the oracle's scale is the rounded double of (hi - lo)/15: leave out the draws within 1e-12 of the band edge
    pts = np.array([float(lo + Fraction(2 * j + 1, 2) * (hi - lo) / 15) for j in range(15)])
    edge = np.abs(np.abs(xv[:, None] - pts[None, :]).min(axis=1) - band) < 1e-12
    np.testing.assert_array_equal(near[~edge], want[~edge])
    assert 20 < near.sum() < 0.2 * x.shape[0]
