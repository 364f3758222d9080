"""Pins for the CPU oracle: every check here is something the paper or the
mathematics fixes independently of the oracle's own code -- closed forms at
special points, identities, automatic differentiation, exact rational
arithmetic, brute force over the whole bf16 domain, and the paper's stated
constants (tests/golden/paper_constants.txt).  A dropped term, a wrong sign,
constant, index or nibble order in oracle/s2a_oracle.c fails at least one.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
from scipy.special import expit, ndtr

import oracle
from paper_2503_08154_amd import workloads as wl


def _paper_constants(golden_dir):
    out = {}
    with open(os.path.join(golden_dir, "paper_constants.txt")) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if line:
                k, v = line.split()
                out[k] = float(v)
    return out


@pytest.fixture(scope="module")
def paper(golden_dir):
    return _paper_constants(golden_dir)


# ----------------------------------------------------------------- Eq. 10 ---

def test_gelu_closed_form_points(paper):
    """sigma takes the rational values 1/4, 1/2, 3/4, 9/10 at known arguments."""
    a = paper["gelu_sigmoid_slope"]
    assert oracle.gelu(0.0) == 0.0
    for odds, sig in ((3.0, 0.75), (9.0, 0.9), (1.0 / 3.0, 0.25), (1.0 / 99.0, 0.01)):
        x = math.log(odds) / a
        assert oracle.gelu(x) == pytest.approx(sig * x, rel=1e-14, abs=0)


def test_gelu_reflection_identity():
    """sigma(-z) = 1 - sigma(z)  =>  y(x) - y(-x) = x, for any slope."""
    for x in np.linspace(0.01, 30.0, 500):
        assert oracle.gelu(x) - oracle.gelu(-x) == pytest.approx(x, rel=1e-14)


def test_gelu_is_scaled_silu(paper):
    """x*sigma(a x) = silu(a x)/a: reduces Eq. 10 to a library routine."""
    a = paper["gelu_sigmoid_slope"]
    xs = torch.linspace(-40.0, 40.0, 4001, dtype=torch.float64)
    ref = torch.nn.functional.silu(a * xs) / a
    got = np.array([oracle.gelu(float(x)) for x in xs])
    np.testing.assert_allclose(got, ref.numpy(), rtol=1e-13, atol=1e-300)


def test_gelu_tracks_erf_gelu():
    """The sigmoid form is the original GELU paper's approximation of x*Phi(x):
    the largest gap is 0.0203 near x = -2.27; a slope other than 1.702 moves it."""
    xs = np.linspace(-8.0, 8.0, 16001)
    y = np.array([oracle.gelu(x) for x in xs])
    gap = np.abs(y - xs * ndtr(xs))
    assert 0.0202 < gap.max() < 0.0205
    assert abs(abs(xs[gap.argmax()]) - 2.27) < 0.02


def test_gelu_tails():
    assert oracle.gelu(50.0) == pytest.approx(50.0, rel=1e-15)
    assert -1e-30 < oracle.gelu(-50.0) < 0.0
    assert math.isinf(oracle.gelu(math.inf)) and oracle.gelu(math.inf) > 0
    assert math.isnan(oracle.gelu(-math.inf))  # -inf * 0 by the literal formula
    assert math.isnan(oracle.gelu(math.nan))


# ----------------------------------------------------------------- Eq. 11 ---

def test_exact_derivative_is_autograd_of_eq10(paper):
    a = paper["gelu_sigmoid_slope"]
    xs = torch.linspace(-12.0, 12.0, 2401, dtype=torch.float64, requires_grad=True)
    (xs * torch.sigmoid(a * xs)).sum().backward()
    got = np.array([oracle.gelu_deriv_exact(float(x)) for x in xs.detach()])
    np.testing.assert_allclose(got, xs.grad.numpy(), rtol=1e-12, atol=1e-15)


def test_exact_derivative_is_slope_of_oracle_gelu():
    h = 1e-5
    for x in np.linspace(-6.0, 6.0, 241):
        fd = (oracle.gelu(x + h) - oracle.gelu(x - h)) / (2 * h)
        assert oracle.gelu_deriv_exact(x) == pytest.approx(fd, abs=2e-9)


def test_exact_derivative_properties_stated_by_the_paper(paper):
    """Property 1: second term odd and vanishing at +-inf.  Property 2: the
    derivative stays roughly inside (-0.1, 1.1)."""
    a = paper["gelu_sigmoid_slope"]
    xs = np.linspace(-30.0, 30.0, 60001)
    d = np.array([oracle.gelu_deriv_exact(x) for x in xs])
    second = d - expit(a * xs)
    np.testing.assert_allclose(second, -second[::-1], atol=1e-14)
    assert abs(second[0]) < 1e-12 and abs(second[-1]) < 1e-12
    assert paper["deriv_range_lo"] - 1e-3 < d.min() < paper["deriv_range_lo"] + 1e-3
    assert paper["deriv_range_hi"] - 1e-3 < d.max() < paper["deriv_range_hi"] + 1e-3


# ----------------------------------------------------------------- Eq. 12 ---

def test_approx_derivative_special_points(paper):
    a, amp, w = paper["gelu_sigmoid_slope"], paper["sine_amplitude"], paper["sine_frequency"]
    assert oracle.gelu_deriv_approx(0.0) == 0.5
    # sine term = +amp, 0, -amp where w*x = pi/2, pi, -pi/2
    x = math.pi / (2 * w)
    assert oracle.gelu_deriv_approx(x) == pytest.approx(expit(a * x) + amp, rel=1e-15)
    x = math.pi / w
    assert oracle.gelu_deriv_approx(x) == pytest.approx(expit(a * x), abs=1e-15)
    x = -math.pi / (2 * w)
    assert oracle.gelu_deriv_approx(x) == pytest.approx(expit(a * x) - amp, abs=1e-15)


def test_approx_derivative_reflection():
    """sigma(-z) = 1 - sigma(z) and sin odd  =>  D(x) + D(-x) = 1."""
    for x in np.linspace(0.0, 5.0, 501):
        assert oracle.gelu_deriv_approx(x) + oracle.gelu_deriv_approx(-x) == pytest.approx(1.0, abs=1e-15)


def test_approx_fits_exact_on_the_clip_range(paper):
    """Fig. 4 right: on [-2, 2] the sine term follows the second term of Eq. 11
    (same sign, one period) and the two derivatives stay within 0.075."""
    a = paper["gelu_sigmoid_slope"]
    xs = np.linspace(paper["clip_lo"], paper["clip_hi"], 4001)
    ap = np.array([oracle.gelu_deriv_approx(x) for x in xs])
    ex = np.array([oracle.gelu_deriv_exact(x) for x in xs])
    assert np.abs(ap - ex).max() < 0.075
    sine, second = ap - expit(a * xs), ex - expit(a * xs)
    inner = np.abs(xs) > 1e-9
    assert np.all(np.sign(sine[inner]) == np.sign(second[inner]))
    # one period over the clip range: a single sign change, at the origin
    assert np.count_nonzero(np.diff(np.sign(sine[inner])) != 0) == 1


# -------------------------------------------------------------- quantizer ---

def _exact_code(x: float, paper) -> int:
    """Clip + Eq. 8 in exact rational arithmetic, ties to even."""
    lo, hi = Fraction(int(paper["clip_lo"])), Fraction(int(paper["clip_hi"]))
    levels = 2 ** int(paper["bits"]) - 1
    xc = min(max(Fraction(x), lo), hi)
    t = (xc - lo) * levels / (hi - lo)
    fl = t.numerator // t.denominator
    frac = t - fl
    if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return int(fl)


def test_quantizer_exhaustive_bf16_against_exact_rationals(paper):
    """Every finite bf16 bit pattern.  Double rounding in the oracle can only
    differ from exact arithmetic inside the 1e-6 band around a decision point
    (in fact only for negative x so small that x + 2 rounds to 2)."""
    bits = np.arange(65536, dtype=np.uint16)
    vals = wl.bf16_bits_to_f32(bits).astype(np.float64)
    _, _, bounds = oracle.table()
    mismatched = 0
    for v in vals:
        if not math.isfinite(v):
            continue
        got, want = oracle.quantize(v), _exact_code(v, paper)
        if got != want:
            mismatched += 1
            assert np.abs(bounds - v).min() <= 1e-6 and -2.0 ** -52 <= v < 0
            assert abs(got - want) == 1
    # bf16 has about 9.5k negative patterns below 2^-52 in magnitude
    assert mismatched < 10000


def test_quantizer_random_fp32_against_exact_rationals(paper):
    g = np.random.default_rng(7)
    xs = np.concatenate([g.standard_normal(4000) * 1.5, g.uniform(-2.2, 2.2, 4000)]).astype(np.float32)
    _, _, bounds = oracle.table()
    for v in xs.astype(np.float64):
        if np.abs(bounds - v).min() > 1e-12:
            assert oracle.quantize(v) == _exact_code(v, paper)


def test_quantizer_invariants(paper):
    xs = np.linspace(-3.0, 3.0, 60001)
    codes = np.array([oracle.quantize(x) for x in xs])
    assert np.all(np.diff(codes) >= 0)                       # monotone bins
    assert sorted(set(codes.tolist())) == list(range(2 ** int(paper["bits"])))  # 16 levels
    xhat, _, bounds = oracle.table()
    for k in range(16):                                      # representatives reproduce themselves
        assert oracle.quantize(xhat[k]) == k
        assert oracle.dequantize(k) == xhat[k]
    # mirror symmetry away from decision points
    for x in xs:
        if np.abs(bounds - x).min() > 1e-9 and np.abs(bounds + x).min() > 1e-9:
            assert oracle.quantize(-x) == 15 - oracle.quantize(x)
    # reconstruction error of the clipped input is at most half a step
    step = (paper["clip_hi"] - paper["clip_lo"]) / 15
    recon = np.array([oracle.dequantize(c) for c in codes])
    assert np.all(np.abs(np.clip(xs, -2, 2) - recon) <= step / 2 + 1e-12)


def test_quantizer_levels_and_bounds(paper):
    xhat, _, bounds = oracle.table()
    np.testing.assert_allclose(xhat, np.linspace(paper["clip_lo"], paper["clip_hi"], 16), atol=1e-15)
    np.testing.assert_allclose(bounds, (xhat[:-1] + xhat[1:]) / 2, atol=1e-15)
    assert bounds[7] == 0.0
    # a point just either side of each decision point falls in neighbouring bins
    for j, b in enumerate(bounds):
        assert oracle.quantize(b - 1e-9) == j and oracle.quantize(b + 1e-9) == j + 1


def test_quantizer_special_values():
    assert oracle.quantize(0.0) == 8 and oracle.quantize(-0.0) == 8   # the only exact tie: 7.5 -> 8
    assert oracle.quantize(math.inf) == 15 and oracle.quantize(1e30) == 15
    assert oracle.quantize(-math.inf) == 0 and oracle.quantize(-1e30) == 0
    assert oracle.quantize(math.nan) == 0                              # fmax/fmin drop the NaN
    assert [oracle.quantize(v) for v in (-3, -2, -1, -0.5, 0.5, 1, 2, 3)] == [0, 0, 4, 6, 9, 11, 15, 15]


# ----------------------------------------------------------- table (Eq. 9+12)

def test_table_antisymmetry_and_consistency(paper):
    xhat, deriv, _ = oracle.table()
    np.testing.assert_allclose(deriv + deriv[::-1], 1.0, atol=1e-15)
    for k in range(16):
        assert deriv[k] == oracle.gelu_deriv_approx(xhat[k])
    exact = np.array([oracle.gelu_deriv_exact(x) for x in xhat])
    assert np.abs(deriv - exact).max() < 0.075
    # the 16 derivative levels stay in the paper's "roughly (-0.1, 1.1)" band
    assert deriv.min() > paper["deriv_range_lo"] - 0.01 and deriv.max() < paper["deriv_range_hi"] + 0.01
    # the two outermost levels are where the derivative has flattened out
    assert 0 < deriv[0] < 0.01 and 0.99 < deriv[15] < 1


def test_stored_table_matches_oracle(golden_dir):
    """tests/golden/oracle_table.txt is written by tests/golden/make_oracle_table.py,
    which calls only oracle/; it guards against silent drift of the oracle."""
    rows = np.loadtxt(os.path.join(golden_dir, "oracle_table.txt"))
    xhat, deriv, _ = oracle.table()
    np.testing.assert_array_equal(rows[:, 1], xhat)
    np.testing.assert_array_equal(rows[:, 2], deriv)


# ------------------------------------------------------------ array passes --

def _unpack_little_endian(packed: np.ndarray, n: int) -> np.ndarray:
    """Codes as 4-bit fields of a little-endian bit stream: code i = bits 4i..4i+3."""
    bits = np.unpackbits(packed, bitorder="little")[: 4 * n].reshape(n, 4)
    return (bits * np.array([1, 2, 4, 8], dtype=np.uint8)).sum(axis=1).astype(np.uint8)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("n", [0, 1, 2, 3, 16, 17, 1001])
def test_fwd_array_pass(dtype, n):
    x = wl.draw_x(n, "student_t", 2.0, dtype, seed=11 + n)
    y, code, packed, near = oracle.fwd(x, dtype)
    xv = wl.storage_to_f64(x, dtype)
    assert packed.shape == ((n + 1) // 2,)
    for i in range(n):
        assert y[i] == oracle.gelu(xv[i]) and code[i] == oracle.quantize(xv[i])
    np.testing.assert_array_equal(_unpack_little_endian(packed, n), code)
    if n % 2:
        assert packed[-1] >> 4 == 0                         # pad nibble is zero
    assert near.sum() == 0 or n > 0


def test_packing_hand_example():
    """Codes (4, 11, 8) -> bytes 0xB4, 0x08: element 0 in the low nibble."""
    x = np.array([-1.0, 1.0, 0.0], dtype=np.float32)
    _, code, packed, _ = oracle.fwd(x, wl.F32)
    assert code.tolist() == [4, 11, 8]
    assert packed.tolist() == [0xB4, 0x08]


def test_fwd_bwd_on_the_representatives():
    """x = the 16 representatives, dy = 1: codes 0..15, bytes 0x10, 0x32, ..., 0xFE, dx = the table."""
    xhat, deriv, _ = oracle.table()
    x = xhat.astype(np.float32)
    _, code, packed, _ = oracle.fwd(x, wl.F32)
    assert code.tolist() == list(range(16))
    assert packed.tolist() == [0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE]
    dx = oracle.bwd(np.ones(16, np.float32), wl.F32, packed)
    np.testing.assert_array_equal(dx, deriv)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_bwd_is_linear_in_dy_and_reads_the_right_nibble(dtype):
    n = 999
    x = wl.draw_x(n, "normal", 1.0, dtype, seed=3)
    dy = wl.draw_dy(n, 1.0, dtype, seed=4)
    _, code, packed, _ = oracle.fwd(x, dtype)
    _, deriv, _ = oracle.table()
    dx = oracle.bwd(dy, dtype, packed)
    np.testing.assert_array_equal(dx, wl.storage_to_f64(dy, dtype) * deriv[_unpack_little_endian(packed, n)])
    ones = wl.to_storage(np.ones(n), dtype)
    np.testing.assert_array_equal(oracle.bwd(ones, dtype, packed), deriv[code])


def test_near_flag_marks_exactly_the_band():
    _, _, bounds = oracle.table()
    x = np.array([bounds[3] + 5e-7, bounds[3] + 2e-6, 0.0, 1e-7, -1e-5, 1.0], dtype=np.float64)
    x32 = x.astype(np.float32)
    _, _, _, near = oracle.fwd(x32, wl.F32, band=1e-6)
    want = [np.abs(bounds - float(v)).min() <= 1e-6 for v in x32]
    assert near.tolist() == [int(w) for w in want]
    assert near.tolist()[2:5] == [1, 1, 0]


def test_code_histogram_of_a_normal_draw():
    """N(0,1) inputs: the end bins hold P(|x| > 28/15) / 2 = 3.10 % each and the
    two centre bins P(0 < x < 4/15) = 10.51 % each -- a check on the synthetic
    data and on the bin edges at once."""
    n = 400_000
    x = wl.draw_x(n, "normal", 1.0, wl.F32, seed=99)
    _, code, _, _ = oracle.fwd(x, wl.F32)
    h = np.bincount(code, minlength=16) / n
    p_end = ndtr(-28.0 / 15.0)
    p_mid = ndtr(4.0 / 15.0) - 0.5
    assert abs(h[0] - p_end) < 0.002 and abs(h[15] - p_end) < 0.002
    assert abs(h[7] - p_mid) < 0.003 and abs(h[8] - p_mid) < 0.003


def test_saved_bytes_ratio(paper):
    """4-bit codes are 8x smaller than 32-bit activations (Sec. 4.3)."""
    n = 4096
    x = wl.draw_x(n, "normal", 1.0, wl.F32, seed=1)
    _, _, packed, _ = oracle.fwd(x, wl.F32)
    assert x.nbytes / packed.nbytes == paper["memory_ratio_32bit"]
