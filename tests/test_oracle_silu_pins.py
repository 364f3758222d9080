"""Pins for the SiLU variant of the oracle: a library SiLU and its autograd, and
exact agreement with the (pinned) GELU functions under x -> x / 1.702."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_08154_amd import workloads as wl

A = 1.702


def test_silu_is_library_silu():
    xs = torch.linspace(-40.0, 40.0, 4001, dtype=torch.float64)
    got = np.array([oracle.silu(float(x)) for x in xs])
    np.testing.assert_allclose(got, torch.nn.functional.silu(xs).numpy(), rtol=1e-13, atol=1e-300)


def test_substitution_maps_silu_onto_the_gelu_scheme():
    xs = np.linspace(-9.0, 9.0, 3601)
    for x in xs:
        assert oracle.silu(x) == pytest.approx(A * oracle.gelu(x / A), rel=1e-14, abs=1e-300)
        assert oracle.silu_deriv_approx(x) == pytest.approx(oracle.gelu_deriv_approx(x / A), abs=2e-15)
    _, _, bounds = oracle.table()
    for x in xs:
        if np.abs(bounds - x / A).min() > 1e-9:
            assert oracle.silu_quantize(x) == oracle.quantize(x / A)
    for k in range(16):
        assert oracle.silu_dequantize(k) == pytest.approx(A * oracle.dequantize(k), rel=1e-15, abs=1e-15)
        assert oracle.silu_quantize(oracle.silu_dequantize(k)) == k
    assert oracle.silu_dequantize(0) == -2 * A and oracle.silu_dequantize(15) == pytest.approx(2 * A, rel=1e-15)


def test_fit_tracks_the_true_silu_derivative_on_the_clip_range():
    xs = torch.linspace(-2 * A, 2 * A, 2001, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.silu(xs).sum().backward()
    ap = np.array([oracle.silu_deriv_approx(float(x)) for x in xs.detach()])
    assert np.abs(ap - xs.grad.numpy()).max() < 0.075


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_array_passes(dtype):
    n = 1001
    x = wl.draw_x(n, "student_t", 2.0, dtype, seed=8)
    dy = wl.draw_dy(n, 1.0, dtype, seed=9)
    y, code, packed, near = oracle.silu_fwd(x, dtype)
    xv = wl.storage_to_f64(x, dtype)
    for i in range(n):
        assert y[i] == oracle.silu(xv[i]) and code[i] == oracle.silu_quantize(xv[i])
    bits = np.unpackbits(packed, bitorder="little")[:4 * n].reshape(n, 4)
    np.testing.assert_array_equal((bits * np.array([1, 2, 4, 8], np.uint8)).sum(axis=1), code)
    dx = oracle.silu_bwd(dy, dtype, packed)
    levels = np.array([oracle.silu_deriv_approx(oracle.silu_dequantize(k)) for k in range(16)])
    np.testing.assert_array_equal(dx, wl.storage_to_f64(dy, dtype) * levels[code])


def test_near_flag_marks_exactly_the_band():
    """The decision points of the SiLU quantizer are -3.404 + (j + 1/2) * 6.808/15 (the GELU
    points times 1.702).  Hand-placed inputs either side of several of them, judged in exact
    rational arithmetic on the stored fp32 values."""
    from fractions import Fraction

    clip, band = Fraction("3.404"), Fraction(1, 10 ** 6)
    step = 2 * clip / 15
    pts = [-clip + Fraction(2 * j + 1, 2) * step for j in range(15)]
    vals, placed = [], []
    for j in (0, 4, 7, 9, 14):
        for off, flag in ((5e-7, 1), (-5e-7, 1), (2e-6, 0), (-2e-6, 0), (0.05, 0)):
            vals.append(float(pts[j]) + off)
            placed.append(flag)
    vals += [0.0, 1e-7, -1e-5, 50.0, -50.0, 3.404, -3.404]
    placed += [1, 1, 0, 0, 0, 0, 0]
    x = np.array(vals, np.float32)
    _, _, _, near = oracle.silu_fwd(x, wl.F32, band=1e-6)
    exact = [int(min(abs(Fraction(float(v)) - p) for p in pts) <= band) for v in x]
    assert near.tolist() == exact == placed
    # scaled GELU points: a value is in the SiLU band exactly when value / 1.702 is in the
    # GELU band of width band / 1.702 (the fixed-range flag has its own pin)
    g = np.random.default_rng(5)
    xs = g.uniform(-4.0, 4.0, 20000).astype(np.float32)
    _, _, _, near_s = oracle.silu_fwd(xs, wl.F32, band=3e-3)
    _, _, bounds = oracle.table()
    dist = np.abs(xs.astype(np.float64)[:, None] - A * bounds[None, :]).min(axis=1)
    sure = np.abs(dist - 3e-3) > 1e-9
    np.testing.assert_array_equal(near_s[sure], (dist <= 3e-3)[sure].astype(np.uint8))
    assert 100 < near_s.sum() < 2000
