"""Randomised parity of the headline forward / backward kernels against the
oracle: seeded random sizes (vector path with every leftover count, partial
last waves, the element-wise path through unaligned pointers), value mixes
(bin boundaries, clip limits, zeros, denormals, huge and non-finite values
sprinkled into Gaussian data) and both storage types.  Every case is a full
element-by-element comparison under the usual tolerances.

The number of cases per storage type is S2A_RANDOM_CASES (default 120).
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2503_08154_amd import s2a
from paper_2503_08154_amd import workloads as wl

import gpu_util as gu
import parity

pytestmark = pytest.mark.gpu
CASES = int(os.environ.get("S2A_RANDOM_CASES", "120"))


@pytest.fixture(scope="module", autouse=True)
def _init():
    s2a.qtable_init(16)


def _values(g, n, dtype):
    """Gaussian body of a random width with special values planted at random places."""
    a = g.standard_normal(n) * g.choice([0.3, 1.0, 1.5, 4.0, 30.0])
    k = max(1, n // 8)
    bounds = -2.0 + (np.arange(15) + 0.5) * (4.0 / 15.0)
    planted = np.concatenate([
        bounds, bounds * (1 + 2.0 ** -20), bounds * (1 - 2.0 ** -20),       # decision points and neighbours
        [-2.0, 2.0, -2.0000002, 2.0000002, 0.0, -0.0],                      # clip limits, zeros
        [1e-40, -1e-40, 1e-30, -88.0, -104.0, 90.0, 3e38, -3e38],           # denormal, tiny, large
        [np.inf, -np.inf, np.nan],
    ])
    idx = g.integers(0, n, size=min(k, 4 * planted.shape[0]))
    a[idx] = g.choice(planted, size=idx.shape[0])
    return wl.to_storage(a, dtype)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_random_cases(dtype):
    g = np.random.Generator(np.random.Philox(20250308 + dtype))
    worst_y = worst_dx = 0.0
    in_band = differing = 0
    for case in range(CASES):
        kind = case % 4
        if kind == 0:
            n = int(g.integers(1, 600))                    # less than a few waves
        elif kind == 1:
            n = int(g.integers(600, 40_000))
        elif kind == 2:
            n = int(g.integers(40_000, 400_000))
        else:
            n = int(g.integers(1, 64)) * 512 + int(g.integers(0, 9))   # whole waves plus 0..8 leftovers
        off = (0, 0) if g.random() < 0.6 else (int(g.integers(0, 8)), int(g.integers(0, 4)))
        x = _values(g, n, dtype)
        dy = wl.to_storage(g.standard_normal(n) * g.choice([1e-3, 1.0, 1e3]), dtype)
        y_ref, code_ref, packed_ref, near = oracle.fwd(x, dtype, band=parity.BAND)
        y, packed = gu.run_fwd(x, dtype, offset_elems=off[0], code_offset=off[1])
        finite = np.isfinite(wl.storage_to_f64(x, dtype))
        try:
            rep = parity.check_codes(packed, code_ref, near, n, parity.band_mask(wl.storage_to_f64(x, dtype), parity.GELU_POINTS))
            worst_y = max(worst_y, parity.check_values(y, y_ref, dtype, "y", finite_in=finite))
            dx_ref = oracle.bwd(dy, dtype, packed_ref)
            dx = gu.run_bwd(dy, packed_ref, dtype, offset_elems=off[0], code_offset=off[1])
            worst_dx = max(worst_dx, parity.check_values(dx, dx_ref, dtype, "dx"))
        except AssertionError as e:
            raise AssertionError(f"case {case}: n={n} offsets={off} dtype={dtype}: {e}") from e
        in_band += rep.flagged
        differing += rep.differing
    print(f"\n[random dtype={dtype}] {CASES} cases, in-band {in_band}, differing {differing}, "
          f"worst y {worst_y:.3f}, worst dx {worst_dx:.3f} of the tolerance")
