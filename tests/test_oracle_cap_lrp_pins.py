"""Pins for the Channel-Average-Pooling (Eq. 5) and Low-Rank-Prompt (Eq. 3-4)
parts of the oracle: library pooling / matmul and automatic differentiation."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_08154_amd import workloads as wl


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("r", [1, 2, 8, 16])
def test_cap_is_average_pooling_and_its_adjoint(dtype, r):
    N, C = 13, 16 * r
    x = wl.draw_x(N * C, "normal", 1.0, dtype, seed=r)
    g = wl.draw_dy(N * C // r, 1.0, dtype, seed=r + 1)
    xt = torch.from_numpy(wl.storage_to_f64(x, dtype)).reshape(1, N, C).requires_grad_(True)
    yt = torch.nn.functional.avg_pool1d(xt, kernel_size=r, stride=r)            # pools the last (channel) axis
    np.testing.assert_allclose(oracle.cap_fwd(x, dtype, r), yt.detach().reshape(-1).numpy(), rtol=1e-15, atol=1e-17)
    gt = torch.from_numpy(wl.storage_to_f64(g, dtype)).reshape(1, N, C // r)
    yt.backward(gt)
    dx = oracle.cap_bwd(g, dtype, r)
    np.testing.assert_allclose(dx, xt.grad.reshape(-1).numpy(), rtol=1e-15, atol=0)
    # adjoint identity
    lhs = float(np.dot(oracle.cap_fwd(x, dtype, r), wl.storage_to_f64(g, dtype)))
    rhs = float(np.dot(wl.storage_to_f64(x, dtype), dx))
    assert lhs == pytest.approx(rhs, rel=1e-12)


def test_cap_hand_example():
    x = np.array([1, 2, 3, 4, 10, 20, 30, 40], np.float32)
    np.testing.assert_array_equal(oracle.cap_fwd(x, wl.F32, 4), [2.5, 25.0])
    np.testing.assert_array_equal(oracle.cap_bwd(np.array([8.0, -4.0], np.float32), wl.F32, 4),
                                  [2, 2, 2, 2, -1, -1, -1, -1])


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_lrp_is_matmul_plus_x_and_its_autograd(dtype):
    batch, N, C, r = 3, 7, 12, 5
    g = np.random.default_rng(0)
    A = g.standard_normal((N, r)).astype(np.float32)
    B = g.standard_normal((r, C)).astype(np.float32)
    x = wl.draw_x(batch * N * C, "normal", 1.0, dtype, seed=3)
    dy = wl.draw_dy(batch * N * C, 1.0, dtype, seed=4)
    At = torch.from_numpy(A.astype(np.float64)).requires_grad_(True)
    Bt = torch.from_numpy(B.astype(np.float64)).requires_grad_(True)
    xt = torch.from_numpy(wl.storage_to_f64(x, dtype)).reshape(batch, N, C).requires_grad_(True)
    yt = xt + At @ Bt
    np.testing.assert_allclose(oracle.lrp_fwd(x, dtype, A, B, batch, N, C), yt.detach().reshape(-1).numpy(), rtol=1e-14, atol=1e-15)
    yt.backward(torch.from_numpy(wl.storage_to_f64(dy, dtype)).reshape(batch, N, C))
    dA, dB = oracle.lrp_bwd(dy, dtype, A, B, batch, N, C)
    np.testing.assert_allclose(dA, At.grad.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dB, Bt.grad.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_array_equal(xt.grad.reshape(-1).numpy(), wl.storage_to_f64(dy, dtype))   # dL/dx = dL/dy


def test_lrp_starts_as_the_identity():
    """A is initialised to 0, so the activation is unchanged at the start of fine-tuning."""
    batch, N, C, r = 2, 5, 8, 3
    A = np.zeros((N, r), np.float32)
    B = np.random.default_rng(1).standard_normal((r, C)).astype(np.float32)
    x = wl.draw_x(batch * N * C, "normal", 1.0, wl.F32, seed=5)
    np.testing.assert_array_equal(oracle.lrp_fwd(x, wl.F32, A, B, batch, N, C), x.astype(np.float64))
