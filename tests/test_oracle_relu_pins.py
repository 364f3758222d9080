"""Pins for the ReLU part of the oracle (Sec. 3.2, "ReLU layer"): library ReLU,
numpy bit packing, automatic differentiation."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_08154_amd import workloads as wl


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 63, 64, 65, 1000])
def test_forward_is_library_relu_and_mask_is_x_gt_0(dtype, n):
    x = wl.draw_x(n, "normal", 1.0, dtype, seed=50 + n)
    if n > 3:
        x[:3] = wl.to_storage(np.array([0.0, -0.0, 1e-30]), dtype)
    xv = wl.storage_to_f64(x, dtype)
    y, bit, packed = oracle.relu_fwd(x, dtype)
    np.testing.assert_array_equal(y, torch.relu(torch.from_numpy(xv)).numpy())
    np.testing.assert_array_equal(bit, (xv > 0).astype(np.uint8))
    np.testing.assert_array_equal(packed, np.packbits(xv > 0, bitorder="little"))
    assert packed.shape == ((n + 7) // 8,)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_backward_is_autograd_of_library_relu(dtype):
    n = 777
    x = wl.draw_x(n, "normal", 1.0, dtype, seed=1)
    x[5] = 0                                             # derivative 0 at the kink
    dy = wl.draw_dy(n, 1.0, dtype, seed=2)
    _, bit, packed = oracle.relu_fwd(x, dtype)
    xt = torch.from_numpy(wl.storage_to_f64(x, dtype)).requires_grad_(True)
    torch.relu(xt).backward(torch.from_numpy(wl.storage_to_f64(dy, dtype)))
    np.testing.assert_array_equal(oracle.relu_bwd(dy, dtype, packed), xt.grad.numpy())
    ones = wl.to_storage(np.ones(n), dtype)
    np.testing.assert_array_equal(oracle.relu_bwd(ones, dtype, packed), bit.astype(np.float64))


def test_special_values_and_size_ratio():
    x = np.array([np.nan, np.inf, -np.inf, 3.4e38, -1e-45, 1e-45, 0.0, -0.0, 2.0], np.float32)
    y, bit, packed = oracle.relu_fwd(x, wl.F32)
    assert bit.tolist() == [0, 1, 0, 1, 0, 1, 0, 0, 1]
    assert y[0] == 0.0 and y[1] == np.inf and y[2] == 0.0 and y[5] == float(np.float32(1e-45))
    assert packed.tolist() == [0b00101010, 0b1]
    big = np.zeros(4096, np.float32)
    assert big.nbytes / oracle.relu_fwd(big, wl.F32)[2].nbytes == 32   # 32-bit -> 1-bit
