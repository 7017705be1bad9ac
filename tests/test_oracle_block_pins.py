"""Pins for the depthwise-separable block of the CPU oracle (depthwise 3x3 + bias + rectifier, then pointwise 1x1 +
bias + rectifier): hand-worked numbers, the composition of the separately pinned entry points, torch in double
precision.  None needs a GPU."""
import numpy as np


def test_hand_worked_block(oracle):
    # one 3 x 3 plane per channel, two channels; depthwise filters that pick the centre tap and the left neighbour
    x = np.zeros((1, 2, 3, 3), np.float32)
    x[0, 0] = [[1, 2, 3], [4, 5, 6], [7, 8, 9]]
    x[0, 1] = [[-1, -2, -3], [-4, -5, -6], [-7, -8, -9]]
    w_dw = np.zeros((2, 1, 3, 3), np.float32)
    w_dw[0, 0, 1, 1] = 2.0                      # t0 = 2 * x0
    w_dw[1, 0, 1, 0] = 1.0                      # t1[i, j] = x1[i, j - 1] (zero in the first column)
    b_dw = np.array([0.0, 3.0], np.float32)     # t1 += 3, then the rectifier
    w_pw = np.array([[1.0, 10.0], [-1.0, 0.5]], np.float32).reshape(2, 2, 1, 1)
    b_pw = np.array([0.25, 0.0], np.float32)
    y, d = oracle.dw_pw_block(x, w_dw, b_dw, w_pw, b_pw, True, False)
    t0 = 2.0 * x[0, 0].astype(np.float64)
    t1 = np.maximum(np.array([[3, 2, 1], [3, -1, -2], [3, -4, -5]], np.float64), 0.0)
    assert np.array_equal(y[0, 0], t0 + 10.0 * t1 + 0.25)
    assert np.array_equal(y[0, 1], -t0 + 0.5 * t1)
    # magnitude: |w_pw| times (sum |x * w_dw| + |b_dw|), plus |b_pw|
    d1 = np.abs(np.array([[0, 1, 2], [0, 4, 5], [0, 7, 8]], np.float64)) + 3.0
    assert np.array_equal(d[0, 0], t0 + 10.0 * d1 + 0.25)
    y2, _ = oracle.dw_pw_block(x, w_dw, b_dw, w_pw, b_pw, True, True)
    assert np.array_equal(y2, np.maximum(y, 0.0))
    # without the first rectifier the negative depthwise outputs pass through
    y3, _ = oracle.dw_pw_block(x, w_dw, b_dw, w_pw, b_pw, False, False)
    t1n = np.array([[3, 2, 1], [3, -1, -2], [3, -4, -5]], np.float64)
    assert np.array_equal(y3[0, 0], t0 + 10.0 * t1n + 0.25)


def test_block_is_the_composition_of_the_pinned_entry_points_and_matches_torch(oracle):
    import torch

    rng = np.random.default_rng(7100)
    x = rng.standard_normal((2, 5, 9, 7)).astype(np.float32)
    w_dw = rng.standard_normal((5, 1, 3, 3)).astype(np.float32)
    b_dw = rng.standard_normal(5).astype(np.float32)
    w_pw = rng.standard_normal((4, 5, 1, 1)).astype(np.float32)
    b_pw = rng.standard_normal(4).astype(np.float32)
    y, d = oracle.dw_pw_block(x, w_dw, b_dw, w_pw, b_pw, True, True)
    # second stage through the oracle's own convolution on the (fp32-rounded) intermediate: agreement to fp32 rounding
    t, _ = oracle.conv2d_depthwise_bias_relu(x, w_dw, b_dw, 1, 1, True)
    y2, _ = oracle.conv2d_bias_relu(t.astype(np.float32), w_pw, b_pw, 1, 0, True)
    assert np.max(np.abs(y - y2) / d) < 1e-6
    td = torch.relu(torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w_dw).double(),
                                               torch.from_numpy(b_dw).double(), padding=1, groups=5))
    ty = torch.relu(torch.nn.functional.conv2d(td, torch.from_numpy(w_pw).double(), torch.from_numpy(b_pw).double()))
    assert np.max(np.abs(y - ty.numpy())) < 1e-12
    assert np.all(d >= np.abs(y) - 1e-12)
