"""Pins for the bias + rectifier step of the CPU oracle (fp32 convolution followed by y = act(y + bias[co])).
The paper gives no formula (section 1 names the layers these kernels serve); the definition is the usual one.
Each test fixes it to something other than itself; none needs a GPU."""
import numpy as np
import pytest


def test_hand_worked_example(oracle):
    # one 1x1 filter per output channel over one input channel: y[co] = w[co] * x + bias[co]
    x = np.array([[[[1.0, -2.0, 0.5, 4.0]]]], np.float32)                 # [1,1,1,4]
    w = np.array([2.0, -1.0], np.float32).reshape(2, 1, 1, 1)
    bias = np.array([0.5, -1.0], np.float32)
    y, d = oracle.conv2d_bias_relu(x, w, bias, 1, 0, False)
    assert y.tolist() == [[[[2.5, -3.5, 1.5, 8.5]], [[-2.0, 1.0, -1.5, -5.0]]]]
    # the bias is one more term of the magnitude sum
    assert d.tolist() == [[[[2.5, 4.5, 1.5, 8.5]], [[2.0, 3.0, 1.5, 5.0]]]]
    y, _ = oracle.conv2d_bias_relu(x, w, bias, 1, 0, True)
    assert y.tolist() == [[[[2.5, 0.0, 1.5, 8.5]], [[0.0, 1.0, 0.0, 0.0]]]]
    # the rectifier acts after the bias: w*x = -2 with bias +3 is 1, not 3
    y, _ = oracle.conv2d_bias_relu(np.array([[[[1.0]]]], np.float32), np.array([[[[-2.0]]]], np.float32),
                                   np.array([3.0], np.float32), 1, 0, True)
    assert y.item() == 1.0


@pytest.mark.parametrize("relu", [False, True])
def test_against_torch_conv2d_with_bias(oracle, relu):
    import torch

    rng = np.random.default_rng(777 + relu)
    x = rng.standard_normal((2, 3, 9, 8)).astype(np.float32)
    w = rng.standard_normal((5, 3, 3, 2)).astype(np.float32)
    bias = rng.standard_normal(5).astype(np.float32) * 3
    y, d = oracle.conv2d_bias_relu(x, w, bias, 2, 1, relu)
    t = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                   torch.from_numpy(bias).double(), stride=2, padding=1)
    if relu:
        t = torch.relu(t)
    assert y.shape == tuple(t.shape)
    assert np.max(np.abs(y - t.numpy())) <= 1e-12
    assert relu or np.all(d >= np.abs(y) - 1e-12)
    if relu:
        assert y.min() == 0.0 and (y == 0).mean() > 0.2


def test_no_bias_and_no_rectifier_is_the_plain_convolution(oracle):
    rng = np.random.default_rng(778)
    x = rng.standard_normal((1, 2, 6, 6)).astype(np.float32)
    w = rng.standard_normal((3, 2, 3, 3)).astype(np.float32)
    y0, d0 = oracle.conv2d(x, w, 1, 1)
    y1, d1 = oracle.conv2d_bias_relu(x, w, None, 1, 1, False)
    assert np.array_equal(y0, y1) and np.array_equal(d0, d1)
    y2, _ = oracle.conv2d_bias_relu(x, w, None, 1, 1, True)
    assert np.array_equal(y2, np.maximum(y0, 0.0))
    with pytest.raises(ValueError):
        oracle.conv2d_bias_relu(x, w, np.zeros(2, np.float32), 1, 1, False)


def test_depthwise_variant_hand_worked(oracle):
    # two channels, each its own 1x1 filter and bias: y[c] = act(w[c] * x[c] + bias[c])
    x = np.array([[[[1.0, -2.0]], [[3.0, -4.0]]]], np.float32)            # [1,2,1,2]
    w = np.array([2.0, -1.0], np.float32).reshape(2, 1, 1, 1)
    bias = np.array([0.5, 2.0], np.float32)
    y, d = oracle.conv2d_depthwise_bias_relu(x, w, bias, 1, 0, False)
    assert y.tolist() == [[[[2.5, -3.5]], [[-1.0, 6.0]]]]
    assert d.tolist() == [[[[2.5, 4.5]], [[5.0, 6.0]]]]
    y, _ = oracle.conv2d_depthwise_bias_relu(x, w, bias, 1, 0, True)
    assert y.tolist() == [[[[2.5, 0.0]], [[0.0, 6.0]]]]
