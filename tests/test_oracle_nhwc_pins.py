"""Pins for the channel-last entry points of the CPU oracle: they permute axes around the separately pinned
channel-first functions, so what needs pinning is the permutation itself -- a hand-worked example in which every
axis has a different extent and every element a different weight, and a brute-force loop written directly on the
channel-last arrays.  None needs a GPU."""
import numpy as np


def test_hand_worked_channel_last_example(oracle):
    # one image of 1 x 2 pixels with 3 channels, two 1 x 1 filters: y[pixel, co] = sum_ci x[pixel, ci] * w[co, ci]
    x = np.array([[[[1, 2, 3], [4, 5, 6]]]], np.int8)                      # [N=1, H=1, W=2, C_in=3]
    w = np.array([[[[1, 10, 100]]], [[[-1, 0, 2]]]], np.int8)              # [C_out=2, R=1, S=1, C_in=3]
    y = oracle.conv2d_s8_nhwc(x, w, 1, 0)
    assert y.shape == (1, 1, 2, 2)
    assert y[0, 0].tolist() == [[321, 5], [654, 8]]
    # a 1 x 2 filter over the two pixels: taps along W, channels innermost
    w2 = np.array([[[[1, 0, 0], [0, 0, 10]]]], np.int8)                    # [1, 1, 2, 3]: x[.,0,c0] + 10 * x[.,1,c2]
    assert oracle.conv2d_s8_nhwc(x, w2, 1, 0).tolist() == [[[[61]]]]
    # requantised: (321, 5, 654, 8) + bias (0, 100) times scale (0.25, 0.5)
    q = oracle.conv2d_s8_nhwc_requant(x, w, np.array([0, 100], np.int32), np.array([0.25, 0.5], np.float32), 1, 0, False)
    assert q[0, 0].tolist() == [[80, 52], [127, 54]]


def test_channel_last_brute_force(oracle):
    rng = np.random.default_rng(5150)
    N, H, W, Ci, Co, R, S, stride, pad = 2, 6, 5, 3, 4, 3, 2, 2, 1
    x = rng.integers(-128, 128, size=(N, H, W, Ci)).astype(np.int8)
    w = rng.integers(-128, 128, size=(Co, R, S, Ci)).astype(np.int8)
    y = oracle.conv2d_s8_nhwc(x, w, stride, pad)
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    assert y.shape == (N, Ho, Wo, Co)
    ref = np.zeros((N, Ho, Wo, Co), np.int64)
    for n in range(N):
        for i in range(Ho):
            for j in range(Wo):
                for r in range(R):
                    for s in range(S):
                        h, v = i * stride + r - pad, j * stride + s - pad
                        if 0 <= h < H and 0 <= v < W:
                            ref[n, i, j] += w[:, r, s, :].astype(np.int64) @ x[n, h, v].astype(np.int64)
    assert np.array_equal(y, ref)
