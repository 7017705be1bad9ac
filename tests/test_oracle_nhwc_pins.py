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


def test_hand_worked_channel_last_float_example(oracle):
    # the same 1 x 2 image with 3 channels in fp32; dilation 1 and a bias + rectifier
    x = np.array([[[[1, 2, 3], [4, 5, 6]]]], np.float32)
    w = np.array([[[[1, 10, 100]]], [[[-1, 0, 2]]]], np.float32)
    y, d = oracle.conv2d_nhwc(x, w, 1, 0)
    assert y[0, 0].tolist() == [[321.0, 5.0], [654.0, 8.0]] and d[0, 0].tolist() == [[321.0, 7.0], [654.0, 16.0]]
    y, d = oracle.conv2d_nhwc(x, w, 1, 0, 1, np.array([-400.0, 1.5], np.float32), True)
    assert y[0, 0].tolist() == [[0.0, 6.5], [254.0, 9.5]] and d[0, 0].tolist() == [[721.0, 8.5], [1054.0, 17.5]]
    # a 1 x 2 filter at dilation 2 over a row of four pixels: taps two pixels apart, channels innermost
    x4 = np.arange(1, 13, dtype=np.float32).reshape(1, 1, 4, 3)            # pixels (1,2,3) (4,5,6) (7,8,9) (10,11,12)
    w2 = np.array([[[[1, 0, 0], [0, 0, 10]]]], np.float32)                 # x[., j, c0] + 10 * x[., j + 2, c2]
    y, _ = oracle.conv2d_nhwc(x4, w2, 1, 0, 2)
    assert y.tolist() == [[[[91.0], [124.0]]]]
    # bf16 bit patterns: 0x3F80 = 1, 0x4000 = 2, 0xC040 = -3; widened exactly, summed in fp64, not rounded
    xb = np.array([[[[0x3F80, 0x4000]]]], np.uint16)
    wb = np.array([[[[0x4000, 0xC040]]]], np.uint16)
    y, d = oracle.conv2d_bf16_nhwc(xb, wb, 1, 0)
    assert y.tolist() == [[[[-4.0]]]] and d.tolist() == [[[[8.0]]]]
    # half-precision bit patterns: 0x3C00 = 1, 0x4000 = 2, 0xC200 = -3, 0x3800 = 0.5, 0x0001 = 2^-24 (the smallest
    # denormal): 1 * 2 + 2 * (-3) = -4 with magnitude 8; 0.5 * 2^-24 = 2^-25 is kept (fp64 sums, no rounding)
    xh = np.array([[[[0x3C00, 0x4000]]]], np.uint16)
    wh = np.array([[[[0x4000, 0xC200]]]], np.uint16)
    y, d = oracle.conv2d_f16_nhwc(xh, wh, 1, 0)
    assert y.tolist() == [[[[-4.0]]]] and d.tolist() == [[[[8.0]]]]
    y, d = oracle.conv2d_f16_nhwc(np.array([[[[0x3800]]]], np.uint16), np.array([[[[0x0001]]]], np.uint16), 1, 0)
    assert y.tolist() == [[[[2.0 ** -25]]]] and d.tolist() == [[[[2.0 ** -25]]]]
    assert oracle.f16_to_f32(np.array([0x7BFF, 0xFBFF, 0x0400], np.uint16)).tolist() == [65504.0, -65504.0, 2.0 ** -14]


def test_channel_last_float_brute_force(oracle):
    rng = np.random.default_rng(5151)
    N, H, W, Ci, Co, R, S, stride, pad, dil = 2, 9, 8, 3, 4, 3, 2, 2, 2, 2
    x = rng.integers(-8, 9, size=(N, H, W, Ci)).astype(np.float32)          # small integers: every sum is exact
    w = rng.integers(-8, 9, size=(Co, R, S, Ci)).astype(np.float32)
    b = rng.integers(-20, 21, size=Co).astype(np.float32)
    y, d = oracle.conv2d_nhwc(x, w, stride, pad, dil, b, True)
    Ho, Wo = (H + 2 * pad - (dil * (R - 1) + 1)) // stride + 1, (W + 2 * pad - (dil * (S - 1) + 1)) // stride + 1
    assert y.shape == (N, Ho, Wo, Co)
    ref = np.zeros((N, Ho, Wo, Co), np.int64)
    mag = np.zeros((N, Ho, Wo, Co), np.int64)
    for n in range(N):
        for i in range(Ho):
            for j in range(Wo):
                for r in range(R):
                    for s in range(S):
                        h, v = i * stride + r * dil - pad, j * stride + s * dil - pad
                        if 0 <= h < H and 0 <= v < W:
                            ref[n, i, j] += w[:, r, s, :].astype(np.int64) @ x[n, h, v].astype(np.int64)
                            mag[n, i, j] += np.abs(w[:, r, s, :]).astype(np.int64) @ np.abs(x[n, h, v]).astype(np.int64)
    ref += b.astype(np.int64)
    mag += np.abs(b).astype(np.int64)
    assert np.array_equal(y, np.maximum(ref, 0)) and np.array_equal(d, mag)
    # the same integers as half-precision bit patterns (exact in 11 bits): the 16-bit entry points' oracle is the same sum
    yh, dh = oracle.conv2d_f16_nhwc(x.astype(np.float16).view(np.uint16), w.astype(np.float16).view(np.uint16), stride, pad, dil, b, True)
    assert np.array_equal(yh, y) and np.array_equal(dh, d)
