"""Pins for the 2-D pooling oracle (abstract of the paper: pooling is a sliding window sum).  Each
test fixes it to something other than itself; none needs a GPU."""
import itertools

import numpy as np
import pytest

from paper_2310_05218_amd import inputs

# (N, C, H, W, R, S, stride, pad)
CASES = [
    (1, 1, 4, 4, 2, 2, 2, 0),
    (2, 3, 7, 9, 3, 3, 2, 1),
    (1, 2, 8, 6, 2, 3, 1, 1),
    (1, 1, 9, 9, 3, 3, 1, 0),
    (1, 2, 11, 5, 5, 2, 3, 1),
    (1, 1, 6, 6, 4, 4, 2, 2),
    (1, 1, 5, 7, 1, 1, 2, 0),
]


def scatter_pool_sum(x, R, S, stride, pad):
    """Window sums and in-plane counts by scattering every INPUT pixel into the outputs whose window
    holds it (the oracle gathers per output).  Python integers: exact."""
    N, C, H, W = x.shape
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    tot = np.zeros((N, C, Ho, Wo), dtype=object)
    tot[...] = 0
    cnt = np.zeros((Ho, Wo), dtype=np.int64)
    for h, v in itertools.product(range(H), range(W)):
        for r, s in itertools.product(range(R), range(S)):
            ti, tj = h + pad - r, v + pad - s
            if ti < 0 or tj < 0 or ti % stride or tj % stride:
                continue
            i, j = ti // stride, tj // stride
            if i >= Ho or j >= Wo:
                continue
            cnt[i, j] += 1
            for n, c in itertools.product(range(N), range(C)):
                tot[n, c, i, j] += int(x[n, c, h, v])
    return tot.astype(np.int64), cnt


@pytest.mark.parametrize("case", CASES)
def test_average_matches_scatter_brute_force(oracle, case):
    N, C, H, W, R, S, stride, pad = case
    x = inputs.small_ints_f32((N, C, H, W), 900 + H * W + R)
    y, d = oracle.pool2d(x, R, S, stride, pad, oracle.POOL_AVG)
    tot, _ = scatter_pool_sum(x, R, S, stride, pad)
    assert y.shape == tot.shape
    assert np.array_equal(y * (R * S), tot.astype(np.float64))          # small integers: exact
    totabs, _ = scatter_pool_sum(np.abs(x), R, S, stride, pad)
    assert np.array_equal(d * (R * S), totabs.astype(np.float64))


@pytest.mark.parametrize("case", CASES)
def test_maximum_matches_slices_of_a_minus_infinity_padded_copy(oracle, case):
    N, C, H, W, R, S, stride, pad = case
    x = inputs.normal_f32((N, C, H, W), 950 + H + 3 * W + S)
    y, d = oracle.pool2d(x, R, S, stride, pad, oracle.POOL_MAX)
    xp = np.full((N, C, H + 2 * pad, W + 2 * pad), -np.inf, np.float64)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    Ho, Wo = y.shape[2:]
    for i, j in itertools.product(range(Ho), range(Wo)):
        ref = xp[:, :, i * stride:i * stride + R, j * stride:j * stride + S].max(axis=(2, 3))
        assert np.array_equal(y[:, :, i, j], ref)
    assert np.array_equal(d, np.abs(y))


def test_closed_forms(oracle):
    # a constant plane: the average is c * (positions inside) / (R*S); the maximum is c everywhere,
    # also for a negative c next to the padding (padding must not win with its zero)
    c = np.full((1, 1, 6, 7), -2.5, np.float32)
    ya, _ = oracle.pool2d(c, 3, 3, 1, 1, oracle.POOL_AVG)
    _, cnt = scatter_pool_sum(np.ones((1, 1, 6, 7)), 3, 3, 1, 1)
    assert cnt[0, 0] == 4 and cnt[0, 3] == 6 and cnt[2, 3] == 9
    assert np.array_equal(ya[0, 0], -2.5 * cnt / 9.0)
    ym, _ = oracle.pool2d(c, 3, 3, 1, 1, oracle.POOL_MAX)
    assert np.array_equal(ym, np.full((1, 1, 6, 7), -2.5))
    # x[h, v] = 10 h + v grows along both axes: the maximum sits at the window's last in-plane corner
    H, W, R, S, st, pad = 9, 8, 3, 2, 2, 1
    x = (10.0 * np.arange(H)[:, None] + np.arange(W)[None, :]).astype(np.float32)[None, None]
    y, _ = oracle.pool2d(x, R, S, st, pad, oracle.POOL_MAX)
    Ho, Wo = (H + 2 * pad - R) // st + 1, (W + 2 * pad - S) // st + 1
    ref = np.array([[10.0 * min(i * st - pad + R - 1, H - 1) + min(j * st - pad + S - 1, W - 1)
                     for j in range(Wo)] for i in range(Ho)])
    assert np.array_equal(y[0, 0], ref)
    y, _ = oracle.pool2d(-x, R, S, st, pad, oracle.POOL_MAX)      # decreasing: the first in-plane corner
    ref = np.array([[-(10.0 * max(i * st - pad, 0) + max(j * st - pad, 0)) for j in range(Wo)] for i in range(Ho)])
    assert np.array_equal(y[0, 0], ref)


def test_special_cases_reduce_to_the_other_entry_points(oracle):
    x = inputs.normal_f32((2, 3, 12, 14), 960)
    # one row, window one row high: the 1-D pooling of each row
    x1 = inputs.normal_f32((5, 40), 961)
    for mode in (oracle.POOL_AVG, oracle.POOL_MAX):
        y2, d2 = oracle.pool2d(x1[None, :, None, :], 1, 8, 3, 0, mode)
        y1, d1 = oracle.pool1d(x1, 8, 3, mode)
        assert np.array_equal(y2[0, :, 0, :], y1) and np.array_equal(d2[0, :, 0, :], d1)
    # the average is the depthwise convolution with the constant filter 1/(R*S) (a power of two here,
    # so the products are exact and the sums agree to rounding order)
    w = np.full((3, 1, 4, 2), 1.0 / 8.0, np.float32)
    ya, da = oracle.pool2d(x, 4, 2, 2, 1, oracle.POOL_AVG)
    yc, dc = oracle.conv2d_depthwise(x, w, 2, 1)
    assert np.max(np.abs(ya - yc)) < 1e-14 and np.max(np.abs(da - dc)) < 1e-14
    # a window that covers the whole plane: global average and maximum
    yg, _ = oracle.pool2d(x, 12, 14, 1, 0, oracle.POOL_AVG)
    assert np.allclose(yg[:, :, 0, 0], x.astype(np.float64).mean(axis=(2, 3)), rtol=0, atol=1e-15)
    yg, _ = oracle.pool2d(x, 12, 14, 1, 0, oracle.POOL_MAX)
    assert np.array_equal(yg[:, :, 0, 0], x.max(axis=(2, 3)).astype(np.float64))
    # window 1, stride 1: identity for both modes
    for mode in (oracle.POOL_AVG, oracle.POOL_MAX):
        assert np.array_equal(oracle.pool2d(x, 1, 1, 1, 0, mode)[0], x.astype(np.float64))


def test_library_routine_in_float64(oracle):
    import torch
    import torch.nn.functional as F

    x = inputs.normal_f32((2, 8, 56, 56), 970)
    t = torch.from_numpy(x.astype(np.float64))
    for R, st, pad in [(2, 2, 0), (3, 2, 1), (3, 1, 1), (5, 1, 2)]:
        ya, _ = oracle.pool2d(x, R, R, st, pad, oracle.POOL_AVG)
        ref = F.avg_pool2d(t, R, st, pad, count_include_pad=True).numpy()
        assert np.max(np.abs(ya - ref)) < 1e-14
        ym, _ = oracle.pool2d(x, R, R, st, pad, oracle.POOL_MAX)
        assert np.array_equal(ym, F.max_pool2d(t, R, st, pad).numpy())


def test_arguments(oracle):
    x = np.zeros((1, 1, 4, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.pool2d(x, 5, 5, 1, 0, oracle.POOL_AVG)          # window larger than the plane
    with pytest.raises(ValueError):
        oracle.pool2d(x, 2, 2, 1, 3, oracle.POOL_MAX)          # windows that lie wholly in the padding
    with pytest.raises(ValueError):
        oracle.pool2d(x, 2, 2, 1, 0, 7)
