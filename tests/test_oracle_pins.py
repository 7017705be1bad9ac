"""Pins for the CPU oracle: each test fixes the oracle to something other than
itself (hand-worked values, closed forms, brute force in a different
formulation, invariants, library routines).  None of them needs a GPU.
"""
import itertools
import json
import os

import numpy as np
import pytest

from paper_2310_05218_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")


# ---------------------------------------------------------------------------
# An independent formulation: loop over INPUT pixels and scatter each product
# into the outputs it belongs to (the oracle gathers per output).  Pure Python
# integers, so the result is exact.
# ---------------------------------------------------------------------------

def scatter_conv2d(x, w, stride, pad):
    N, C_in, H, W = x.shape
    C_out, _, R, S = w.shape
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - S) // stride + 1
    y = [[[[0] * Wo for _ in range(Ho)] for _ in range(C_out)] for _ in range(N)]
    for n, ci, h, v in itertools.product(range(N), range(C_in), range(H), range(W)):
        xv = int(x[n, ci, h, v])
        for r, s in itertools.product(range(R), range(S)):
            ti, tj = h + pad - r, v + pad - s      # = i*stride, j*stride
            if ti < 0 or tj < 0 or ti % stride or tj % stride:
                continue
            i, j = ti // stride, tj // stride
            if i >= Ho or j >= Wo:
                continue
            for co in range(C_out):
                y[n][co][i][j] += xv * int(w[co, ci, r, s])
    return np.array(y, dtype=np.int64).reshape(N, C_out, Ho, Wo)


CASES_2D = [
    # N, C_in, C_out, H, W, R, S, stride, pad
    (1, 1, 1, 5, 5, 3, 3, 1, 0),
    (2, 3, 2, 7, 6, 3, 3, 1, 1),
    (1, 2, 3, 7, 7, 3, 2, 2, 1),
    (2, 1, 2, 6, 7, 2, 3, 2, 2),
    (1, 3, 1, 4, 5, 1, 1, 1, 0),
    (1, 2, 2, 7, 7, 3, 3, 2, 0),
    (1, 1, 1, 3, 3, 3, 3, 1, 2),
    (1, 2, 1, 5, 4, 5, 4, 1, 0),
]


@pytest.mark.parametrize("case", CASES_2D)
def test_conv2d_matches_scatter_brute_force(oracle, case):
    N, C_in, C_out, H, W, R, S, stride, pad = case
    x = inputs.small_ints_f32((N, C_in, H, W), 11)
    w = inputs.small_ints_f32((C_out, C_in, R, S), 12)
    y, d = oracle.conv2d(x, w, stride, pad)
    ref = scatter_conv2d(x, w, stride, pad)
    assert y.shape == ref.shape
    assert np.array_equal(y, ref.astype(np.float64))
    assert np.array_equal(d, scatter_conv2d(np.abs(x), np.abs(w), stride, pad).astype(np.float64))


@pytest.mark.parametrize("case", CASES_2D)
def test_conv2d_s8_matches_scatter_brute_force(oracle, case):
    N, C_in, C_out, H, W, R, S, stride, pad = case
    x = inputs.uniform_s8((N, C_in, H, W), 21)
    w = inputs.uniform_s8((C_out, C_in, R, S), 22)
    y = oracle.conv2d_s8(x, w, stride, pad)
    assert y.dtype == np.int32
    assert np.array_equal(y.astype(np.int64), scatter_conv2d(x, w, stride, pad))


@pytest.mark.parametrize("case", [(2, 3, 7, 6, 3, 3, 1, 1), (1, 2, 7, 7, 3, 2, 2, 1), (1, 4, 5, 5, 5, 5, 1, 2)])
def test_depthwise_matches_scatter_brute_force(oracle, case):
    N, C, H, W, R, S, stride, pad = case
    x = inputs.small_ints_f32((N, C, H, W), 31)
    w = inputs.small_ints_f32((C, 1, R, S), 32)
    y, _ = oracle.conv2d_depthwise(x, w, stride, pad)
    for c in range(C):
        ref = scatter_conv2d(x[:, c:c + 1], w[c:c + 1], stride, pad)
        assert np.array_equal(y[:, c:c + 1], ref.astype(np.float64))


@pytest.mark.parametrize("k,stride,pad", [(1, 1, 0), (3, 1, 0), (3, 2, 1), (4, 3, 2), (9, 1, 0), (5, 1, 4)])
def test_conv1d_matches_scatter_brute_force(oracle, k, stride, pad):
    x = inputs.small_ints_f32((3, 17), 41)
    w = inputs.small_ints_f32((k,), 42)
    y, _ = oracle.conv1d(x, w, stride, pad)
    ref = scatter_conv2d(x[:, None, None, :], w[None, None, None, :], stride, 0) if pad == 0 else None
    # 1-D scatter with padding written out directly
    Lo = (17 + 2 * pad - k) // stride + 1
    out = np.zeros((3, Lo), np.int64)
    for row in range(3):
        for t in range(17):
            for j in range(k):
                ti = t + pad - j
                if ti >= 0 and ti % stride == 0 and ti // stride < Lo:
                    out[row, ti // stride] += int(x[row, t]) * int(w[j])
    assert np.array_equal(y, out.astype(np.float64))
    if ref is not None:
        assert np.array_equal(ref[:, 0, 0, :], out)


# ---------------------------------------------------------------------------
# Hand-worked examples.
# ---------------------------------------------------------------------------

def test_hand_worked_examples(oracle):
    g = json.load(open(GOLDEN))
    for name in ("conv2d_valid_2x2", "conv2d_pad1_asymmetric"):
        c = g[name]
        x = np.array(c["x"], np.float32)[None, None]
        w = np.array(c["w"], np.float32)[None, None]
        y, _ = oracle.conv2d(x, w, c["stride"], c["pad"])
        assert np.array_equal(y[0, 0], np.array(c["y"], np.float64)), name
        yd, _ = oracle.conv2d_depthwise(x, w, c["stride"], c["pad"])
        assert np.array_equal(yd[0, 0], np.array(c["y"], np.float64)), name
        ys = oracle.conv2d_s8(x.astype(np.int8), w.astype(np.int8), c["stride"], c["pad"])
        assert np.array_equal(ys[0, 0], np.array(c["y"], np.int32)), name
    c = g["conv1d_stride2"]
    y, _ = oracle.conv1d(np.array([c["x"]], np.float32), np.array(c["w"], np.float32), c["stride"], c["pad"])
    assert np.array_equal(y[0], np.array(c["y"], np.float64))
    c = g["pool1d_window3"]
    x = np.array([c["x"]], np.float32)
    ya, _ = oracle.pool1d(x, c["window"], c["stride"], oracle.POOL_AVG)
    ym, _ = oracle.pool1d(x, c["window"], c["stride"], oracle.POOL_MAX)
    assert np.allclose(ya[0], c["avg"], rtol=0, atol=1e-15)
    assert np.array_equal(ym[0], np.array(c["max"], np.float64))


# ---------------------------------------------------------------------------
# Special cases with closed forms.
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("pad", [0, 1, 2])
def test_impulse_reproduces_the_filter_without_flip(oracle, pad):
    H, W, R, S = 12, 13, 3, 5
    i0, j0 = 5, 6      # every tap lands inside the output for each pad
    x = np.zeros((1, 1, H, W), np.float32)
    x[0, 0, i0, j0] = 1.0
    w = inputs.uniform_f32((1, 1, R, S), 51)
    y, d = oracle.conv2d(x, w, 1, pad)
    expect = np.zeros_like(y)
    for r in range(R):
        for s in range(S):
            expect[0, 0, i0 - r + pad, j0 - s + pad] = float(w[0, 0, r, s])
    assert np.array_equal(y, expect)
    assert np.array_equal(d, np.abs(expect))


def _box_sums_from_prefix(x, R, S):
    """Valid box sums through a summed-area table (exact for integer-valued x)."""
    H, W = x.shape
    sat = np.zeros((H + 1, W + 1), np.float64)
    sat[1:, 1:] = np.cumsum(np.cumsum(x.astype(np.float64), axis=0), axis=1)
    return sat[R:, S:] - sat[:-R, S:] - sat[R:, :-S] + sat[:-R, :-S]


@pytest.mark.parametrize("R,S", [(3, 3), (5, 5), (7, 7), (2, 6), (1, 4)])
def test_all_ones_filter_equals_box_sums(oracle, R, S):
    x = inputs.small_ints_f32((2, 2, 19, 23), 61, -9, 9)
    w = np.ones((1, 2, R, S), np.float32)
    y, _ = oracle.conv2d(x, w, 1, 0)
    for n in range(2):
        expect = _box_sums_from_prefix(x[n, 0], R, S) + _box_sums_from_prefix(x[n, 1], R, S)
        assert np.array_equal(y[n, 0], expect)
    # depthwise: per-channel box sums, with padding realised by an explicit zero frame
    wd = np.ones((2, 1, R, S), np.float32)
    pad = 2
    yd, _ = oracle.conv2d_depthwise(x, wd, 1, pad)
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    for n, c in itertools.product(range(2), range(2)):
        assert np.array_equal(yd[n, c], _box_sums_from_prefix(xp[n, c], R, S))
    # 1-D: sliding sum through a 1-D prefix sum; the average is that sum / window
    x1 = x[0, 0]
    ps = np.concatenate([np.zeros((x1.shape[0], 1)), np.cumsum(x1.astype(np.float64), axis=1)], axis=1)
    y1, _ = oracle.conv1d(x1, np.ones(S, np.float32), 1, 0)
    assert np.array_equal(y1, ps[:, S:] - ps[:, :-S])
    ya, _ = oracle.pool1d(x1, S, 1, oracle.POOL_AVG)
    assert np.allclose(ya, (ps[:, S:] - ps[:, :-S]) / S, rtol=0, atol=1e-14)


def test_linearity_in_input_and_filter(oracle):
    x1 = inputs.small_ints_f32((2, 3, 8, 9), 71)
    x2 = inputs.small_ints_f32((2, 3, 8, 9), 72)
    w1 = inputs.small_ints_f32((4, 3, 3, 3), 73)
    w2 = inputs.small_ints_f32((4, 3, 3, 3), 74)
    a, b = 3.0, -2.0
    f = lambda x, w: oracle.conv2d(x, w, 1, 1)[0]
    assert np.array_equal(f((a * x1 + b * x2).astype(np.float32), w1), a * f(x1, w1) + b * f(x2, w1))
    assert np.array_equal(f(x1, (a * w1 + b * w2).astype(np.float32)), a * f(x1, w1) + b * f(x1, w2))


@pytest.mark.parametrize("stride,pad", [(1, 1), (1, 3), (2, 2)])
def test_padding_equals_valid_on_zero_framed_copy(oracle, stride, pad):
    x = inputs.normal_f32((2, 3, 10, 11), 81)
    w = inputs.normal_f32((2, 3, 3, 4), 82)
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    y, d = oracle.conv2d(x, w, stride, pad)
    yv, dv = oracle.conv2d(xp, w, stride, 0)
    assert np.array_equal(y, yv) and np.array_equal(d, dv)
    x1 = x[0, 0]
    y1, _ = oracle.conv1d(x1, w[0, 0, 0], stride, pad)
    y1v, _ = oracle.conv1d(np.pad(x1, ((0, 0), (pad, pad))), w[0, 0, 0], stride, 0)
    assert np.array_equal(y1, y1v)


def test_entry_points_agree_with_each_other(oracle):
    # depthwise == full convolution with block-diagonal weights
    x = inputs.normal_f32((2, 4, 9, 9), 91)
    wd = inputs.normal_f32((4, 1, 3, 3), 92)
    wfull = np.zeros((4, 4, 3, 3), np.float32)
    for c in range(4):
        wfull[c, c] = wd[c, 0]
    yd, dd = oracle.conv2d_depthwise(x, wd, 1, 1)
    yf, df = oracle.conv2d(x, wfull, 1, 1)
    assert np.array_equal(yd, yf) and np.array_equal(dd, df)
    # conv1d == conv2d with H = R = 1
    x1 = inputs.normal_f32((5, 40), 93)
    w1 = inputs.normal_f32((9,), 94)
    y1, d1 = oracle.conv1d(x1, w1, 1, 0)
    y2, d2 = oracle.conv2d(x1[:, None, None, :], w1[None, None, None, :], 1, 0)
    assert np.array_equal(y1, y2[:, 0, 0, :]) and np.array_equal(d1, d2[:, 0, 0, :])
    # average pooling == conv1d with taps 1/window (1/8 is exact, so products are too)
    ya, _ = oracle.pool1d(x1, 8, 1, oracle.POOL_AVG)
    yc, _ = oracle.conv1d(x1, np.full(8, 0.125, np.float32), 1, 0)
    assert np.allclose(ya, yc, rtol=0, atol=1e-15)
    # 1x1 filter == one matrix product per pixel
    wp = inputs.normal_f32((3, 4, 1, 1), 95)
    yp, _ = oracle.conv2d(x, wp, 1, 0)
    ref = np.einsum("oc,nchw->nohw", wp[:, :, 0, 0].astype(np.float64), x.astype(np.float64))
    assert np.allclose(yp, ref, rtol=0, atol=1e-14)


def test_separable_filter_is_two_1d_passes(oracle):
    x = inputs.small_ints_f32((1, 1, 12, 13), 101)
    u = inputs.small_ints_f32((3,), 102)
    v = inputs.small_ints_f32((5,), 103)
    w = np.outer(u, v).astype(np.float32)[None, None]
    y, _ = oracle.conv2d(x, w, 1, 0)
    rows, _ = oracle.conv1d(x[0, 0], v, 1, 0)                       # along W
    cols, _ = oracle.conv1d(np.ascontiguousarray(rows.T).astype(np.float32), u, 1, 0)  # along H
    assert np.array_equal(y[0, 0], cols.T)


def test_shift_equivariance_valid_mode(oracle):
    x = inputs.normal_f32((1, 2, 14, 15), 111)
    w = inputs.normal_f32((2, 2, 3, 3), 112)
    a, b = 2, 3
    y, _ = oracle.conv2d(x, w, 1, 0)
    ys, _ = oracle.conv2d(np.ascontiguousarray(x[:, :, a:, b:]), w, 1, 0)
    assert np.array_equal(ys, y[:, :, a:, b:])


def test_max_pool_semantics(oracle):
    x = inputs.normal_f32((4, 50), 121)
    for window, stride in [(8, 1), (3, 2), (1, 1), (50, 1)]:
        y, _ = oracle.pool1d(x, window, stride, oracle.POOL_MAX)
        Lo = (50 - window) // stride + 1
        ref = np.stack([x[:, i * stride:i * stride + window].max(axis=1) for i in range(Lo)], axis=1)
        assert np.array_equal(y, ref.astype(np.float64))
    c = np.full((2, 20), -3.25, np.float32)
    assert np.array_equal(oracle.pool1d(c, 8, 1, oracle.POOL_MAX)[0], np.full((2, 13), -3.25))
    assert np.array_equal(oracle.pool1d(c, 8, 1, oracle.POOL_AVG)[0], np.full((2, 13), -3.25))
    up = np.arange(20, dtype=np.float32)[None]
    assert np.array_equal(oracle.pool1d(up, 8, 1, oracle.POOL_MAX)[0][0], np.arange(7, 20))      # window end
    assert np.array_equal(oracle.pool1d(-up, 8, 1, oracle.POOL_MAX)[0][0], -np.arange(0, 13.0))   # window start


def test_s8_extremes_and_agreement_with_float_oracle(oracle):
    N, C_in, C_out, H, W = 1, 128, 2, 5, 5
    lo = np.full((N, C_in, H, W), -128, np.int8)
    wlo = np.full((C_out, C_in, 3, 3), -128, np.int8)
    whi = np.full((C_out, C_in, 3, 3), 127, np.int8)
    y = oracle.conv2d_s8(lo, wlo, 1, 1)
    assert y[0, 0, 2, 2] == 128 * 9 * 16384 == 18874368      # interior: all 1152 taps
    assert y[0, 0, 0, 0] == 128 * 4 * 16384                  # corner: 2x2 taps remain
    assert y[0, 1, 0, 2] == 128 * 6 * 16384                  # edge: 2x3 taps remain
    y = oracle.conv2d_s8(lo, whi, 1, 1)
    assert y[0, 0, 2, 2] == 128 * 9 * (-128 * 127)
    alt = lo.copy()
    alt[:, 1::2] = 127                                        # alternate sign by channel
    y = oracle.conv2d_s8(alt, wlo, 1, 1)
    assert y[0, 0, 2, 2] == 64 * 9 * 16384 + 64 * 9 * (127 * -128)
    x = inputs.uniform_s8((2, 16, 7, 7), 131)
    w = inputs.uniform_s8((3, 16, 3, 3), 132)
    yi = oracle.conv2d_s8(x, w, 1, 1)
    yf, _ = oracle.conv2d(x.astype(np.float32), w.astype(np.float32), 1, 1)
    assert np.array_equal(yi.astype(np.float64), yf)


def test_s8_overflow_is_refused(oracle):
    # 131072 terms of (-128)*(-128) = 2**31 exactly: one past INT32_MAX.
    x = np.full((1, 131072 // 4, 2, 2), -128, np.int8)
    w = np.full((1, 131072 // 4, 2, 2), -128, np.int8)
    with pytest.raises(OverflowError):
        oracle.conv2d_s8(x, w, 1, 0)


def test_out_dim_formula(oracle):
    for n_in, k, st, pad in itertools.product(range(1, 12), range(1, 6), range(1, 4), range(0, 3)):
        starts = [t for t in range(0, n_in + 2 * pad - k + 1, st)]   # window starts that fit
        assert oracle.out_dim(n_in, k, st, pad) == len(starts)
    assert oracle.out_dim(56, 3, 1, 1) == 56 and oracle.out_dim(56, 7, 1, 3) == 56
    assert oracle.out_dim(65536, 9, 1, 0) == 65528 and oracle.out_dim(65536, 8, 1, 0) == 65529
    assert oracle.out_dim(2, 3, 1, 0) == 0


# ---------------------------------------------------------------------------
# Library routines (float64) on the seeded workload distributions.
# ---------------------------------------------------------------------------

def test_against_torch_float64_routines(oracle):
    import torch
    import torch.nn.functional as F

    t = lambda a: torch.from_numpy(a.astype(np.float64))
    x, w = inputs.workload3(N=2)
    y, d = oracle.conv2d(x, w, 1, 1)
    ref = F.conv2d(t(x), t(w), stride=1, padding=1).numpy()
    refd = F.conv2d(t(np.abs(x)), t(np.abs(w)), stride=1, padding=1).numpy()
    assert np.max(np.abs(y - ref) / d) < 1e-12
    assert np.max(np.abs(d - refd) / d) < 1e-12

    x, w3, w7 = inputs.workload4(N=1, C=16)
    for wd, pad in ((w3, 1), (w7, 3)):
        y, d = oracle.conv2d_depthwise(x, wd, 1, pad)
        ref = F.conv2d(t(x), t(wd), stride=1, padding=pad, groups=16).numpy()
        assert np.max(np.abs(y - ref) / d) < 1e-12

    x, w = inputs.workload2(rows=4, length=4096)
    y, d = oracle.conv1d(x, w, 1, 0)
    ref = F.conv1d(t(x)[:, None], t(w)[None, None]).numpy()[:, 0]
    assert np.max(np.abs(y - ref) / d) < 1e-12
    ya, da = oracle.pool1d(x, 8, 1, oracle.POOL_AVG)
    assert np.max(np.abs(ya - F.avg_pool1d(t(x)[:, None], 8, 1).numpy()[:, 0])) < 1e-14
    ym, _ = oracle.pool1d(x, 8, 1, oracle.POOL_MAX)
    assert np.array_equal(ym, F.max_pool1d(t(x)[:, None], 8, 1).numpy()[:, 0])
    assert np.allclose(da, F.avg_pool1d(t(np.abs(x))[:, None], 8, 1).numpy()[:, 0], rtol=0, atol=1e-14)

    x, w = inputs.workload1()
    y, d = oracle.conv2d(x, w, 1, 0)
    assert np.max(np.abs(y - F.conv2d(t(x), t(w)).numpy()) / np.maximum(d, 1e-300)) < 1e-12

    x, w = inputs.workload5(N=1)
    yi = oracle.conv2d_s8(x, w, 1, 1)
    ref = F.conv2d(t(x), t(w), padding=1).numpy()          # exact: |sum| < 2**53
    assert np.array_equal(yi.astype(np.float64), ref)

    # strided / non-square
    x = inputs.normal_f32((2, 3, 11, 13), 141)
    w = inputs.normal_f32((4, 3, 3, 5), 142)
    y, d = oracle.conv2d(x, w, 2, 2)
    assert np.max(np.abs(y - F.conv2d(t(x), t(w), stride=2, padding=2).numpy()) / d) < 1e-12


def test_threading_does_not_change_a_value(oracle):
    x, w = inputs.workload3(N=2)
    n = oracle.max_threads()
    oracle.set_threads(1)
    y1, d1 = oracle.conv2d(x, w, 1, 1)
    oracle.set_threads(n)
    yn, dn = oracle.conv2d(x, w, 1, 1)
    assert np.array_equal(y1, yn) and np.array_equal(d1, dn)
