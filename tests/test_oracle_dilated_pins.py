"""Pins for the dilated convolution of the CPU oracle (taps `dilation` input positions apart).  Each test fixes
it to something other than itself: the a-trous identity (a dilated filter is the plain convolution with zeros
stuffed between the taps, computed by the separately pinned plain entry points), an input-driven scatter,
hand-worked numbers and torch's double-precision convolution.  None needs a GPU."""
import numpy as np
import pytest

CASES = [
    # N, C_in, C_out, H, W, R, S, stride, pad, dilation
    (1, 1, 1, 7, 7, 3, 3, 1, 0, 2),
    (2, 3, 4, 11, 9, 3, 2, 1, 2, 2),
    (1, 2, 3, 13, 12, 2, 3, 2, 3, 3),
    (1, 4, 2, 9, 14, 3, 3, 3, 4, 4),
    (2, 2, 2, 8, 8, 1, 1, 1, 0, 5),      # one tap: dilation changes nothing
    (1, 3, 3, 10, 10, 3, 1, 1, 1, 2),    # dilation acts on rows only when S = 1
]


def _stuffed(w, dil):
    Co, Ci, R, S = w.shape
    z = np.zeros((Co, Ci, dil * (R - 1) + 1, dil * (S - 1) + 1), np.float32)
    z[:, :, ::dil, ::dil] = w
    return z


@pytest.mark.parametrize("case", CASES)
def test_dilated_equals_plain_convolution_with_a_zero_stuffed_filter(oracle, case):
    N, Ci, Co, H, W, R, S, stride, pad, dil = case
    rng = np.random.default_rng(9000 + sum(case))
    x = rng.standard_normal((N, Ci, H, W)).astype(np.float32)
    w = rng.standard_normal((Co, Ci, R, S)).astype(np.float32)
    y, d = oracle.conv2d_dilated(x, w, stride, pad, dil)
    y0, d0 = oracle.conv2d(x, _stuffed(w, dil), stride, pad)
    assert y.shape == y0.shape
    assert np.array_equal(y, y0) and np.array_equal(d, d0)     # the same products in the same order
    # depthwise: channel c of x with filter c
    wd = rng.standard_normal((Ci, 1, R, S)).astype(np.float32)
    yd, dd = oracle.conv2d_dilated(x, wd, stride, pad, dil, depthwise=True)
    yd0, dd0 = oracle.conv2d_depthwise(x, _stuffed(wd, dil), stride, pad)
    assert np.array_equal(yd, yd0) and np.array_equal(dd, dd0)


@pytest.mark.parametrize("case", CASES[:4])
def test_dilated_matches_input_driven_scatter(oracle, case):
    """Every input element is pushed to the outputs it contributes to (the loop nest runs over inputs and taps
    and solves for the output index, the reverse of the oracle's)."""
    N, Ci, Co, H, W, R, S, stride, pad, dil = case
    rng = np.random.default_rng(9100 + sum(case))
    x = rng.integers(-3, 4, size=(N, Ci, H, W)).astype(np.float32)
    w = rng.integers(-3, 4, size=(Co, Ci, R, S)).astype(np.float32)
    y, _ = oracle.conv2d_dilated(x, w, stride, pad, dil)
    Ho, Wo = y.shape[2:]
    ref = np.zeros_like(y)
    for h in range(H):
        for v in range(W):
            for r in range(R):
                for s in range(S):
                    ti, tj = h + pad - r * dil, v + pad - s * dil
                    if ti < 0 or tj < 0 or ti % stride or tj % stride:
                        continue
                    i, j = ti // stride, tj // stride
                    if i >= Ho or j >= Wo:
                        continue
                    ref[:, :, i, j] += np.einsum("nc,oc->no", x[:, :, h, v].astype(np.float64), w[:, :, r, s].astype(np.float64))
    assert np.array_equal(y, ref)      # small integers: exact


def test_hand_worked_example(oracle):
    # 1-D in disguise: a row 1..7, filter [1, 10, 100] with dilation 2 reads positions j, j+2, j+4
    x = np.arange(1, 8, dtype=np.float32).reshape(1, 1, 1, 7)
    w = np.array([1, 10, 100], np.float32).reshape(1, 1, 1, 3)
    y, d = oracle.conv2d_dilated(x, w, 1, 0, 2)
    assert y.reshape(-1).tolist() == [531.0, 642.0, 753.0]
    assert d.reshape(-1).tolist() == [531.0, 642.0, 753.0]
    # padding 2 on every side: five output rows, the middle one sees the data row; its first outputs see zeros
    # on the left, its last ones on the right
    y, _ = oracle.conv2d_dilated(x, w, 1, 2, 2)
    assert y.shape == (1, 1, 5, 7)
    assert y[0, 0, 2].tolist() == [310.0, 420.0, 531.0, 642.0, 753.0, 64.0, 75.0]
    assert not y[0, 0, [0, 1, 3, 4]].any()
    # stride 2: windows start at 0 and 2
    y, _ = oracle.conv2d_dilated(x, w, 2, 0, 2)
    assert y.reshape(-1).tolist() == [531.0, 753.0]
    # columns: the same along H
    y, _ = oracle.conv2d_dilated(x.reshape(1, 1, 7, 1), w.reshape(1, 1, 3, 1), 1, 0, 3)
    assert y.reshape(-1).tolist() == [741.0]
    with pytest.raises(ValueError):
        oracle.conv2d_dilated(x, w, 1, 0, 4)        # span 9 > 7
    with pytest.raises(ValueError):
        oracle.conv2d_dilated(x, w, 1, 0, 0)


def test_against_torch_double(oracle):
    import torch

    rng = np.random.default_rng(9200)
    x = rng.standard_normal((2, 4, 15, 13)).astype(np.float32)
    w = rng.standard_normal((6, 4, 3, 3)).astype(np.float32)
    for stride, pad, dil in [(1, 2, 2), (2, 3, 3), (1, 0, 4)]:
        y, _ = oracle.conv2d_dilated(x, w, stride, pad, dil)
        t = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), None,
                                       stride=stride, padding=pad, dilation=dil).numpy()
        assert y.shape == t.shape and np.max(np.abs(y - t)) <= 1e-12
    wd = rng.standard_normal((4, 1, 3, 3)).astype(np.float32)
    y, _ = oracle.conv2d_dilated(x, wd, 1, 2, 2, depthwise=True)
    t = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(wd).double(), None, stride=1,
                                   padding=2, dilation=2, groups=4).numpy()
    assert np.max(np.abs(y - t)) <= 1e-12
