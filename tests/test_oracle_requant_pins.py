"""Pins for the requantisation step of the CPU oracle (exact int32 sums -> int8).  The paper gives no formula
(section 1.1 only says that quantised inference keeps activations in 8 bits), so the definition is this
library's: q = clamp(rne(scale[co] * float(acc + bias[co])), 0 if relu else -128, 127), every step in fp32.
Each test fixes it to something other than itself; none needs a GPU."""
import numpy as np
import pytest


def _acc_as_conv(oracle, acc, bias, scale, relu):
    """Feeds chosen accumulator values through the oracle: a 1x1 filter of weight 1 over one input channel per
    output channel would need int8 inputs, so the values are split as acc = 127 * a + b with int8 a, b and two
    input channels weighted 127 and 1."""
    acc = np.asarray(acc, np.int64)
    a = np.trunc(acc / 127).astype(np.int64)
    b = acc - 127 * a
    assert np.all(np.abs(a) <= 127) and np.all(np.abs(b) <= 127)
    x = np.stack([a, b]).astype(np.int8)[None, :, None, :]             # [1, 2, 1, n]
    w = np.array([127, 1], np.int8).reshape(1, 2, 1, 1)
    return oracle.conv2d_s8_requant(x, w, bias, scale, 1, 0, relu)[0, 0, 0]


def test_hand_worked_ties_and_saturation(oracle):
    sc = np.array([0.5], np.float32)
    # 0.5 -> 0, 1.5 -> 2, 2.5 -> 2, 3.5 -> 4, -0.5 -> 0, -1.5 -> -2, -2.5 -> -2 (ties to even), 3 * 0.5 rounds 1.5 -> 2
    assert list(_acc_as_conv(oracle, [1, 3, 5, 7, -1, -3, -5, 4, -4], None, sc, False)) == [0, 2, 2, 4, 0, -2, -2, 2, -2]
    # bias shifts the sum before scaling: (acc + 1) * 0.5
    assert list(_acc_as_conv(oracle, [0, 2, 4, -2], np.array([1], np.int32), sc, False)) == [0, 2, 2, 0]
    # saturation and the rectifier
    sc2 = np.array([2.0], np.float32)
    assert list(_acc_as_conv(oracle, [100, 63, 64, -64, -65, -100], None, sc2, False)) == [127, 126, 127, -128, -128, -128]
    assert list(_acc_as_conv(oracle, [100, 3, 0, -1, -100], None, sc2, True)) == [127, 6, 0, 0, 0]


def test_conversion_to_fp32_comes_before_the_product(oracle):
    # 33554434 = 2^25 + 2 is halfway between two fp32 values and becomes 2^25 (even mantissa); times 2^-26 that
    # is exactly 0.5 and rounds to 0.  A product taken in double would be 0.50000003 and round to 1.
    acc = np.array([[[[33554434]]]], np.int32)
    q = np.empty((1, 1, 1, 1), np.int8)
    _load, _p = oracle._load, oracle._p
    rc = _load().oracle_requant_s8(_p(acc), None, _p(np.array([2.0 ** -26], np.float32)), _p(q), 1, 1, 1, 0)
    assert rc == 0 and q[0, 0, 0, 0] == 0
    # ... and the product is rounded to fp32 before it is rounded to an integer: 3 * 0.16666667 (fp32 of 1/6)
    # is 0.50000001 in exact arithmetic but exactly 0.5 in fp32, which ties to 0
    acc[...] = 3
    rc = _load().oracle_requant_s8(_p(acc), None, _p(np.array([1.0 / 6.0], np.float32)), _p(q), 1, 1, 1, 0)
    assert np.float32(3.0) * np.float32(1.0 / 6.0) == np.float32(0.5)
    assert rc == 0 and q[0, 0, 0, 0] == 0


@pytest.mark.parametrize("relu", [False, True])
def test_against_numpy_float32_arithmetic(oracle, relu):
    _load, _p = oracle._load, oracle._p
    rng = np.random.default_rng(4242 + relu)
    N, C, P = 3, 7, 501
    acc = rng.integers(-2 ** 30, 2 ** 30, size=(N, C, P), dtype=np.int64).astype(np.int32)
    acc[:, :3] = rng.integers(-300, 300, size=(N, 3, P))
    bias = rng.integers(-1000, 1000, size=C).astype(np.int32)
    scale = np.concatenate([[0.5, 0.25, 1.5], 2.0 ** -rng.integers(20, 28, size=C - 3) * rng.uniform(0.5, 1.5, C - 3)]).astype(np.float32)
    q = np.empty((N, C, P), np.int8)
    assert _load().oracle_requant_s8(_p(acc), _p(bias), _p(scale), _p(q), N, C, P, int(relu)) == 0
    t = (acc.astype(np.int64) + bias[None, :, None]).astype(np.int32)
    prod = t.astype(np.float32) * scale[None, :, None]                 # numpy: IEEE fp32 conversion and product
    assert prod.dtype == np.float32
    ref = np.clip(np.rint(prod), 0 if relu else -128, 127).astype(np.int8)
    assert np.array_equal(q, ref)
    import torch
    tref = torch.clamp(torch.round(torch.from_numpy(t).to(torch.float32) * torch.from_numpy(scale)[None, :, None]),
                       0 if relu else -128, 127).to(torch.int8).numpy()
    assert np.array_equal(q, tref)


def test_identity_monotonicity_and_overflow(oracle):
    _load, _p = oracle._load, oracle._p
    acc = np.arange(-128, 128, dtype=np.int32).reshape(1, 1, 256)
    q = np.empty((1, 1, 256), np.int8)
    one = np.array([1.0], np.float32)
    assert _load().oracle_requant_s8(_p(acc), None, _p(one), _p(q), 1, 1, 256, 0) == 0
    assert np.array_equal(q[0, 0], np.arange(-128, 128).astype(np.int8))            # scale 1, no bias: identity
    acc = np.sort(np.random.default_rng(5).integers(-10 ** 6, 10 ** 6, size=(1, 1, 4000))).astype(np.int32)
    q = np.empty(acc.shape, np.int8)
    assert _load().oracle_requant_s8(_p(acc), None, _p(np.array([1e-4], np.float32)), _p(q), 1, 1, 4000, 0) == 0
    assert np.all(np.diff(q[0, 0].astype(int)) >= 0)                               # positive scale: non-decreasing
    big = np.array([[[2 ** 31 - 1]]], np.int32)
    q1 = np.empty((1, 1, 1), np.int8)
    assert _load().oracle_requant_s8(_p(big), _p(np.array([1], np.int32)), _p(one), _p(q1), 1, 1, 1, 0) == 2


def test_two_channels_use_their_own_scale_and_bias(oracle):
    x = np.array([10, -10, 3], np.int8).reshape(1, 1, 1, 3)
    w = np.array([1, 2], np.int8).reshape(2, 1, 1, 1)
    q = oracle.conv2d_s8_requant(x, w, np.array([1, -1], np.int32), np.array([0.5, 2.0], np.float32), 1, 0, False)
    assert q[0, 0, 0].tolist() == [6, -4, 2]         # (10+1)/2 = 5.5 -> 6, (-10+1)/2 = -4.5 -> -4, (3+1)/2 = 2
    assert q[0, 1, 0].tolist() == [38, -42, 10]      # (20-1)*2, (-20-1)*2, (6-1)*2
