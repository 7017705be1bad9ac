"""GPU parity of the bf16-activation depthwise convolution (bf16 in, fp32 filter and accumulation, one rounding to
bf16 out) against the CPU oracle on the widened inputs.  In value space the result must lie within the fp32
parity bound plus half a bf16 unit of the exact sum: |y - y_oracle| <= 2e-5 * sum|x*w| + 2^-8 * |y_oracle|; where
the exact sum is representable in bf16 (small integers, identity filters) it must be bit-exact."""
import numpy as np
import pytest

from paper_2310_05218_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as _t

    assert _t.cuda.is_available(), "these tests need the GPU"
    return _t


@pytest.fixture(scope="module")
def sw():
    import paper_2310_05218_amd as _sw
    from paper_2310_05218_amd import binding

    binding.lib()            # fails loudly if the library is not built
    return _sw


def bf16_dev(torch, bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bits_of(torch, t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def run(torch, sw, xb, w, stride, pad):
    y = sw.sw_conv2d_depthwise_bf16(bf16_dev(torch, xb), torch.from_numpy(w).cuda(), stride, pad)
    torch.cuda.synchronize()
    return bits_of(torch, y)


CASES = [
    # N, C, H, W, R, S, stride, pad
    (2, 9, 56, 56, 3, 3, 1, 1),      # whole-plane kernel, 56 x 56 specialisation
    (2, 9, 56, 56, 5, 5, 1, 2),
    (2, 9, 56, 56, 7, 7, 1, 3),
    (3, 5, 48, 56, 3, 3, 1, 1),      # ... general variant: fewer rows
    (2, 5, 28, 32, 5, 5, 1, 2),
    (2, 5, 40, 40, 7, 7, 1, 3),
    (2, 5, 56, 56, 3, 3, 1, 0),      # valid mode: 54 x 54 output is not a multiple of 8 -> one thread per output
    (2, 5, 30, 30, 3, 3, 2, 1),      # stride 2
    (1, 4, 20, 23, 9, 4, 1, 3),      # other extents, ragged width
    (1, 3, 64, 64, 3, 3, 1, 1),      # larger than a tile
    (1, 2, 3, 3, 3, 3, 1, 0),        # a single output
]


@pytest.mark.parametrize("case", CASES)
def test_bf16_depthwise_matches_the_oracle(torch, sw, oracle, case):
    N, C, H, W, R, S, stride, pad = case
    xb = inputs.normal_bf16((N, C, H, W), 4001)
    w = inputs.normal_f32((C, 1, R, S), 4002, 1.0 / (R * S) ** 0.5)
    y_ref, d = oracle.conv2d_depthwise(oracle.bf16_to_f32(xb), w, stride, pad)
    y = oracle.bf16_to_f32(run(torch, sw, xb, w, stride, pad)).astype(np.float64)
    assert y.shape == y_ref.shape
    bound = 2e-5 * d + 2.0 ** -8 * np.abs(y_ref) + 1e-37
    worst = float(np.max(np.abs(y - y_ref) / bound))
    assert worst <= 1.0, f"bf16 depthwise {case}: {worst:.3f} of the bound"
    # and it really is rounded, not truncated: truncation would bias the error towards zero by 2^-9 on average
    if y.size >= 10000:
        err = (y - y_ref) * np.sign(y_ref)
        assert abs(float(np.mean(err / (np.abs(y_ref) + 1e-30)))) < 2.0 ** -11


@pytest.mark.parametrize("case", [(3, 7, 56, 56, 3, 3, 1, 1), (2, 5, 48, 48, 7, 7, 1, 3), (2, 5, 31, 29, 5, 5, 2, 2)])
def test_bf16_exact_where_the_sum_is_representable(torch, sw, oracle, case):
    """Small integers: every product and sum is exact in fp32 and the result (|y| <= 196) is a bf16 value."""
    N, C, H, W, R, S, stride, pad = case
    rng = np.random.default_rng(4010)
    x = rng.integers(-2, 3, size=(N, C, H, W)).astype(np.float32)
    w = rng.integers(-2, 3, size=(C, 1, R, S)).astype(np.float32)
    y_ref, _ = oracle.conv2d_depthwise(x, w, stride, pad)
    assert np.abs(y_ref).max() <= 256
    y = oracle.bf16_to_f32(run(torch, sw, oracle.f32_to_bf16_rne(x), w, stride, pad))
    assert np.array_equal(y.astype(np.float64), y_ref)


def test_bf16_identity_ties_and_many_planes(torch, sw, oracle):
    # centre tap 1: the output is the input, bit for bit; 2105 planes: several planes per wavefront
    N, C = 5, 421
    xb = inputs.normal_bf16((N, C, 56, 56), 4021)
    w = np.zeros((C, 1, 3, 3), np.float32)
    w[:, 0, 1, 1] = 1.0
    assert np.array_equal(run(torch, sw, xb, w, 1, 1), xb)
    # centre tap 1 + 2^-8 on x = 1: the exact product 1.00390625 lies halfway between the bf16 values 1.0 and
    # 1.0078125 and goes to the even one (1.0); with x = 1.0078125 (odd mantissa) the product
    # 1.011749267578125 lies above the halfway point 1.01171875 and goes up to 1.015625
    w[:, 0, 1, 1] = 1.0 + 2.0 ** -8
    ones = oracle.f32_to_bf16_rne(np.full((1, C, 56, 56), 1.0, np.float32))
    assert np.all(oracle.bf16_to_f32(run(torch, sw, ones, w, 1, 1)) == 1.0)
    odd = oracle.f32_to_bf16_rne(np.full((1, C, 56, 56), 1.0078125, np.float32))
    assert np.all(oracle.bf16_to_f32(run(torch, sw, odd, w, 1, 1)) == 1.015625)


def test_bf16_full_size_workload(torch, sw, oracle):
    """Workload 4's shape (32 x 256 planes of 56 x 56, 3x3 and 7x7) in bf16: every output against the oracle."""
    N, C = 32, 256
    xb = inputs.normal_bf16((N, C, 56, 56), 4031)
    xd = bf16_dev(torch, xb)
    xw = oracle.bf16_to_f32(xb)
    for k in (3, 7):
        w = inputs.normal_f32((C, 1, k, k), 4032 + k, 1.0 / k)
        y = bits_of(torch, sw.sw_conv2d_depthwise_bf16(xd, torch.from_numpy(w).cuda(), 1, k // 2))
        y_ref, d = oracle.conv2d_depthwise(xw, w, 1, k // 2)
        yv = oracle.bf16_to_f32(y).astype(np.float64)
        bound = 2e-5 * d + 2.0 ** -8 * np.abs(y_ref) + 1e-37
        worst = float(np.max(np.abs(yv - y_ref) / bound))
        print(f"bf16 {k}x{k} full size: largest error / bound = {worst:.3f}")
        assert worst <= 1.0, (k, worst)
