"""Seeded random shapes through every entry point, each checked element by element against the CPU oracle.
The shapes are drawn so that every kernel selection rule of the library is crossed many times (small and
ragged planes, strides, paddings up to the filter extent, odd channel counts, wide rows)."""
import numpy as np
import pytest

from paper_2310_05218_amd import inputs
from parity import assert_f32_parity, guarded_empty, assert_guards_intact

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    if not t.cuda.is_available():
        pytest.skip("no GPU")
    return t


@pytest.fixture(scope="module")
def sw():
    import paper_2310_05218_amd as m
    from paper_2310_05218_amd import binding
    binding.lib()
    return m


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _shape(rng, max_hw, max_k, max_stride=3):
    R, S = int(rng.integers(1, max_k + 1)), int(rng.integers(1, max_k + 1))
    if rng.random() < 0.5:
        S = R
    stride = int(rng.integers(1, max_stride + 1))
    pad = int(rng.integers(0, max(R, S)))
    H = int(rng.integers(max(1, R - 2 * pad), max_hw + 1))
    W = int(rng.integers(max(1, S - 2 * pad), max_hw + 1))
    if rng.random() < 0.4:
        W = (W + 3) // 4 * 4
    return H, W, R, S, stride, pad


def _cases(seed, n, **kw):
    rng = np.random.default_rng(seed)
    return [(i,) + _shape(rng, **kw) + (int(rng.integers(0, 1 << 30)),) for i in range(n)]


@pytest.mark.parametrize("case", _cases(71, 40, max_hw=70, max_k=9), ids=lambda c: "x".join(map(str, c[1:7])))
def test_depthwise_random(torch, sw, oracle, case):
    _, H, W, R, S, stride, pad, seed = case
    rng = np.random.default_rng(seed)
    N, C = int(rng.integers(1, 4)), int(rng.choice([1, 3, 8, 70, 130]))
    x = inputs.normal_f32((N, C, H, W), seed % 100000)
    w = inputs.normal_f32((C, 1, R, S), seed % 100000 + 1)
    y_ref, d = oracle.conv2d_depthwise(x, w, stride, pad)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_depthwise(dev(torch, x), dev(torch, w), stride, pad, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"depthwise {case} N={N} C={C}")


@pytest.mark.parametrize("case", _cases(72, 40, max_hw=40, max_k=7), ids=lambda c: "x".join(map(str, c[1:7])))
def test_conv2d_random(torch, sw, oracle, case):
    _, H, W, R, S, stride, pad, seed = case
    rng = np.random.default_rng(seed)
    N = int(rng.integers(1, 3))
    C_in, C_out = int(rng.choice([1, 2, 3, 7, 16, 24, 33])), int(rng.choice([1, 5, 32, 64, 70]))
    x = inputs.normal_f32((N, C_in, H, W), seed % 100000)
    w = inputs.normal_f32((C_out, C_in, R, S), seed % 100000 + 1)
    y_ref, d = oracle.conv2d(x, w, stride, pad)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d(dev(torch, x), dev(torch, w), stride, pad, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"conv2d {case} N={N} C_in={C_in} C_out={C_out}")


@pytest.mark.parametrize("case", _cases(73, 30, max_hw=36, max_k=5), ids=lambda c: "x".join(map(str, c[1:7])))
def test_conv2d_s8_random(torch, sw, oracle, case):
    _, H, W, R, S, stride, pad, seed = case
    rng = np.random.default_rng(seed)
    N = int(rng.integers(1, 3))
    C_in, C_out = int(rng.choice([1, 3, 16, 40, 64, 100])), int(rng.choice([1, 5, 64, 70]))
    x = inputs.uniform_s8((N, C_in, H, W), seed % 100000)
    w = inputs.uniform_s8((C_out, C_in, R, S), seed % 100000 + 1)
    y_ref = oracle.conv2d_s8(x, w, stride, pad)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.int32)
    sw.sw_conv2d_s8(dev(torch, x), dev(torch, w), stride, pad, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert np.array_equal(out.cpu().numpy(), y_ref), f"conv2d_s8 {case} N={N} C_in={C_in} C_out={C_out}"


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("case", _cases(74, 30, max_hw=70, max_k=6), ids=lambda c: "x".join(map(str, c[1:7])))
def test_pool2d_random(torch, sw, oracle, case, mode):
    _, H, W, R, S, stride, pad, seed = case
    pad = min(pad, min(R, S) // 2)          # the library's contract: no window wholly inside the padding
    if H + 2 * pad < R or W + 2 * pad < S:
        pytest.skip("window larger than the padded plane")
    rng = np.random.default_rng(seed)
    N, C = int(rng.integers(1, 3)), int(rng.choice([1, 3, 64, 100]))
    x = inputs.normal_f32((N, C, H, W), seed % 100000) - (2.0 if mode else 0.0)
    y_ref, d = oracle.pool2d(x, R, S, stride, pad, mode)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_pool2d(dev(torch, x), R, S, stride, pad, mode, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    y = out.cpu().numpy()
    if mode == 1:
        assert np.array_equal(y.astype(np.float64), y_ref), f"max pool2d {case}"
    else:
        assert_f32_parity(y, y_ref, d, f"avg pool2d {case}")


@pytest.mark.parametrize("case", list(range(30)))
def test_conv1d_and_pool1d_random(torch, sw, oracle, case):
    rng = np.random.default_rng(7500 + case)
    rows = int(rng.integers(1, 6))
    k = int(rng.integers(1, 40))
    stride = int(rng.choice([1, 1, 1, 2, 3]))
    pad = int(rng.integers(0, k))
    length = int(rng.integers(max(1, k - 2 * pad), 9000))
    x = inputs.normal_f32((rows, length), 7600 + case)
    w = inputs.normal_f32((k,), 7700 + case)
    y_ref, d = oracle.conv1d(x, w, stride, pad)
    y = sw.sw_conv1d(dev(torch, x), dev(torch, w), stride, pad).cpu().numpy()
    assert_f32_parity(y, y_ref, d, f"conv1d k={k} stride={stride} pad={pad} len={length}")
    if length >= k:
        for mode in (0, 1):
            y_ref, d = oracle.pool1d(x, k, stride, mode)
            y = sw.sw_pool1d(dev(torch, x), k, stride, mode).cpu().numpy()
            if mode == 1:
                assert np.array_equal(y.astype(np.float64), y_ref)
            else:
                assert_f32_parity(y, y_ref, d, f"avg pool1d window={k} stride={stride} len={length}")


@pytest.mark.parametrize("case", _cases(81, 30, max_hw=40, max_k=5), ids=lambda c: "x".join(map(str, c[1:7])))
def test_conv2d_dilated_random(torch, sw, oracle, case):
    _, H, W, R, S, stride, pad, seed = case
    rng = np.random.default_rng(seed)
    dil = int(rng.integers(1, 5))
    # keep the dilated filter inside the padded plane
    H = max(H, dil * (R - 1) + 1 - 2 * pad)
    W = max(W, dil * (S - 1) + 1 - 2 * pad)
    N = int(rng.integers(1, 3))
    depthwise = bool(rng.random() < 0.3)
    C_in, C_out = int(rng.choice([1, 2, 3, 7, 16, 33])), int(rng.choice([1, 5, 32, 64, 70]))
    if depthwise:
        C_out = C_in
    x = inputs.normal_f32((N, C_in, H, W), seed % 100000)
    w = inputs.normal_f32((C_out, 1 if depthwise else C_in, R, S), seed % 100000 + 1)
    y_ref, d = oracle.conv2d_dilated(x, w, stride, pad, dil, depthwise=depthwise)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    call = sw.sw_conv2d_depthwise_dilated if depthwise else sw.sw_conv2d_dilated
    call(dev(torch, x), dev(torch, w), stride, pad, dil, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"dilated {case} dil={dil} dw={depthwise} C_in={C_in} C_out={C_out}")


@pytest.mark.parametrize("case", _cases(82, 40, max_hw=60, max_k=7), ids=lambda c: "x".join(map(str, c[1:7])))
def test_bias_relu_random(torch, sw, oracle, case):
    """Both fused-epilogue entry points (multi-channel and depthwise), bias present or not, rectifier on or off."""
    _, H, W, R, S, stride, pad, seed = case
    rng = np.random.default_rng(seed)
    N = int(rng.integers(1, 3))
    depthwise = bool(rng.random() < 0.5)
    C_in, C_out = int(rng.choice([1, 3, 8, 16, 40])), int(rng.choice([1, 5, 64, 70]))
    if depthwise:
        C_in = C_out = int(rng.choice([1, 3, 8, 70, 130]))
    relu, with_bias = bool(rng.random() < 0.6), bool(rng.random() < 0.8)
    x = inputs.normal_f32((N, C_in, H, W), seed % 100000)
    w = inputs.normal_f32((C_out, 1 if depthwise else C_in, R, S), seed % 100000 + 1)
    bias = inputs.normal_f32((C_out,), seed % 100000 + 2, 0.8) if with_bias else None
    if depthwise:
        y_ref, d = oracle.conv2d_depthwise_bias_relu(x, w, bias, stride, pad, relu)
        call = sw.sw_conv2d_depthwise_bias_relu
    else:
        y_ref, d = oracle.conv2d_bias_relu(x, w, bias, stride, pad, relu)
        call = sw.sw_conv2d_bias_relu
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    call(dev(torch, x), dev(torch, w), dev(torch, bias) if with_bias else None, stride, pad, relu, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"bias_relu {case} dw={depthwise} relu={relu} bias={with_bias}")


@pytest.mark.parametrize("case", _cases(83, 30, max_hw=60, max_k=7), ids=lambda c: "x".join(map(str, c[1:7])))
def test_depthwise_bf16_random(torch, sw, oracle, case):
    _, H, W, R, S, stride, pad, seed = case
    rng = np.random.default_rng(seed)
    if rng.random() < 0.5:          # steer half of the cases to the whole-plane kernel's range
        R = S = int(rng.choice([3, 5, 7]))
        stride, pad = 1, R // 2
        H, W = int(rng.integers(R, 57)), int(rng.choice([8, 16, 24, 32, 40, 48, 56]))
    N, C = int(rng.integers(1, 4)), int(rng.choice([1, 3, 8, 70]))
    xb = inputs.normal_bf16((N, C, H, W), seed % 100000)
    w = inputs.normal_f32((C, 1, R, S), seed % 100000 + 1, 1.0 / (R * S) ** 0.5)
    y_ref, d = oracle.conv2d_depthwise(oracle.bf16_to_f32(xb), w, stride, pad)
    xd = torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.bfloat16)
    sw.sw_conv2d_depthwise_bf16(xd, dev(torch, w), stride, pad, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    y = oracle.bf16_to_f32(out.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    assert np.all(np.abs(y - y_ref) <= 2e-5 * d + 2.0 ** -8 * np.abs(y_ref) + 1e-37), f"bf16 depthwise {case} N={N} C={C}"


def _jit_cases(seed, n):
    """Geometries inside the generated kernel's range: stride 1, W and W_out multiples of 4, output at most
    56 x 56 and at least half of that, 2 * pad <= min(R, S) - 1."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        R, S = int(rng.integers(1, 20)), int(rng.integers(1, 20))
        pad = int(rng.integers(0, (min(R, S) - 1) // 2 + 1))
        Ho, Wo = int(rng.integers(40, 57)), int(rng.choice([40, 44, 48, 52, 56]))
        H, W = Ho + R - 1 - 2 * pad, Wo + S - 1 - 2 * pad
        if W % 4 or H * W > 4096:
            continue
        out.append((len(out), H, W, R, S, pad, int(rng.integers(0, 1 << 30))))
    return out


@pytest.mark.parametrize("case", _jit_cases(84, 16), ids=lambda c: "x".join(map(str, c[1:6])))
def test_depthwise_jit_random(torch, sw, oracle, case):
    _, H, W, R, S, pad, seed = case
    assert sw.sw_jit_prepare_depthwise(H, W, R, S, 1, pad) == 0, "geometry expected inside the generated kernel's range"
    rng = np.random.default_rng(seed)
    N, C = int(rng.integers(1, 3)), int(rng.choice([1, 3, 9]))
    x = inputs.normal_f32((N, C, H, W), seed % 100000)
    w = inputs.normal_f32((C, 1, R, S), seed % 100000 + 1, 1.0 / (R * S) ** 0.5)
    y_ref, d = oracle.conv2d_depthwise(x, w, 1, pad)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_depthwise_jit(dev(torch, x), dev(torch, w), 1, pad, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"jit depthwise {case} N={N} C={C}")


# ---- channel-last tensors: fp32, bf16, IEEE half, int8 (int32 and requantised int8 out) ----
# Channel counts on and off the grids the matrix-core kernels want (whole 32-byte pixels, C_out % 4), small and ragged
# planes, several images per tile, strides, paddings and (float formats) dilations: the window-in-LDS kernel's planner,
# its older companions and the one-thread-per-output kernel all take their share.

def _nhwc_cases(seed, n):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        H, W, R, S, stride, pad = _shape(rng, max_hw=34, max_k=5)
        N = int(rng.integers(1, 7))
        C_in = int(rng.choice([8, 16, 24, 32, 48, 64, 96, 160, 192]))
        C_out = int(rng.choice([4, 8, 20, 30, 32, 36, 64, 72, 100, 128]))
        dil = int(rng.choice([1, 1, 2, 3]))
        out.append((N, H, W, C_in, C_out, R, S, stride, pad, dil, int(rng.integers(0, 100000))))
    return out


def _fits(H, W, R, S, pad, dil):
    return H + 2 * pad >= dil * (R - 1) + 1 and W + 2 * pad >= dil * (S - 1) + 1


@pytest.mark.parametrize("case", _nhwc_cases(81, 40), ids=lambda c: "x".join(map(str, c[:10])))
def test_conv2d_nhwc_random(torch, sw, oracle, case):
    N, H, W, C_in, C_out, R, S, stride, pad, dil, seed = case
    if not _fits(H, W, R, S, pad, dil):
        dil = 1
    x = inputs.normal_f32((N, H, W, C_in), seed)
    w = inputs.normal_f32((C_out, R, S, C_in), seed + 1, (2.0 / (C_in * R * S)) ** 0.5)
    b = inputs.normal_f32((C_out,), seed + 2, 0.5)
    relu = bool(seed & 1)
    y_ref, d = oracle.conv2d_nhwc(x, w, stride, pad, dil, b, relu)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_nhwc(dev(torch, x), dev(torch, w), stride, pad, dil, dev(torch, b), relu, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"nhwc fp32 {case} ({sw.sw_last_kernel()})")


@pytest.mark.parametrize("half", [False, True], ids=["bf16", "f16"])
@pytest.mark.parametrize("case", _nhwc_cases(82, 40), ids=lambda c: "x".join(map(str, c[:10])))
def test_conv2d_nhwc_16bit_random(torch, sw, oracle, case, half):
    N, H, W, C_in, C_out, R, S, stride, pad, dil, seed = case
    if not _fits(H, W, R, S, pad, dil):
        dil = 1
    gen = inputs.normal_f16 if half else inputs.normal_bf16
    xb = gen((N, H, W, C_in), seed)
    wb = gen((C_out, R, S, C_in), seed + 1, (2.0 / (C_in * R * S)) ** 0.5)
    b = inputs.normal_f32((C_out,), seed + 2, 0.5)
    relu = bool(seed & 1)
    ref = oracle.conv2d_f16_nhwc if half else oracle.conv2d_bf16_nhwc
    y_ref, d = ref(xb, wb, stride, pad, dil, b, relu)
    tdt = torch.float16 if half else torch.bfloat16
    as_t = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(tdt)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, tdt, fill=77)
    (sw.sw_conv2d_f16_nhwc if half else sw.sw_conv2d_bf16_nhwc)(as_t(xb), as_t(wb), stride, pad, dil, dev(torch, b), relu, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    bits = out.view(torch.int16).cpu().numpy().view(np.uint16)
    y = (oracle.f16_to_f32(bits) if half else oracle.bf16_to_f32(bits)).astype(np.float64)
    # fp32 sums (2e-5 D) and one rounding of the result to the 16-bit format (half a unit in the last place)
    ulp = 2.0 ** -11 if half else 2.0 ** -8
    floor = 2.0 ** -25 if half else 1e-37
    assert np.all(np.abs(y - y_ref) <= 2e-5 * d + ulp * np.abs(y_ref) + floor), f"nhwc 16-bit {case} ({sw.sw_last_kernel()})"


@pytest.mark.parametrize("case", _nhwc_cases(83, 40), ids=lambda c: "x".join(map(str, c[:9])))
def test_conv2d_s8_nhwc_random(torch, sw, oracle, case):
    N, H, W, C_in, C_out, R, S, stride, pad, _, seed = case
    x = inputs.uniform_s8((N, H, W, C_in), seed)
    w = inputs.uniform_s8((C_out, R, S, C_in), seed + 1)
    y_ref = oracle.conv2d_s8_nhwc(x, w, stride, pad)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.int32)
    sw.sw_conv2d_s8_nhwc(dev(torch, x), dev(torch, w), stride, pad, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert np.array_equal(out.cpu().numpy(), y_ref), f"s8 nhwc {case} ({sw.sw_last_kernel()})"
    rng = np.random.default_rng(seed)
    std = (C_in * R * S) ** 0.5 * 5461.0
    bias = rng.integers(-int(std), int(std), size=C_out).astype(np.int32)
    scale = (rng.uniform(0.5, 2.0, size=C_out) * 60.0 / std).astype(np.float32)
    relu = bool(seed & 1)
    q_ref = oracle.conv2d_s8_nhwc_requant(x, w, bias, scale, stride, pad, relu)
    buf, out, front, n, s = guarded_empty(torch, q_ref.shape, torch.int8, fill=77)
    sw.sw_conv2d_s8_nhwc(dev(torch, x), dev(torch, w), stride, pad, bias=dev(torch, bias), scale=dev(torch, scale), relu=relu, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert np.array_equal(out.cpu().numpy(), q_ref), f"s8 nhwc requant {case} ({sw.sw_last_kernel()})"
