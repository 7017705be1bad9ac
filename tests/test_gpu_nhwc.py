"""GPU parity of the channel-last int8 convolution (sw_conv2d_s8_nhwc, int32 and requantised int8 output) against
the CPU oracle: bit-exact."""
import numpy as np
import pytest

from paper_2310_05218_amd import inputs
from parity import assert_guards_intact, guarded_empty

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


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


CASES = [
    # N, H, W, C_in, C_out, R, S, stride, pad, kernel (int32 out; the int8-out call runs its requantising twin:
    # mfma_s8q_nhwc_lds_kernel with the same arguments, mfma_s8_nhwc_kernel<1,KS>, direct_s8_nhwc_kernel<1>)
    (2, 28, 28, 128, 128, 3, 3, 1, 1, "mfma_s8_nhwc_lds_kernel<2,1,1,4>"),   # workload 5's layer, channel-last
    (1, 28, 28, 32, 64, 3, 3, 1, 1, "mfma_s8_nhwc_lds_kernel<2,1,1,4>"),     # one K step
    (2, 14, 14, 64, 96, 3, 3, 1, 1, "mfma_s8_nhwc_lds_kernel<2,1,1,7>"),     # the whole image in one tile, ragged channel block
    (1, 56, 56, 64, 64, 3, 3, 1, 1, "mfma_s8_nhwc_lds_kernel<2,1,1,2>"),     # 2-row tiles
    (2, 30, 41, 32, 40, 3, 3, 1, 1, "mfma_s8_nhwc_lds_kernel<2,1,1,3>"),     # blocks of 32 pixels that span rows, ragged last block
    (1, 57, 57, 64, 128, 3, 3, 2, 1, "mfma_s8_nhwc_lds_kernel<2,1,1,4>"),    # stride 2
    (1, 20, 20, 32, 32, 5, 5, 1, 2, "mfma_s8_nhwc_lds_kernel<1,1,1,5>"),     # 25 taps
    (2, 19, 23, 64, 70, 1, 1, 1, 0, "mfma_s8_nhwc_kernel<0,2>"),     # pointwise, an output channel count off the grid of four: window copied through registers
    (1, 33, 17, 32, 5, 7, 3, 2, 3, "mfma_s8_nhwc_kernel<0,1>"),      # rectangular filter, few output channels
    (1, 14, 14, 128, 30, 3, 3, 1, 1, "mfma_s8_nhwc_kernel<0,4>"),    # four K steps per tap in the register-copy kernel
    (1, 10, 10, 256, 6, 1, 1, 1, 0, "mfma_s8_nhwc_kernel<0,0>"),     # its run-time K loop
    (1, 9, 300, 32, 64, 3, 3, 1, 1, "direct_s8_nhwc_kernel<0>"),     # rows wider than 256 outputs: one thread per output
    (1, 12, 12, 24, 16, 3, 3, 1, 1, "direct_s8_nhwc_kernel<0>"),     # C_in not a multiple of 32: one thread per output
    (1, 5, 5, 32, 8, 5, 5, 1, 0, "mfma_s8_nhwc_lds_kernel<1,1,1,1>"),        # a single output pixel
    (32, 28, 28, 128, 128, 3, 3, 1, 1, "mfma_s8_nhwc_lds_kernel<2,2,1,7>"),  # workload 5 at full size: two pixel blocks per wavefront
    (4, 14, 14, 256, 64, 3, 3, 1, 1, "mfma_s8_nhwc_lds_kernel<1,1,1,7>"),    # one channel block per workgroup
    (2, 14, 14, 512, 64, 3, 3, 1, 1, "mfma_s8_nhwc_lds_kernel<12,1,1,7>"),   # filters fetched per chunk with the window
    (8, 56, 56, 64, 256, 1, 1, 1, 0, "mfma_s8_nhwc_lds_kernel<2,1,1,2>"),    # pointwise, four channel-block rows of workgroups
    (5, 7, 7, 64, 64, 3, 3, 1, 1, "mfma_s8_nhwc_lds_kernel<2,1,2,7>"),       # whole small images, two per tile, the last tile short
    (1, 12, 12, 32, 36, 3, 3, 1, 1, "mfma_s8_nhwc_lds_kernel<2,1,1,6>"),     # C_out % 16 != 0: int8 results leave in 4-byte stores
    (3, 9, 9, 96, 44, 3, 3, 2, 1, "mfma_s8_nhwc_lds_kernel<2,1,3,5>"),       # three images per tile, stride 2, three chunks
]


def _requant_twin(kernel):
    return (kernel.replace("mfma_s8_nhwc_lds_kernel", "mfma_s8q_nhwc_lds_kernel").replace("mfma_s8_nhwc_kernel<0,", "mfma_s8_nhwc_kernel<1,")
            .replace("direct_s8_nhwc_kernel<0>", "direct_s8_nhwc_kernel<1>"))


@pytest.mark.parametrize("case", CASES, ids=lambda c: "x".join(map(str, c[:9])))
def test_s8_nhwc_is_bit_exact(torch, sw, oracle, case):
    N, H, W, C_in, C_out, R, S, stride, pad, kernel = case
    x = inputs.uniform_s8((N, H, W, C_in), 5001)
    w = inputs.uniform_s8((C_out, R, S, C_in), 5002)
    y_ref = oracle.conv2d_s8_nhwc(x, w, stride, pad)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.int32)
    sw.sw_conv2d_s8_nhwc(dev(torch, x), dev(torch, w), stride, pad, out=out)
    assert sw.sw_last_kernel() == kernel, sw.sw_last_kernel()
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert np.array_equal(out.cpu().numpy(), y_ref), f"s8 nhwc {case}"


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "x".join(map(str, c[:9])))
def test_s8_nhwc_requant_is_bit_exact(torch, sw, oracle, case, relu):
    N, H, W, C_in, C_out, R, S, stride, pad, kernel = case
    x = inputs.uniform_s8((N, H, W, C_in), 5011)
    w = inputs.uniform_s8((C_out, R, S, C_in), 5012)
    rng = np.random.default_rng(5013)
    std = (C_in * R * S) ** 0.5 * 5461.0                       # of a sum of products of two uniform int8
    bias = rng.integers(-int(std), int(std), size=C_out).astype(np.int32)
    scale = (rng.uniform(0.5, 2.0, size=C_out) * 60.0 / std).astype(np.float32)
    q_ref = oracle.conv2d_s8_nhwc_requant(x, w, bias, scale, stride, pad, relu)
    buf, out, front, n, s = guarded_empty(torch, q_ref.shape, torch.int8, fill=77)
    sw.sw_conv2d_s8_nhwc(dev(torch, x), dev(torch, w), stride, pad, bias=dev(torch, bias), scale=dev(torch, scale),
                         relu=relu, out=out)
    assert sw.sw_last_kernel() == _requant_twin(kernel), sw.sw_last_kernel()
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    q = out.cpu().numpy()
    assert np.array_equal(q, q_ref), f"s8 nhwc requant {case} relu={relu}"
    assert len(np.unique(q)) > (50 if q.size > 2000 else 5)


def test_s8_nhwc_extremes(torch, sw, oracle):
    """All -128: every product is +16384, the largest sum a 3x3 x 128-channel layer can reach."""
    x = np.full((1, 8, 8, 128), -128, np.int8)
    w = np.full((64, 3, 3, 128), -128, np.int8)
    y = sw.sw_conv2d_s8_nhwc(dev(torch, x), dev(torch, w), 1, 1).cpu().numpy()
    assert y.max() == 9 * 128 * 16384 and np.array_equal(y, oracle.conv2d_s8_nhwc(x, w, 1, 1))


def test_s8_nhwc_full_size_agrees_with_the_channel_first_call(torch, sw, oracle):
    """Workload 5 at full size in both layouts: the two entry points must give the same sums; sampled images are
    also checked against the oracle."""
    x, w = inputs.workload5()
    xd, wd = dev(torch, x), dev(torch, w)
    y_cf = sw.sw_conv2d_s8(xd, wd, 1, 1)
    y_cl = sw.sw_conv2d_s8_nhwc(xd.permute(0, 2, 3, 1).contiguous(), wd.permute(0, 2, 3, 1).contiguous(), 1, 1)
    assert torch.equal(y_cl.permute(0, 3, 1, 2), y_cf)
    for n in (0, 31):
        assert np.array_equal(y_cf[n:n + 1].cpu().numpy(), oracle.conv2d_s8(x[n:n + 1], w, 1, 1))


# ----------------------------------------------------------------------------- fp32 and bf16, channel-last

FLOAT_CASES = [
    # N, H, W, C_in, C_out, R, S, stride, pad, dilation, kernel for fp32, kernel for bf16 (the window-in-LDS kernel:
    # <channel blocks per workgroup, pixel blocks per wavefront, images per tile, rows per tile>)
    (2, 28, 28, 64, 64, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,4>", "mfma_bf16_nhwc_lds_kernel<2,1,1,4>"),    # two fp32 chunks of 32 channels, one bf16 chunk
    (1, 56, 56, 32, 64, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,2>", "mfma_bf16_nhwc_lds_kernel<2,1,1,2>"),    # 4-row bands (224 pixels)
    (2, 14, 14, 128, 96, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,7>", "mfma_bf16_nhwc_lds_kernel<1,1,1,7>"),   # four / two chunks, ragged channel block
    (2, 30, 41, 16, 40, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,3>", "mfma_bf16_nhwc_lds_kernel<2,1,1,3>"),    # blocks that span rows, ragged last block
    (1, 57, 57, 64, 128, 3, 3, 2, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,2>", "mfma_bf16_nhwc_lds_kernel<2,1,1,1>"),   # stride 2
    (1, 20, 20, 16, 32, 5, 5, 1, 2, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,5>", "mfma_bf16_nhwc_lds_kernel<1,1,1,5>"),    # 25 taps: two rounds of filter pieces
    (1, 12, 12, 48, 64, 7, 7, 1, 3, 1, "mfma_nhwc_kernel<0,1>", "mfma_bf16_nhwc_direct_kernel<1,2>"),    # 49 taps: LDS bounds the chunk
    (2, 19, 23, 64, 70, 1, 1, 1, 0, 1, "mfma_nhwc_kernel<0,4>", "mfma_nhwc_kernel<1,4>"),    # pointwise
    (1, 33, 17, 16, 5, 7, 3, 2, 3, 1, "mfma_nhwc_kernel<0,2>", "mfma_nhwc_kernel<1,1>"),     # rectangular filter, few output channels
    (1, 28, 28, 32, 64, 3, 3, 1, 2, 2, "mfma_f32_nhwc_lds_kernel<11,1,1,4>", "mfma_bf16_nhwc_lds_kernel<2,1,1,4>"),    # dilation 2
    (1, 40, 40, 16, 64, 3, 3, 2, 6, 6, "mfma_f32_nhwc_lds_kernel<11,1,1,1>", "mfma_bf16_nhwc_lds_kernel<2,1,1,5>"),    # dilation 6 with stride 2
    (1, 9, 300, 16, 64, 3, 3, 1, 1, 1, "direct_nhwc_kernel<0>", "mfma_bf16_nhwc_direct_kernel<1,2>"),    # rows wider than 256 outputs
    (1, 12, 12, 12, 16, 3, 3, 1, 1, 1, "direct_nhwc_kernel<0>", "direct_nhwc_kernel<1>"),    # pixels that are not whole K steps
    (1, 12, 12, 8, 16, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,6>", "direct_nhwc_kernel<1>"),     # 32 bytes per pixel in fp32, 16 in bf16
    (1, 5, 5, 16, 8, 5, 5, 1, 0, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,1>", "mfma_bf16_nhwc_lds_kernel<1,1,1,1>"),       # a single output pixel
    (16, 56, 56, 32, 64, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<12,2,1,4>", "mfma_bf16_nhwc_lds_kernel<2,2,1,4>"),   # enough tiles for two channel blocks per wavefront
    (3, 21, 21, 48, 36, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,6>", "mfma_bf16_nhwc_lds_kernel<2,1,1,6>"),    # three K steps per tap (27 iterations), ragged channel block
    (2, 16, 16, 32, 64, 2, 2, 1, 0, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,8>", "mfma_bf16_nhwc_lds_kernel<2,1,1,8>"),    # 8 iterations: two left over after the ring's trips
    (1, 20, 20, 32, 30, 3, 3, 1, 1, 1, "mfma_nhwc_kernel<0,4>", "mfma_nhwc_kernel<1,2>"),    # an output channel count the 8-byte stores do not take: window in LDS
    (5, 7, 7, 32, 64, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,2,7>", "mfma_bf16_nhwc_lds_kernel<2,1,2,7>"),        # whole small images, several per tile, the last tile short
    (9, 4, 4, 64, 40, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,5,4>", "mfma_bf16_nhwc_lds_kernel<2,1,5,4>"),    # five 4 x 4 images per tile, 9 = 5 + 4
    # filters too large to stay in LDS whole: the window-in-LDS kernel fetches each chunk's part with the window (first
    # number + 10)
    (2, 14, 14, 160, 64, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,7>", "mfma_bf16_nhwc_lds_kernel<12,1,1,7>"),   # ten chunks of 16 channels
    (1, 16, 16, 320, 32, 2, 2, 1, 0, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,8>", "mfma_bf16_nhwc_lds_kernel<11,1,1,8>"),   # one channel block, 2 x 2
    (32, 28, 28, 128, 128, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<12,2,1,7>", "mfma_bf16_nhwc_lds_kernel<12,2,1,7>"),  # two pixel blocks per wavefront
    (4, 7, 7, 256, 64, 3, 3, 1, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,2,7>", "mfma_bf16_nhwc_lds_kernel<12,1,2,7>"),     # two images per tile
    (1, 15, 15, 192, 44, 3, 3, 2, 1, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,8>", "mfma_bf16_nhwc_lds_kernel<12,1,1,8>"),   # stride 2, ragged channel block
    (1, 14, 14, 144, 64, 3, 3, 1, 2, 2, "mfma_f32_nhwc_lds_kernel<11,1,1,7>", "mfma_bf16_nhwc_lds_kernel<12,1,1,7>"),   # dilation 2, nine chunks
    (2, 10, 10, 96, 64, 5, 5, 1, 2, 1, "mfma_f32_nhwc_lds_kernel<11,1,1,10>", "mfma_bf16_nhwc_lds_kernel<11,1,1,10>"),   # 25 taps
    # single taps, where fp32 keeps its filters resident as well (its other cases fetch them per chunk)
    (8, 56, 56, 64, 64, 1, 1, 1, 0, 1, "mfma_f32_nhwc_lds_kernel<2,1,1,2>", "mfma_bf16_nhwc_lds_kernel<2,1,1,2>"),
    (16, 14, 14, 64, 96, 1, 1, 1, 0, 1, "mfma_f32_nhwc_lds_kernel<1,1,1,4>", "mfma_bf16_nhwc_lds_kernel<2,1,1,7>"),
    (32, 56, 56, 256, 64, 1, 1, 1, 0, 1, "mfma_f32_nhwc_lds_kernel<2,2,1,4>", "mfma_bf16_nhwc_lds_kernel<2,1,1,2>"),   # eight chunks of 32 channels, two pixel blocks per wavefront
    # rows too wide for a window tile: operands straight from global memory
    (1, 4, 300, 160, 32, 3, 3, 1, 1, 1, "direct_nhwc_kernel<0>", "mfma_bf16_nhwc_direct_kernel<1,2>"),     # ten K steps per tap (90 iterations)
    (1, 3, 300, 320, 32, 2, 2, 1, 0, 1, "direct_nhwc_kernel<0>", "mfma_bf16_nhwc_direct_kernel<1,2>"),     # 80 iterations: two left over after the ring's trips
    (20, 9, 300, 16, 64, 3, 3, 1, 1, 1, "direct_nhwc_kernel<0>", "mfma_bf16_nhwc_direct_kernel<2,2>"),     # enough tiles for two channel blocks per wavefront
]


@pytest.mark.parametrize("case", FLOAT_CASES, ids=lambda c: "x".join(map(str, c[:10])))
def test_conv2d_nhwc_fp32(torch, sw, oracle, case):
    N, H, W, C_in, C_out, R, S, stride, pad, dil, kernel, _ = case
    x = inputs.normal_f32((N, H, W, C_in), 5201)
    w = inputs.normal_f32((C_out, R, S, C_in), 5202, (2.0 / (C_in * R * S)) ** 0.5)
    b = inputs.normal_f32((C_out,), 5203, 0.5)
    for bias, relu in ((None, False), (b, True)):
        y_ref, d = oracle.conv2d_nhwc(x, w, stride, pad, dil, bias, relu)
        buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
        sw.sw_conv2d_nhwc(dev(torch, x), dev(torch, w), stride, pad, dil, None if bias is None else dev(torch, bias), relu,
                          out=out)
        assert sw.sw_last_kernel() == kernel, sw.sw_last_kernel()
        torch.cuda.synchronize()
        assert_guards_intact(buf, front, n, s)
        err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - y_ref) / np.maximum(d, 1e-300)))
        assert err <= 2e-5, f"nhwc fp32 {case} relu={relu}: normalised error {err:.3e}"


@pytest.mark.parametrize("case", FLOAT_CASES, ids=lambda c: "x".join(map(str, c[:10])))
def test_conv2d_nhwc_bf16(torch, sw, oracle, case):
    """bf16 in and out, fp32 accumulation: |y - oracle| <= 2e-5 * D (the fp32 sums) + 2^-8 |oracle| (one rounding of the
    result to bf16: half a unit in the last of 8 significant bits)."""
    N, H, W, C_in, C_out, R, S, stride, pad, dil, _, kernel = case
    xb = inputs.normal_bf16((N, H, W, C_in), 5211)
    wb = inputs.normal_bf16((C_out, R, S, C_in), 5212, (2.0 / (C_in * R * S)) ** 0.5)
    b = inputs.normal_f32((C_out,), 5213, 0.5)
    as_bf16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    for bias, relu in ((None, False), (b, True)):
        y_ref, d = oracle.conv2d_bf16_nhwc(xb, wb, stride, pad, dil, bias, relu)
        n = y_ref.size
        buf = torch.full((128 + n + 64,), 12345.0, dtype=torch.bfloat16, device="cuda")
        out = buf[128:128 + n].view(y_ref.shape)
        sw.sw_conv2d_bf16_nhwc(as_bf16(xb), as_bf16(wb), stride, pad, dil, None if bias is None else dev(torch, bias), relu,
                               out=out)
        assert sw.sw_last_kernel() == kernel, sw.sw_last_kernel()
        torch.cuda.synchronize()
        guard = buf.view(torch.int16)
        assert bool((guard[:128] == guard[0]).all()) and bool((guard[128 + n:] == guard[0]).all()), "write outside y"
        y = oracle.bf16_to_f32(out.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
        assert np.all(np.abs(y - y_ref) <= 2e-5 * d + 2.0 ** -8 * np.abs(y_ref) + 1e-37), \
            f"nhwc bf16 {case} relu={relu}: max excess {np.max(np.abs(y - y_ref) - 2e-5 * d - 2.0 ** -8 * np.abs(y_ref)):.3e}"


def _f16_case(torch, sw, oracle, xh, wh, stride, pad, dil, bias, relu, kernel, what):
    """One half-precision call against the oracle: |y - oracle| <= 2e-5 * D (the fp32 sums) + 2^-11 |oracle| (one rounding
    to half precision: half a unit in the last of 11 significant bits) + 2^-25 (half the spacing of its denormals)."""
    as_f16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    y_ref, d = oracle.conv2d_f16_nhwc(xh, wh, stride, pad, dil, bias, relu)
    n = y_ref.size
    buf = torch.full((128 + n + 64,), 12345.0, dtype=torch.float16, device="cuda")
    out = buf[128:128 + n].view(y_ref.shape)
    sw.sw_conv2d_f16_nhwc(as_f16(xh), as_f16(wh), stride, pad, dil, None if bias is None else dev(torch, bias), relu, out=out)
    if kernel is not None:
        assert sw.sw_last_kernel() == kernel, sw.sw_last_kernel()
    torch.cuda.synchronize()
    guard = buf.view(torch.int16)
    assert bool((guard[:128] == guard[0]).all()) and bool((guard[128 + n:] == guard[0]).all()), "write outside y"
    y = oracle.f16_to_f32(out.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    bound = 2e-5 * d + 2.0 ** -11 * np.abs(y_ref) + 2.0 ** -25
    assert np.all(np.abs(y - y_ref) <= bound), f"nhwc f16 {what} relu={relu}: max excess {np.max(np.abs(y - y_ref) - bound):.3e}"
    return y, y_ref


@pytest.mark.parametrize("case", FLOAT_CASES, ids=lambda c: "x".join(map(str, c[:10])))
def test_conv2d_nhwc_f16(torch, sw, oracle, case):
    """IEEE half precision in and out, fp32 accumulation, on every shape of the bf16 cases (the same kernels with the
    half-precision matrix instruction and rounding)."""
    N, H, W, C_in, C_out, R, S, stride, pad, dil, _, kernel = case
    kernel = kernel.replace("mfma_bf16_nhwc_direct", "mfma_f16_nhwc_direct").replace("mfma_bf16_nhwc_lds", "mfma_f16_nhwc_lds").replace("mfma_nhwc_kernel<1,", "mfma_nhwc_kernel<2,") \
        .replace("direct_nhwc_kernel<1>", "direct_nhwc_kernel<2>")
    xh = inputs.normal_f16((N, H, W, C_in), 5231)
    wh = inputs.normal_f16((C_out, R, S, C_in), 5232, (2.0 / (C_in * R * S)) ** 0.5)
    b = inputs.normal_f32((C_out,), 5233, 0.5)
    for bias, relu in ((None, False), (b, True)):
        _f16_case(torch, sw, oracle, xh, wh, stride, pad, dil, bias, relu, kernel, case)


@pytest.mark.parametrize("shape", [(2, 14, 14, 32, 32, "mfma_f16_nhwc_lds_kernel<1,1,1,7>"), (1, 9, 9, 160, 32, "mfma_f16_nhwc_lds_kernel<11,1,1,9>"),
                                   (1, 3, 300, 160, 32, "mfma_f16_nhwc_direct_kernel<1,2>"),
                                   (1, 14, 14, 32, 30, "mfma_nhwc_kernel<2,2>"), (1, 9, 9, 12, 8, "direct_nhwc_kernel<2>")], ids=lambda s: s[5])
def test_conv2d_nhwc_f16_denormals_and_overflow(torch, sw, oracle, shape):
    """What half precision has and bf16 has not: denormal inputs count (activations of about 2^-16 against filters of
    about 2^6: were the denormals flushed the sums would vanish), results below 2^-14 are kept as denormals, results
    beyond 65504 become infinities of the right sign."""
    N, H, W, C_in, C_out, kernel = shape
    x_small = inputs.normal_f16((N, H, W, C_in), 5241, 2.0 ** -16)
    assert np.mean((x_small & 0x7C00) == 0) > 0.9                      # nearly all denormal
    w_big = inputs.normal_f16((C_out, 3, 3, C_in), 5242, 64.0)
    y, y_ref = _f16_case(torch, sw, oracle, x_small, w_big, 1, 1, 1, None, False, kernel, "denormal x")
    assert np.median(np.abs(y_ref)) > 2.0 ** -10 and np.count_nonzero(y) > 0.99 * y.size
    w_small = inputs.normal_f16((C_out, 3, 3, C_in), 5243, 2.0 ** -6 * (32.0 / max(C_in, 32)) ** 0.5)
    y, y_ref = _f16_case(torch, sw, oracle, x_small, w_small, 1, 1, 1, None, False, kernel, "denormal y")
    assert np.max(np.abs(y_ref)) < 2.0 ** -14 and np.count_nonzero(y) > 0.5 * y.size
    # overflow: every product 200 * 200, so a full window sums to 9 * C_in * 40000 > 65504; the sign follows the filter
    as_f16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    xo = np.full((N, H, W, C_in), 200.0, np.float16).view(np.uint16)
    wo = np.full((C_out, 3, 3, C_in), 200.0, np.float16)
    wo[1::2] = -200.0
    out = sw.sw_conv2d_f16_nhwc(as_f16(xo), as_f16(wo.view(np.uint16)), 1, 1)
    assert sw.sw_last_kernel() == kernel
    yo = out.float().cpu().numpy()
    y_ref, _ = oracle.conv2d_f16_nhwc(xo, wo.view(np.uint16), 1, 1)
    with np.errstate(over="ignore"):
        assert np.array_equal(yo, y_ref.astype(np.float16).astype(np.float32)) and np.isinf(yo).all()
    assert (yo[..., 0::2] > 0).all() and (yo[..., 1::2] < 0).all()


def test_nhwc_is_the_channel_first_call_on_permuted_tensors(torch, sw):
    """Same sums, other layout: the two fp32 entry points agree to rounding order on a layer both take."""
    x = inputs.normal_f32((2, 64, 28, 28), 5221)
    w = inputs.normal_f32((64, 64, 3, 3), 5222, 0.06)
    y_cf = sw.sw_conv2d(dev(torch, x), dev(torch, w), 1, 1).cpu().numpy()
    y_cl = sw.sw_conv2d_nhwc(dev(torch, x.transpose(0, 2, 3, 1)), dev(torch, w.transpose(0, 2, 3, 1)), 1, 1).cpu().numpy()
    assert np.allclose(y_cl.transpose(0, 3, 1, 2), y_cf, rtol=0, atol=2e-5 * 40)


# ----------------------------------------------------------------------------- views that are only element-aligned

def _offset_view(torch, a, off):
    """A copy of `a` that starts `off` elements into a fresh allocation (element-aligned, not 16-byte aligned)."""
    flat = torch.empty(a.numel() + off + 8, dtype=a.dtype, device="cuda")
    v = flat[off:off + a.numel()].view(a.shape)
    v.copy_(a)
    return v


@pytest.mark.parametrize("which", ["x", "w", "y"])
def test_conv2d_nhwc_element_aligned_views(torch, sw, oracle, which):
    """The matrix-core kernels want 16-byte aligned operands; a view that is only element-aligned must still give the
    oracle's result (through whichever kernel takes it), in every format, and write nothing outside y."""
    N, H, W, C_in, C_out = 2, 14, 14, 64, 64
    x = inputs.normal_f32((N, H, W, C_in), 5301)
    w = inputs.normal_f32((C_out, 3, 3, C_in), 5302, 0.05)
    y_ref, d = oracle.conv2d_nhwc(x, w, 1, 1)
    xd, wd = dev(torch, x), dev(torch, w)
    if which == "x": xd = _offset_view(torch, xd, 1)
    if which == "w": wd = _offset_view(torch, wd, 1)
    n = y_ref.size
    off = 1 if which == "y" else 0
    buf = torch.full((64 + off + n + 64,), 12345.0, device="cuda")
    out = buf[64 + off:64 + off + n].view(y_ref.shape)
    sw.sw_conv2d_nhwc(xd, wd, 1, 1, out=out)
    torch.cuda.synchronize()
    assert bool((buf[:64 + off] == 12345.0).all()) and bool((buf[64 + off + n:] == 12345.0).all()), "write outside y"
    err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - y_ref) / np.maximum(d, 1e-300)))
    assert err <= 2e-5, f"fp32, {which} offset: {err:.3e} ({sw.sw_last_kernel()})"
    # bf16: one element is two bytes
    xb, wb = inputs.normal_bf16((N, H, W, C_in), 5303), inputs.normal_bf16((C_out, 3, 3, C_in), 5304, 0.05)
    yb_ref, db = oracle.conv2d_bf16_nhwc(xb, wb, 1, 1)
    as_bf16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    xt, wt = as_bf16(xb), as_bf16(wb)
    if which == "x": xt = _offset_view(torch, xt, 1)
    if which == "w": wt = _offset_view(torch, wt, 1)
    bufb = torch.full((64 + off + n + 64,), 77.0, dtype=torch.bfloat16, device="cuda")
    outb = bufb[64 + off:64 + off + n].view(yb_ref.shape)
    sw.sw_conv2d_bf16_nhwc(xt, wt, 1, 1, out=outb)
    torch.cuda.synchronize()
    assert bool((bufb[:64 + off] == 77.0).all()) and bool((bufb[64 + off + n:] == 77.0).all()), "write outside y (bf16)"
    yv = oracle.bf16_to_f32(outb.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    assert np.all(np.abs(yv - yb_ref) <= 2e-5 * db + 2.0 ** -8 * np.abs(yb_ref) + 1e-37), f"bf16, {which} offset ({sw.sw_last_kernel()})"
    # int8 in, int32 out
    xs, ws = inputs.uniform_s8((N, H, W, C_in), 5305), inputs.uniform_s8((C_out, 3, 3, C_in), 5306)
    ys_ref = oracle.conv2d_s8_nhwc(xs, ws, 1, 1)
    xq, wq = dev(torch, xs), dev(torch, ws)
    if which == "x": xq = _offset_view(torch, xq, 1)
    if which == "w": wq = _offset_view(torch, wq, 1)
    bufs = torch.full((64 + off + n + 64,), 12345, dtype=torch.int32, device="cuda")
    outs = bufs[64 + off:64 + off + n].view(ys_ref.shape)
    sw.sw_conv2d_s8_nhwc(xq, wq, 1, 1, out=outs)
    torch.cuda.synchronize()
    assert bool((bufs[:64 + off] == 12345).all()) and bool((bufs[64 + off + n:] == 12345).all()), "write outside y (int8)"
    assert np.array_equal(outs.cpu().numpy(), ys_ref), f"int8, {which} offset ({sw.sw_last_kernel()})"


@pytest.mark.parametrize("shape", [(2, 14, 14, 64, 64, "mfma_s8q_nhwc_lds_kernel"), (1, 10, 10, 64, 6, "mfma_s8_nhwc_kernel")],
                         ids=lambda s: s[5])
def test_s8_nhwc_requant_without_bias(torch, sw, oracle, shape):
    """scale without a bias: the requantisation adds nothing before it scales (a null bias pointer in the C call)."""
    N, H, W, C_in, C_out, kernel = shape
    x = inputs.uniform_s8((N, H, W, C_in), 5401)
    w = inputs.uniform_s8((C_out, 3, 3, C_in), 5402)
    scale = np.full((C_out,), 60.0 / ((C_in * 9) ** 0.5 * 5461.0), np.float32)
    q_ref = oracle.conv2d_s8_nhwc_requant(x, w, np.zeros(C_out, np.int32), scale, 1, 1, False)
    buf, out, front, n, s = guarded_empty(torch, q_ref.shape, torch.int8, fill=77)
    sw.sw_conv2d_s8_nhwc(dev(torch, x), dev(torch, w), 1, 1, scale=dev(torch, scale), out=out)
    assert sw.sw_last_kernel().startswith(kernel), sw.sw_last_kernel()
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert np.array_equal(out.cpu().numpy(), q_ref)


@pytest.mark.parametrize("N,kernel", [(63, "mfma_bf16_nhwc_lds_kernel"), (64, "mfma_nhwc_kernel<1,")], ids=["below", "at"])
def test_conv2d_bf16_nhwc_around_two_gib(torch, sw, oracle, N, kernel):
    """x of 2.11e9 bytes, just below the 2 GiB the buffer descriptors of the window-in-LDS kernel address (byte offsets up
    to 2^31 - 3.6e7 in its unsigned arithmetic), and x of exactly 2 GiB, which that kernel must leave to the one that
    addresses image by image in 64 bits.  A 1 x 1 filter, so that sampled output pixels can be checked by the oracle on
    the sampled input pixels alone (the pixels as a 1 x P image)."""
    H, W, C_in, C_out = 128, 128, 1024, 8
    g = torch.Generator(device="cuda"); g.manual_seed(5501)
    x = torch.empty((N, H, W, C_in), device="cuda", dtype=torch.bfloat16)
    for n in range(N):                                               # (image by image: no 4 GiB fp32 temporary)
        x[n] = torch.randn((H, W, C_in), generator=g, device="cuda").bfloat16()
    w = (torch.randn((C_out, 1, 1, C_in), generator=g, device="cuda") * 0.03).bfloat16()
    assert (x.numel() * 2 < 2 ** 31) == (N == 63) and x.numel() * 2 > 2.1e9
    y = sw.sw_conv2d_bf16_nhwc(x, w, 1, 0)
    assert sw.sw_last_kernel().startswith(kernel), sw.sw_last_kernel()
    torch.cuda.synchronize()
    rng = np.random.default_rng(5502)
    P = 512
    idx = np.stack([rng.integers(0, N, P), rng.integers(0, H, P), rng.integers(0, W, P)], axis=1)
    idx[:4] = [[0, 0, 0], [N - 1, H - 1, W - 1], [N - 1, 0, 0], [N // 2, H - 1, 0]]          # the corners of the address range
    ti = torch.from_numpy(idx).cuda()
    xs = x[ti[:, 0], ti[:, 1], ti[:, 2]].view(torch.int16).cpu().numpy().view(np.uint16).reshape(1, 1, P, C_in)
    ys = y[ti[:, 0], ti[:, 1], ti[:, 2]].view(torch.int16).cpu().numpy().view(np.uint16).reshape(1, 1, P, C_out)
    wb = w.view(torch.int16).cpu().numpy().view(np.uint16)
    y_ref, d = oracle.conv2d_bf16_nhwc(xs, wb, 1, 0)
    yv = oracle.bf16_to_f32(ys).astype(np.float64)
    assert np.all(np.abs(yv - y_ref) <= 2e-5 * d + 2.0 ** -8 * np.abs(y_ref) + 1e-37)
    assert np.count_nonzero(yv) > 0.99 * yv.size
