"""GPU parity of the int8 convolution with filters packed once (sw_s8_pack_filter + sw_conv2d_s8_packed[_requant])
against the CPU oracle's plain int8 convolution on the unpacked filters: bit-exact, through the C ABI."""
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


BAND = "mfma_s8_band_kernel"        # full-width row bands (H * W a multiple of 16, at most 64 output columns)
FAST = "mfma_s8_packed_kernel"      # any other tiling of a 3x3 stride-1 problem
DIRECT = "direct_s8_packed_kernel"

PACKED_CASES = [
    # N, C_in, C_out, H, W, R, S, stride, pad, kernel
    (1, 128, 128, 28, 28, 3, 3, 1, 1, BAND),     # the quantised workload's layer, one image
    (2, 64, 64, 28, 28, 3, 3, 1, 1, BAND),
    (2, 32, 64, 28, 28, 3, 3, 1, 1, BAND),       # a single K step per tap
    (2, 64, 64, 56, 56, 3, 3, 1, 1, BAND),       # three-row bands, the last one ragged
    (1, 128, 64, 56, 56, 3, 3, 1, 1, BAND),      # ... the longest band per channel (19 pieces)
    (2, 128, 64, 20, 28, 3, 3, 1, 1, BAND),      # last row band ragged
    (1, 128, 64, 8, 8, 3, 3, 1, 1, BAND),        # one tile, two blocks
    (1, 64, 128, 12, 16, 3, 3, 1, 0, BAND),      # valid mode: no padding cells at all
    (1, 32, 64, 4, 4, 3, 3, 1, 1, BAND),         # 16 pixels
    (1, 128, 64, 8, 64, 3, 3, 1, 1, BAND),       # 64 columns: two-row bands, the second wavefront pair idle
    (1, 64, 64, 16, 20, 3, 3, 1, 2, BAND),       # padding wider than the filter needs, 22 output columns
    (1, 128, 64, 16, 36, 3, 3, 1, 1, BAND),      # six-row bands: seven blocks, the last one partial
    (3, 128, 128, 28, 28, 3, 3, 1, 1, BAND),
    (1, 128, 64, 13, 20, 3, 3, 1, 1, FAST),      # ragged row bands
    (1, 64, 128, 30, 12, 3, 3, 1, 0, FAST),      # valid mode
    (1, 64, 64, 9, 100, 3, 3, 1, 1, FAST),       # two column tiles
    (1, 128, 64, 18, 200, 3, 3, 1, 1, FAST),     # four staging items per thread
    (1, 128, 64, 7, 8, 3, 3, 1, 2, FAST),        # padding wider than the filter needs
    (2, 128, 64, 21, 28, 3, 3, 1, 1, FAST),      # last row band ragged
    (1, 128, 128, 9, 12, 3, 3, 1, 0, FAST),      # tile with a single live pixel block pair
    (1, 128, 64, 5, 40, 3, 3, 1, 1, FAST),       # odd block count
    (1, 32, 128, 3, 4, 3, 3, 1, 0, FAST),        # a single output row of two pixels
    (1, 64, 128, 30, 9, 3, 3, 1, 0, DIRECT),     # width not a multiple of 4
    (1, 128, 64, 13, 17, 3, 3, 1, 1, DIRECT),
    (1, 192, 64, 10, 12, 3, 3, 1, 1, DIRECT),    # C_in outside the resident kernel's set
    (1, 64, 64, 16, 16, 3, 3, 2, 1, DIRECT),     # stride 2
    (2, 40, 33, 12, 15, 5, 3, 1, 2, DIRECT),     # ragged channel counts (zero-filled in the packed copy)
    (1, 30, 16, 16, 16, 1, 1, 1, 0, DIRECT),
    (1, 3, 70, 9, 11, 2, 5, 2, 2, DIRECT),
]


@pytest.mark.parametrize("case", PACKED_CASES, ids=lambda c: "x".join(map(str, c[:9])))
def test_conv2d_s8_packed(torch, sw, oracle, case):
    N, C_in, C_out, H, W, R, S, stride, pad, kernel = case
    x = inputs.uniform_s8((N, C_in, H, W), 5101)
    w = inputs.uniform_s8((C_out, C_in, R, S), 5102)
    y_ref = oracle.conv2d_s8(x, w, stride, pad)
    nbytes = sw.sw_s8_packed_filter_bytes(C_in, C_out, R, S)
    assert nbytes == -(-C_out // 32) * R * S * -(-C_in // 32) * 1024
    pbuf, packed, pfront, pn, ps = guarded_empty(torch, (nbytes,), torch.int8, fill=55)
    sw.sw_s8_pack_filter(dev(torch, w), out=packed)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.int32)
    sw.sw_conv2d_s8_packed(dev(torch, x), packed, C_out, R, S, stride, pad, out=out)
    assert sw.sw_last_kernel().startswith(kernel), sw.sw_last_kernel()
    torch.cuda.synchronize()
    assert_guards_intact(pbuf, pfront, pn, ps)
    assert_guards_intact(buf, front, n, s)
    assert np.array_equal(out.cpu().numpy(), y_ref), f"packed s8 {case} is not bit-exact"


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("case", [
    (2, 128, 128, 28, 28, 3, 3, 1, 1, BAND),
    (1, 128, 64, 20, 28, 3, 3, 1, 1, BAND),      # ragged last row band
    (2, 64, 64, 28, 28, 3, 3, 1, 1, BAND),
    (1, 32, 64, 16, 36, 3, 3, 1, 1, BAND),       # two stores per step
    (1, 64, 64, 12, 28, 3, 3, 1, 0, BAND),       # output rows that are not whole dwords of int8: byte stores
    (1, 128, 64, 21, 28, 3, 3, 1, 1, FAST),
    (1, 32, 64, 9, 100, 3, 3, 1, 1, FAST),       # two column tiles, stores of four per step
    (1, 64, 64, 13, 28, 3, 3, 1, 0, FAST),       # byte stores
    (1, 40, 70, 12, 15, 3, 3, 2, 1, DIRECT),
], ids=lambda c: "x".join(map(str, c[:9])))
def test_conv2d_s8_packed_requant(torch, sw, oracle, case, relu):
    N, C_in, C_out, H, W, R, S, stride, pad, kernel = case
    x = inputs.uniform_s8((N, C_in, H, W), 5111)
    w = inputs.uniform_s8((C_out, C_in, R, S), 5112)
    rng = np.random.default_rng(5113)
    bias = rng.integers(-20000, 20000, size=C_out).astype(np.int32)
    std = np.sqrt(C_in * R * S) * 5461.0                   # of the sums: uniform int8 operands have variance 5461
    scale = (rng.uniform(0.5, 2.0, size=C_out) * 40.0 / std).astype(np.float32)
    scale[::3] = np.float32(2.0 ** np.round(np.log2(40.0 / std)))
    q_ref = oracle.conv2d_s8_requant(x, w, bias, scale, stride, pad, relu)
    packed = sw.sw_s8_pack_filter(dev(torch, w))
    buf, out, front, n, s = guarded_empty(torch, q_ref.shape, torch.int8, fill=77)
    sw.sw_conv2d_s8_packed(dev(torch, x), packed, C_out, R, S, stride, pad, dev(torch, bias), dev(torch, scale), relu,
                           out=out)
    assert sw.sw_last_kernel().startswith(kernel), sw.sw_last_kernel()
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    q = out.cpu().numpy()
    assert np.array_equal(q, q_ref), f"packed requant {case}: {np.count_nonzero(q != q_ref)} of {q.size} differ"
    q0 = sw.sw_conv2d_s8_packed(dev(torch, x), packed, C_out, R, S, stride, pad, None, dev(torch, scale), relu)
    assert np.array_equal(q0.cpu().numpy(), oracle.conv2d_s8_requant(x, w, None, scale, stride, pad, relu))


def test_workload5_full_size_packed(torch, sw, oracle):
    x, w = inputs.workload5()
    y_ref = oracle.conv2d_s8(x, w, 1, 1)
    packed = sw.sw_s8_pack_filter(dev(torch, w))
    y = sw.sw_conv2d_s8_packed(dev(torch, x), packed, 128, 3, 3, 1, 1)
    assert sw.sw_last_kernel() == "mfma_s8_band_kernel<4,0,0>"
    assert np.array_equal(y.cpu().numpy(), y_ref)
    # the packed copy depends on the filters only: a second, different batch with the same buffer
    x2 = inputs.uniform_s8((3, 128, 28, 28), 5121)
    y2 = sw.sw_conv2d_s8_packed(dev(torch, x2), packed, 128, 3, 3, 1, 1)
    assert np.array_equal(y2.cpu().numpy(), oracle.conv2d_s8(x2, w, 1, 1))


def test_packed_extremes(torch, sw):
    """All -128 * -128: every interior output of the quantised workload's layer is 128 * 9 * 16384."""
    x = np.full((1, 128, 28, 28), -128, np.int8)
    w = np.full((128, 128, 3, 3), -128, np.int8)
    packed = sw.sw_s8_pack_filter(dev(torch, w))
    y = sw.sw_conv2d_s8_packed(dev(torch, x), packed, 128, 3, 3, 1, 1).cpu().numpy()
    assert np.all(y[:, :, 1:-1, 1:-1] == 128 * 9 * 16384)
    assert np.all(y[:, :, 0, 0] == 128 * 4 * 16384)


@pytest.mark.parametrize("raw_filters", [False, True], ids=["packed", "caller-filters"])
@pytest.mark.parametrize("case", [
    # N, C_in, C_out, H, W, pad, byte offset of y8, store variant the band kernel must take
    (32, 128, 128, 28, 28, 1, 0, 2),    # the quantised workload at full size: through LDS, 16-byte pieces
    (2, 128, 64, 28, 28, 1, 0, 2),
    (3, 64, 128, 28, 28, 1, 0, 2),      # C_in = 64, no helper wavefronts
    (2, 64, 64, 56, 56, 1, 0, 2),       # several tiles per image, the last one ragged
    (1, 128, 64, 12, 16, 1, 0, 2),      # a single tile of six blocks
    (1, 64, 64, 20, 20, 1, 0, 2),       # 400 pixels: the last block holds 16
    (2, 128, 64, 28, 28, 1, 4, 1),      # y8 not 16-byte aligned: dword stores from the registers
    (2, 128, 64, 28, 28, 1, 1, 1),      # ... not even 4-byte aligned: byte stores
    (2, 64, 64, 28, 28, 0, 0, 1),       # 26 x 26 outputs: planes of 676 pixels, not a multiple of 16
], ids=lambda c: "x".join(map(str, c)))
def test_band_kernel_requantised_store_variants(torch, sw, oracle, case, raw_filters):
    N, C_in, C_out, H, W, pad, offset, variant = case
    if raw_filters and C_in % 64:
        pytest.skip("the band kernel takes the caller's filters in chunks of 64 input channels")
    x = inputs.uniform_s8((N, C_in, H, W), 5131)
    w = inputs.uniform_s8((C_out, C_in, 3, 3), 5132)
    rng = np.random.default_rng(5133)
    bias = rng.integers(-30000, 30000, size=C_out).astype(np.int32)
    std = np.sqrt(C_in * 9) * 5461.0
    scale = (rng.uniform(0.5, 2.0, size=C_out) * 40.0 / std).astype(np.float32)
    scale[::3] = np.float32(2.0 ** np.round(np.log2(40.0 / std)))      # powers of two produce exact ties
    scale[1::5] *= np.float32(-1.0)                                    # negative scales are legal
    for relu in (False, True):
        q_ref = oracle.conv2d_s8_requant(x, w, bias, scale, 1, pad, relu)
        n = q_ref.size
        buf = torch.full((256 + n + 64,), 77, dtype=torch.int8, device="cuda")
        out = buf[256 + offset:256 + offset + n].view(q_ref.shape)
        if raw_filters:
            sw.sw_conv2d_s8_requant(dev(torch, x), dev(torch, w), dev(torch, bias), dev(torch, scale), 1, pad, relu, out=out)
        else:
            sw.sw_conv2d_s8_packed(dev(torch, x), sw.sw_s8_pack_filter(dev(torch, w)), C_out, 3, 3, 1, pad,
                                   dev(torch, bias), dev(torch, scale), relu, out=out)
        assert sw.sw_last_kernel() == f"mfma_s8_band_kernel<{C_in // 32},{variant},{int(raw_filters)}>", sw.sw_last_kernel()
        torch.cuda.synchronize()
        assert bool((buf[:256 + offset] == 77).all()) and bool((buf[256 + offset + n:] == 77).all()), "write outside y8"
        q = out.cpu().numpy()
        assert np.array_equal(q, q_ref), f"{case} relu={relu}: {np.count_nonzero(q != q_ref)} of {q.size} differ"
