"""GPU parity: libswconv.so (through the C ABI) against the CPU oracle, element by element, on the
same seeded inputs.  fp32: max |y_gpu - y_oracle| / sum|x*w| <= 2e-5 per output; maximum pooling and
the int8 path: bit-exact."""
import numpy as np
import pytest

from paper_2310_05218_amd import inputs
from parity import assert_f32_parity, assert_guards_intact, guarded_empty

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


# ----------------------------------------------------------------------------- 1-D ---------------

CONV1D_CASES = [
    # rows, len, k, stride, pad
    (1, 9, 9, 1, 0),            # a single output
    (3, 17, 3, 1, 0),
    (2, 4173, 9, 1, 0),         # two tiles and a ragged tail, row length not a multiple of 4
    (3, 6144 + 8, 9, 1, 0),
    (2, 8300, 9, 1, 0),         # two tiles of 4096 and a ragged tail
    (3, 12288 + 8, 9, 1, 0),    # output length an exact multiple of the tile
    (5, 5000, 1, 1, 0),
    (4, 5000, 2, 1, 1),
    (4, 4100, 5, 1, 4),
    (2, 4096, 16, 1, 7),
    (2, 4099, 17, 1, 16),
    (2, 4500, 18, 1, 3),        # beyond the unrolled sizes: run-time tap count
    (3, 3000, 33, 1, 32),
    (2, 2500, 64, 1, 63),
    (2, 8301, 25, 1, 3),        # unrolled long filters: 25, 32, 49 taps (33 and 64 above)
    (3, 4100, 32, 1, 31),
    (2, 9000, 49, 1, 0),
    (2, 2049, 12, 1, 0),
    (3, 1000, 9, 2, 0),         # strided kernel
    (3, 1001, 4, 3, 2),
    (5, 4099, 2, 2, 0),         # ... several tiles, rows that start at every alignment
    (3, 9001, 7, 2, 6),
    (2, 20000, 64, 8, 63),      # ... widest window, largest stride
    (2, 700, 3, 9, 1),          # stride 9: one thread per output
]


@pytest.mark.parametrize("case", CONV1D_CASES)
def test_conv1d(torch, sw, oracle, case):
    rows, length, k, stride, pad = case
    x = inputs.normal_f32((rows, length), 1001)
    w = inputs.normal_f32((k,), 1002)
    y_ref, d = oracle.conv1d(x, w, stride, pad)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv1d(dev(torch, x), dev(torch, w), stride, pad, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"conv1d {case}")


def test_conv1d_more_tiles_than_workgroups(torch, sw, oracle):
    # 9000 tiles (one per row) > 8192 workgroups: some workgroups walk over two tiles (prefetch path)
    x = inputs.normal_f32((9000, 2051), 1003)
    w = inputs.normal_f32((5,), 1004)
    y_ref, d = oracle.conv1d(x, w, 1, 1)
    y = sw.sw_conv1d(dev(torch, x), dev(torch, w), 1, 1)
    assert_f32_parity(y.cpu().numpy(), y_ref, d, "conv1d 9000 x 2051")


POOL_CASES = [(1, 8, 8, 1), (3, 4173, 8, 1), (2, 6144 + 7, 8, 1), (2, 12288 + 7, 8, 1), (3, 9001, 8, 1), (4, 5000, 3, 1), (2, 5000, 1, 1),
              (3, 4099, 2, 2), (5, 9000, 3, 2), (2, 10001, 4, 4), (2, 30000, 8, 8),
              (3, 4100, 2, 2), (5, 9000, 4, 4), (7, 10008, 8, 8), (1, 8, 8, 8), (64, 8192, 2, 2),   # windows tile the rows
              (2, 4100, 17, 1), (2, 4100, 40, 1), (2, 3000, 64, 1), (3, 1000, 8, 2), (3, 1001, 3, 3),
              (2, 8301, 25, 1), (3, 4100, 32, 1), (2, 4173, 33, 1), (2, 9000, 49, 1)]          # unrolled long windows


@pytest.mark.parametrize("case", POOL_CASES)
@pytest.mark.parametrize("mode", [0, 1])
def test_pool1d(torch, sw, oracle, case, mode):
    rows, length, window, stride = case
    x = inputs.normal_f32((rows, length), 1011)
    y_ref, d = oracle.pool1d(x, window, stride, mode)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_pool1d(dev(torch, x), window, stride, mode, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    y = out.cpu().numpy()
    if mode == 1:
        assert np.array_equal(y.astype(np.float64), y_ref), f"max pool {case} is not bit-exact"
    else:
        assert_f32_parity(y, y_ref, d, f"avg pool {case}")


def test_avg_pool_equals_conv1d_with_constant_taps(torch, sw):
    x = dev(torch, inputs.normal_f32((4, 5000), 1021))
    w = torch.full((8,), 0.125, device="cuda")
    a = sw.sw_pool1d(x, 8, 1, 0)
    c = sw.sw_conv1d(x, w, 1, 0)
    assert float((a - c).abs().max()) <= 2e-6


def test_workload2_full_size(torch, sw, oracle):
    x, w = inputs.workload2()
    xd, wd = dev(torch, x), dev(torch, w)
    y_ref, d = oracle.conv1d(x, w, 1, 0)
    assert_f32_parity(sw.sw_conv1d(xd, wd).cpu().numpy(), y_ref, d, "workload 2 conv1d")
    y_ref, d = oracle.pool1d(x, 8, 1, 0)
    assert_f32_parity(sw.sw_pool1d(xd, 8, 1, 0).cpu().numpy(), y_ref, d, "workload 2 avg")
    y_ref, _ = oracle.pool1d(x, 8, 1, 1)
    assert np.array_equal(sw.sw_pool1d(xd, 8, 1, 1).cpu().numpy().astype(np.float64), y_ref)


# ----------------------------------------------------------------------------- 2-D single filter per plane

PLANE_CASES = [
    # N, C, H, W, R, S, stride, pad
    (1, 1, 3, 3, 3, 3, 1, 0),       # a single output
    (2, 3, 56, 56, 3, 3, 1, 1),
    (2, 3, 56, 56, 5, 5, 1, 2),
    (2, 3, 56, 56, 7, 7, 1, 3),
    (1, 2, 57, 59, 3, 3, 1, 1),     # ragged tiles
    (1, 2, 61, 70, 7, 7, 1, 3),
    (1, 2, 130, 131, 5, 5, 1, 0),
    (1, 2, 33, 47, 3, 3, 1, 0),
    (2, 2, 28, 28, 3, 3, 1, 1),
    (1, 3, 20, 21, 2, 6, 1, 1),     # filter extent without a fixed-size kernel
    (1, 2, 40, 40, 9, 9, 1, 4),
    (1, 2, 30, 30, 17, 17, 1, 8),
    (1, 2, 60, 61, 21, 21, 1, 10),  # beyond 17: the wide-window generic kernel
    (1, 1, 70, 64, 33, 29, 1, 14),
    (1, 1, 56, 56, 51, 51, 1, 25),
    (1, 2, 64, 64, 13, 4, 1, 0),
    (1, 2, 20, 520, 3, 3, 1, 1),    # rows kernel, three overlapping strips
    (1, 1, 30, 260, 5, 5, 1, 2),    # rows kernel, second strip of one lane
    (2, 1, 37, 512, 3, 3, 1, 0),
    (1, 3, 19, 256, 5, 5, 1, 1),
    (1, 2, 11, 252, 5, 5, 1, 0),
    (8, 64, 64, 64, 3, 3, 1, 1),    # rows kernel, 8-row bands
    (1, 3, 21, 23, 3, 3, 2, 1),     # strided, W not a multiple of 4: direct kernel
    (2, 3, 56, 56, 3, 3, 2, 1),     # strided rows kernel
    (1, 2, 57, 60, 3, 3, 2, 0),
    (1, 2, 30, 64, 5, 5, 2, 2),
    (1, 3, 23, 260, 5, 5, 2, 1),    # ... a second strip of one lane
    (1, 2, 21, 520, 3, 3, 2, 1),    # ... three strips
    (1, 1, 18, 252, 5, 5, 2, 0),
    (4, 64, 112, 112, 3, 3, 2, 1),  # ... 4-row bands
    (2, 3, 112, 112, 7, 7, 1, 3),   # rows kernel, 7x7: three columns from either neighbour lane
    (1, 2, 61, 300, 7, 7, 1, 2),    # ... two strips
    (1, 2, 64, 68, 7, 7, 2, 3),
    (1, 2, 33, 520, 7, 7, 2, 1),
    (1, 2, 64, 64, 7, 7, 1, 1),     # 7x7 with padding 1: tile kernel
    (1, 2, 9, 8, 3, 3, 3, 1),       # stride 3: direct kernel
    (2, 70, 14, 14, 3, 3, 1, 1),    # small planes: a run of planes per workgroup
    (1, 100, 7, 7, 3, 3, 1, 1),
    (1, 65, 7, 7, 5, 5, 1, 2),
    (1, 64, 14, 14, 3, 3, 2, 1),
    (1, 64, 13, 11, 4, 2, 2, 2),    # ... run-time filter extent, padding beyond the filter's need
    (1, 64, 30, 30, 3, 3, 1, 1),    # ... ragged 30 x 30 planes
    (3, 50, 5, 9, 5, 7, 1, 3),
    (1, 2, 7, 5, 7, 5, 1, 0),
    (1, 2, 16, 16, 3, 3, 1, 2),     # padding wider than the usual (R-1)/2
    (1, 2, 60, 60, 7, 7, 1, 1),     # one 56 x 56 tile of outputs from a plane larger than 56 x 56
    (8, 64, 60, 60, 5, 5, 1, 0),    # ... on enough planes for the whole-plane kernels to be considered
    (8, 64, 56, 60, 5, 5, 1, 0),
    (8, 64, 58, 58, 3, 3, 1, 0),
    (8, 64, 62, 62, 7, 7, 1, 0),
]


def _enough_planes_for_the_sliding_kernel(N, C, H, W, R, S, stride, pad):
    """The library sends problems of fewer than 64 tiles with small filters to the one-thread-per-output
    kernel (launch-latency regime).  Returns a batch size that keeps the case on the sliding kernel."""
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    tiles = -(-Ho // 56) * -(-Wo // 56)
    return N * -(-64 // (N * C * tiles))


@pytest.mark.parametrize("batch", ["as given", "sliding-kernel batch"])
@pytest.mark.parametrize("case", PLANE_CASES)
def test_depthwise(torch, sw, oracle, case, batch):
    N, C, H, W, R, S, stride, pad = case
    if batch != "as given":
        N = _enough_planes_for_the_sliding_kernel(*case)
    x = inputs.normal_f32((N, C, H, W), 2001)
    w = inputs.normal_f32((C, 1, R, S), 2002)
    y_ref, d = oracle.conv2d_depthwise(x, w, stride, pad)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_depthwise(dev(torch, x), dev(torch, w), stride, pad, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"depthwise {case}")


@pytest.mark.parametrize("batch", ["as given", "sliding-kernel batch"])
@pytest.mark.parametrize("case", PLANE_CASES)
def test_conv2d_single_input_channel(torch, sw, oracle, case, batch):
    N, C_out, H, W, R, S, stride, pad = case
    if batch != "as given":
        N = _enough_planes_for_the_sliding_kernel(*case)
    x = inputs.normal_f32((N, 1, H, W), 2011)
    w = inputs.normal_f32((C_out, 1, R, S), 2012)
    y_ref, d = oracle.conv2d(x, w, stride, pad)
    y = sw.sw_conv2d(dev(torch, x), dev(torch, w), stride, pad)
    assert_f32_parity(y.cpu().numpy(), y_ref, d, f"conv2d C_in=1 {case}")


# ----------------------------------------------------------------------------- 2-D pooling

POOL2D_CASES = [
    # N, C, H, W, R, S, stride, pad
    (1, 1, 2, 4, 2, 2, 2, 0),       # a row of two outputs
    (2, 3, 56, 56, 2, 2, 2, 0),     # register-only kernel
    (2, 3, 56, 56, 3, 3, 2, 1),
    (1, 2, 57, 60, 3, 3, 2, 0),
    (1, 2, 31, 64, 3, 3, 1, 1),
    (1, 2, 30, 44, 3, 3, 1, 0),
    (1, 2, 21, 520, 3, 3, 2, 1),    # ... three strips
    (1, 3, 23, 260, 2, 2, 2, 0),    # ... a second strip of one lane
    (1, 1, 19, 256, 3, 3, 1, 1),
    (4, 64, 112, 112, 3, 3, 2, 1),  # ... long bands
    (2, 16, 112, 112, 2, 2, 2, 0),
    (1, 3, 21, 23, 3, 3, 2, 1),     # W not a multiple of 4: one thread per output
    (1, 2, 20, 20, 2, 2, 1, 0),
    (1, 2, 20, 24, 5, 3, 2, 1),
    (1, 2, 14, 14, 14, 14, 1, 0),   # global pooling of small planes: 64 planes per wavefront
    (3, 40, 7, 7, 7, 7, 1, 0),
    (2, 100, 16, 16, 16, 16, 1, 0),
    (1, 65, 3, 5, 3, 5, 1, 0),
    (1, 3, 20, 20, 20, 20, 1, 0),   # global pooling of larger planes: a wavefront per output
    (1, 2, 30, 33, 9, 11, 2, 4),    # ... large windows with padding and stride
    (1, 1, 70, 66, 64, 64, 1, 1),
    (1, 2, 17, 16, 4, 4, 4, 2),
    (1, 2, 9, 12, 1, 1, 2, 0),
]


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("case", POOL2D_CASES)
def test_pool2d(torch, sw, oracle, case, mode):
    N, C, H, W, R, S, stride, pad = case
    x = inputs.normal_f32((N, C, H, W), 2101)
    if mode == 1:
        x = x - 3.0          # mostly negative: padding must not win the maximum with a zero
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


def test_pool2d_misaligned_views(torch, sw, oracle):
    """Input and output that start 4 bytes off a 16-byte boundary: the one-thread-per-output kernel (input)
    and the scalar stores of the register-only kernel (output) give the same values."""
    x = inputs.normal_f32((2, 4, 24, 32), 2102)
    for mode in (0, 1):
        y_ref, d = oracle.pool2d(x, 3, 3, 2, 1, mode)
        xb = torch.empty(x.size + 1, dtype=torch.float32, device="cuda")
        xv = xb[1:].view(x.shape)
        xv.copy_(torch.from_numpy(x))
        y1 = sw.sw_pool2d(xv, 3, 3, 2, 1, mode).cpu().numpy()
        yb = torch.empty(y_ref.size + 1, dtype=torch.float32, device="cuda")
        yv = yb[1:].view(y_ref.shape)
        sw.sw_pool2d(dev(torch, x), 3, 3, 2, 1, mode, out=yv)
        for y in (y1, yv.cpu().numpy()):
            if mode == 1:
                assert np.array_equal(y.astype(np.float64), y_ref)
            else:
                assert_f32_parity(y, y_ref, d, "avg pool2d, misaligned")


@pytest.mark.parametrize("layer", [("max", 3, 2, 1), ("avg", 2, 2, 0), ("max", 2, 2, 0), ("dw", 3, 2, 1), ("dw", 5, 2, 2)],
                         ids=lambda l: "%s%dx%ds%d" % (l[0], l[1], l[1], l[2]))
def test_strided_layers_full_size(torch, sw, oracle, layer):
    """The stride-2 layers of the benchmark's layer table at their full size (8 x 64 x 112 x 112 planes here:
    the same launch configuration, a quarter of the batch), every output against the oracle."""
    kind, R, stride, pad = layer
    x = inputs.normal_f32((8, 64, 112, 112), 2201)
    if kind == "dw":
        w = inputs.normal_f32((64, 1, R, R), 2202, 1.0 / R)
        y_ref, d = oracle.conv2d_depthwise(x, w, stride, pad)
        y = sw.sw_conv2d_depthwise(dev(torch, x), dev(torch, w), stride, pad).cpu().numpy()
        assert_f32_parity(y, y_ref, d, f"depthwise {layer}")
    else:
        mode = 1 if kind == "max" else 0
        y_ref, d = oracle.pool2d(x, R, R, stride, pad, mode)
        y = sw.sw_pool2d(dev(torch, x), R, R, stride, pad, mode).cpu().numpy()
        if mode == 1:
            assert np.array_equal(y.astype(np.float64), y_ref)
        else:
            assert_f32_parity(y, y_ref, d, f"avg pool2d {layer}")


def test_workload1_full_size(torch, sw, oracle):
    x, w = inputs.workload1()
    y_ref, d = oracle.conv2d(x, w, 1, 0)
    y = sw.sw_conv2d(dev(torch, x), dev(torch, w), 1, 0)
    assert y.shape == (1, 1, 254, 254)
    assert_f32_parity(y.cpu().numpy(), y_ref, d, "workload 1")


def test_impulse_reproduces_filter_on_gpu(torch, sw):
    x = np.zeros((1, 64, 40, 40), np.float32)      # 64 planes: runs on the sliding kernel
    x[0, :, 20, 21] = 1.0
    w = inputs.uniform_f32((64, 1, 7, 7), 2021)
    y = sw.sw_conv2d_depthwise(dev(torch, x), dev(torch, w), 1, 3).cpu().numpy()
    expect = np.zeros_like(y)
    for r in range(7):
        for s in range(7):
            expect[0, :, 20 - r + 3, 21 - s + 3] = w[:, 0, r, s]
    assert np.array_equal(y, expect)


@pytest.mark.parametrize("which", ["3x3", "7x7"])
def test_workload4_full_size(torch, sw, oracle, which):
    x, w3, w7 = inputs.workload4()
    w, pad = (w3, 1) if which == "3x3" else (w7, 3)
    y_ref, d = oracle.conv2d_depthwise(x, w, 1, pad)
    y = sw.sw_conv2d_depthwise(dev(torch, x), dev(torch, w), 1, pad)
    assert_f32_parity(y.cpu().numpy(), y_ref, d, f"workload 4 {which}")


# ----------------------------------------------------------------------------- 2-D multi-channel fp32

CONV2D_CASES = [
    # N, C_in, C_out, H, W, R, S, stride, pad
    (1, 3, 5, 9, 11, 3, 3, 1, 1),        # small odd shapes: the any-shape matrix-core kernel
    (2, 4, 3, 12, 10, 2, 5, 2, 2),
    (1, 7, 2, 8, 8, 1, 1, 1, 0),
    (2, 16, 64, 56, 56, 3, 3, 1, 1),     # matrix-core path, one channel block
    (1, 64, 64, 56, 56, 3, 3, 1, 1),
    (2, 32, 128, 28, 28, 3, 3, 1, 1),    # two output-channel blocks
    (1, 32, 64, 30, 41, 3, 3, 1, 1),     # ragged row bands and widths
    (1, 16, 64, 9, 100, 3, 3, 1, 1),
    (1, 48, 64, 14, 14, 3, 3, 1, 0),     # valid mode
    (1, 16, 64, 20, 20, 5, 5, 1, 2),
    (1, 16, 64, 12, 12, 1, 1, 1, 0),
    (1, 32, 64, 17, 19, 3, 3, 2, 1),     # strided: the any-shape matrix-core kernel
    (2, 3, 10, 23, 21, 3, 3, 1, 1),      # odd channel counts on both sides (zero-filled in LDS)
    (1, 3, 64, 60, 60, 7, 7, 2, 3),      # a CNN stem: 7x7, stride 2, three input channels
    (1, 3, 70, 35, 35, 11, 11, 4, 2),    # 11x11 stride 4
    (2, 5, 33, 12, 150, 3, 3, 1, 1),     # output rows wider than a tile: column tiles
    (1, 7, 65, 40, 9, 5, 3, 1, 2),       # rectangular filter, padding beyond (S-1)/2
    (3, 64, 96, 7, 7, 3, 3, 1, 1),       # small images
    (2, 40, 64, 14, 14, 1, 1, 1, 0),     # pointwise, C_in not a multiple of 8
    (1, 24, 64, 14, 14, 1, 1, 2, 0),     # pointwise with stride
    (1, 6, 8, 30, 30, 13, 13, 1, 6),     # 169 taps: channel chunks of two
    (1, 6, 64, 30, 30, 11, 11, 1, 5),    # filter rows beyond 64 KB of LDS: one workgroup per CU
    (2, 4, 70, 24, 24, 13, 13, 1, 6),
    (1, 3, 64, 40, 40, 17, 17, 2, 8),    # the largest filter of the matrix-core kernel
    (1, 2, 5, 40, 40, 18, 18, 1, 9),     # beyond it: the compound (filter-row) kernel
    (1, 2, 4, 5, 5, 5, 5, 1, 0),         # a single output pixel
    (1, 9, 130, 16, 16, 2, 2, 2, 0),     # even filter, three channel blocks with a ragged last one
]


DILATED_CASES = [
    # N, C_in, C_out, H, W, R, S, stride, pad, dilation
    (2, 16, 64, 28, 28, 3, 3, 1, 2, 2),      # "same" 3x3 at dilation 2: matrix-core kernel, window grows by 2
    (1, 32, 70, 33, 31, 3, 3, 1, 4, 4),      # dilation 4 (segmentation heads), ragged channel block
    (2, 8, 16, 40, 40, 3, 3, 2, 3, 3),       # with stride 2
    (1, 3, 5, 25, 27, 5, 2, 1, 3, 2),        # rectangular filter
    (1, 6, 64, 64, 64, 3, 3, 1, 12, 12),     # dilation 12: window 25 rows taller than the tile
    (1, 4, 8, 20, 20, 7, 7, 1, 9, 3),        # 49 taps, span 19
    (2, 5, 9, 12, 12, 1, 1, 1, 0, 5),        # one tap: dilation changes nothing
    (1, 2, 3, 9, 9, 3, 3, 1, 0, 4),          # span 9 = the plane: a single output
    (2, 1, 6, 20, 22, 3, 3, 1, 2, 2),        # one input channel: one thread per output
]


@pytest.mark.parametrize("case", DILATED_CASES)
def test_conv2d_dilated(torch, sw, oracle, case):
    N, C_in, C_out, H, W, R, S, stride, pad, dil = case
    x = inputs.normal_f32((N, C_in, H, W), 3201)
    w = inputs.normal_f32((C_out, C_in, R, S), 3202, (2.0 / (C_in * R * S)) ** 0.5)
    y_ref, d = oracle.conv2d_dilated(x, w, stride, pad, dil)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_dilated(dev(torch, x), dev(torch, w), stride, pad, dil, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"conv2d_dilated {case}")


@pytest.mark.parametrize("case", [(2, 7, 30, 28, 3, 3, 1, 2, 2), (1, 5, 21, 40, 5, 3, 2, 4, 3), (3, 4, 14, 14, 3, 3, 1, 0, 6),
                                  (1, 6, 56, 56, 3, 3, 1, 1, 1)])
def test_conv2d_depthwise_dilated(torch, sw, oracle, case):
    N, C, H, W, R, S, stride, pad, dil = case
    x = inputs.normal_f32((N, C, H, W), 3211)
    w = inputs.normal_f32((C, 1, R, S), 3212)
    y_ref, d = oracle.conv2d_dilated(x, w, stride, pad, dil, depthwise=True)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_depthwise_dilated(dev(torch, x), dev(torch, w), stride, pad, dil, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"depthwise_dilated {case}")


@pytest.mark.parametrize("case", [
    # N, C, H, W, R, S, pad, dilation, kernel the call must reach
    (2, 64, 56, 56, 3, 3, 2, 2, "sliding_plane_kernel<3,3,2>"),      # 3x3 at dilation 2 and 4: unrolled kernels
    (1, 64, 57, 59, 3, 3, 0, 2, "sliding_plane_kernel<3,3,2>"),      # ... ragged tiles, no padding
    (1, 64, 40, 44, 4, 4, 3, 2, "sliding_plane_kernel<0,0,17>"),     # dilation 2, other extents: taps in groups of four
    (1, 64, 57, 59, 5, 5, 4, 2, "sliding_plane_kernel<0,0,17>"),     # ... a group of four and one more, ragged tiles
    (1, 70, 40, 44, 2, 7, 3, 2, "sliding_plane_kernel<0,0,17>"),     # ... and three more; two filter rows
    (1, 64, 65, 70, 3, 3, 6, 6, "sliding_plane_kernel<0,0,17>"),     # any other dilation: one tap at a time, span 13
    (1, 64, 60, 60, 3, 3, 12, 12, "sliding_plane_kernel<0,0,51>"),   # span 25: the wide window
    (1, 64, 64, 64, 3, 3, 18, 18, "sliding_plane_kernel<0,0,51>"),   # span 37
    (1, 64, 112, 112, 3, 3, 4, 4, "sliding_plane_kernel<3,3,4>"),    # four tiles per plane
    (1, 8, 30, 30, 7, 7, 9, 3, "sliding_plane_kernel<0,0,51>"),      # 49 taps, span 19, few planes
    (1, 64, 80, 80, 3, 3, 0, 30, "direct_conv2d_kernel"),            # span 61: no window holds it
], ids=lambda c: "x".join(map(str, c[:8])))
def test_depthwise_dilated_sliding_kernel(torch, sw, oracle, case):
    """Dilated one-filter-per-plane convolution on the sliding tile kernel (enough planes to fill the chip)."""
    N, C, H, W, R, S, pad, dil, kernel = case
    x = inputs.normal_f32((N, C, H, W), 3221)
    w = inputs.normal_f32((C, 1, R, S), 3222)
    b = inputs.normal_f32((C,), 3223, 0.5)
    y_ref, d = oracle.conv2d_dilated(x, w, 1, pad, dil, depthwise=True)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_depthwise_dilated(dev(torch, x), dev(torch, w), 1, pad, dil, out=out)
    assert sw.sw_last_kernel().startswith(kernel), sw.sw_last_kernel()
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"depthwise_dilated {case}")
    # one input channel, C filters: the same planes through sw_conv2d_dilated
    x1 = inputs.normal_f32((N, 1, H, W), 3224)
    y_ref, d = oracle.conv2d_dilated(x1, w, 1, pad, dil)
    y = sw.sw_conv2d_dilated(dev(torch, x1), dev(torch, w), 1, pad, dil)
    assert sw.sw_last_kernel().startswith(kernel), sw.sw_last_kernel()
    assert_f32_parity(y.cpu().numpy(), y_ref, d, f"conv2d_dilated C_in=1 {case}")


# (N, C, H, W, R, S, stride, pad, floats the input is shifted by): plane sizes that are and are not multiples of four
# floats, runs whose last workgroup holds fewer planes, an input off the 16-byte grid (4-byte loads), a frame smaller
# than the padded image (stride 2)
SMALL_PLANE_CASES = [
    (3, 50, 13, 13, 3, 3, 1, 1, 0), (2, 65, 7, 7, 3, 3, 1, 1, 0), (1, 130, 7, 7, 5, 5, 1, 2, 0), (5, 13, 14, 14, 7, 7, 1, 3, 0),
    (2, 67, 14, 14, 3, 3, 2, 1, 0), (1, 70, 9, 11, 3, 3, 1, 0, 0), (3, 50, 13, 13, 3, 3, 1, 1, 1), (2, 64, 14, 14, 3, 3, 1, 1, 2),
    (32, 16, 28, 28, 5, 5, 1, 2, 0),
]


@pytest.mark.parametrize("case", SMALL_PLANE_CASES, ids=lambda c: "x".join(map(str, c)))
def test_depthwise_small_planes(torch, sw, oracle, case):
    N, C, H, W, R, S, stride, pad, shift = case
    x = inputs.normal_f32((N, C, H, W), 3231)
    w = inputs.normal_f32((C, 1, R, S), 3232)
    y_ref, d = oracle.conv2d_depthwise(x, w, stride, pad)
    xbuf = torch.empty((x.size + 4,), device="cuda")
    xd = xbuf[shift:shift + x.size].view(x.shape)
    xd.copy_(dev(torch, x))
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_depthwise(xd, dev(torch, w), stride, pad, out=out)
    assert sw.sw_last_kernel().startswith("small_planes_kernel"), sw.sw_last_kernel()
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"depthwise on small planes {case}")


def test_dilation_one_is_the_undilated_call(torch, sw):
    x = dev(torch, inputs.normal_f32((2, 16, 28, 28), 3221))
    w = dev(torch, inputs.normal_f32((64, 16, 3, 3), 3222, 0.1))
    assert torch.equal(sw.sw_conv2d_dilated(x, w, 1, 1, 1), sw.sw_conv2d(x, w, 1, 1))


DMA_KERNEL_CASES = [
    # N, C_in, C_out, H, W, R, S, stride, pad, dilation,
    # kernel<100 K parts + 10 block columns + blocks per wavefront, channels per chunk, images and rows per tile>
    (1, 8, 64, 12, 12, 3, 3, 1, 1, 1, "mfma_f32_dma_kernel<421,8,1,2>"),       # one chunk, row pairs of 24 pixels
    (2, 16, 40, 14, 14, 3, 3, 1, 1, 1, "mfma_f32_dma_kernel<421,8,1,2>"),      # two chunks, channel block with 24 dead channels
    (3, 32, 70, 7, 7, 3, 3, 1, 1, 1, "mfma_f32_dma_kernel<421,8,1,4>"),        # tiles of four and three rows of a 7 x 7 image, ragged channel block
    (7, 16, 64, 5, 6, 3, 3, 1, 1, 1, "mfma_f32_dma_kernel<421,8,1,5>"),        # one whole 5 x 6 image per tile
    (2, 16, 64, 30, 41, 3, 3, 1, 1, 1, "mfma_f32_dma_kernel<421,8,1,1>"),      # one row of 41 pixels per tile: two blocks, the second ragged
    (1, 24, 96, 57, 57, 3, 3, 2, 1, 1, "mfma_f32_dma_kernel<421,8,1,1>"),      # stride 2, three chunks, ragged channel block
    (1, 8, 64, 28, 28, 3, 3, 1, 2, 2, "mfma_f32_dma_kernel<421,8,1,1>"),       # dilation 2
    (1, 16, 64, 40, 40, 3, 3, 2, 3, 3, "mfma_f32_dma_kernel<421,8,1,3>"),      # dilation 3 with stride 2
    (2, 64, 64, 19, 23, 1, 1, 2, 0, 1, "mfma_f32_dma_kernel<421,32,1,2>"),     # one tap at stride 2: chunks of 32 channels
    (1, 16, 32, 20, 20, 4, 4, 1, 2, 1, "mfma_f32_dma_kernel<421,8,1,3>"),      # 16 taps, even extents
    (1, 8, 16, 9, 200, 3, 3, 1, 1, 1, "mfma_f32_dma_kernel<142,8,1,1>"),       # rows of 200 pixels: two blocks per wavefront, four window slots
    (5, 8, 64, 5, 5, 2, 2, 1, 0, 1, "mfma_f32_dma_kernel<421,8,2,4>"),         # 2x2, two whole images per tile, the last tile with one
    (2, 40, 64, 16, 16, 3, 1, 1, 1, 1, "mfma_f32_dma_kernel<241,8,1,3>"),      # a column filter (three groups per chunk: at most two wavefronts per block); five chunks
    (5, 8, 256, 56, 56, 3, 3, 1, 1, 1, "mfma_f32_dma_kernel<142,8,1,4>"),      # 224-pixel tiles: two blocks per wavefront, the last wavefront one
    (1, 32, 64, 18, 18, 2, 2, 1, 0, 1, "mfma_f32_dma_kernel<421,16,1,3>"),     # 2x2: chunks of 16 channels
    (1, 8, 64, 3, 3, 3, 3, 1, 0, 1, "mfma_f32_dma_kernel<421,8,1,1>"),         # a single output pixel
    (40, 8, 64, 28, 28, 3, 3, 1, 1, 1, "mfma_f32_dma_kernel<141,8,1,4>"),     # more workgroups than CUs: no K split, unrolled group loop
    (40, 16, 64, 28, 28, 2, 2, 1, 0, 1, "mfma_f32_dma_kernel<141,16,1,4>"),   # ... and the run-time group loop
    (2, 8, 64, 7, 7, 3, 3, 1, 1, 1, "mfma_f32_dma_kernel<421,8,1,4>"),        # two blocks per tile: four wavefronts per block
    (9, 8, 64, 4, 4, 3, 3, 1, 1, 1, "mfma_f32_dma_kernel<421,8,2,4>"),       # whole 4 x 4 images, several per tile, the last tile short
    (6, 8, 64, 7, 9, 3, 1, 1, 0, 1, "mfma_f32_dma_kernel<241,8,2,5>"),       # three groups per chunk: two wavefronts per block; two whole images per tile
    (600, 8, 64, 7, 7, 3, 3, 1, 1, 1, "mfma_f32_dma_kernel<141,8,2,7>"),     # two images per tile without a K split (300 workgroups)
]


@pytest.mark.parametrize("case", DMA_KERNEL_CASES, ids=lambda c: "x".join(map(str, c[:10])))
def test_conv2d_direct_to_lds_kernel(torch, sw, oracle, case):
    """Few taps over whole groups of eight channels: the kernel whose operands come into LDS by direct-to-LDS loads,
    on every tiling it has, with and without the fused epilogue."""
    N, C_in, C_out, H, W, R, S, stride, pad, dil, kernel = case
    x = inputs.normal_f32((N, C_in, H, W), 3401)
    w = inputs.normal_f32((C_out, C_in, R, S), 3402, (2.0 / (C_in * R * S)) ** 0.5)
    y_ref, d = oracle.conv2d_dilated(x, w, stride, pad, dil)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_dilated(dev(torch, x), dev(torch, w), stride, pad, dil, out=out)
    assert sw.sw_last_kernel() == kernel, sw.sw_last_kernel()
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"direct-to-LDS kernel {case}")
    if dil == 1 and N <= 7:
        bias = inputs.normal_f32((C_out,), 3403, 0.7)
        y_ref, d = oracle.conv2d_bias_relu(x, w, bias, stride, pad, True)
        y = sw.sw_conv2d_bias_relu(dev(torch, x), dev(torch, w), dev(torch, bias), stride, pad, True)
        assert sw.sw_last_kernel() == kernel, sw.sw_last_kernel()
        assert_f32_parity(y.cpu().numpy(), y_ref, d, f"direct-to-LDS kernel, bias + rectifier {case}")


def test_conv2d_direct_to_lds_kernel_needs_aligned_filters(torch, sw, oracle):
    """Filters that do not start on a 16-byte boundary (or channel counts off the grid of eight) take the older
    window kernels, with the same results."""
    x = inputs.normal_f32((2, 16, 14, 14), 3411)
    w = inputs.normal_f32((64, 16, 3, 3), 3412, 0.1)
    y_ref, d = oracle.conv2d(x, w, 1, 1)
    wbuf = torch.zeros(w.size + 1, device="cuda")
    wbuf[1:] = dev(torch, w).reshape(-1)
    y = sw.sw_conv2d(dev(torch, x), wbuf[1:].view(64, 16, 3, 3), 1, 1)
    assert sw.sw_last_kernel().startswith("mfma_f32_quad_kernel"), sw.sw_last_kernel()
    assert_f32_parity(y.cpu().numpy(), y_ref, d, "misaligned filters")
    x12 = inputs.normal_f32((2, 12, 14, 14), 3413)
    w12 = inputs.normal_f32((64, 12, 3, 3), 3414, 0.1)
    y = sw.sw_conv2d(dev(torch, x12), dev(torch, w12), 1, 1)
    assert sw.sw_last_kernel().startswith("mfma_f32_quad_kernel"), sw.sw_last_kernel()
    assert_f32_parity(y.cpu().numpy(), *oracle.conv2d(x12, w12, 1, 1), "twelve channels")


DW_BIAS_RELU_CASES = [
    # N, C, H, W, R, S, stride, pad -- one per kernel of the one-filter-per-plane dispatch
    (2, 256, 56, 56, 3, 3, 1, 1),        # whole-plane kernel, 56 x 56 specialisation
    (2, 256, 56, 56, 7, 7, 1, 3),
    (8, 64, 48, 56, 5, 5, 1, 2),         # ... general variant
    (2, 8, 112, 112, 3, 3, 2, 1),        # register-only rows kernel, stride 2
    (2, 40, 28, 28, 3, 3, 1, 1),         # rows kernel, two planes per wavefront
    (4, 32, 14, 14, 3, 3, 1, 1),         # small planes through LDS
    (2, 40, 7, 7, 5, 5, 1, 2),
    (2, 40, 60, 60, 9, 9, 1, 4),         # run-time-extent tile kernel (four wavefronts per tile)
    (1, 70, 100, 60, 4, 6, 1, 2),
    (2, 5, 30, 31, 3, 3, 3, 1),          # one thread per output
]


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("case", DW_BIAS_RELU_CASES)
def test_conv2d_depthwise_bias_relu(torch, sw, oracle, case, relu):
    N, C, H, W, R, S, stride, pad = case
    x = inputs.normal_f32((N, C, H, W), 3301)
    w = inputs.normal_f32((C, 1, R, S), 3302, 1.0 / (R * S) ** 0.5)
    bias = inputs.normal_f32((C,), 3303, 0.7)
    y_ref, d = oracle.conv2d_depthwise_bias_relu(x, w, bias, stride, pad, relu)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_depthwise_bias_relu(dev(torch, x), dev(torch, w), dev(torch, bias), stride, pad, relu, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    y = out.cpu().numpy()
    assert_f32_parity(y, y_ref, d, f"depthwise_bias_relu {case} relu={relu}")
    if relu:
        assert y.min() == 0.0 and 0.2 < (y == 0).mean() < 0.8
    else:
        y0 = sw.sw_conv2d_depthwise(dev(torch, x), dev(torch, w), stride, pad).cpu().numpy()
        assert np.allclose((y - y0).mean(axis=(0, 2, 3)), bias, atol=1e-4)


def test_depthwise_bias_relu_without_either_is_the_plain_call(torch, sw):
    x = dev(torch, inputs.normal_f32((2, 256, 56, 56), 3311))
    w = dev(torch, inputs.normal_f32((256, 1, 3, 3), 3312))
    plain = sw.sw_conv2d_depthwise(x, w, 1, 1)
    assert torch.equal(sw.sw_conv2d_depthwise_bias_relu(x, w, None, 1, 1, False), plain)
    assert torch.equal(sw.sw_conv2d_depthwise_bias_relu(x, w, None, 1, 1, True), torch.clamp_min(plain, 0.0))


ROWS_KERNEL_CASES = [
    # N, C_in, C_out, H, W, R, S, stride, pad, dilation, kernel instance the call must reach
    (2, 16, 64, 56, 56, 5, 5, 1, 2, 1, "mfma_f32_rows_kernel<16,2,8>"),    # 25 taps: sixteen channels per chunk
    (1, 64, 64, 28, 28, 7, 7, 1, 3, 1, "mfma_f32_rows_kernel<16,2,8>"),
    (1, 24, 70, 40, 44, 9, 9, 1, 4, 1, "mfma_f32_rows_kernel<8,2,6>"),     # eight; ragged channel block and channel chunk
    (1, 16, 64, 30, 32, 11, 11, 1, 5, 1, "mfma_f32_rows_kernel<8,2,6>"),
    (1, 16, 64, 30, 32, 13, 13, 1, 6, 1, "mfma_f32_rows_kernel<8,2,8>"),   # longer filter rows: more filter slots per thread
    (1, 12, 130, 24, 24, 17, 17, 1, 8, 1, "mfma_f32_rows_kernel<8,2,10>"),  # three channel blocks, the last one ragged
    (1, 16, 64, 30, 32, 9, 3, 1, 1, 1, "mfma_f32_rows_kernel<16,2,4>"),    # rows of three taps (one thread takes a row)
    (1, 8, 64, 20, 20, 21, 21, 1, 10, 1, "mfma_f32_rows_kernel<4,2,9>"),   # rows beyond 20 taps: four channels per chunk
    (1, 8, 32, 48, 48, 41, 41, 1, 20, 1, "mfma_f32_rows_kernel<4,2,11>"),
    (1, 8, 32, 36, 36, 33, 29, 1, 14, 1, "mfma_f32_rows_kernel<4,2,9>"),   # rectangular
    (1, 6, 64, 32, 32, 51, 51, 1, 25, 1, "mfma_f32_rows_kernel<4,2,13>"),   # (fewer than 8 channels: no other kernel has it)
    (1, 2, 5, 40, 40, 18, 18, 1, 9, 1, "mfma_f32_rows_kernel<2,2,10>"),     # two input channels
    (1, 16, 64, 57, 60, 5, 5, 2, 2, 1, "mfma_f32_rows_kernel<4,2,9>"),     # stride 2: every second input row staged
    (1, 33, 1, 24, 32, 5, 5, 3, 1, 1, "mfma_f32_rows_kernel<16,2,8>"),     # stride 3: image rows wider than the taps reach
    (1, 9, 64, 41, 44, 7, 5, 3, 1, 1, "mfma_f32_rows_kernel<4,2,9>"),      # stride 3, rectangular, odd channel count
    (1, 16, 64, 40, 40, 5, 5, 1, 4, 2, "mfma_f32_rows_kernel<16,2,8>"),    # dilation 2
    (1, 8, 64, 48, 48, 7, 7, 2, 9, 3, "mfma_f32_rows_kernel<4,2,9>"),      # dilation 3 with stride 2
    (1, 16, 64, 5, 8, 5, 5, 1, 0, 1, "mfma_f32_rows_kernel<16,2,8>"),      # a single row of four outputs
    (2, 16, 64, 112, 112, 5, 5, 1, 2, 1, "mfma_f32_rows_kernel<8,2,6>"),   # tiles inside one image row pair
    (40, 8, 128, 56, 56, 5, 5, 1, 2, 1, "mfma_f32_rows_kernel<4,4,9>"),    # enough work for 512-pixel tiles
]


@pytest.mark.parametrize("case", ROWS_KERNEL_CASES, ids=lambda c: "x".join(map(str, c[:10])))
def test_conv2d_large_filters_rows_kernel(torch, sw, oracle, case):
    """The compound kernel (one filter row of a channel chunk at a time), with and without the fused epilogue."""
    N, C_in, C_out, H, W, R, S, stride, pad, dil, kernel = case
    x = inputs.normal_f32((N, C_in, H, W), 3301)
    w = inputs.normal_f32((C_out, C_in, R, S), 3302, (2.0 / (C_in * R * S)) ** 0.5)
    y_ref, d = oracle.conv2d_dilated(x, w, stride, pad, dil)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_dilated(dev(torch, x), dev(torch, w), stride, pad, dil, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"rows kernel {case}")
    assert sw.sw_last_kernel() == kernel, sw.sw_last_kernel()
    if dil == 1 and N <= 2:
        bias = inputs.normal_f32((C_out,), 3303, 0.7)
        y_ref, d = oracle.conv2d_bias_relu(x, w, bias, stride, pad, True)
        y = sw.sw_conv2d_bias_relu(dev(torch, x), dev(torch, w), dev(torch, bias), stride, pad, True)
        assert sw.sw_last_kernel() == kernel, sw.sw_last_kernel()
        assert_f32_parity(y.cpu().numpy(), y_ref, d, f"rows kernel, bias + rectifier {case}")


BIAS_RELU_CASES = [
    # N, C_in, C_out, H, W, R, S, stride, pad
    (8, 16, 256, 56, 56, 3, 3, 1, 1),    # enough large tiles for the fixed 3x3 matrix-core kernel (256 workgroups)
    (4, 16, 256, 56, 56, 5, 5, 1, 2),    # 5x5: the compound (filter-row) kernel
    (2, 16, 64, 56, 56, 3, 3, 1, 1),     # 128-pixel tiles, channel quads
    (1, 3, 5, 9, 11, 3, 3, 1, 1),        # any-shape kernel, ragged channel block
    (2, 4, 3, 12, 10, 2, 5, 2, 2),
    (1, 9, 130, 16, 16, 2, 2, 2, 0),     # three channel blocks with a ragged last one
    (2, 1, 6, 20, 20, 3, 3, 1, 1),       # one input channel: the one-filter-per-plane kernels
    (2, 1, 64, 56, 56, 7, 7, 1, 3),
]


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("case", BIAS_RELU_CASES)
def test_conv2d_bias_relu(torch, sw, oracle, case, relu):
    """Per-channel bias and rectifier fused into the store: y = act(conv + bias[co]); the bias is one more term of
    the magnitude sum the tolerance is relative to."""
    N, C_in, C_out, H, W, R, S, stride, pad = case
    x = inputs.normal_f32((N, C_in, H, W), 3101)
    w = inputs.normal_f32((C_out, C_in, R, S), 3102, (2.0 / (C_in * R * S)) ** 0.5)
    bias = inputs.normal_f32((C_out,), 3103, 0.7)
    y_ref, d = oracle.conv2d_bias_relu(x, w, bias, stride, pad, relu)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_bias_relu(dev(torch, x), dev(torch, w), dev(torch, bias), stride, pad, relu, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    y = out.cpu().numpy()
    assert_f32_parity(y, y_ref, d, f"conv2d_bias_relu {case} relu={relu}")
    if relu:
        assert y.min() == 0.0 and 0.2 < (y == 0).mean() < 0.8
    else:
        # the bias really is per output channel: channel means move by it
        y0 = sw.sw_conv2d(dev(torch, x), dev(torch, w), stride, pad).cpu().numpy()
        shift = (y - y0).mean(axis=(0, 2, 3))
        assert np.allclose(shift, bias, atol=1e-4)


def test_conv2d_bias_relu_without_bias_or_rectifier(torch, sw, oracle):
    x = inputs.normal_f32((2, 16, 28, 28), 3111)
    w = inputs.normal_f32((64, 16, 3, 3), 3112, 0.1)
    xd, wd = dev(torch, x), dev(torch, w)
    plain = sw.sw_conv2d(xd, wd, 1, 1)
    assert torch.equal(sw.sw_conv2d_bias_relu(xd, wd, None, 1, 1, False), plain)
    assert torch.equal(sw.sw_conv2d_bias_relu(xd, wd, None, 1, 1, True), torch.clamp_min(plain, 0.0))


@pytest.mark.parametrize("case", CONV2D_CASES)
def test_conv2d(torch, sw, oracle, case):
    N, C_in, C_out, H, W, R, S, stride, pad = case
    x = inputs.normal_f32((N, C_in, H, W), 3001)
    w = inputs.normal_f32((C_out, C_in, R, S), 3002, (2.0 / (C_in * R * S)) ** 0.5)
    y_ref, d = oracle.conv2d(x, w, stride, pad)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d(dev(torch, x), dev(torch, w), stride, pad, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"conv2d {case}")


def test_workload3_full_size(torch, sw, oracle):
    x, w = inputs.workload3()
    y_ref, d = oracle.conv2d(x, w, 1, 1)
    y = sw.sw_conv2d(dev(torch, x), dev(torch, w), 1, 1)
    assert_f32_parity(y.cpu().numpy(), y_ref, d, "workload 3")


# ----------------------------------------------------------------------------- 2-D int8

S8_CASES = [
    (1, 3, 5, 9, 11, 3, 3, 1, 1),
    (2, 4, 3, 12, 10, 2, 5, 2, 2),
    (1, 128, 128, 28, 28, 3, 3, 1, 1),
    (2, 64, 64, 28, 28, 3, 3, 1, 1),
    (1, 128, 64, 13, 17, 3, 3, 1, 1),    # ragged, width not a multiple of 4: direct kernel
    (1, 128, 64, 13, 20, 3, 3, 1, 1),    # ragged row bands on the matrix-core path
    (1, 64, 128, 30, 12, 3, 3, 1, 0),    # valid mode
    (1, 64, 64, 9, 100, 3, 3, 1, 1),     # two column tiles
    (2, 64, 64, 56, 56, 3, 3, 1, 1),
    (1, 192, 64, 7, 8, 3, 3, 1, 2),      # padding wider than the filter needs
    (2, 128, 64, 20, 28, 3, 3, 1, 1),    # all of K resident in LDS; last row band ragged
    (1, 128, 128, 9, 12, 3, 3, 1, 0),    # resident, tile with a single live pixel block pair
    (1, 128, 64, 5, 40, 3, 3, 1, 1),     # resident, odd block count
    (1, 64, 128, 30, 9, 3, 3, 1, 0),
    (1, 192, 64, 10, 10, 5, 5, 1, 2),
    (1, 64, 64, 15, 15, 3, 3, 2, 1),
    (2, 3, 10, 23, 21, 3, 3, 1, 1),      # any-shape matrix-core kernel: odd channel counts
    (1, 3, 64, 60, 60, 7, 7, 2, 3),      # ... 7x7 stride 2 stem (channel chunks of 32)
    (2, 40, 33, 12, 150, 3, 3, 1, 1),    # ... output rows wider than a tile
    (1, 70, 65, 20, 9, 5, 3, 1, 2),      # ... rectangular filter, two channel chunks, ragged channel block
    (3, 64, 96, 7, 7, 3, 3, 1, 1),       # ... small images
    (2, 100, 64, 14, 14, 1, 1, 1, 0),    # ... pointwise (two chunks, the second ragged; width not a multiple of 4)
    (2, 64, 70, 28, 28, 1, 1, 1, 0),     # ... pointwise, rows read as dwords, ragged output-channel block
    (1, 36, 64, 16, 20, 1, 1, 2, 0),     # ... pointwise with stride, C_in a multiple of 4 but not of the chunk
    (1, 30, 16, 16, 16, 1, 1, 1, 0),     # ... pointwise, C_in not a multiple of 4: byte copy of the filters
    (2, 8, 8, 24, 36, 3, 3, 1, 2),       # ... dword rows with padding on both sides
    (1, 16, 32, 33, 40, 4, 4, 3, 1),     # ... stride 3, even filter
    (1, 64, 64, 17, 19, 3, 3, 2, 1),     # ... stride 2
    (1, 2, 4, 5, 5, 5, 5, 1, 0),         # ... a single output pixel
    (1, 9, 130, 16, 16, 2, 2, 2, 0),
]


@pytest.mark.parametrize("case", S8_CASES)
def test_conv2d_s8(torch, sw, oracle, case):
    N, C_in, C_out, H, W, R, S, stride, pad = case
    x = inputs.uniform_s8((N, C_in, H, W), 5001)
    w = inputs.uniform_s8((C_out, C_in, R, S), 5002)
    y_ref = oracle.conv2d_s8(x, w, stride, pad)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.int32)
    sw.sw_conv2d_s8(dev(torch, x), dev(torch, w), stride, pad, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert np.array_equal(out.cpu().numpy(), y_ref), f"s8 {case} is not bit-exact"


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("case", [
    (2, 128, 128, 28, 28, 3, 3, 1, 1),    # resident-K kernel
    (1, 128, 64, 20, 28, 3, 3, 1, 1),     # ... ragged last row band
    (2, 64, 64, 28, 28, 3, 3, 1, 1),      # any-shape kernel (the chunked large-tile variant has no fused store)
    (1, 40, 70, 12, 15, 3, 3, 2, 1),      # ... odd channel counts, stride 2
    (1, 100, 33, 9, 9, 1, 1, 1, 0),       # ... pointwise
    (1, 8, 5, 20, 20, 7, 7, 1, 3),        # 49 taps: one thread per output
], ids=lambda c: "x".join(map(str, c)))
def test_conv2d_s8_requant(torch, sw, oracle, case, relu):
    N, C_in, C_out, H, W, R, S, stride, pad = case
    x = inputs.uniform_s8((N, C_in, H, W), 4101)
    w = inputs.uniform_s8((C_out, C_in, R, S), 4102)
    rng = np.random.default_rng(4103)
    bias = rng.integers(-20000, 20000, size=C_out).astype(np.int32)
    # scales that bring the sums into the int8 range, with a few exact powers of two (ties do occur)
    std = np.sqrt(C_in * R * S) * 5461.0                   # of the sums: uniform int8 operands have variance 5461
    scale = (rng.uniform(0.5, 2.0, size=C_out) * 40.0 / std).astype(np.float32)
    scale[::3] = np.float32(2.0 ** np.round(np.log2(40.0 / std)))
    q_ref = oracle.conv2d_s8_requant(x, w, bias, scale, stride, pad, relu)
    buf, out, front, n, s = guarded_empty(torch, q_ref.shape, torch.int8, fill=77)
    sw.sw_conv2d_s8_requant(dev(torch, x), dev(torch, w), dev(torch, bias), dev(torch, scale), stride, pad, relu, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    q = out.cpu().numpy()
    assert np.array_equal(q, q_ref), f"requant {case}: {np.count_nonzero(q != q_ref)} of {q.size} differ"
    assert len(np.unique(q_ref)) > (30 if relu else 60)   # the case exercises the range, not just the clamps
    # no bias
    q_ref = oracle.conv2d_s8_requant(x, w, None, scale, stride, pad, relu)
    q = sw.sw_conv2d_s8_requant(dev(torch, x), dev(torch, w), None, dev(torch, scale), stride, pad, relu).cpu().numpy()
    assert np.array_equal(q, q_ref)


def test_workload5_requantised_full_size(torch, sw, oracle):
    x, w = inputs.workload5()
    rng = np.random.default_rng(4104)
    bias = rng.integers(-50000, 50000, size=128).astype(np.int32)
    scale = rng.uniform(1.0, 3.0, size=128).astype(np.float32) * np.float32(2.0 ** -18)
    q_ref = oracle.conv2d_s8_requant(x, w, bias, scale, 1, 1, True)
    q = sw.sw_conv2d_s8_requant(dev(torch, x), dev(torch, w), dev(torch, bias), dev(torch, scale), 1, 1, True).cpu().numpy()
    assert np.array_equal(q, q_ref)


def test_s8_extreme_values(torch, sw):
    x = np.full((1, 128, 28, 28), -128, np.int8)
    w = np.full((128, 128, 3, 3), -128, np.int8)
    y = sw.sw_conv2d_s8(dev(torch, x), dev(torch, w), 1, 1).cpu().numpy()
    assert y[0, 5, 10, 10] == 18874368 and y[0, 0, 0, 0] == 128 * 4 * 16384 and y[0, 127, 27, 13] == 128 * 6 * 16384
    w[:] = 127
    y = sw.sw_conv2d_s8(dev(torch, x), dev(torch, w), 1, 1).cpu().numpy()
    assert y[0, 64, 14, 14] == 1152 * (-128 * 127)


def test_workload5_full_size(torch, sw, oracle):
    x, w = inputs.workload5()
    y_ref = oracle.conv2d_s8(x, w, 1, 1)
    y = sw.sw_conv2d_s8(dev(torch, x), dev(torch, w), 1, 1)
    assert np.array_equal(y.cpu().numpy(), y_ref)


# ----------------------------------------------------------------------------- contract

def test_no_device_allocation_and_side_stream(torch, sw, oracle):
    x, w = inputs.workload3(N=2)
    xd, wd = dev(torch, x), dev(torch, w)
    out = torch.empty((2, 64, 56, 56), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    # first use of a stream and of a kernel makes the HIP runtime set up its own resources
    sw.sw_conv2d(xd, wd, 1, 1, out=out, stream=side)
    torch.cuda.synchronize()
    out.zero_()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    free_before, _ = torch.cuda.mem_get_info()
    with torch.cuda.stream(side):
        sw.sw_conv2d(xd, wd, 1, 1, out=out, stream=side)
    side.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.cuda.mem_get_info()[0] == free_before       # no hipMalloc behind torch's back either
    y_ref, d = oracle.conv2d(x, w, 1, 1)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, "side stream")


def test_bad_arguments_raise(torch, sw):
    x = torch.zeros((2, 16), device="cuda")
    w = torch.zeros((32,), device="cuda")
    with pytest.raises(sw.SwError):
        sw.sw_conv1d(x, w)                       # filter longer than the row
    with pytest.raises(sw.SwError):
        sw.sw_pool1d(x, 4, 1, 7)                 # unknown mode
