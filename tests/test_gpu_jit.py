"""GPU parity of the kernels generated at run time (sw_conv2d_depthwise_jit) against the CPU oracle, element by
element: fp32, max |y_gpu - y_oracle| / sum|x*w| <= 2e-5 per output.  Each geometry compiles its own kernel."""
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


JIT_CASES = [
    # N, C, H, W, R, S, pad      (stride 1; all inside the generated kernel's range)
    (1, 1, 56, 56, 3, 3, 1),     # a single plane
    (2, 5, 56, 56, 5, 5, 2),
    (3, 7, 56, 56, 7, 7, 3),
    (3, 67, 56, 56, 9, 9, 4),    # one pass over the tap columns, three over the rows
    (2, 9, 56, 56, 11, 11, 5),   # unequal passes on both axes (6 + 5)
    (2, 9, 56, 56, 13, 13, 6),
    (2, 9, 56, 56, 17, 17, 8),   # four wavefronts per CU from here on (larger window)
    (1, 6, 56, 56, 25, 25, 12),
    (1, 5, 56, 56, 33, 33, 16),  # the largest window
    (1, 3, 56, 56, 41, 41, 20),  # beyond it -> precompiled path
    (2, 5, 64, 64, 9, 9, 0),     # no padding: the plane is larger than the output tile
    (2, 5, 56, 56, 5, 9, 2),     # rectangular filter, output 56 x 52
    (2, 5, 56, 56, 9, 5, 2),
    (2, 5, 48, 52, 7, 7, 3),     # ragged plane: lanes at the right and bottom have nothing to store
    (2, 5, 40, 44, 3, 3, 1),
    (2, 5, 56, 56, 1, 1, 0),     # one tap
    (2, 5, 56, 56, 12, 12, 4),   # even extent, output 53 x 53 is not a multiple of 4 -> precompiled path
]


@pytest.mark.parametrize("case", JIT_CASES)
def test_generated_kernel_matches_the_oracle(torch, sw, oracle, case):
    N, C, H, W, R, S, pad = case
    x = inputs.normal_f32((N, C, H, W), 2601)
    w = inputs.normal_f32((C, 1, R, S), 2602)
    y_ref, d = oracle.conv2d_depthwise(x, w, 1, pad)
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_depthwise_jit(dev(torch, x), dev(torch, w), 1, pad, out=out)
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"jit depthwise {case}")


STRIDED_DILATED_JIT_CASES = [
    # N, C, H, W, R, S, stride, pad, dilation   (all inside the generated kernel's range)
    (2, 5, 56, 56, 3, 3, 1, 2, 2),      # dilation 2, "same"
    (2, 5, 56, 56, 3, 3, 1, 4, 4),
    (1, 6, 56, 56, 3, 3, 1, 6, 6),
    (1, 6, 56, 56, 3, 3, 1, 12, 12),    # span 25
    (2, 5, 56, 56, 5, 5, 1, 4, 2),      # 5x5 at dilation 2
    (1, 4, 56, 56, 7, 7, 1, 9, 3),      # 49 taps at dilation 3: passes on both axes
    (2, 5, 60, 60, 3, 3, 1, 0, 2),      # no padding: 56 x 56 outputs of a 60 x 60 plane
    (2, 5, 48, 52, 3, 5, 1, 2, 2),      # rectangular filter, ragged plane
    (2, 5, 28, 28, 3, 3, 1, 1, 1),      # a 28 x 28 plane: four outputs per lane and axis
    (2, 5, 28, 28, 5, 5, 1, 4, 2),
    (3, 7, 56, 56, 3, 3, 2, 1, 1),      # stride 2: 28 x 28 outputs
    (2, 5, 64, 64, 3, 3, 2, 1, 1),      # ... 32 x 32
    (2, 5, 56, 56, 5, 5, 2, 2, 1),
    (1, 5, 64, 64, 7, 7, 2, 3, 1),
    (2, 5, 64, 64, 3, 3, 2, 2, 2),      # stride 2 with dilation 2
    (2, 5, 40, 48, 3, 3, 2, 1, 1),      # 20 x 24 outputs: three per lane and axis, ragged
]


@pytest.mark.parametrize("case", STRIDED_DILATED_JIT_CASES, ids=lambda c: "x".join(map(str, c)))
def test_generated_strided_and_dilated_kernels(torch, sw, oracle, case):
    N, C, H, W, R, S, stride, pad, dil = case
    x = inputs.normal_f32((N, C, H, W), 2641)
    w = inputs.normal_f32((C, 1, R, S), 2642)
    y_ref, d = oracle.conv2d_dilated(x, w, stride, pad, dil, depthwise=True)
    assert sw.sw_jit_prepare_depthwise_dilated(H, W, R, S, stride, pad, dil) == 0
    buf, out, front, n, s = guarded_empty(torch, y_ref.shape, torch.float32)
    sw.sw_conv2d_depthwise_dilated_jit(dev(torch, x), dev(torch, w), stride, pad, dil, out=out)
    assert sw.sw_last_kernel() == f"sliding_plane_jit_kernel<{R},{S},{stride},{dil}>", sw.sw_last_kernel()
    torch.cuda.synchronize()
    assert_guards_intact(buf, front, n, s)
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"jit strided / dilated depthwise {case}")


def test_several_planes_per_wavefront(torch, sw, oracle):
    """More planes than the launch has wavefronts (2048): the persistent loop, the prefetch of the next plane and
    the last, partly filled round."""
    N, C, H, W, k = 5, 421, 56, 56, 9          # 2105 planes
    x = inputs.normal_f32((N, C, H, W), 2611)
    w = inputs.normal_f32((C, 1, k, k), 2612)
    y_ref, d = oracle.conv2d_depthwise(x, w, 1, 4)
    y = sw.sw_conv2d_depthwise_jit(dev(torch, x), dev(torch, w), 1, 4)
    assert_f32_parity(y.cpu().numpy(), y_ref, d, "jit depthwise, 2105 planes")
    # four wavefronts per CU (1024): three rounds
    N, C, k = 3, 701, 17                        # 2103 planes
    x = inputs.normal_f32((N, C, H, W), 2613)
    w = inputs.normal_f32((C, 1, k, k), 2614)
    y_ref, d = oracle.conv2d_depthwise(x, w, 1, 8)
    y = sw.sw_conv2d_depthwise_jit(dev(torch, x), dev(torch, w), 1, 8)
    assert_f32_parity(y.cpu().numpy(), y_ref, d, "jit depthwise 17x17, 2103 planes")


def test_a_geometry_is_compiled_once(torch, sw):
    x = dev(torch, inputs.normal_f32((1, 2, 56, 56), 2621))
    w = dev(torch, inputs.normal_f32((2, 1, 15, 15), 2622))
    assert sw.sw_jit_prepare_depthwise(56, 56, 15, 15, 1, 7) == 0
    n = sw.sw_jit_cached_kernels()
    y1 = sw.sw_conv2d_depthwise_jit(x, w, 1, 7)
    y2 = sw.sw_conv2d_depthwise_jit(x, w, 1, 7)
    assert sw.sw_jit_cached_kernels() == n
    assert torch.equal(y1, y2)
    # a shape outside the generated kernel's range compiles nothing and still gives the result
    xs = dev(torch, inputs.normal_f32((1, 2, 8, 8), 2623))
    assert sw.sw_jit_prepare_depthwise(8, 8, 15, 15, 1, 7) == 3
    ys = sw.sw_conv2d_depthwise_jit(xs, w, 1, 7)
    assert sw.sw_jit_cached_kernels() == n
    assert torch.equal(ys, sw.sw_conv2d_depthwise(xs, w, 1, 7))


def test_generated_and_precompiled_kernels_agree_at_full_size(torch, sw, oracle):
    """The sweep's workload (32 x 64 planes of 56 x 56, 13 x 13): every output against the oracle, and against the
    precompiled run-time-extent kernel within twice the parity bound."""
    N, C, k = 32, 64, 13
    x = inputs.normal_f32((N, C, 56, 56), 2631)
    w = inputs.normal_f32((C, 1, k, k), 2632, 1.0 / k)
    xd, wd = dev(torch, x), dev(torch, w)
    y = sw.sw_conv2d_depthwise_jit(xd, wd, 1, 6).cpu().numpy()
    y_ref, d = oracle.conv2d_depthwise(x, w, 1, 6)
    assert_f32_parity(y, y_ref, d, "jit 13x13 full size")
    y_pre = sw.sw_conv2d_depthwise(xd, wd, 1, 6).cpu().numpy()
    dsum = np.abs(x).max() * np.abs(w).reshape(C, -1).sum(axis=1).max()
    assert np.max(np.abs(y - y_pre)) <= 4e-5 * dsum
