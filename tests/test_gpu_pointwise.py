"""GPU parity of the pointwise (1 x 1, stride 1, no padding) matrix-core kernel against the CPU oracle: every variant
(output-channel blocks x pixel blocks per wavefront), channel-group counts of every remainder modulo the register ring,
partial channel blocks, partial tiles, several tiles per wavefront, and the shapes that must fall back to the window
kernels."""
import numpy as np
import pytest
import torch

import paper_2310_05218_amd as sw
from paper_2310_05218_amd import inputs
from parity import assert_f32_parity

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# (N, C_in, C_out, H, W, expected kernel)
CASES = [
    # several tiles per wavefront (more than 2048 tiles): 1, 3 and 6 channel groups
    (5, 8, 32, 256, 256, "mfma_f32_pointwise_kernel<2,4>"),
    (5, 24, 40, 256, 256, "mfma_f32_pointwise_kernel<2,4>"),
    (3, 48, 64, 300, 300, "mfma_f32_pointwise_kernel<2,4>"),
    # few tiles: the smallest variant; 4 and 5 channel groups, partial channel blocks
    (2, 32, 100, 28, 28, "mfma_f32_pointwise_kernel<1,2>"),
    (2, 40, 64, 14, 14, "mfma_f32_pointwise_kernel<1,2>"),
    (1, 8, 1, 2, 2, "mfma_f32_pointwise_kernel<1,2>"),
    # plane size even but no multiple of 4: 8-byte loads
    (120, 16, 128, 15, 14, "mfma_f32_pointwise_kernel<2,2>"),
    (3, 16, 7, 9, 10, "mfma_f32_pointwise_kernel<1,2>"),
    # more input channels than two channel blocks' filters fit beside: one block per wavefront
    (4, 600, 512, 40, 40, "mfma_f32_pointwise_kernel<1,4>"),
    (32, 512, 512, 14, 14, "mfma_f32_pointwise_kernel<1,4>"),
    # one full-size image of a bottleneck layer
    (1, 256, 64, 56, 56, "mfma_f32_pointwise_kernel<1,2>"),
    (8, 256, 64, 56, 56, "mfma_f32_pointwise_kernel<1,2>"),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "x".join(str(v) for v in c[:5]))
def test_pointwise(oracle, case):
    N, Ci, Co, H, W, kernel = case
    x = inputs.normal_f32((N, Ci, H, W), inputs.seed_for(7, 31 * Ci + Co))
    w = inputs.normal_f32((Co, Ci, 1, 1), inputs.seed_for(7, 1000 + Ci), (2.0 / Ci) ** 0.5)
    y_ref, d = oracle.conv2d(x, w, 1, 0)
    guard = torch.full((x.shape[0] * Co * H * W + 64,), 7.25, device="cuda")
    out = guard[32:-32].view(N, Co, H, W)
    sw.sw_conv2d(dev(x), dev(w), 1, 0, out=out)
    assert sw.sw_last_kernel() == kernel
    assert_f32_parity(out.cpu().numpy(), y_ref, d, f"pointwise {case}")
    g = guard.cpu().numpy()
    assert np.all(g[:32] == 7.25) and np.all(g[-32:] == 7.25), "wrote outside the output"


@pytest.mark.parametrize("case", [(3, 24, 130, 10, 14, True), (2, 40, 64, 28, 28, False), (9, 64, 96, 56, 56, True)],
                         ids=lambda c: "x".join(str(v) for v in c))
def test_pointwise_bias_relu(oracle, case):
    N, Ci, Co, H, W, relu = case
    x = inputs.normal_f32((N, Ci, H, W), inputs.seed_for(7, 5))
    w = inputs.normal_f32((Co, Ci, 1, 1), inputs.seed_for(7, 6), (2.0 / Ci) ** 0.5)
    b = inputs.normal_f32((Co,), inputs.seed_for(7, 7))
    y_ref, d = oracle.conv2d_bias_relu(x, w, b, 1, 0, relu)
    y = sw.sw_conv2d_bias_relu(dev(x), dev(w), dev(b), 1, 0, relu)
    assert sw.sw_last_kernel().startswith("mfma_f32_pointwise_kernel")
    assert_f32_parity(y.cpu().numpy(), y_ref, d, f"pointwise bias/relu {case}")


# what the kernel does not take goes to the window kernels: odd plane sizes, channel counts that are no multiple of
# eight, padding, stride, a misaligned input
@pytest.mark.parametrize("case", [(2, 16, 32, 7, 7, 1, 0, 0), (2, 12, 32, 8, 8, 1, 0, 0), (2, 16, 32, 8, 8, 1, 1, 0), (2, 16, 32, 8, 8, 2, 0, 0),
                                  (2, 16, 32, 8, 8, 1, 0, 1)],
                         ids=lambda c: "x".join(str(v) for v in c))
def test_pointwise_fallbacks(oracle, case):
    N, Ci, Co, H, W, stride, pad, shift = case
    x = inputs.normal_f32((N, Ci, H, W), inputs.seed_for(7, 8))
    w = inputs.normal_f32((Co, Ci, 1, 1), inputs.seed_for(7, 9), (2.0 / Ci) ** 0.5)
    y_ref, d = oracle.conv2d(x, w, stride, pad)
    xd = torch.empty((x.size + 4,), device="cuda")
    xv = xd[shift:shift + x.size].view(x.shape)       # shift = 1: four bytes off the 16-byte grid
    xv.copy_(dev(x))
    y = sw.sw_conv2d(xv, dev(w), stride, pad)
    assert not sw.sw_last_kernel().startswith("mfma_f32_pointwise_kernel")
    assert_f32_parity(y.cpu().numpy(), y_ref, d, f"1 x 1 outside the pointwise kernel {case}")
