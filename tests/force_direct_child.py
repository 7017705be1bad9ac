"""Run by tests/test_gpu_force_direct.py in a process of its own with SWCONV_FORCE_DIRECT=1 (the switch is read
once per process): shapes the tiled and matrix-core kernels would normally take must now run on the
one-thread-per-output kernels, and still meet the parity bars."""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import torch  # noqa: E402

import oracle  # noqa: E402
import paper_2310_05218_amd as sw  # noqa: E402
from paper_2310_05218_amd import inputs  # noqa: E402
from parity import assert_f32_parity  # noqa: E402

assert os.environ.get("SWCONV_FORCE_DIRECT") == "1"
oracle.build()
dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()


def ran_direct(what):
    k = sw.sw_last_kernel()
    # wave_pool2d_kernel is the direct pooling launcher's own variant for large windows (one wavefront per output)
    assert k.startswith(("direct", "wave_pool2d")), f"{what}: ran {k}"
    print(f"{what}: {k}", flush=True)


x, w = inputs.workload3(N=1)
assert_f32_parity(sw.sw_conv2d(dev(x), dev(w), 1, 1).cpu().numpy(), *oracle.conv2d(x, w, 1, 1), "conv2d")
ran_direct("sw_conv2d 64->64 3x3")
b = inputs.normal_f32((w.shape[0],), 31, 0.5)
assert_f32_parity(sw.sw_conv2d_bias_relu(dev(x), dev(w), dev(b), 1, 1, True).cpu().numpy(),
                  *oracle.conv2d_bias_relu(x, w, b, 1, 1, True), "conv2d_bias_relu")
ran_direct("sw_conv2d_bias_relu")
x, w3, w7 = inputs.workload4(N=2, C=8)
assert_f32_parity(sw.sw_conv2d_depthwise(dev(x), dev(w7), 1, 3).cpu().numpy(), *oracle.conv2d_depthwise(x, w7, 1, 3), "dw 7x7")
ran_direct("sw_conv2d_depthwise 7x7")
assert_f32_parity(sw.sw_conv2d_depthwise_jit(dev(x), dev(w3), 1, 1).cpu().numpy(), *oracle.conv2d_depthwise(x, w3, 1, 1), "dw jit")
ran_direct("sw_conv2d_depthwise_jit 3x3")
assert_f32_parity(sw.sw_conv2d_depthwise_dilated(dev(x), dev(w3), 1, 2, 2).cpu().numpy(),
                  *oracle.conv2d_dilated(x, w3, 1, 2, 2, depthwise=True), "dw dilated")
ran_direct("sw_conv2d_depthwise_dilated")
x1, w1 = inputs.workload2(rows=3, length=4000)
assert_f32_parity(sw.sw_conv1d(dev(x1), dev(w1), 1, 0).cpu().numpy(), *oracle.conv1d(x1, w1, 1, 0), "conv1d")
ran_direct("sw_conv1d")
assert_f32_parity(sw.sw_pool1d(dev(x1), 8, 2, sw.SW_POOL_AVG).cpu().numpy(), *oracle.pool1d(x1, 8, 2, 0), "pool1d avg")
ran_direct("sw_pool1d avg")
assert np.array_equal(sw.sw_pool1d(dev(x1), 8, 1, sw.SW_POOL_MAX).cpu().numpy().astype(np.float64), oracle.pool1d(x1, 8, 1, 1)[0])
ran_direct("sw_pool1d max")
assert_f32_parity(sw.sw_pool2d(dev(x), 3, 3, 2, 1, sw.SW_POOL_AVG).cpu().numpy(), *oracle.pool2d(x, 3, 3, 2, 1, 0), "pool2d avg")
ran_direct("sw_pool2d avg")
assert np.array_equal(sw.sw_pool2d(dev(x), 7, 7, 1, 0, sw.SW_POOL_MAX).cpu().numpy().astype(np.float64), oracle.pool2d(x, 7, 7, 1, 0, 1)[0])
ran_direct("sw_pool2d max")
x8, w8 = inputs.workload5(N=1)
ref = oracle.conv2d_s8(x8, w8, 1, 1)
assert np.array_equal(sw.sw_conv2d_s8(dev(x8), dev(w8), 1, 1).cpu().numpy(), ref)
ran_direct("sw_conv2d_s8")
packed = sw.sw_s8_pack_filter(dev(w8))
assert np.array_equal(sw.sw_conv2d_s8_packed(dev(x8), packed, 128, 3, 3, 1, 1).cpu().numpy(), ref)
ran_direct("sw_conv2d_s8_packed")
scale = np.full(128, 2.0 ** -12, np.float32)
bias = (np.arange(128, dtype=np.int32) * 1000 - 64000).astype(np.int32)
q = sw.sw_conv2d_s8_requant(dev(x8), dev(w8), dev(bias), dev(scale), 1, 1, True).cpu().numpy()
assert np.array_equal(q, oracle.conv2d_s8_requant(x8, w8, bias, scale, 1, 1, True))
ran_direct("sw_conv2d_s8_requant")
xl, wl = np.ascontiguousarray(x8.transpose(0, 2, 3, 1)), np.ascontiguousarray(w8.transpose(0, 2, 3, 1))
assert np.array_equal(sw.sw_conv2d_s8_nhwc(dev(xl), dev(wl), 1, 1).cpu().numpy(), oracle.conv2d_s8_nhwc(xl, wl, 1, 1))
ran_direct("sw_conv2d_s8_nhwc")
xb = oracle.f32_to_bf16_rne(x)
yb = sw.sw_conv2d_depthwise_bf16(torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16), dev(w3), 1, 1)
yv = oracle.bf16_to_f32(yb.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
y_ref, d = oracle.conv2d_depthwise(oracle.bf16_to_f32(xb), w3, 1, 1)
assert np.all(np.abs(yv - y_ref) <= 2e-5 * d + 2.0 ** -8 * np.abs(y_ref) + 1e-37)
ran_direct("sw_conv2d_depthwise_bf16")
# the 16-bit and fp32 channel-last calls on a shape their matrix-core kernels would take
xh, wh = inputs.normal_f16((1, 10, 10, 32), 5301), inputs.normal_f16((16, 3, 3, 32), 5302, 0.1)
h16 = lambda a, dt: torch.from_numpy(a.view(np.int16)).cuda().view(dt)
yh = sw.sw_conv2d_f16_nhwc(h16(xh, torch.float16), h16(wh, torch.float16), 1, 1)
y_ref, d = oracle.conv2d_f16_nhwc(xh, wh, 1, 1)
yv = oracle.f16_to_f32(yh.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
assert np.all(np.abs(yv - y_ref) <= 2e-5 * d + 2.0 ** -11 * np.abs(y_ref) + 2.0 ** -25)
ran_direct("sw_conv2d_f16_nhwc")
xb2, wb2 = inputs.normal_bf16((1, 10, 10, 32), 5303), inputs.normal_bf16((16, 3, 3, 32), 5304, 0.1)
yb2 = sw.sw_conv2d_bf16_nhwc(h16(xb2, torch.bfloat16), h16(wb2, torch.bfloat16), 1, 1)
y_ref, d = oracle.conv2d_bf16_nhwc(xb2, wb2, 1, 1)
yv = oracle.bf16_to_f32(yb2.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
assert np.all(np.abs(yv - y_ref) <= 2e-5 * d + 2.0 ** -8 * np.abs(y_ref) + 1e-37)
ran_direct("sw_conv2d_bf16_nhwc")
print("force-direct ok", flush=True)
