"""GPU parity of every shape that `bench.py --sweep` and `bench.py --layers` time, against the CPU oracle: the
benchmark modes themselves only time (the oracle is test infrastructure), so the check that what they time is
right lives here.  The cases are built by bench.py's own builders.

What is timed is what is checked, structurally: the library's choice of kernel depends on the batch (planes per
launch, workgroups per launch), so every case first asks which kernel the benchmark's full-size launch runs
(`sw_last_kernel`, on zero-filled tensors of the full size) and then checks parity at the smallest batch that runs
the same kernel -- and fails if no batch up to the full one does."""
import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402  (imports nothing heavy at module level)

from paper_2310_05218_amd import inputs  # noqa: E402
from parity import assert_f32_parity  # noqa: E402

pytestmark = pytest.mark.gpu
BATCHES = (1, 2, 4, 8, 16, 32)


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


def batch_that_runs_the_benchmarks_kernel(torch, sw, full_n, launch_zeros):
    """launch_zeros(n) launches the case on zero-filled tensors with batch n.  Returns (n, kernel): the smallest
    batch whose launch runs the kernel of the full-size launch."""
    launch_zeros(full_n)
    want = sw.sw_last_kernel()
    assert want, "the call recorded no kernel"
    for n in [b for b in BATCHES if b < full_n] + [full_n]:
        launch_zeros(n)
        if sw.sw_last_kernel() == want:
            torch.cuda.synchronize()
            return n, want
    raise AssertionError(f"no batch up to {full_n} runs {want}")


@pytest.mark.parametrize("k", bench.SWEEP_FILTERS)
def test_sweep_one_filter_per_plane(torch, sw, oracle, k):
    pad = (k - 1) // 2
    wz = torch.zeros((64, 1, k, k), device="cuda")
    n, kernel = batch_that_runs_the_benchmarks_kernel(
        torch, sw, 32, lambda b: sw.sw_conv2d_depthwise(torch.zeros((b, 64, 56, 56), device="cuda"), wz, 1, pad))
    x = inputs.normal_f32((n, 64, 56, 56), inputs.seed_for(6, 0))
    w = inputs.normal_f32((64, 1, k, k), inputs.seed_for(6, k), 1.0 / k)
    y_ref, d = oracle.conv2d_depthwise(x, w, 1, pad)
    y = sw.sw_conv2d_depthwise(dev(torch, x), dev(torch, w), 1, pad)
    assert sw.sw_last_kernel() == kernel
    assert_f32_parity(y.cpu().numpy(), y_ref, d, f"sweep {k} ({kernel}, batch {n})")
    if sw.sw_jit_prepare_depthwise(56, 56, k, k, 1, pad) == 0:
        y = sw.sw_conv2d_depthwise_jit(dev(torch, x), dev(torch, w), 1, pad).cpu().numpy()
        assert sw.sw_last_kernel().startswith("sliding_plane_jit_kernel")
        assert_f32_parity(y, y_ref, d, f"sweep {k}, generated kernel")
    else:
        assert k > 33, "sizes up to 33 x 33 are inside the generated kernel's range"


@pytest.mark.parametrize("k", bench.MC_SWEEP_FILTERS)
def test_sweep_multi_channel(torch, sw, oracle, k):
    pad = (k - 1) // 2
    wz = torch.zeros((64, 64, k, k), device="cuda")
    n, kernel = batch_that_runs_the_benchmarks_kernel(
        torch, sw, 32, lambda b: sw.sw_conv2d(torch.zeros((b, 64, 56, 56), device="cuda"), wz, 1, pad))
    w = inputs.normal_f32((64, 64, k, k), inputs.seed_for(6, 1000 + k), (2.0 / (64 * k * k)) ** 0.5)
    # beyond 13 x 13 the CPU oracle needs minutes for a 56 x 56 image (33 G multiply-adds at 51 x 51): the same
    # filters and channel counts on a 20 x 24 image, which must reach the same kernel instance
    H, W = (56, 56) if k <= 13 else (20, 24)
    x = inputs.normal_f32((n, 64, H, W), inputs.seed_for(6, 1000))
    y_ref, d = oracle.conv2d(x, w, 1, pad)
    y = sw.sw_conv2d(dev(torch, x), dev(torch, w), 1, pad)
    assert sw.sw_last_kernel() == kernel
    assert_f32_parity(y.cpu().numpy(), y_ref, d, f"multi-channel sweep {k} ({kernel}, batch {n}, {H} x {W})")


@pytest.mark.parametrize("k", bench.SWEEP_1D)
def test_sweep_1d(torch, sw, oracle, k):
    wz = torch.zeros((k,), device="cuda")
    calls = {"conv": lambda xd, wd: sw.sw_conv1d(xd, wd, 1, 0), "avg": lambda xd, wd: sw.sw_pool1d(xd, k, 1, sw.SW_POOL_AVG),
             "max": lambda xd, wd: sw.sw_pool1d(xd, k, 1, sw.SW_POOL_MAX)}
    for what, call in calls.items():
        rows, kernel = batch_that_runs_the_benchmarks_kernel(
            torch, sw, 64, lambda b: call(torch.zeros((b, 65536), device="cuda"), wz))
        x = inputs.normal_f32((rows, 65536), inputs.seed_for(6, 2000))
        w = inputs.normal_f32((k,), inputs.seed_for(6, 2000 + k), 1.0 / k ** 0.5)
        y = call(dev(torch, x), dev(torch, w)).cpu().numpy()
        assert sw.sw_last_kernel() == kernel
        if what == "conv":
            assert_f32_parity(y, *oracle.conv1d(x, w, 1, 0), f"conv1d {k} ({kernel})")
        elif what == "avg":
            y_ref, mag = oracle.pool1d(x, k, 1, 0)
            assert_f32_parity(y, y_ref, np.maximum(mag, 1e-300), f"avg {k} ({kernel})")
        else:
            assert np.array_equal(y.astype(np.float64), oracle.pool1d(x, k, 1, 1)[0]), f"max {k} ({kernel})"


@pytest.mark.parametrize("idx", range(len(bench.LAYERS)), ids=[layer[0] for layer in bench.LAYERS])
def test_layer(torch, sw, oracle, idx):
    full_n = bench.LAYERS[idx][2][0]

    def launch_zeros(b):
        cz = bench.layer_case(idx, n_images=b, data=False)
        bench.layer_call(sw, cz, bench.layer_device(torch, cz))

    n, kernel = batch_that_runs_the_benchmarks_kernel(torch, sw, full_n, launch_zeros)
    c = bench.layer_case(idx, n_images=n)
    d = bench.layer_device(torch, c)
    y = bench.layer_call(sw, c, d)
    assert sw.sw_last_kernel() == kernel
    torch.cuda.synchronize()
    name = f"{c['name']} ({kernel}, batch {n})"
    kind, st, p, x, w = c["kind"], c["stride"], c["pad"], c["x"], c["w"]
    if kind in ("max", "avg"):
        y_ref, mag = oracle.pool2d(x, c["R"], c["R"], st, p, 1 if kind == "max" else 0)
        if kind == "max":
            assert np.array_equal(y.cpu().numpy().astype(np.float64), y_ref), name
        else:
            assert_f32_parity(y.cpu().numpy(), y_ref, np.maximum(mag, 1e-300), name)
    elif kind in ("block", "block2"):
        y_ref, mag = oracle.dw_pw_block(x, w, c["bias"], c["w_pw"], c["bias_pw"], True, True)
        err = float(np.max(np.abs(y.cpu().numpy().astype(np.float64) - y_ref) / np.maximum(mag, 1e-300)))
        assert err <= 2e-5, (name, err)
    elif kind == "dw":
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d_depthwise(x, w, st, p), name)
    elif kind in ("dw_dil", "dw_dil_jit"):
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d_dilated(x, w, st, p, c["dil"], depthwise=True), name)
    elif kind == "dw_br":
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d_depthwise_bias_relu(x, w, c["bias"], st, p, True), name)
    elif kind == "dw_bf16":
        y_ref, mag = oracle.conv2d_depthwise(oracle.bf16_to_f32(x), w, st, p)
        yv = oracle.bf16_to_f32(y.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
        assert np.all(np.abs(yv - y_ref) <= 2e-5 * mag + 2.0 ** -8 * np.abs(y_ref) + 1e-37), name
    elif kind == "conv":
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d(x, w, st, p), name)
    elif kind == "conv_br":
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d_bias_relu(x, w, c["bias"], st, p, True), name)
    elif kind == "conv_dil":
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d_dilated(x, w, st, p, c["dil"]), name)
    elif kind == "conv_nhwc":
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d_nhwc(x, w, st, p), name)
    elif kind == "conv_bf16_nhwc":
        y_ref, mag = oracle.conv2d_bf16_nhwc(x, w, st, p)
        yv = oracle.bf16_to_f32(y.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
        assert np.all(np.abs(yv - y_ref) <= 2e-5 * mag + 2.0 ** -8 * np.abs(y_ref) + 1e-37), name
    elif kind == "conv_f16_nhwc":
        y_ref, mag = oracle.conv2d_f16_nhwc(x, w, st, p)
        yv = oracle.f16_to_f32(y.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
        assert np.all(np.abs(yv - y_ref) <= 2e-5 * mag + 2.0 ** -11 * np.abs(y_ref) + 2.0 ** -25), name
    elif kind in ("conv_s8", "conv_s8_pk"):
        assert np.array_equal(y.cpu().numpy(), oracle.conv2d_s8(x, w, st, p)), name
    elif kind in ("conv_s8_rq", "conv_s8_pk_rq"):
        assert np.array_equal(y.cpu().numpy(), oracle.conv2d_s8_requant(x, w, c["bias"], c["scale"], st, p, True)), name
    elif kind == "conv_s8_nhwc":
        assert np.array_equal(y.cpu().numpy(), oracle.conv2d_s8_nhwc(x, w, st, p)), name
    elif kind == "conv_s8_nhwc_rq":
        assert np.array_equal(y.cpu().numpy(), oracle.conv2d_s8_nhwc_requant(x, w, c["bias"], c["scale"], st, p, True)), name
    else:
        raise AssertionError(kind)
