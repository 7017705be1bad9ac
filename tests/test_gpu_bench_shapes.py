"""GPU parity of every shape that `bench.py --sweep` and `bench.py --layers` time, against the CPU oracle: the
benchmark modes themselves only time (the oracle is test infrastructure), so the check that what they time is
right lives here.  Full channel counts and plane sizes, one image (two planes for the one-filter-per-plane sweep);
the cases are built by bench.py's own builders, so what is timed is what is checked."""
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


@pytest.mark.parametrize("k", bench.SWEEP_FILTERS)
def test_sweep_one_filter_per_plane(torch, sw, oracle, k):
    x = inputs.normal_f32((1, 2, 56, 56), inputs.seed_for(6, 0))
    w = inputs.normal_f32((2, 1, k, k), inputs.seed_for(6, k), 1.0 / k)
    pad = (k - 1) // 2
    y_ref, d = oracle.conv2d_depthwise(x, w, 1, pad)
    assert_f32_parity(sw.sw_conv2d_depthwise(dev(torch, x), dev(torch, w), 1, pad).cpu().numpy(), y_ref, d, f"sweep {k}")
    if sw.sw_jit_prepare_depthwise(56, 56, k, k, 1, pad) == 0:
        y = sw.sw_conv2d_depthwise_jit(dev(torch, x), dev(torch, w), 1, pad).cpu().numpy()
        assert_f32_parity(y, y_ref, d, f"sweep {k}, generated kernel")
    else:
        assert k > 33, "sizes up to 33 x 33 are inside the generated kernel's range"


@pytest.mark.parametrize("k", bench.MC_SWEEP_FILTERS)
def test_sweep_multi_channel(torch, sw, oracle, k):
    x = inputs.normal_f32((1, 64, 56, 56), inputs.seed_for(6, 1000))
    w = inputs.normal_f32((64, 64, k, k), inputs.seed_for(6, 1000 + k), (2.0 / (64 * k * k)) ** 0.5)
    pad = (k - 1) // 2
    y_ref, d = oracle.conv2d(x, w, 1, pad)
    assert_f32_parity(sw.sw_conv2d(dev(torch, x), dev(torch, w), 1, pad).cpu().numpy(), y_ref, d, f"multi-channel sweep {k}")


@pytest.mark.parametrize("k", bench.SWEEP_1D)
def test_sweep_1d(torch, sw, oracle, k):
    x = inputs.normal_f32((2, 65536), inputs.seed_for(6, 2000))
    w = inputs.normal_f32((k,), inputs.seed_for(6, 2000 + k), 1.0 / k ** 0.5)
    xd = dev(torch, x)
    assert_f32_parity(sw.sw_conv1d(xd, dev(torch, w), 1, 0).cpu().numpy(), *oracle.conv1d(x, w, 1, 0), f"conv1d {k}")
    y_ref, mag = oracle.pool1d(x, k, 1, 0)
    assert_f32_parity(sw.sw_pool1d(xd, k, 1, sw.SW_POOL_AVG).cpu().numpy(), y_ref, np.maximum(mag, 1e-300), f"avg {k}")
    ym = sw.sw_pool1d(xd, k, 1, sw.SW_POOL_MAX).cpu().numpy().astype(np.float64)
    assert np.array_equal(ym, oracle.pool1d(x, k, 1, 1)[0]), f"max {k}"


@pytest.mark.parametrize("idx", range(len(bench.LAYERS)), ids=[layer[0] for layer in bench.LAYERS])
def test_layer(torch, sw, oracle, idx):
    c = bench.layer_case(idx, n_images=1)
    d = bench.layer_device(torch, c)
    y = bench.layer_call(sw, c, d)
    torch.cuda.synchronize()
    kind, st, p, x, w = c["kind"], c["stride"], c["pad"], c["x"], c["w"]
    if kind in ("max", "avg"):
        y_ref, mag = oracle.pool2d(x, c["R"], c["R"], st, p, 1 if kind == "max" else 0)
        if kind == "max":
            assert np.array_equal(y.cpu().numpy().astype(np.float64), y_ref), c["name"]
        else:
            assert_f32_parity(y.cpu().numpy(), y_ref, np.maximum(mag, 1e-300), c["name"])
    elif kind in ("block", "block2"):
        y_ref, mag = oracle.dw_pw_block(x, w, c["bias"], c["w_pw"], c["bias_pw"], True, True)
        err = float(np.max(np.abs(y.cpu().numpy().astype(np.float64) - y_ref) / np.maximum(mag, 1e-300)))
        assert err <= 4e-5, (c["name"], err)
    elif kind == "dw":
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d_depthwise(x, w, st, p), c["name"])
    elif kind == "dw_br":
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d_depthwise_bias_relu(x, w, c["bias"], st, p, True), c["name"])
    elif kind == "dw_bf16":
        y_ref, mag = oracle.conv2d_depthwise(inputs.bf16_bits_to_f32(x), w, st, p)
        yv = inputs.bf16_bits_to_f32(y.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
        assert np.all(np.abs(yv - y_ref) <= 2e-5 * mag + 2.0 ** -8 * np.abs(y_ref) + 1e-37), c["name"]
    elif kind == "conv":
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d(x, w, st, p), c["name"])
    elif kind == "conv_br":
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d_bias_relu(x, w, c["bias"], st, p, True), c["name"])
    elif kind == "conv_dil":
        assert_f32_parity(y.cpu().numpy(), *oracle.conv2d_dilated(x, w, st, p, c["dil"]), c["name"])
    elif kind == "conv_s8":
        assert np.array_equal(y.cpu().numpy(), oracle.conv2d_s8(x, w, st, p)), c["name"]
    elif kind == "conv_s8_rq":
        assert np.array_equal(y.cpu().numpy(), oracle.conv2d_s8_requant(x, w, c["bias"], c["scale"], st, p, True)), c["name"]
    elif kind == "conv_s8_nhwc":
        assert np.array_equal(y.cpu().numpy(), oracle.conv2d_s8_nhwc(x, w, st, p)), c["name"]
    elif kind == "conv_s8_nhwc_rq":
        assert np.array_equal(y.cpu().numpy(), oracle.conv2d_s8_nhwc_requant(x, w, c["bias"], c["scale"], st, p, True)), c["name"]
    else:
        raise AssertionError(kind)
