"""The library under HIP graph capture: every entry point of the benchmark step (and the run-time-generated kernel,
prepared beforehand) is captured once and replayed several times on changing inputs, with the program's own eager
work and synchronisations between the replays; every replay must give exactly what the eager call gives.  The
library allocates nothing and records no memset node, so a captured launch is just its kernel."""
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


def test_replays_equal_eager_calls(torch, sw):
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    # static buffers of the graph
    x1 = dev(inputs.normal_f32((2, 5000), 6001)); w1 = dev(inputs.normal_f32((9,), 6002))
    x3 = dev(inputs.normal_f32((2, 16, 56, 56), 6003)); w3 = dev(inputs.normal_f32((64, 16, 3, 3), 6004, 0.1))
    b3 = dev(inputs.normal_f32((64,), 6005))
    x4 = dev(inputs.normal_f32((2, 8, 56, 56), 6006)); w4 = dev(inputs.normal_f32((8, 1, 7, 7), 6007, 0.15))
    w9 = dev(inputs.normal_f32((8, 1, 9, 9), 6008, 0.1))
    x5 = dev(inputs.uniform_s8((2, 128, 28, 28), 6009)); w5 = dev(inputs.uniform_s8((128, 128, 3, 3), 6010))
    # channel-last tensors: the window-in-LDS kernel in fp32, bf16 and int8 (int32 and requantised int8 out)
    x6 = dev(inputs.normal_f32((2, 28, 28, 64), 6012)); w6 = dev(inputs.normal_f32((64, 3, 3, 64), 6013, 0.05))
    x6b, w6b = x6.bfloat16(), w6.bfloat16()
    x7 = dev(inputs.uniform_s8((2, 28, 28, 128), 6014)); w7 = dev(inputs.uniform_s8((128, 3, 3, 128), 6015))
    b7 = dev(np.arange(128, dtype=np.int32) * 100 - 6400); s7 = dev(np.full((128,), 3e-4, np.float32))
    assert sw.sw_jit_prepare_depthwise(56, 56, 9, 9, 1, 4) == 0        # compiled before the capture

    def run():
        return [sw.sw_conv1d(x1, w1, 1, 0), sw.sw_pool1d(x1, 8, 1, sw.SW_POOL_AVG), sw.sw_pool1d(x1, 8, 1, sw.SW_POOL_MAX),
                sw.sw_conv2d(x3, w3, 1, 1), sw.sw_conv2d_bias_relu(x3, w3, b3, 1, 1, True),
                sw.sw_conv2d_depthwise(x4, w4, 1, 3), sw.sw_conv2d_depthwise_jit(x4, w9, 1, 4),
                sw.sw_pool2d(x4, 3, 3, 2, 1, sw.SW_POOL_MAX), sw.sw_conv2d_s8(x5, w5, 1, 1),
                sw.sw_conv2d_nhwc(x6, w6, 1, 1, 1, b3, True), sw.sw_conv2d_bf16_nhwc(x6b, w6b, 1, 1, 1, b3, True),
                sw.sw_conv2d_s8_nhwc(x7, w7, 1, 1), sw.sw_conv2d_s8_nhwc(x7, w7, 1, 1, bias=b7, scale=s7, relu=True)]

    run()                                                             # warm-up outside the capture
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(st):
        with torch.cuda.graph(g, stream=st):
            outs = run()
    torch.cuda.current_stream().wait_stream(st)
    rng = np.random.default_rng(6011)
    for replay in range(4):
        # new data in the static inputs, some eager work of the program in between
        for t in (x1, x3, x4):
            t.copy_(torch.from_numpy(rng.standard_normal(tuple(t.shape)).astype(np.float32)))
        x5.copy_(torch.from_numpy(rng.integers(-128, 128, size=tuple(x5.shape)).astype(np.int8)))
        x6.copy_(torch.from_numpy(rng.standard_normal(tuple(x6.shape)).astype(np.float32)))
        x6b.copy_(x6)
        x7.copy_(torch.from_numpy(rng.integers(-128, 128, size=tuple(x7.shape)).astype(np.int8)))
        scratch = (x3 * 2.0).sum().item()                              # eager kernels and a synchronisation
        assert np.isfinite(scratch)
        g.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        want = run()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(got, want)):
            assert torch.equal(a, b), f"replay {replay}: output {i} differs from the eager call"
