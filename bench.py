#!/usr/bin/env python3
"""Benchmark of the sliding-window convolution / pooling library on one MI355X.

A *step* is one pass of the whole hot path over one batch of synthetic input: the eight kernel
launches that cover the five workloads (single-channel 3x3; 1-D conv + avg + max pooling;
multi-channel fp32 3x3; depthwise 3x3 and 7x7; int8 3x3).  Inputs are resident in HBM before the
timed region starts.  Steps rotate over several buffer sets so that the ~0.44 GB a step touches
is not served from the 256 MB Infinity Cache.

Prints ONE JSON line.  `value` is useful operations per second over the whole step (2 per
multiply-add of the direct definition, window-1 adds/compares per pooled output ... the counts
are in WORK below); `roofline` is for the kernel that takes the largest share of a step, timed
with HIP events on the launch stream inside the timed region; `cpu_baseline` is the CPU oracle
(naive fp64 / int64 loops, OpenMP) on the same step, timed on this host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published peaks
HBM_GBS = 8000.0
MFMA_F32_TFLOPS = 157.3
MFMA_I8_TOPS = 5000.0
VALU_F32_TFLOPS = 78.6     # 256 CU x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz, no packed FP32


def work_table():
    """name -> (useful ops per launch, algorithmic bytes per launch, bound, peak, unit)."""
    f = 4
    t = {}
    t["conv2d_1ch_3x3"] = (2 * 9 * 254 * 254, 256 * 256 * f + 9 * f + 254 * 254 * f, "hbm", HBM_GBS, "GB/s")
    t["conv1d_k9"] = (2 * 9 * 64 * 65528, 64 * 65536 * f + 9 * f + 64 * 65528 * f, "hbm", HBM_GBS, "GB/s")
    t["avgpool1d_w8"] = (8 * 64 * 65529, 64 * 65536 * f + 64 * 65529 * f, "hbm", HBM_GBS, "GB/s")
    t["maxpool1d_w8"] = (7 * 64 * 65529, 64 * 65536 * f + 64 * 65529 * f, "hbm", HBM_GBS, "GB/s")
    px = 32 * 56 * 56
    t["conv2d_64x64_3x3"] = (2 * 64 * 64 * 9 * px, 2 * 64 * px * f + 64 * 64 * 9 * f, "mfma", MFMA_F32_TFLOPS, "TFLOP/s")
    t["depthwise_3x3"] = (2 * 9 * 256 * px, 2 * 256 * px * f + 256 * 9 * f, "hbm", HBM_GBS, "GB/s")
    t["depthwise_7x7"] = (2 * 49 * 256 * px, 2 * 256 * px * f + 256 * 49 * f, "hbm", HBM_GBS, "GB/s")
    px8 = 32 * 28 * 28
    # 456.6 op/B is below the int8 ridge (5000 TOP/s / 8 TB/s = 625 op/B): the applicable roof is HBM
    t["conv2d_s8_128x128_3x3"] = (2 * 128 * 128 * 9 * px8, 128 * px8 + 128 * 128 * 9 + 128 * px8 * 4, "hbm",
                                  HBM_GBS, "GB/s")
    return t


# second roof quoted beside the bounding one: name -> (peak in T(FL)OP/s, label)
SECOND_ROOF = {"depthwise_7x7": (VALU_F32_TFLOPS, "frac_alu_f32_plain_fma"),
               "conv2d_s8_128x128_3x3": (MFMA_I8_TOPS, "frac_mfma_i8")}


# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a plain copy kernel, see
# profiles/hbm_traffic_all_kernels.txt), with the kernel source and its sha256 prefix at the time the
# counters were taken.  A kernel whose source has changed since reports traffic = null.
TRAFFIC = {
    "depthwise_3x3": (207363275, "sw_sliding_plane.hip", "c19725ff48dea175"),
    "depthwise_7x7": (206176097, "sw_sliding_plane.hip", "c19725ff48dea175"),
    "conv2d_64x64_3x3": (62452409, "sw_mfma_f32.hip", "c33152360085e7c7"),
    "conv2d_s8_128x128_3x3": (21142296, "sw_mfma_s8.hip", "83bf83c186c5e9f3"),
    "conv1d_k9": (33896573, "sw_sliding1d.hip", "eeb6f644a27cb890"),
    "avgpool1d_w8": (34163235, "sw_sliding1d.hip", "eeb6f644a27cb890"),
    "maxpool1d_w8": (34136887, "sw_sliding1d.hip", "eeb6f644a27cb890"),
    "conv2d_1ch_3x3": (660935, "sw_sliding_rows.hip", "21935214a73b4290"),
}


def measured_traffic(name):
    import hashlib

    if name not in TRAFFIC:
        return None
    nbytes, src, digest = TRAFFIC[name]
    path = os.path.join(ROOT, "paper_2310_05218_amd", "csrc", src)
    try:
        now = hashlib.sha256(open(path, "rb").read()).hexdigest()[:16]
    except OSError:
        return None
    return nbytes if now == digest else None


def make_sets(torch, nsets):
    from paper_2310_05218_amd import inputs

    host = {}
    host["x1"], host["w1"] = inputs.workload1()
    host["x2"], host["w2"] = inputs.workload2()
    host["x3"], host["w3"] = inputs.workload3()
    host["x4"], host["w4a"], host["w4b"] = inputs.workload4()
    host["x5"], host["w5"] = inputs.workload5()
    sets = []
    for _ in range(nsets):
        d = {k: torch.from_numpy(v).cuda() for k, v in host.items()}
        e = lambda *s, dt=torch.float32: torch.empty(s, dtype=dt, device="cuda")
        d["y1"] = e(1, 1, 254, 254)
        d["y2a"], d["y2b"], d["y2c"] = e(64, 65528), e(64, 65529), e(64, 65529)
        d["y3"] = e(32, 64, 56, 56)
        d["y4a"], d["y4b"] = e(32, 256, 56, 56), e(32, 256, 56, 56)
        d["y5"] = e(32, 128, 28, 28, dt=torch.int32)
        sets.append(d)
    return host, sets


def launches(sw):
    # Order inside a step.  The long launches come first: the host enqueues a launch in about 8 us, so it is ahead
    # of the GPU after them and the short launches that follow never wait for their enqueue.  The matrix-core fp32
    # launch follows the 7x7 depthwise one: measured right after a light kernel it takes 70-74 us, right after an
    # arithmetic-heavy one 66 us (the chip's clock and matrix units are already at their loaded state).
    return [
        ("depthwise_3x3", lambda d: sw.sw_conv2d_depthwise(d["x4"], d["w4a"], 1, 1, out=d["y4a"])),
        ("depthwise_7x7", lambda d: sw.sw_conv2d_depthwise(d["x4"], d["w4b"], 1, 3, out=d["y4b"])),
        ("conv2d_64x64_3x3", lambda d: sw.sw_conv2d(d["x3"], d["w3"], 1, 1, out=d["y3"])),
        ("conv2d_s8_128x128_3x3", lambda d: sw.sw_conv2d_s8(d["x5"], d["w5"], 1, 1, out=d["y5"])),
        ("conv1d_k9", lambda d: sw.sw_conv1d(d["x2"], d["w2"], 1, 0, out=d["y2a"])),
        ("avgpool1d_w8", lambda d: sw.sw_pool1d(d["x2"], 8, 1, sw.SW_POOL_AVG, out=d["y2b"])),
        ("maxpool1d_w8", lambda d: sw.sw_pool1d(d["x2"], 8, 1, sw.SW_POOL_MAX, out=d["y2c"])),
        ("conv2d_1ch_3x3", lambda d: sw.sw_conv2d(d["x1"], d["w1"], 1, 0, out=d["y1"])),
    ]


# buffers each launch touches (for building rotations that are larger than the Infinity Cache)
BUFFERS = {
    "conv2d_1ch_3x3": ("x1", "w1", "y1"), "conv1d_k9": ("x2", "w2", "y2a"), "avgpool1d_w8": ("x2", "y2b"),
    "maxpool1d_w8": ("x2", "y2c"), "conv2d_64x64_3x3": ("x3", "w3", "y3"), "depthwise_3x3": ("x4", "w4a", "y4a"),
    "depthwise_7x7": ("x4", "w4b", "y4b"), "conv2d_s8_128x128_3x3": ("x5", "w5", "y5"),
}
COLD_ROTATION_BYTES = 768 * 1024 * 1024      # 3 x the 256 MB Infinity Cache


def cold_rotation(torch, sets, name):
    """Buffer sets for one launch whose total footprint exceeds COLD_ROTATION_BYTES, so that no launch of the
    rotation finds its data in the Infinity Cache or in L2 (the three full sets come first)."""
    keys = BUFFERS[name]
    per_set = sum(sets[0][k].numel() * sets[0][k].element_size() for k in keys)
    need = min(32, max(len(sets), -(-COLD_ROTATION_BYTES // per_set)))
    rot = [{k: d[k] for k in keys} for d in sets]
    while len(rot) < need:
        rot.append({k: sets[0][k].clone() for k in keys})
    return rot


def time_kernel(torch, fn, sets, reps, batches=5):
    """Per-launch time in us: `reps` back-to-back launches (rotating over `sets`) are captured into one HIP
    graph, so that the host's launch cost does not bound microsecond kernels; each batch replays the graph
    between two events on the launch stream.  Median over batches."""
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        for i in range(len(sets)):
            fn(sets[i])                      # warm-up outside capture
        st.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            for i in range(reps):
                fn(sets[i % len(sets)])
        out = []
        g.replay()
        st.synchronize()
        for _ in range(batches):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            g.replay()
            e1.record(st)
            e1.synchronize()
            out.append(e0.elapsed_time(e1) * 1e3 / reps)
    torch.cuda.current_stream().wait_stream(st)
    out.sort()
    return out[len(out) // 2]


def filter_size_sweep(torch, sw):
    """Throughput against filter size on one plane-per-filter workload (N=32, C=64, 56x56, stride 1, 'same'
    padding, fp32 N(0,1), weights N(0, 1/k^2)): sizes 3, 5, 7 run the fixed-size kernels, up to 17 the first
    generic kernel, beyond that the wide-window generic kernel.  Sizes up to 33 are also timed through the kernel
    generated at run time for the geometry (`jit_*` columns; paper, section 2); its compilation happens in the
    warm-up call, outside the timed launches.  Each size and path is first checked against the CPU oracle on two
    planes."""
    import numpy as np

    import oracle
    from paper_2310_05218_amd import inputs

    N, C, H = 32, 64, 56
    x = inputs.normal_f32((N, C, H, H), inputs.seed_for(6, 0))
    sets = [{"x": torch.from_numpy(x).cuda(), "y": torch.empty((N, C, H, H), device="cuda")} for _ in range(4)]
    rows = []
    for k in (3, 5, 7, 9, 11, 13, 15, 17, 21, 25, 29, 33, 37, 45, 51):
        w = inputs.normal_f32((C, 1, k, k), inputs.seed_for(6, k), 1.0 / k)
        wd = torch.from_numpy(w).cuda()
        pad = (k - 1) // 2
        y = sw.sw_conv2d_depthwise(sets[0]["x"][:1, :2].contiguous(), wd[:2].contiguous(), 1, pad).cpu().numpy()
        y_ref, d = oracle.conv2d_depthwise(x[:1, :2], w[:2], 1, pad)
        err = float(np.max(np.abs(y - y_ref) / d))
        assert err <= 2e-5, (k, err)
        us = time_kernel(torch, lambda s_: sw.sw_conv2d_depthwise(s_["x"], wd, 1, pad, out=s_["y"]), sets,
                         50 if k < 20 else 10)
        flop = 2.0 * k * k * N * C * H * H
        nbytes = 2 * N * C * H * H * 4 + C * k * k * 4
        row = {"filter": k, "us": round(us, 2), "gflops": round(flop / us / 1e3, 1),
               "gbs": round(nbytes / us / 1e3, 1), "frac_hbm": round(nbytes / us / 1e3 / HBM_GBS, 4),
               "frac_alu_f32_plain_fma": round(flop / us / 1e6 / VALU_F32_TFLOPS, 4),
               "max_norm_err": float("%.2e" % err)}
        if sw.sw_jit_prepare_depthwise(H, H, k, k, 1, pad) == 0:
            y = sw.sw_conv2d_depthwise_jit(sets[0]["x"][:1, :2].contiguous(), wd[:2].contiguous(), 1, pad).cpu().numpy()
            err = float(np.max(np.abs(y - y_ref) / d))
            assert err <= 2e-5, ("jit", k, err)
            us = time_kernel(torch, lambda s_: sw.sw_conv2d_depthwise_jit(s_["x"], wd, 1, pad, out=s_["y"]), sets,
                             50 if k < 20 else 10)
            row.update({"jit_us": round(us, 2), "jit_gflops": round(flop / us / 1e3, 1),
                        "jit_frac_alu_f32_plain_fma": round(flop / us / 1e6 / VALU_F32_TFLOPS, 4),
                        "jit_max_norm_err": float("%.2e" % err)})
        rows.append(row)
    # the same axis with a C_in reduction (matrix cores): workload 3's shape with growing filters
    mc_rows = []
    Ci = Co = 64
    xm = inputs.normal_f32((N, Ci, H, H), inputs.seed_for(6, 1000))
    msets = [{"x": torch.from_numpy(xm).cuda(), "y": torch.empty((N, Co, H, H), device="cuda")} for _ in range(6)]
    for k in (1, 3, 5, 7, 9, 11, 13):
        w = inputs.normal_f32((Co, Ci, k, k), inputs.seed_for(6, 1000 + k), (2.0 / (Ci * k * k)) ** 0.5)
        wd = torch.from_numpy(w).cuda()
        pad = (k - 1) // 2
        y = sw.sw_conv2d(msets[0]["x"][:1].contiguous(), wd, 1, pad).cpu().numpy()
        y_ref, d = oracle.conv2d(xm[:1], w, 1, pad)
        err = float(np.max(np.abs(y - y_ref) / d))
        assert err <= 2e-5, ("multi-channel", k, err)
        us = time_kernel(torch, lambda s_: sw.sw_conv2d(s_["x"], wd, 1, pad, out=s_["y"]), msets, 12 if k < 7 else 6)
        flop = 2.0 * k * k * Ci * Co * N * H * H
        mc_rows.append({"filter": k, "us": round(us, 2), "gflops": round(flop / us / 1e3, 1),
                        "frac_mfma_f32": round(flop / us / 1e6 / MFMA_F32_TFLOPS, 4),
                        "max_norm_err": float("%.2e" % err)})
    return {"sweep": "depthwise-shaped 32x64x56x56 fp32, square filter, stride 1, same padding", "rows": rows,
            "multi_channel_sweep": "32x64x56x56 -> 64 channels fp32, square filter, stride 1, same padding",
            "multi_channel_rows": mc_rows}


def _conv_layer_row(torch, sw, oracle, inputs, np, idx, name, kind, shape, R, stride, pad, C_out):
    """One multi-channel layer of the table below (fp32 or int8), checked on one image against the oracle."""
    N, C, H, W = shape
    dil = 2 if kind == "conv_dil" else 1            # the dilated row: taps two positions apart
    Ho, Wo = (H + 2 * pad - dil * (R - 1) - 1) // stride + 1, (W + 2 * pad - dil * (R - 1) - 1) // stride + 1
    s8 = kind in ("conv_s8", "conv_s8_rq", "conv_s8_nhwc", "conv_s8_nhwc_rq")
    rq = kind in ("conv_s8_rq", "conv_s8_nhwc_rq")
    nhwc = kind in ("conv_s8_nhwc", "conv_s8_nhwc_rq")      # the same layer on channel-last tensors
    br = kind == "conv_br"
    if s8:
        x = inputs.uniform_s8(shape, inputs.seed_for(7, idx))
        w = inputs.uniform_s8((C_out, C, R, R), inputs.seed_for(7, 100 + idx))
        call, odt, esz = sw.sw_conv2d_s8, torch.int32, 1
        if rq:      # workload 5 with the requantisation fused into the store: int8 out instead of int32
            rng = np.random.default_rng(inputs.seed_for(7, 200 + idx))
            bias = rng.integers(-50000, 50000, size=C_out).astype(np.int32)
            scale = (rng.uniform(1.0, 3.0, size=C_out) * 2.0 ** -18).astype(np.float32)
            bd, sd = torch.from_numpy(bias).cuda(), torch.from_numpy(scale).cuda()
            call = lambda a, b, st_, p_, out=None: sw.sw_conv2d_s8_requant(a, b, bd, sd, st_, p_, True, out=out)
            odt = torch.int8
        if nhwc:
            x = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
            w = np.ascontiguousarray(w.transpose(0, 2, 3, 1))
            if rq:
                call = lambda a, b, st_, p_, out=None: sw.sw_conv2d_s8_nhwc(a, b, st_, p_, bias=bd, scale=sd, relu=True, out=out)
            else:
                call = lambda a, b, st_, p_, out=None: sw.sw_conv2d_s8_nhwc(a, b, st_, p_, out=out)
    else:
        x = inputs.normal_f32(shape, inputs.seed_for(7, idx))
        w = inputs.normal_f32((C_out, C, R, R), inputs.seed_for(7, 100 + idx), (2.0 / (C * R * R)) ** 0.5)
        call, odt, esz = sw.sw_conv2d, torch.float32, 4
        if dil > 1:
            call = lambda a, b, st_, p_, out=None: sw.sw_conv2d_dilated(a, b, st_, p_, dil, out=out)
        if br:      # bias and rectifier fused into the store
            bias = inputs.normal_f32((C_out,), inputs.seed_for(7, 200 + idx), 0.5)
            bd = torch.from_numpy(bias).cuda()
            call = lambda a, b, st_, p_, out=None: sw.sw_conv2d_bias_relu(a, b, bd, st_, p_, True, out=out)
    xs, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    y = call(xs[:1].contiguous(), wd, stride, pad).cpu().numpy()
    if nhwc and rq:
        assert np.array_equal(y, oracle.conv2d_s8_nhwc_requant(x[:1], w, bias, scale, stride, pad, True)), name
        err = 0.0
    elif nhwc:
        assert np.array_equal(y, oracle.conv2d_s8_nhwc(x[:1], w, stride, pad)), name
        err = 0.0
    elif rq:
        assert np.array_equal(y, oracle.conv2d_s8_requant(x[:1], w, bias, scale, stride, pad, True)), name
        err = 0.0
    elif s8:
        assert np.array_equal(y, oracle.conv2d_s8(x[:1], w, stride, pad)), name
        err = 0.0
    else:
        if br:
            y_ref, d = oracle.conv2d_bias_relu(x[:1], w, bias, stride, pad, True)
        elif dil > 1:
            y_ref, d = oracle.conv2d_dilated(x[:1], w, stride, pad, dil)
        else:
            y_ref, d = oracle.conv2d(x[:1], w, stride, pad)
        err = float(np.max(np.abs(y - y_ref) / d))
        assert err <= 2e-5, (name, err)
    nbytes = x.nbytes + w.nbytes + N * C_out * Ho * Wo * (1 if rq else 4)
    nsets = min(16, max(3, -(-COLD_ROTATION_BYTES // nbytes)))
    oshape = (N, Ho, Wo, C_out) if nhwc else (N, C_out, Ho, Wo)
    sets = [{"x": xs if i == 0 else xs.clone(), "y": torch.empty(oshape, dtype=odt, device="cuda")}
            for i in range(nsets)]
    us = time_kernel(torch, lambda s_: call(s_["x"], wd, stride, pad, out=s_["y"]), sets, 2 * nsets)
    ops = 2.0 * N * C_out * Ho * Wo * C * R * R
    peak = MFMA_I8_TOPS if s8 else MFMA_F32_TFLOPS
    return {"layer": name, "shape": list(shape) + [C_out], "us_cold": round(us, 2), "gbs": round(nbytes / us / 1e3, 1),
            "frac_hbm": round(nbytes / us / 1e3 / HBM_GBS, 4), "gops": round(ops / us / 1e3, 1),
            "frac_mfma": round(ops / us / 1e6 / peak, 4), "max_norm_err": float("%.2e" % err)}


def strided_and_pooling_table(torch, sw):
    """2-D pooling and stride-2 layers of common CNN shapes (fp32 N(0,1) activations), timed cold like the
    step's kernels; each is first checked against the CPU oracle on two planes.  All are bound by HBM:
    bytes = input once + output once (+ filters)."""
    import numpy as np

    import oracle
    from paper_2310_05218_amd import inputs

    layers = [  # name, kind, (N, C, H, W), R, stride, pad
        ("maxpool_3x3_s2", "max", (32, 64, 112, 112), 3, 2, 1),
        ("maxpool_2x2_s2", "max", (32, 64, 112, 112), 2, 2, 0),
        ("avgpool_2x2_s2", "avg", (32, 64, 112, 112), 2, 2, 0),
        ("avgpool_3x3_s1", "avg", (32, 64, 56, 56), 3, 1, 1),
        ("depthwise_3x3_s2", "dw", (32, 128, 112, 112), 3, 2, 1),
        ("depthwise_5x5_s2", "dw", (32, 128, 112, 112), 5, 2, 2),
        ("depthwise_3x3_bias_relu", "dw_br", (32, 256, 56, 56), 3, 1, 1),
        ("depthwise_3x3_s2_bias_relu", "dw_br", (32, 128, 112, 112), 3, 2, 1),
        ("depthwise_3x3_bf16", "dw_bf16", (32, 256, 56, 56), 3, 1, 1),
        ("depthwise_7x7_bf16", "dw_bf16", (32, 256, 56, 56), 7, 1, 3),
        ("global_avgpool_7x7", "avg", (32, 2048, 7, 7), 7, 1, 0),
        ("depthwise_3x3_28x28", "dw", (32, 256, 28, 28), 3, 1, 1),
        ("depthwise_3x3_14x14", "dw", (32, 512, 14, 14), 3, 1, 1),
        ("depthwise_7x7_14x14", "dw", (32, 384, 14, 14), 7, 1, 3),
        ("conv_7x7_s2_3to64", "conv", (32, 3, 224, 224), 7, 2, 3, 64),
        ("conv_3x3_s2_64to128", "conv", (32, 64, 56, 56), 3, 2, 1, 128),
        ("conv_1x1_256to64", "conv", (32, 256, 56, 56), 1, 1, 0, 64),
        ("conv_3x3_14x14_256", "conv", (32, 256, 14, 14), 3, 1, 1, 256),
        ("conv_3x3_64to64", "conv", (32, 64, 56, 56), 3, 1, 1, 64),
        ("conv_3x3_64to64_bias_relu", "conv_br", (32, 64, 56, 56), 3, 1, 1, 64),
        ("conv_3x3_14x14_256_bias_relu", "conv_br", (32, 256, 14, 14), 3, 1, 1, 256),
        ("conv_3x3_dilation2_64to64", "conv_dil", (32, 64, 56, 56), 3, 1, 2, 64),
        ("conv_s8_3x3_s2_64to128", "conv_s8", (32, 64, 56, 56), 3, 2, 1, 128),
        ("conv_s8_1x1_64to256", "conv_s8", (32, 64, 56, 56), 1, 1, 0, 256),
        ("conv_s8_requant_3x3_128to128", "conv_s8_rq", (32, 128, 28, 28), 3, 1, 1, 128),
        ("conv_s8_nhwc_3x3_128to128", "conv_s8_nhwc", (32, 128, 28, 28), 3, 1, 1, 128),
        ("conv_s8_nhwc_requant_3x3_128to128", "conv_s8_nhwc_rq", (32, 128, 28, 28), 3, 1, 1, 128),
        ("conv_s8_nhwc_3x3_s2_64to128", "conv_s8_nhwc", (32, 64, 56, 56), 3, 2, 1, 128),
        ("conv_s8_nhwc_1x1_64to256", "conv_s8_nhwc", (32, 64, 56, 56), 1, 1, 0, 256),
    ]
    rows = []
    for idx, (name, kind, shape, R, stride, pad, *more) in enumerate(layers):
        N, C, H, W = shape
        if kind in ("conv", "conv_br", "conv_dil", "conv_s8", "conv_s8_rq", "conv_s8_nhwc", "conv_s8_nhwc_rq"):
            rows.append(_conv_layer_row(torch, sw, oracle, inputs, np, idx, name, kind, shape, R, stride, pad, more[0]))
            continue
        Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
        x = inputs.normal_f32(shape, inputs.seed_for(7, idx))
        in_bytes, out_bytes = x.nbytes, N * C * Ho * Wo * 4
        nsets = min(32, max(3, -(-COLD_ROTATION_BYTES // (in_bytes + out_bytes))))
        xs = torch.from_numpy(x).cuda()
        sets = [{"x": xs if i == 0 else xs.clone(), "y": torch.empty((N, C, Ho, Wo), device="cuda")}
                for i in range(nsets)]
        if kind == "dw_bf16":       # bf16 planes, fp32 filter and accumulation: half the bytes of the fp32 layer
            xb = inputs.to_bf16_bits(x)
            xs = torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16)
            in_bytes, out_bytes = xb.nbytes, N * C * Ho * Wo * 2
            nsets = min(32, max(3, -(-COLD_ROTATION_BYTES // (in_bytes + out_bytes))))
            sets = [{"x": xs if i == 0 else xs.clone(),
                     "y": torch.empty((N, C, Ho, Wo), dtype=torch.bfloat16, device="cuda")} for i in range(nsets)]
            w = inputs.normal_f32((C, 1, R, R), inputs.seed_for(7, 100 + idx), 1.0 / R)
            wd = torch.from_numpy(w).cuda()
            fn = lambda s_: sw.sw_conv2d_depthwise_bf16(s_["x"], wd, stride, pad, out=s_["y"])
            yb = sw.sw_conv2d_depthwise_bf16(xs[:1, :2].contiguous(), wd[:2].contiguous(), stride, pad)
            y = inputs.bf16_bits_to_f32(yb.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
            y_ref, d = oracle.conv2d_depthwise(inputs.bf16_bits_to_f32(xb[:1, :2]), w[:2], stride, pad)
            # fp32 parity bound plus half a bf16 unit of the exact sum, normalised to the usual 2e-5
            err = float(np.max(np.abs(y - y_ref) / (d + 2.0 ** -8 * np.abs(y_ref) / 2e-5 + 1e-30)))
            ops, extra = 2.0 * R * R * N * C * Ho * Wo, w.nbytes
        elif kind == "dw_br":       # depthwise with bias and rectifier fused into the store
            w = inputs.normal_f32((C, 1, R, R), inputs.seed_for(7, 100 + idx), 1.0 / R)
            bias = inputs.normal_f32((C,), inputs.seed_for(7, 200 + idx), 0.5)
            wd, bd = torch.from_numpy(w).cuda(), torch.from_numpy(bias).cuda()
            fn = lambda s_: sw.sw_conv2d_depthwise_bias_relu(s_["x"], wd, bd, stride, pad, True, out=s_["y"])
            y = sw.sw_conv2d_depthwise_bias_relu(xs[:1, :2].contiguous(), wd[:2].contiguous(), bd[:2].contiguous(),
                                                 stride, pad, True).cpu().numpy()
            y_ref, d = oracle.conv2d_depthwise_bias_relu(x[:1, :2], w[:2], bias[:2], stride, pad, True)
            err = float(np.max(np.abs(y - y_ref) / d))
            ops, extra = 2.0 * R * R * N * C * Ho * Wo, w.nbytes
        elif kind == "dw":
            w = inputs.normal_f32((C, 1, R, R), inputs.seed_for(7, 100 + idx), 1.0 / R)
            wd = torch.from_numpy(w).cuda()
            fn = lambda s_: sw.sw_conv2d_depthwise(s_["x"], wd, stride, pad, out=s_["y"])
            y = sw.sw_conv2d_depthwise(xs[:1, :2].contiguous(), wd[:2].contiguous(), stride, pad).cpu().numpy()
            y_ref, d = oracle.conv2d_depthwise(x[:1, :2], w[:2], stride, pad)
            err = float(np.max(np.abs(y - y_ref) / d))
            ops, extra = 2.0 * R * R * N * C * Ho * Wo, w.nbytes
        else:
            mode = sw.SW_POOL_MAX if kind == "max" else sw.SW_POOL_AVG
            fn = lambda s_: sw.sw_pool2d(s_["x"], R, R, stride, pad, mode, out=s_["y"])
            y = sw.sw_pool2d(xs[:1, :2].contiguous(), R, R, stride, pad, mode).cpu().numpy()
            y_ref, d = oracle.pool2d(x[:1, :2], R, R, stride, pad, mode)
            err = float(np.max(np.abs(y - y_ref) / np.maximum(d, 1e-300)))
            if kind == "max":
                assert np.array_equal(y.astype(np.float64), y_ref), name
            ops, extra = float(R * R * N * C * Ho * Wo), 0
        assert err <= 2e-5, (name, err)
        us = time_kernel(torch, fn, sets, 4 * nsets)
        nbytes = in_bytes + out_bytes + extra
        rows.append({"layer": name, "shape": list(shape), "us_cold": round(us, 2), "gbs": round(nbytes / us / 1e3, 1),
                     "frac_hbm": round(nbytes / us / 1e3 / HBM_GBS, 4), "gops": round(ops / us / 1e3, 1),
                     "max_norm_err": float("%.2e" % err)})
        del sets, xs
        torch.cuda.empty_cache()
    return {"table": "2-D pooling, stride-2, small-plane and other multi-channel layers, cold (rotation larger than the Infinity Cache)",
            "rows": rows}


def cpu_baseline(host, total_ops):
    import oracle

    oracle.build()

    def one_step():
        t0 = time.perf_counter()
        oracle.conv2d(host["x1"], host["w1"], 1, 0)
        oracle.conv1d(host["x2"], host["w2"], 1, 0)
        oracle.pool1d(host["x2"], 8, 1, oracle.POOL_AVG)
        oracle.pool1d(host["x2"], 8, 1, oracle.POOL_MAX)
        oracle.conv2d(host["x3"], host["w3"], 1, 1)
        oracle.conv2d_depthwise(host["x4"], host["w4a"], 1, 1)
        oracle.conv2d_depthwise(host["x4"], host["w4b"], 1, 3)
        oracle.conv2d_s8(host["x5"], host["w5"], 1, 1)
        return time.perf_counter() - t0

    cores = oracle.max_threads()
    times = [one_step() for _ in range(3)]
    dt = min(times)
    oracle.set_threads(1)                 # the same step once more on a single thread
    dt1 = one_step()
    oracle.set_threads(cores)
    return {"value": round(total_ops / dt / 1e9, 2), "unit": "GFLOP/s", "cores": cores, "kind": "oracle",
            "single_thread_value": round(total_ops / dt1 / 1e9, 2),
            "sample": "one full step (all eight launches at full size) run 3 times on %d OpenMP threads, best %.2f s "
                      "wall, and once on one thread, %.2f s (about %.0f s of CPU work in all); naive fp64/int64 loops, "
                      "not a tuned CPU library" % (cores, dt, dt1, sum(times) * cores + dt1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--sets", type=int, default=3, help="buffer sets rotated over (cold-cache timing)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-detail", action="store_true", help="skip the per-kernel hot/cold table")
    ap.add_argument("--sweep", action="store_true",
                    help="filter-size sweep (the paper's experiment axis, section 2): depthwise-shaped "
                         "32x64x56x56 fp32, square filters 3..51, 'same' padding; prints one JSON line")
    ap.add_argument("--layers", action="store_true",
                    help="2-D pooling and stride-2 layers of common CNN shapes; prints one JSON line")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for counter runs under rocprofv3 --pmc: one 64 MiB device copy (calibration), then "
                         "every kernel of the step twice; prints nothing but a marker line")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch

    import paper_2310_05218_amd as sw
    from paper_2310_05218_amd import binding

    binding.lib()     # raises if libswconv.so has not been built: there is no fallback
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    if args.sweep:
        print(json.dumps(filter_size_sweep(torch, sw)))
        return
    if args.layers:
        print(json.dumps(strided_and_pooling_table(torch, sw)))
        return

    work = work_table()
    host, sets = make_sets(torch, args.sets)
    ls = launches(sw)
    total_ops = sum(work[n][0] for n, _ in ls)

    if args.pmc_probe:
        a = torch.empty(16 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.mul(a, 1.0, out=b)        # plain copy kernel, 64 MiB read + 64 MiB written: scales FETCH_SIZE / WRITE_SIZE
        torch.cuda.synchronize()
        for _, fn in ls:
            fn(sets[0])
            fn(sets[1 % len(sets)])
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": "done", "copy_bytes_each_way": a.numel() * 4}))
        return

    def step(i):
        d = sets[i % len(sets)]
        for _, fn in ls:
            fn(d)

    # pick the kernel with the largest share of a step (cold buffers)
    for i in range(3):
        step(i)
    torch.cuda.synchronize()
    probe = {n: time_kernel(torch, fn, sets, 21, 3) for n, fn in ls}
    dominant = max(probe, key=probe.get)

    for i in range(args.warmup):
        step(i)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        d = sets[i % len(sets)]
        for n, fn in ls:
            if n == dominant:
                ev[i][0].record()
                fn(d)
                ev[i][1].record()
            else:
                fn(d)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    dom_us = sum(a.elapsed_time(b) for a, b in ev) * 1e3 / args.steps

    ops, nbytes, bound, peak, unit = work[dominant]
    achieved = (nbytes / dom_us / 1e3) if bound == "hbm" else (ops / dom_us / 1e6)   # GB/s or T(FL)OP/s
    roofline = {"kernel": dominant, "bound": bound, "achieved": round(achieved, 2), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "avg_launch_us": round(dom_us, 2),
                "traffic": measured_traffic(dominant), "algorithmic_bytes": nbytes, "useful_ops": ops}

    result = {
        "metric": "conv GFLOP/s (or GB/s for 1-D/depthwise) and % of roofline, 1 MI355X",
        "value": round(total_ops / (dt / args.steps) / 1e9, 1),
        "unit": "GFLOP/s (useful ops of the direct definition, int8 multiply-adds counted as 2)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (int8 -> int32 for the quantised launch)", "data": "synthetic",
        "config": {"workload": "all five workloads back to back, 8 launches per step: 1x1x256x256 3x3; "
                               "64x65536 conv1d k=9 + avg/max pool w=8; 32x64x56x56->64 3x3; depthwise "
                               "32x256x56x56 3x3 and 7x7; int8 32x128x28x28->128 3x3",
                   "buffer_sets": args.sets},
        "roofline": roofline,
    }

    if not args.no_detail:
        table = []
        copy_cache = {}

        def copy_gbs(nbytes):
            """What a plain device copy that moves the same number of bytes reaches on this GPU, cold (half read,
            half written; torch's elementwise kernel): the measured-achievable HBM rate beside the datasheet's."""
            n_el = max(1024, int(nbytes) // 8)
            if n_el not in copy_cache:
                need = min(32, max(3, -(-COLD_ROTATION_BYTES // (8 * n_el))))
                cs = [{"a": torch.empty(n_el, device="cuda").normal_(), "b": torch.empty(n_el, device="cuda")}
                      for _ in range(need)]
                us = time_kernel(torch, lambda d: torch.mul(d["a"], 1.0, out=d["b"]), cs, max(50, 2 * need))
                copy_cache[n_el] = 8.0 * n_el / us / 1e3
                del cs
            return copy_cache[n_el]

        for n, fn in ls:
            ops, nbytes, bound, peak, unit = work[n]
            reps = 200 if probe[n] < 200 else 50
            rot = cold_rotation(torch, sets, n)
            cold = time_kernel(torch, fn, rot, max(reps, 2 * len(rot)))
            del rot
            hot = time_kernel(torch, fn, sets[:1], reps)
            row = {"kernel": n, "us_cold": round(cold, 2), "us_hot": round(hot, 2),
                   "gflops_cold": round(ops / cold / 1e3, 1), "gbs_cold": round(nbytes / cold / 1e3, 1),
                   "bound": bound}
            row["frac_cold"] = round((nbytes / cold / 1e3) / peak if bound == "hbm" else (ops / cold / 1e6) / peak, 4)
            row["frac_hot"] = round((nbytes / hot / 1e3) / peak if bound == "hbm" else (ops / hot / 1e6) / peak, 4)
            if n in SECOND_ROOF:
                row[SECOND_ROOF[n][1]] = round(ops / cold / 1e6 / SECOND_ROOF[n][0], 4)
            if bound == "hbm":
                row["copy_gbs_same_bytes"] = round(copy_gbs(nbytes), 1)
                row["frac_of_copy"] = round((nbytes / cold / 1e3) / row["copy_gbs_same_bytes"], 4)
            row["traffic"] = measured_traffic(n)
            table.append(row)
        result["kernels"] = table

    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(host, total_ops)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
