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
MFMA_BF16_TFLOPS = 2500.0
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
    # the quantised launch is quoted against the int8 matrix peak (its target is the compute roofline); 456.6 op/B is
    # below the int8 ridge (5000 TOP/s / 8 TB/s = 625 op/B), so the HBM fraction is quoted beside it (SECOND_ROOF)
    t["conv2d_s8_128x128_3x3"] = (2 * 128 * 128 * 9 * px8, 128 * px8 + 128 * 128 * 9 + 128 * px8 * 4, "mfma",
                                  MFMA_I8_TOPS, "TOP/s")
    t["conv2d_s8_128x128_3x3_packed"] = t["conv2d_s8_128x128_3x3"]      # filters packed once, outside the timed region
    return t


# second roof quoted beside the bounding one: name -> (peak in T(FL)OP/s, label)
SECOND_ROOF = {"depthwise_7x7": (VALU_F32_TFLOPS, "frac_alu_f32_plain_fma")}
# launches whose bytes are quoted against HBM beside their compute roof
ALSO_HBM = ("conv2d_s8_128x128_3x3", "conv2d_s8_128x128_3x3_packed")
# measured-achievable peak (see measured_peaks) each launch's compute fraction is also quoted against
MEASURED_ROOF = {"conv2d_64x64_3x3": "mfma_f32_tflops", "conv2d_s8_128x128_3x3": "mfma_i8_tops",
                 "conv2d_s8_128x128_3x3_packed": "mfma_i8_tops", "depthwise_7x7": "fma_f32_tflops"}


# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a plain copy kernel, see
# profiles/hbm_traffic_all_kernels.txt), with the kernel source and its sha256 prefix at the time the
# counters were taken.  A kernel whose source has changed since reports traffic = null.
TRAFFIC_SOURCE = ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs made by the builder (profiles/hbm_traffic_all_kernels.txt), "
                  "not measured by this run; null where the kernel's source has changed since")
TRAFFIC = {
    "depthwise_3x3": (207413237, "sw_sliding_plane.hip", "1d24ebdfa6df1cef"),
    "depthwise_7x7": (206183315, "sw_sliding_plane.hip", "1d24ebdfa6df1cef"),
    "conv2d_64x64_3x3": (62550964, "sw_mfma_f32.hip", "20a2d4cb31e9e833"),
    "conv2d_s8_128x128_3x3": (22096535, "sw_mfma_s8_band.hip", "efae7346fdd97c23"),
    "conv1d_k9": (33974646, "sw_sliding1d.hip", "b574d6ab8949af6c"),
    "avgpool1d_w8": (34237947, "sw_sliding1d.hip", "b574d6ab8949af6c"),
    "maxpool1d_w8": (34207183, "sw_sliding1d.hip", "b574d6ab8949af6c"),
    "conv2d_1ch_3x3": (660943, "sw_sliding_rows.hip", "0e35510846c9b8a1"),
    "conv2d_s8_128x128_3x3_packed": (21953725, "sw_mfma_s8_band.hip", "efae7346fdd97c23"),
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


def measured_peaks(torch, sw):
    """Rates this GPU sustains on arithmetic-only kernels of the library (sw_probe: nothing but the instruction, no
    memory), timed like everything else here: the measured-achievable peaks beside the datasheet's."""
    out = {}
    for key, kind, iters in (("mfma_f32_tflops", sw.SW_PROBE_MFMA_F32, 4000), ("mfma_i8_tops", sw.SW_PROBE_MFMA_I8, 8000),
                             ("fma_f32_tflops", sw.SW_PROBE_FMA_F32, 1000),
                             # plain FMAs and fp32 matrix instructions in one stream: the sum of the two rates if the
                             # pipes overlapped; measured, a round takes the sum of the two times instead
                             ("fma_plus_mfma_f32_tflops", sw.SW_PROBE_FMA_MFMA_F32, 2000),
                             # fp32 matrix instructions fed from LDS (one 4-byte operand read behind each), one and two
                             # wavefronts per SIMD: what a stream of them sustains once it has operands to fetch
                             ("mfma_bf16_tflops", sw.SW_PROBE_MFMA_BF16, 8000),
                             ("mfma_f32_fed_tflops", sw.SW_PROBE_MFMA_F32_FED, 4000),
                             ("mfma_f32_fed_two_wavefronts_tflops", sw.SW_PROBE_MFMA_F32_FED2, 4000)):
        ops = sw.sw_probe(kind, iters)
        us = time_kernel(torch, lambda d: sw.sw_probe(kind, iters), [None], 10, 3)
        out[key] = round(ops / us / 1e6, 1)
    return out


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


def extra_launches(sw):
    """Launches timed in the per-kernel table only (not part of the step): the quantised layer with its filters
    packed once (sw_s8_pack_filter, done when the buffer sets are built)."""
    return [("conv2d_s8_128x128_3x3_packed",
             lambda d: sw.sw_conv2d_s8_packed(d["x5"], d["w5p"], 128, 3, 3, 1, 1, out=d["y5"]))]


# buffers each launch touches (for building rotations that are larger than the Infinity Cache)
BUFFERS = {
    "conv2d_1ch_3x3": ("x1", "w1", "y1"), "conv1d_k9": ("x2", "w2", "y2a"), "avgpool1d_w8": ("x2", "y2b"),
    "maxpool1d_w8": ("x2", "y2c"), "conv2d_64x64_3x3": ("x3", "w3", "y3"), "depthwise_3x3": ("x4", "w4a", "y4a"),
    "depthwise_7x7": ("x4", "w4b", "y4b"), "conv2d_s8_128x128_3x3": ("x5", "w5", "y5"),
    "conv2d_s8_128x128_3x3_packed": ("x5", "w5p", "y5"),
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


# filter sizes of `--sweep`: one filter per plane, and with a C_in reduction
SWEEP_FILTERS = (3, 5, 7, 9, 11, 13, 15, 17, 21, 25, 29, 33, 37, 45, 51)
MC_SWEEP_FILTERS = (1, 3, 5, 7, 9, 11, 13, 15, 17, 21, 25, 29, 33, 37, 45, 51)
SWEEP_1D = (2, 3, 5, 9, 13, 17, 25, 33, 49, 64)        # 1-D filter lengths / pooling windows


def filter_size_sweep(torch, sw):
    """Throughput against filter size on one plane-per-filter workload (N=32, C=64, 56x56, stride 1, 'same'
    padding, fp32 N(0,1), weights N(0, 1/k^2)): sizes 3, 5, 7 run the fixed-size kernels, up to 17 the first
    generic kernel, beyond that the wide-window generic kernel.  Sizes up to 33 are also timed through the kernel
    generated at run time for the geometry (`jit_*` columns; paper, section 2); its compilation happens in the
    warm-up call, outside the timed launches.  (Parity of every size and path of this sweep against the CPU oracle
    is a GPU test: tests/test_gpu_bench_shapes.py.)"""
    from paper_2310_05218_amd import inputs

    N, C, H = 32, 64, 56
    x = inputs.normal_f32((N, C, H, H), inputs.seed_for(6, 0))
    sets = [{"x": torch.from_numpy(x).cuda(), "y": torch.empty((N, C, H, H), device="cuda")} for _ in range(4)]
    rows = []
    for k in SWEEP_FILTERS:
        w = inputs.normal_f32((C, 1, k, k), inputs.seed_for(6, k), 1.0 / k)
        wd = torch.from_numpy(w).cuda()
        pad = (k - 1) // 2
        us = time_kernel(torch, lambda s_: sw.sw_conv2d_depthwise(s_["x"], wd, 1, pad, out=s_["y"]), sets,
                         50 if k < 20 else 10)
        flop = 2.0 * k * k * N * C * H * H
        nbytes = 2 * N * C * H * H * 4 + C * k * k * 4
        row = {"filter": k, "us": round(us, 2), "gflops": round(flop / us / 1e3, 1),
               "gbs": round(nbytes / us / 1e3, 1), "frac_hbm": round(nbytes / us / 1e3 / HBM_GBS, 4),
               "frac_alu_f32_plain_fma": round(flop / us / 1e6 / VALU_F32_TFLOPS, 4)}
        if sw.sw_jit_prepare_depthwise(H, H, k, k, 1, pad) == 0:
            us = time_kernel(torch, lambda s_: sw.sw_conv2d_depthwise_jit(s_["x"], wd, 1, pad, out=s_["y"]), sets,
                             50 if k < 20 else 10)
            row.update({"jit_us": round(us, 2), "jit_gflops": round(flop / us / 1e3, 1),
                        "jit_frac_alu_f32_plain_fma": round(flop / us / 1e6 / VALU_F32_TFLOPS, 4)})
        rows.append(row)
    # the same axis with a C_in reduction (matrix cores): workload 3's shape with growing filters
    mc_rows = []
    Ci = Co = 64
    xm = inputs.normal_f32((N, Ci, H, H), inputs.seed_for(6, 1000))
    msets = [{"x": torch.from_numpy(xm).cuda(), "y": torch.empty((N, Co, H, H), device="cuda")} for _ in range(6)]
    for k in MC_SWEEP_FILTERS:
        w = inputs.normal_f32((Co, Ci, k, k), inputs.seed_for(6, 1000 + k), (2.0 / (Ci * k * k)) ** 0.5)
        wd = torch.from_numpy(w).cuda()
        pad = (k - 1) // 2
        us = time_kernel(torch, lambda s_: sw.sw_conv2d(s_["x"], wd, 1, pad, out=s_["y"]), msets, 12 if k < 7 else 6)
        flop = 2.0 * k * k * Ci * Co * N * H * H
        mc_rows.append({"filter": k, "us": round(us, 2), "gflops": round(flop / us / 1e3, 1),
                        "frac_mfma_f32": round(flop / us / 1e6 / MFMA_F32_TFLOPS, 4)})
    # the 1-D axis (the paper's first experiment): workload 2's rows with growing filters / windows
    rows_1d = []
    x2 = inputs.normal_f32((64, 65536), inputs.seed_for(6, 2000))
    nb = x2.nbytes
    s1 = [{"x": torch.from_numpy(x2).cuda()} for _ in range(12)]
    for k in SWEEP_1D:
        w = torch.from_numpy(inputs.normal_f32((k,), inputs.seed_for(6, 2000 + k), 1.0 / k ** 0.5)).cuda()
        Lo = 65536 - k + 1
        for s_ in s1:
            s_["y"] = torch.empty((64, Lo), device="cuda")
        row = {"taps": k}
        for name, fn, ops in (("conv", lambda d: sw.sw_conv1d(d["x"], w, 1, 0, out=d["y"]), 2.0 * k),
                              ("avg", lambda d: sw.sw_pool1d(d["x"], k, 1, sw.SW_POOL_AVG, out=d["y"]), float(k)),
                              ("max", lambda d: sw.sw_pool1d(d["x"], k, 1, sw.SW_POOL_MAX, out=d["y"]), float(k - 1))):
            us = time_kernel(torch, fn, s1, 60)
            nbytes = nb + 64 * Lo * 4
            row[name + "_us"] = round(us, 2)
            row[name + "_frac_hbm"] = round(nbytes / us / 1e3 / HBM_GBS, 4)
            row[name + "_gops"] = round(ops * 64 * Lo / us / 1e3, 1)
        rows_1d.append(row)
    return {"sweep": "depthwise-shaped 32x64x56x56 fp32, square filter, stride 1, same padding", "rows": rows,
            "sweep_1d": "64 rows x 65536 fp32, stride 1, no padding: convolution, average and maximum by window length",
            "rows_1d": rows_1d,
            "multi_channel_sweep": "32x64x56x56 -> 64 channels fp32, square filter, stride 1, same padding",
            "multi_channel_rows": mc_rows}


# layers of `--layers`: name, kind, (N, C, H, W), R (= S), stride, pad[, C_out]
LAYERS = [
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
    ("conv_1x1_64to256", "conv", (32, 64, 56, 56), 1, 1, 0, 256),
    ("conv_1x1_256to256_28x28", "conv", (32, 256, 28, 28), 1, 1, 0, 256),
    ("conv_1x1_512to512_14x14", "conv", (32, 512, 14, 14), 1, 1, 0, 512),
    ("conv_3x3_14x14_256", "conv", (32, 256, 14, 14), 3, 1, 1, 256),
    ("conv_3x3_64to64", "conv", (32, 64, 56, 56), 3, 1, 1, 64),
    ("conv_3x3_64to64_bias_relu", "conv_br", (32, 64, 56, 56), 3, 1, 1, 64),
    ("conv_3x3_14x14_256_bias_relu", "conv_br", (32, 256, 14, 14), 3, 1, 1, 256),
    ("conv_3x3_dilation2_64to64", "conv_dil", (32, 64, 56, 56), 3, 1, 2, 64),
    ("depthwise_3x3_dilation2", "dw_dil", (32, 256, 56, 56), 3, 1, 2, 2),       # (last entry: the dilation)
    ("depthwise_3x3_dilation6", "dw_dil", (32, 256, 56, 56), 3, 1, 6, 6),
    ("depthwise_3x3_dilation2_generated", "dw_dil_jit", (32, 256, 56, 56), 3, 1, 2, 2),   # kernels generated at run time
    ("depthwise_3x3_dilation6_generated", "dw_dil_jit", (32, 256, 56, 56), 3, 1, 6, 6),
    ("depthwise_3x3_s2_56x56", "dw", (32, 256, 56, 56), 3, 2, 1),
    ("depthwise_3x3_s2_56x56_generated", "dw_dil_jit", (32, 256, 56, 56), 3, 2, 1, 1),
    ("depthwise_5x5_s2_56x56_generated", "dw_dil_jit", (32, 256, 56, 56), 5, 2, 2, 1),
    ("block_dw3x3_pw_128to128_56x56", "block", (32, 128, 56, 56), 3, 1, 1, 128),
    ("block_two_launches_128to128_56x56", "block2", (32, 128, 56, 56), 3, 1, 1, 128),
    ("block_dw3x3_pw_256to256_28x28", "block", (32, 256, 28, 28), 3, 1, 1, 256),
    ("block_two_launches_256to256_28x28", "block2", (32, 256, 28, 28), 3, 1, 1, 256),
    ("block_dw3x3_pw_512to512_14x14", "block", (32, 512, 14, 14), 3, 1, 1, 512),
    ("block_two_launches_512to512_14x14", "block2", (32, 512, 14, 14), 3, 1, 1, 512),
    ("conv_nhwc_3x3_64to64", "conv_nhwc", (32, 64, 56, 56), 3, 1, 1, 64),              # channel-last fp32
    ("conv_nhwc_3x3_128to128_28x28", "conv_nhwc", (32, 128, 28, 28), 3, 1, 1, 128),
    ("conv_bf16_nhwc_3x3_64to64", "conv_bf16_nhwc", (32, 64, 56, 56), 3, 1, 1, 64),    # channel-last bf16, fp32 accumulation
    ("conv_bf16_nhwc_3x3_128to128_28x28", "conv_bf16_nhwc", (32, 128, 28, 28), 3, 1, 1, 128),
    ("conv_bf16_nhwc_3x3_s2_64to128", "conv_bf16_nhwc", (32, 64, 56, 56), 3, 2, 1, 128),
    ("conv_bf16_nhwc_1x1_256to64", "conv_bf16_nhwc", (32, 256, 56, 56), 1, 1, 0, 64),
    ("conv_bf16_nhwc_3x3_256to256_14x14", "conv_bf16_nhwc", (32, 256, 14, 14), 3, 1, 1, 256),
    ("conv_f16_nhwc_3x3_64to64", "conv_f16_nhwc", (32, 64, 56, 56), 3, 1, 1, 64),      # channel-last IEEE half, fp32 accumulation
    ("conv_f16_nhwc_3x3_128to128_28x28", "conv_f16_nhwc", (32, 128, 28, 28), 3, 1, 1, 128),
    ("conv_s8_3x3_s2_64to128", "conv_s8", (32, 64, 56, 56), 3, 2, 1, 128),
    ("conv_s8_1x1_64to256", "conv_s8", (32, 64, 56, 56), 1, 1, 0, 256),
    ("conv_s8_requant_3x3_128to128", "conv_s8_rq", (32, 128, 28, 28), 3, 1, 1, 128),
    ("conv_s8_packed_3x3_128to128", "conv_s8_pk", (32, 128, 28, 28), 3, 1, 1, 128),
    ("conv_s8_packed_requant_3x3_128to128", "conv_s8_pk_rq", (32, 128, 28, 28), 3, 1, 1, 128),
    ("conv_s8_3x3_64to64_56x56", "conv_s8", (32, 64, 56, 56), 3, 1, 1, 64),
    ("conv_s8_packed_3x3_64to64_56x56", "conv_s8_pk", (32, 64, 56, 56), 3, 1, 1, 64),
    ("conv_s8_nhwc_3x3_128to128", "conv_s8_nhwc", (32, 128, 28, 28), 3, 1, 1, 128),
    ("conv_s8_nhwc_requant_3x3_128to128", "conv_s8_nhwc_rq", (32, 128, 28, 28), 3, 1, 1, 128),
    ("conv_s8_nhwc_3x3_s2_64to128", "conv_s8_nhwc", (32, 64, 56, 56), 3, 2, 1, 128),
    ("conv_s8_nhwc_1x1_64to256", "conv_s8_nhwc", (32, 64, 56, 56), 1, 1, 0, 256),
    ("conv_s8_nhwc_3x3_256to256_14x14", "conv_s8_nhwc", (32, 256, 14, 14), 3, 1, 1, 256),
    ("conv_nhwc_1x1_256to64", "conv_nhwc", (32, 256, 56, 56), 1, 1, 0, 64),
]


def layer_case(idx, n_images=None, data=True):
    """Host-side description of layer LAYERS[idx] (optionally with fewer images): seeded inputs and everything
    needed to call it.  Shared by `--layers` (timing) and tests/test_gpu_bench_shapes.py (parity against the CPU
    oracle), so that what is timed is what is checked.  data=False: arrays of zeros with the same shapes and types
    (the library's choice of kernel looks at shapes and addresses only)."""
    import numpy as np

    from paper_2310_05218_amd import inputs

    if not data:
        class inputs:       # noqa: F811  (same generators, zeros)
            seed_for = staticmethod(lambda *a: 0)
            normal_f32 = staticmethod(lambda shape, seed, std=1.0: np.zeros(shape, np.float32))
            uniform_s8 = staticmethod(lambda shape, seed: np.zeros(shape, np.int8))
            normal_bf16 = staticmethod(lambda shape, seed, std=1.0: np.zeros(shape, np.uint16))
            normal_f16 = staticmethod(lambda shape, seed, std=1.0: np.zeros(shape, np.uint16))

    name, kind, shape, R, stride, pad, *more = LAYERS[idx]
    N, C, H, W = shape
    if n_images is not None:
        N = n_images
    c = {"name": name, "kind": kind, "N": N, "C": C, "H": H, "W": W, "R": R, "stride": stride, "pad": pad,
         "dil": more[0] if kind.startswith("dw_dil") else 2 if kind == "conv_dil" else 1,
         "C_out": more[0] if more and not kind.startswith("dw_dil") else C}
    span = c["dil"] * (R - 1) + 1
    c["Ho"], c["Wo"] = (H + 2 * pad - span) // stride + 1, (W + 2 * pad - span) // stride + 1
    rng = np.random.default_rng(inputs.seed_for(7, 200 + idx))
    if kind.startswith("conv_s8"):
        x = inputs.uniform_s8((N, C, H, W), inputs.seed_for(7, idx))
        w = inputs.uniform_s8((c["C_out"], C, R, R), inputs.seed_for(7, 100 + idx))
        if kind.endswith("rq"):
            c["bias"] = rng.integers(-50000, 50000, size=c["C_out"]).astype(np.int32)
            c["scale"] = (rng.uniform(1.0, 3.0, size=c["C_out"]) * 2.0 ** -18).astype(np.float32)
        if "nhwc" in kind:
            x = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
            w = np.ascontiguousarray(w.transpose(0, 2, 3, 1))
    elif kind.startswith("block"):      # depthwise 3x3 + bias + ReLU, pointwise 1x1 + bias + ReLU: fused, or two launches
        x = inputs.normal_f32((N, C, H, W), inputs.seed_for(7, idx))
        w = inputs.normal_f32((C, 1, 3, 3), inputs.seed_for(7, 100 + idx), 1.0 / 3)
        c["w_pw"] = inputs.normal_f32((c["C_out"], C, 1, 1), inputs.seed_for(7, 300 + idx), (2.0 / C) ** 0.5)
        c["bias"] = inputs.normal_f32((C,), inputs.seed_for(7, 200 + idx), 0.3)
        c["bias_pw"] = inputs.normal_f32((c["C_out"],), inputs.seed_for(7, 400 + idx), 0.3)
    elif kind.startswith("conv"):
        x = inputs.normal_f32((N, C, H, W), inputs.seed_for(7, idx))
        w = inputs.normal_f32((c["C_out"], C, R, R), inputs.seed_for(7, 100 + idx), (2.0 / (C * R * R)) ** 0.5)
        if kind == "conv_br":
            c["bias"] = inputs.normal_f32((c["C_out"],), inputs.seed_for(7, 200 + idx), 0.5)
        if kind == "conv_bf16_nhwc":        # (the same draws, truncated to bf16 bit patterns)
            x = inputs.normal_bf16((N, C, H, W), inputs.seed_for(7, idx))
            w = inputs.normal_bf16((c["C_out"], C, R, R), inputs.seed_for(7, 100 + idx), (2.0 / (C * R * R)) ** 0.5)
        if kind == "conv_f16_nhwc":         # (the same draws, rounded to half-precision bit patterns)
            x = inputs.normal_f16((N, C, H, W), inputs.seed_for(7, idx))
            w = inputs.normal_f16((c["C_out"], C, R, R), inputs.seed_for(7, 100 + idx), (2.0 / (C * R * R)) ** 0.5)
        if "nhwc" in kind:
            x = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
            w = np.ascontiguousarray(w.transpose(0, 2, 3, 1))
    else:
        x = inputs.normal_f32((N, C, H, W), inputs.seed_for(7, idx))
        w = inputs.normal_f32((C, 1, R, R), inputs.seed_for(7, 100 + idx), 1.0 / R) if kind.startswith("dw") else None
        if kind == "dw_br":
            c["bias"] = inputs.normal_f32((C,), inputs.seed_for(7, 200 + idx), 0.5)
        if kind == "dw_bf16":
            x = inputs.normal_bf16((N, C, H, W), inputs.seed_for(7, idx))
    c["x"], c["w"] = x, w
    return c


def layer_device(torch, c):
    """Device tensors of a layer case: x, w, bias, scale (None where the layer has none) and an empty output."""
    import numpy as np

    def dev(a):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()

    x = c["x"]
    kind = c["kind"]
    as_bf16 = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    as_f16 = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.float16)
    xd = as_bf16(x) if kind in ("dw_bf16", "conv_bf16_nhwc") else as_f16(x) if kind == "conv_f16_nhwc" else dev(x)
    odt = (torch.bfloat16 if kind in ("dw_bf16", "conv_bf16_nhwc") else torch.float16 if kind == "conv_f16_nhwc" else
           torch.int8 if kind.endswith("rq") else torch.int32 if kind.startswith("conv_s8") else torch.float32)
    oshape = ((c["N"], c["Ho"], c["Wo"], c["C_out"]) if "nhwc" in kind else (c["N"], c["C_out"], c["Ho"], c["Wo"]))
    d = {"x": xd, "w": as_bf16(c["w"]) if kind == "conv_bf16_nhwc" else as_f16(c["w"]) if kind == "conv_f16_nhwc" else dev(c["w"]), "bias": dev(c.get("bias")), "scale": dev(c.get("scale")),
         "y": torch.empty(oshape, dtype=odt, device="cuda")}
    if kind.startswith("block"):
        d["w_pw"], d["bias_pw"] = dev(c["w_pw"]), dev(c["bias_pw"])
        if kind == "block2":            # the intermediate of the two-launch form lives in device memory
            d["t"] = torch.empty((c["N"], c["C"], c["H"], c["W"]), device="cuda")
    return d


def layer_call(sw, c, d, x=None, y=None):
    """Runs the layer on device tensors d (x / y override the input and output, for buffer rotations)."""
    x = d["x"] if x is None else x
    y = d["y"] if y is None else y
    kind, st, p = c["kind"], c["stride"], c["pad"]
    if kind in ("max", "avg"):
        return sw.sw_pool2d(x, c["R"], c["R"], st, p, sw.SW_POOL_MAX if kind == "max" else sw.SW_POOL_AVG, out=y)
    if kind == "dw":
        return sw.sw_conv2d_depthwise(x, d["w"], st, p, out=y)
    if kind == "dw_dil":
        return sw.sw_conv2d_depthwise_dilated(x, d["w"], st, p, c["dil"], out=y)
    if kind == "dw_dil_jit":
        return sw.sw_conv2d_depthwise_dilated_jit(x, d["w"], st, p, c["dil"], out=y)
    if kind == "dw_br":
        return sw.sw_conv2d_depthwise_bias_relu(x, d["w"], d["bias"], st, p, True, out=y)
    if kind == "dw_bf16":
        return sw.sw_conv2d_depthwise_bf16(x, d["w"], st, p, out=y)
    if kind == "block":
        return sw.sw_dw_pw_block(x, d["w"], d["bias"], d["w_pw"], d["bias_pw"], True, True, out=y)
    if kind == "block2":
        sw.sw_conv2d_depthwise_bias_relu(x, d["w"], d["bias"], 1, 1, True, out=d["t"])
        return sw.sw_conv2d_bias_relu(d["t"], d["w_pw"], d["bias_pw"], 1, 0, True, out=y)
    if kind == "conv":
        return sw.sw_conv2d(x, d["w"], st, p, out=y)
    if kind == "conv_br":
        return sw.sw_conv2d_bias_relu(x, d["w"], d["bias"], st, p, True, out=y)
    if kind == "conv_dil":
        return sw.sw_conv2d_dilated(x, d["w"], st, p, c["dil"], out=y)
    if kind in ("conv_nhwc", "conv_bf16_nhwc", "conv_f16_nhwc"):
        return sw.sw_conv2d_nhwc(x, d["w"], st, p, 1, out=y)
    if kind == "conv_s8":
        return sw.sw_conv2d_s8(x, d["w"], st, p, out=y)
    if kind == "conv_s8_rq":
        return sw.sw_conv2d_s8_requant(x, d["w"], d["bias"], d["scale"], st, p, True, out=y)
    if kind in ("conv_s8_pk", "conv_s8_pk_rq"):
        if "packed" not in d:            # the filters are packed once, outside every timed region
            d["packed"] = sw.sw_s8_pack_filter(d["w"])
        if kind == "conv_s8_pk":
            return sw.sw_conv2d_s8_packed(x, d["packed"], c["C_out"], c["R"], c["R"], st, p, out=y)
        return sw.sw_conv2d_s8_packed(x, d["packed"], c["C_out"], c["R"], c["R"], st, p, d["bias"], d["scale"], True, out=y)
    if kind == "conv_s8_nhwc":
        return sw.sw_conv2d_s8_nhwc(x, d["w"], st, p, out=y)
    if kind == "conv_s8_nhwc_rq":
        return sw.sw_conv2d_s8_nhwc(x, d["w"], st, p, bias=d["bias"], scale=d["scale"], relu=True, out=y)
    raise ValueError(kind)


def strided_and_pooling_table(torch, sw, only=None):
    """Layers of common CNN shapes beyond the five workloads (2-D pooling, strides, small planes, fused epilogues,
    dilation, bf16 planes, int8 in both layouts), timed cold like the step's kernels.  bytes = input once + output
    once (+ filters); multi-channel rows also give the fraction of the matrix peak.  (Parity of every row against
    the CPU oracle is a GPU test: tests/test_gpu_bench_shapes.py.)"""
    rows = []
    for idx in range(len(LAYERS)):
        if only is not None and only not in LAYERS[idx][0]:
            continue
        c = layer_case(idx)
        d = layer_device(torch, c)
        kind, N, C, R = c["kind"], c["N"], c["C"], c["R"]
        w_bytes = 0 if c["w"] is None else c["w"].nbytes
        nbytes = c["x"].nbytes + w_bytes + d["y"].numel() * d["y"].element_size()
        nsets = min(32, max(3, -(-COLD_ROTATION_BYTES // nbytes)))
        sets = [{"x": d["x"] if i == 0 else d["x"].clone(), "y": torch.empty_like(d["y"])} for i in range(nsets)]
        us = time_kernel(torch, lambda s_: layer_call(sw, c, d, s_["x"], s_["y"]), sets, 4 * nsets)
        outs = N * c["C_out"] * c["Ho"] * c["Wo"]
        if kind.startswith("block"):
            ops = 2.0 * N * C * c["H"] * c["W"] * 9 + 2.0 * outs * C
            nbytes += c["w_pw"].nbytes
        elif kind.startswith("conv"):
            ops = 2.0 * outs * C * R * R
        elif kind.startswith("dw"):
            ops = 2.0 * outs * R * R
        else:
            ops = float(outs * R * R)
        row = {"layer": c["name"], "shape": [N, C, c["H"], c["W"]] + ([c["C_out"]] if kind.startswith("conv") else []),
               "us_cold": round(us, 2), "gbs": round(nbytes / us / 1e3, 1),
               "frac_hbm": round(nbytes / us / 1e3 / HBM_GBS, 4), "gops": round(ops / us / 1e3, 1)}
        if kind.startswith("conv") or kind.startswith("block"):
            row["frac_mfma"] = round(ops / us / 1e6 / (MFMA_I8_TOPS if "s8" in kind else MFMA_BF16_TFLOPS if "bf16" in kind or "f16" in kind
                                                       else MFMA_F32_TFLOPS), 4)
        rows.append(row)
        del sets, d
        torch.cuda.empty_cache()
    return {"table": "layers of common CNN shapes beyond the five workloads, cold (rotation larger than the Infinity Cache)",
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
    ap.add_argument("--only", default=None, metavar="TEXT",
                    help="with --layers: only the rows whose name contains TEXT (short runs under a profiler)")
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
        print(json.dumps(strided_and_pooling_table(torch, sw, args.only)))
        return

    work = work_table()
    host, sets = make_sets(torch, args.sets)
    for d in sets:
        d["w5p"] = sw.sw_s8_pack_filter(d["w5"])
    torch.cuda.synchronize()
    ls = launches(sw)
    total_ops = sum(work[n][0] for n, _ in ls)

    if args.pmc_probe:
        a = torch.empty(16 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.mul(a, 1.0, out=b)        # plain copy kernel, 64 MiB read + 64 MiB written: scales FETCH_SIZE / WRITE_SIZE
        torch.cuda.synchronize()
        for _, fn in ls + extra_launches(sw):
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
                "traffic": measured_traffic(dominant), "traffic_source": TRAFFIC_SOURCE, "algorithmic_bytes": nbytes,
                "useful_ops": ops}

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

        peaks = measured_peaks(torch, sw)
        result["measured_peaks"] = dict(peaks, note="arithmetic-only probe kernels of the library (sw_probe), timed in this run")
        for n, fn in ls + extra_launches(sw):
            ops, nbytes, bound, peak, unit = work[n]
            if n not in probe:
                probe[n] = time_kernel(torch, fn, sets, 21, 3)
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
            if n in MEASURED_ROOF:
                row["frac_of_measured_" + MEASURED_ROOF[n]] = round(ops / cold / 1e6 / peaks[MEASURED_ROOF[n]], 4)
            if n == "conv2d_64x64_3x3":      # one multiplying wavefront per SIMD: against the operand-fed stream as well
                row["frac_of_measured_mfma_f32_fed_tflops"] = round(ops / cold / 1e6 / peaks["mfma_f32_fed_tflops"], 4)
            if bound == "hbm" or n in ALSO_HBM:
                row["frac_hbm"] = round(nbytes / cold / 1e3 / HBM_GBS, 4)
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
