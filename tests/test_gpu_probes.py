"""The arithmetic-only probe kernels run, report the kernel they enqueued, and the mixed fp32 probe shows what the
one-filter-per-plane kernels rely on: plain FMAs and fp32 matrix instructions of one stream do not overlap."""
import pytest
import torch

import paper_2310_05218_amd as sw

pytestmark = pytest.mark.gpu


def timed_us(kind, iters):
    sw.sw_probe(kind, iters)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    sw.sw_probe(kind, iters)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3


@pytest.mark.parametrize("kind, name", [(sw.SW_PROBE_MFMA_F32, "probe_mfma_f32_kernel"), (sw.SW_PROBE_MFMA_I8, "probe_mfma_i8_kernel"),
                                        (sw.SW_PROBE_FMA_F32, "probe_fma_f32_kernel"), (sw.SW_PROBE_FMA_MFMA_F32, "probe_fma_mfma_f32_kernel"),
                                        (sw.SW_PROBE_MFMA_F32_FED, "probe_mfma_f32_fed_kernel<1>"),
                                        (sw.SW_PROBE_MFMA_F32_FED2, "probe_mfma_f32_fed_kernel<2>"),
                                        (sw.SW_PROBE_MFMA_BF16, "probe_mfma_bf16_kernel")])
def test_probe_runs(kind, name):
    ops = sw.sw_probe(kind, 50)
    torch.cuda.synchronize()
    assert ops > 0 and sw.sw_last_kernel() == name


def test_fp32_matrix_and_vector_pipes_do_not_overlap():
    # FLOP/us of plain FMAs alone and of the mixed stream (9 FMAs of 128 FLOP + one matrix product of 2048 FLOP a round).
    # Side by side, a round would take its slower part (the 9 FMAs: 36 cycles against 32) and the mixed rate would be
    # (1152 + 2048) / 1152 = 2.8 x the FMA rate; one after the other it is 3200 / (36 + 32) cycles = 1.5 x.
    iters = 2000
    fma = sw.sw_probe(sw.SW_PROBE_FMA_F32, iters) / timed_us(sw.SW_PROBE_FMA_F32, iters)
    mix = sw.sw_probe(sw.SW_PROBE_FMA_MFMA_F32, iters) / timed_us(sw.SW_PROBE_FMA_MFMA_F32, iters)
    print(f"plain FMA {fma / 1e6:.1f} TFLOP/s, mixed stream {mix / 1e6:.1f} TFLOP/s, ratio {mix / fma:.2f}")
    assert 1.1 < mix / fma < 2.0


def test_operand_reads_slow_the_fp32_matrix_stream_and_a_second_wavefront_hides_part_of_it():
    # One 4-byte LDS read behind every matrix instruction, its result the next-but-three instruction's operand: with one
    # wavefront per SIMD the stream loses a few percent of the bare instruction's rate (measured 0.94 - 0.96), with two
    # about half of that.
    iters = 4000
    bare = sw.sw_probe(sw.SW_PROBE_MFMA_F32, iters) / timed_us(sw.SW_PROBE_MFMA_F32, iters)
    fed1 = sw.sw_probe(sw.SW_PROBE_MFMA_F32_FED, iters) / timed_us(sw.SW_PROBE_MFMA_F32_FED, iters)
    fed2 = sw.sw_probe(sw.SW_PROBE_MFMA_F32_FED2, iters) / timed_us(sw.SW_PROBE_MFMA_F32_FED2, iters)
    print(f"bare {bare / 1e6:.1f} TFLOP/s, fed with one wavefront per SIMD {fed1 / 1e6:.1f}, with two {fed2 / 1e6:.1f}")
    assert 0.6 < fed1 / bare < 0.995 and fed1 <= 1.01 * fed2 and fed2 <= 1.03 * bare
