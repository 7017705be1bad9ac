// Measurement aids: kernels that issue one kind of arithmetic instruction and nothing else, so that a benchmark
// can quote the rate this chip sustains (at the clock it holds under that instruction) beside the datasheet
// peak.  They read and write no memory (the sink is only there to keep the arithmetic alive); the "fed" probe reads
// its operands from LDS, as every convolution kernel must.
#include "../../include/swconv.h"

#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx16 __attribute__((ext_vector_type(16)));
typedef int intx4 __attribute__((ext_vector_type(4)));

constexpr int kProbeGroups = 256 * 8;    // workgroups of one wavefront: eight per compute unit, two per SIMD
constexpr int kMfmaPerIter = 8;          // matrix instructions per loop turn (four independent accumulators, twice)
constexpr int kFmaAcc = 48;              // independent fp32 accumulators of the vector probe
constexpr int kFmaPerIter = kFmaAcc * 4;
constexpr int kMixRounds = 16;           // rounds per loop turn of the mixed probe:
constexpr int kMixFma = 9;               // nine plain FMAs, then one 16 x 16 x 4 matrix instruction

__global__ __launch_bounds__(64) void probe_mfma_f32_kernel(int iters, float* sink)
{
    floatx16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const float a = 1.0f + threadIdx.x * 1e-3f, b = 0.5f;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kMfmaPerIter; ++u) acc[u & 3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[u & 3], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i) s += acc[i][0] + acc[i][15];
    if (sink && s == 12345.678f) *sink = s;
}

__global__ __launch_bounds__(64) void probe_mfma_i8_kernel(int iters, float* sink)
{
    intx16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0;
    const intx4 a = {(int)threadIdx.x, 0x01020304, 0x7f807f80, 0x11111111}, b = {0x01010101, 0x02020202, (int)blockIdx.x, 0x04040404};
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kMfmaPerIter; ++u) acc[u & 3] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[u & 3], 0, 0, 0);
    }
    int s = 0;
    for (int i = 0; i < 4; ++i) s += acc[i][0] + acc[i][15];
    if (sink && s == 123456789) *sink = (float)s;
}

__global__ __launch_bounds__(64) void probe_mfma_bf16_kernel(int iters, float* sink)
{
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    floatx16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const intx4 ai = {0x3f803f80, 0x3f003f00, (int)(0x3f800000u | threadIdx.x), 0x3f803f00}, bi = {0x3f803f80, 0x3f803f80, 0x3f003f80, 0x3f803f80};
    const bf16x8 a = __builtin_bit_cast(bf16x8, ai), b = __builtin_bit_cast(bf16x8, bi);
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kMfmaPerIter; ++u) acc[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[u & 3], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i) s += acc[i][0] + acc[i][15];
    if (sink && s == 12345.678f) *sink = s;
}

// plain v_fma_f32 with a wave-uniform multiplicand, as in the one-filter-per-plane kernels (no packed forms)
__global__ __launch_bounds__(64) void probe_fma_f32_kernel(int iters, float* sink, float tap0, float tap1)
{
    float acc[kFmaAcc];
    for (int i = 0; i < kFmaAcc; ++i) acc[i] = threadIdx.x * 1e-3f + i;
    float in[4] = {1.0f + threadIdx.x * 1e-4f, 0.999f, 1.001f, 0.5f};
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < kFmaAcc; ++i) acc[i] = fmaf((u & 1) ? tap1 : tap0, in[u], acc[i]);
    }
    float s = 0.f;
    for (int i = 0; i < kFmaAcc; ++i) s += acc[i];
    if (sink && s == 12345.678f) *sink = s;
}

// Plain FMAs and independent fp32 matrix instructions in one stream (nine v_fma_f32, one v_mfma_f32_16x16x4_f32, ...):
// if the vector and the matrix pipe worked side by side on fp32, a round would take as long as its slower part; on this
// chip it takes the sum of the two, which is why the one-filter-per-plane kernels leave the matrix cores alone.
__global__ __launch_bounds__(64) void probe_fma_mfma_f32_kernel(int iters, float* sink, float tap0)
{
    float acc[kFmaAcc];
    for (int i = 0; i < kFmaAcc; ++i) acc[i] = threadIdx.x * 1e-3f + i;
    float in[8];
    for (int j = 0; j < 8; ++j) in[j] = 1.0f + threadIdx.x * 1e-4f + j * 1e-3f;
    floatx4 d[8];
    for (int t = 0; t < 8; ++t) d[t] = floatx4{0.f, 0.f, 0.f, 0.f};
    const float a = 1.0f + threadIdx.x * 1e-3f, b = 0.5f;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int g = 0; g < kMixRounds; ++g) {
#pragma unroll
            for (int i = 0; i < kMixFma; ++i) {
                const int k = (g * kMixFma + i) % kFmaAcc;
                acc[k] = fmaf(tap0, in[(k + g) & 7], acc[k]);
            }
            d[g & 7] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, d[g & 7], 0, 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, kMixFma, 0);     // keep the two kinds interleaved as written
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
    }
    float s = 0.f;
    for (int i = 0; i < kFmaAcc; ++i) s += acc[i];
    for (int t = 0; t < 8; ++t) s += d[t][0] + d[t][3];
    if (sink && s == 12345.678f) *sink = s;
}

// fp32 matrix instructions whose A operand comes from LDS, one 4-byte read behind each instruction, consumed four
// instructions later (its latency hidden): what a matrix-instruction stream sustains when it is fed at the lowest
// rate a 64-channel x 32-pixel tile allows (half an operand dword per instruction from each side).  WAVES
// wavefronts per SIMD: one (a workgroup alone on its CU) or two.
template <int WAVES>
__global__ __launch_bounds__(256 * WAVES) void probe_mfma_f32_fed_kernel(int iters, float* sink)
{
    __shared__ float lds[4096];
    for (int i = threadIdx.x; i < 4096; i += 256 * WAVES) lds[i] = 1.0f + i * 1e-6f;
    __syncthreads();
    floatx16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const float b = 0.5f;
    const int at = threadIdx.x & 1023;
    float ring[4];
    for (int r = 0; r < 4; ++r) ring[r] = lds[at + 64 * r];
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kMfmaPerIter; ++u) {
            acc[u & 3] = __builtin_amdgcn_mfma_f32_32x32x2f32(ring[u & 3], b, acc[u & 3], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            ring[u & 3] = lds[at + 256 * u + (it & 1023)];
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i) s += acc[i][0] + acc[i][15];
    if (sink && s == 12345.678f) *sink = s;
}

}  // namespace

}  // namespace swconv

using namespace swconv;

extern "C" {

int64_t sw_probe_ops(int kind, int iters)
{
    if (iters <= 0) return 0;
    const int64_t waves = kProbeGroups;
    switch (kind) {
        case SW_PROBE_MFMA_F32: return waves * iters * kMfmaPerIter * (2LL * 32 * 32 * 2);
        case SW_PROBE_MFMA_I8: return waves * iters * kMfmaPerIter * (2LL * 32 * 32 * 32);
        case SW_PROBE_FMA_F32: return waves * iters * kFmaPerIter * (2LL * 64);
        case SW_PROBE_FMA_MFMA_F32: return waves * iters * kMixRounds * (kMixFma * 2LL * 64 + 2LL * 16 * 16 * 4);
        case SW_PROBE_MFMA_BF16: return waves * iters * kMfmaPerIter * (2LL * 32 * 32 * 16);
        case SW_PROBE_MFMA_F32_FED: return 256LL * 4 * iters * kMfmaPerIter * (2LL * 32 * 32 * 2);
        case SW_PROBE_MFMA_F32_FED2: return 256LL * 8 * iters * kMfmaPerIter * (2LL * 32 * 32 * 2);
        default: return 0;
    }
}

int sw_probe(int kind, int iters, void* hip_stream)
{
    if (iters <= 0) return SW_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    float* none = nullptr;
    switch (kind) {
        case SW_PROBE_MFMA_F32:
            SW_NOTED_LAUNCH(note_kernel("probe_mfma_f32_kernel"), probe_mfma_f32_kernel, dim3(kProbeGroups), dim3(64), 0, st, iters, none);
            break;
        case SW_PROBE_MFMA_I8:
            SW_NOTED_LAUNCH(note_kernel("probe_mfma_i8_kernel"), probe_mfma_i8_kernel, dim3(kProbeGroups), dim3(64), 0, st, iters, none);
            break;
        case SW_PROBE_FMA_F32:
            SW_NOTED_LAUNCH(note_kernel("probe_fma_f32_kernel"), probe_fma_f32_kernel, dim3(kProbeGroups), dim3(64), 0, st, iters, none,
                            1.0000001f, 0.9999999f);
            break;
        case SW_PROBE_FMA_MFMA_F32:
            SW_NOTED_LAUNCH(note_kernel("probe_fma_mfma_f32_kernel"), probe_fma_mfma_f32_kernel, dim3(kProbeGroups), dim3(64), 0, st, iters,
                            none, 1.0000001f);
            break;
        case SW_PROBE_MFMA_BF16:
            SW_NOTED_LAUNCH(note_kernel("probe_mfma_bf16_kernel"), probe_mfma_bf16_kernel, dim3(kProbeGroups), dim3(64), 0, st, iters, none);
            break;
        case SW_PROBE_MFMA_F32_FED:
            SW_NOTED_LAUNCH(note_kernel("probe_mfma_f32_fed_kernel", 1), probe_mfma_f32_fed_kernel<1>, dim3(256), dim3(256), 0, st, iters, none);
            break;
        case SW_PROBE_MFMA_F32_FED2:
            SW_NOTED_LAUNCH(note_kernel("probe_mfma_f32_fed_kernel", 2), probe_mfma_f32_fed_kernel<2>, dim3(256), dim3(512), 0, st, iters, none);
            break;
        default: return SW_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? SW_OK : SW_ERR_LAUNCH;
}

}  // extern "C"
