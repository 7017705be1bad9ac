// Multi-channel convolution on channel-last tensors, fp32, bf16 and IEEE half, on the matrix cores: any filter extent,
// stride, padding and dilation (paper, section 3: the taps as small matrix products; section 1.1: reduced
// precision applied to the same sliding formulation).
//
//   x [N, H, W, C_in]     w [C_out, R, S, C_in]     y [N, H_out, W_out, C_out]
//   fp32: fp32 everywhere, v_mfma_f32_32x32x2_f32.
//   bf16: x, w and y are bf16 bit patterns, products and sums are fp32 (v_mfma_f32_32x32x16_bf16: a bf16 product
//         is exact in fp32), one rounding of the finished sum (+ bias, rectifier) to bf16, nearest even.
//   half: the same with v_mfma_f32_32x32x16_f16 (a product of two halves is exact in fp32 as well) and one rounding
//         to half precision, nearest even, overflow to infinity, denormals kept.
//
// With the channel as the fastest axis of both tensors the K operand of a matrix instruction is 16 consecutive
// bytes of memory per lane (four fp32 channels = the operands of four K steps, or eight bf16 channels = one), so
// nothing is transposed on the way: the rows of the input a band of outputs touches and the filters of 64 output
// channels go to LDS with plain 16-byte loads, a chunk of CB bytes per pixel at a time (all loads of a chunk are
// issued before the first LDS write: one memory round trip), and every tap (r, s) contributes W_rs[co, ci] times
// the window shifted by (r, s) * dilation: the shift is an address offset, no column matrix exists.
//
// Workgroup = 4 wavefronts = 64 output channels x a band of TH output rows of one image, taken as up to 8 blocks
// of 32 consecutive output pixels (row-major: each lane computes its own pixel's window address).  A = pixels,
// B = filters: a lane of the result holds one output channel for 16 pixels, so a store instruction writes runs of
// 32 consecutive channels, the fastest axis of the output.  LDS pitches: a pixel takes CB + 16 bytes, an output
// channel's filters R*S*CB + 16 (+ what makes that 16 modulo 128).
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

constexpr int kMaxBlocks = 8;          // 32-pixel blocks per workgroup
constexpr int kBlocksPerWave = 4;      // a wavefront takes every second block of one 32-channel half
constexpr int kLdsBudget = 156 * 1024;
constexpr int kXSlots = 12;            // 16-byte pieces of the window per thread and chunk
constexpr int kWSlots = 24;            // 16-byte pieces of the filters per thread and chunk

struct NhwcFParams {
    Epilogue ep;                       // fp32 bias and rectifier applied in the store
    int H, W, C_out, R, S, stride, pad, dil, Ho, Wo;
    int PB, CB, chunks;                // bytes per pixel (C_in * element size), per pixel and chunk, chunks
    int TH, IH, IWp;                   // output rows per band; window rows and columns in LDS
    int CP, WPITCH;                    // bytes per pixel / per output channel's filters in LDS
    int c16;                           // 16-byte pieces per pixel and chunk
    int wrow16;                        // 16-byte pieces per output channel's filters and chunk (R * S * c16)
    int x_bytes;                       // window bytes in LDS (filters follow)
    FastDiv by_c16, by_IWp, by_wrow16, by_Wo;
};

__device__ __forceinline__ unsigned short bf16_rne(float f)
{
    unsigned u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

// the one rounding of a finished value to the tensor's 16-bit format
template <int EK>
__device__ __forceinline__ unsigned short round16(float f)
{
    if constexpr (EK == kElemF16) return __builtin_bit_cast(unsigned short, (_Float16)f);      // v_cvt_f16_f32: nearest even
    else return bf16_rne(f);
}

// a 16-bit element widened to fp32 (exact)
template <int EK>
__device__ __forceinline__ float widen16(unsigned short h)
{
    if constexpr (EK == kElemF16) return (float)__builtin_bit_cast(_Float16, h);
    else return __uint_as_float((unsigned)h << 16);
}

// EK: element format (Elem).  KS: K steps of 32 bytes per tap and chunk (CB / 32): 1, 2 or 4.
template <int EK, int KS>
__global__ __launch_bounds__(256, 1) void mfma_nhwc_kernel(const unsigned char* __restrict__ x,
                                                           const unsigned char* __restrict__ w, void* __restrict__ yv,
                                                           const NhwcFParams P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* lx = smem;                 // [window row][window column][chunk bytes], pitch CP
    unsigned char* lw = smem + P.x_bytes;     // [co][tap][chunk bytes], pitch WPITCH
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lg = lane >> 5, lj = lane & 31;          // K half; pixel (A) or channel (B, D) inside a block
    const int band = blockIdx.x, n = blockIdx.y, cb = blockIdx.z;
    const int oi0 = band * P.TH;                        // first output row of the band
    const int rows = min(P.TH, P.Ho - oi0);
    const int npix = rows * P.Wo;                       // output pixels of this band
    const int co0 = cb * 64;
    const int RS = P.R * P.S;

    // ---- staging plan (the same for every chunk): window piece = (window pixel, 16-byte piece c of the chunk)
    const int gr0 = oi0 * P.stride - P.pad;             // image row / column of window position (0, 0)
    const int n_x = P.IH * P.IWp * P.c16;
    const unsigned char* xn = x + (int64_t)n * P.H * P.W * P.PB;
    int xsrc[kXSlots], xdst[kXSlots];                   // source byte offset in the image (< 0: zero), LDS byte offset (< 0: none)
#pragma unroll
    for (int u = 0; u < kXSlots; ++u) {
        const int idx = tid + 256 * u;
        const int pix = fast_div(idx, P.by_c16);
        const int c = idx - pix * P.c16;
        const int e = fast_div(pix, P.by_IWp), f = pix - e * P.IWp;
        const int gr = gr0 + e, gc = f - P.pad;
        xdst[u] = idx < n_x ? pix * P.CP + 16 * c : -1;
        xsrc[u] = (idx < n_x && gr >= 0 && gr < P.H && gc >= 0 && gc < P.W) ? (gr * P.W + gc) * P.PB + 16 * c : -1;
    }
    // filter piece = (output channel, tap, 16-byte piece c of the chunk)
    const int n_w = 64 * P.wrow16;
    const unsigned char* wb = w + (int64_t)co0 * RS * P.PB;

    // ---- this wavefront: channel half wn, pixel blocks wp, wp + 2, wp + 4, wp + 6 ----
    const int wn = wave & 1, wp = wave >> 1;
    const int nblocks = (npix + 31) >> 5;
    int aoff[kBlocksPerWave];                           // byte offset in lx of the lane's pixel, tap (0, 0)
#pragma unroll
    for (int b = 0; b < kBlocksPerWave; ++b) {
        int p = 32 * (wp + 2 * b) + lj;
        if (p > npix - 1) p = npix - 1;                 // lanes past the band read a valid pixel, store nothing
        const int oi = fast_div(p, P.by_Wo), oj = p - oi * P.Wo;
        aoff[b] = ((oi * P.stride) * P.IWp + oj * P.stride) * P.CP + 16 * lg;
    }
    const unsigned char* bsrc = lw + (32 * wn + lj) * P.WPITCH + 16 * lg;
    floatx16 acc[kBlocksPerWave];
#pragma unroll
    for (int b = 0; b < kBlocksPerWave; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;

    struct Ops {
        intx4 bq[KS];
        intx4 aq[KS][kBlocksPerWave];
    };
    auto load_ops = [&](Ops& o, int tap_x, int tap_w) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < KS; ++k) {
            o.bq[k] = *reinterpret_cast<const intx4*>(bsrc + tap_w + 32 * k);
#pragma unroll
            for (int b = 0; b < kBlocksPerWave; ++b)
                o.aq[k][b] = *reinterpret_cast<const intx4*>(lx + aoff[b] + tap_x + 32 * k);
        }
    };
    auto multiply = [&](const Ops& o) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < KS; ++k)
#pragma unroll
            for (int b = 0; b < kBlocksPerWave; ++b)
                if (wp + 2 * b < nblocks) {             // (wave-uniform)
                    if constexpr (EK == kElemF16) {
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, o.aq[k][b]),
                                                                        __builtin_bit_cast(halfx8, o.bq[k]), acc[b], 0, 0, 0);
                    } else if constexpr (EK == kElemBF16) {
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, o.aq[k][b]),
                                                                         __builtin_bit_cast(bf16x8, o.bq[k]), acc[b], 0, 0, 0);
                    } else {
                        const floatx4 af = __builtin_bit_cast(floatx4, o.aq[k][b]), bf = __builtin_bit_cast(floatx4, o.bq[k]);
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bf[t], acc[b], 0, 0, 0);
                    }
                }
    };

    for (int ch = 0; ch < P.chunks; ++ch) {
        // ---- global -> registers -> LDS: every piece of the chunk before any LDS write
        const int cb0 = ch * P.CB;
        intx4 xv[kXSlots];
#pragma unroll
        for (int u = 0; u < kXSlots; ++u) {
            xv[u] = intx4{0, 0, 0, 0};
            if (xsrc[u] >= 0) xv[u] = *reinterpret_cast<const intx4*>(xn + xsrc[u] + cb0);
        }
        if (ch > 0) __syncthreads();                    // everybody has finished the multiplications of the chunk before
#pragma unroll
        for (int u = 0; u < kXSlots; ++u)
            if (xdst[u] >= 0) *reinterpret_cast<intx4*>(lx + xdst[u]) = xv[u];
        // the filters in rounds of kWSlots pieces per thread (one round for up to 96 pieces per output channel)
        for (int base = 0; base < n_w; base += 256 * kWSlots) {
            intx4 wv[kWSlots];
            int wdst[kWSlots];
#pragma unroll
            for (int u = 0; u < kWSlots; ++u) {
                const int idx = base + tid + 256 * u;
                const int co = fast_div(idx, P.by_wrow16);
                const int q = idx - co * P.wrow16;
                const int tap = fast_div(q, P.by_c16), c = q - tap * P.c16;
                wdst[u] = idx < n_w ? co * P.WPITCH + tap * P.CB + 16 * c : -1;
                wv[u] = intx4{0, 0, 0, 0};              // channels beyond C_out: zero filters
                if (idx < n_w && co0 + co < P.C_out)
                    wv[u] = *reinterpret_cast<const intx4*>(wb + (co * RS + tap) * P.PB + 16 * c + cb0);
            }
#pragma unroll
            for (int u = 0; u < kWSlots; ++u)
                if (wdst[u] >= 0) *reinterpret_cast<intx4*>(lw + wdst[u]) = wv[u];
        }
        __syncthreads();

        // ---- every tap: the operands of the next tap are on their way from LDS while this one multiplies
        int tap_x = 0, tap_w = 0, s = 0;
        auto next_tap = [&]() __attribute__((always_inline)) {
            tap_w += P.CB;
            tap_x += P.dil * P.CP;
            if (++s == P.S) { s = 0; tap_x += P.dil * (P.IWp - P.S) * P.CP; }
        };
        Ops o0, o1;
        load_ops(o0, tap_x, tap_w);
        int tap = 0;
#pragma unroll 1
        for (; tap + 2 <= RS; tap += 2) {
            next_tap();
            load_ops(o1, tap_x, tap_w);
            __builtin_amdgcn_sched_barrier(0);
            multiply(o0);
            __builtin_amdgcn_sched_barrier(0);
            if (tap + 2 < RS) {
                next_tap();
                load_ops(o0, tap_x, tap_w);
            }
            __builtin_amdgcn_sched_barrier(0);
            multiply(o1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (tap < RS) multiply(o0);                     // odd tap count: the last tap is already in o0
    }

    // ---- store: register v of a lane is pixel 8*(v/4) + 4*lg + v%4 of the block, channel lj ----
    const int co = co0 + 32 * wn + lj;
    if (co >= P.C_out) return;
    const int64_t pix0 = ((int64_t)n * P.Ho + oi0) * P.Wo;
    const float bias = P.ep.bias ? P.ep.bias[co] : 0.f;
#pragma unroll
    for (int b = 0; b < kBlocksPerWave; ++b) {
        if (wp + 2 * b >= nblocks) break;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int p = 32 * (wp + 2 * b) + 8 * (v >> 2) + 4 * lg + (v & 3);
            float t = acc[b][v];
            if (P.ep.bias) t += bias;
            if (P.ep.relu) t = fmaxf(t, 0.f);
            if (p < npix) {
                if constexpr (EK != kElemF32) static_cast<unsigned short*>(yv)[(pix0 + p) * P.C_out + co] = round16<EK>(t);
                else static_cast<float*>(yv)[(pix0 + p) * P.C_out + co] = t;
            }
        }
    }
}

// One thread per output, any shape: the channel loop runs over contiguous elements of both tensors.
template <int EK>
__global__ __launch_bounds__(256) void direct_nhwc_kernel(const void* __restrict__ xv, const void* __restrict__ wv,
                                                          void* __restrict__ yv, Conv2dShape s, Epilogue ep)
{
    const int64_t total = (int64_t)s.N * s.Ho * s.Wo * s.C_out;
    for (int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (int64_t)gridDim.x * 256) {
        const int co = (int)(o % s.C_out);
        int64_t t = o / s.C_out;
        const int oj = (int)(t % s.Wo);
        t /= s.Wo;
        const int oi = (int)(t % s.Ho);
        const int n = (int)(t / s.Ho);
        float acc = 0.f;
        for (int r = 0; r < s.R; ++r) {
            const int h = oi * s.stride + r * s.dil - s.pad;
            if (h < 0 || h >= s.H) continue;
            for (int q = 0; q < s.S; ++q) {
                const int v = oj * s.stride + q * s.dil - s.pad;
                if (v < 0 || v >= s.W) continue;
                const int64_t xo = (((int64_t)n * s.H + h) * s.W + v) * s.C_in, wo = (((int64_t)co * s.R + r) * s.S + q) * s.C_in;
                if constexpr (EK != kElemF32) {
                    const unsigned short* xp = static_cast<const unsigned short*>(xv) + xo;
                    const unsigned short* wp = static_cast<const unsigned short*>(wv) + wo;
                    for (int ci = 0; ci < s.C_in; ++ci)
                        acc = fmaf(widen16<EK>(xp[ci]), widen16<EK>(wp[ci]), acc);
                } else {
                    const float* xp = static_cast<const float*>(xv) + xo;
                    const float* wp = static_cast<const float*>(wv) + wo;
                    for (int ci = 0; ci < s.C_in; ++ci) acc = fmaf(xp[ci], wp[ci], acc);
                }
            }
        }
        if (ep.bias) acc += ep.bias[co];
        if (ep.relu) acc = fmaxf(acc, 0.f);
        if constexpr (EK != kElemF32) static_cast<unsigned short*>(yv)[o] = round16<EK>(acc);
        else static_cast<float*>(yv)[o] = acc;
    }
}

struct NhwcFPlan {
    NhwcFParams P;
    size_t lds;
    int bands, KS;
    bool ok;
};

NhwcFPlan plan_nhwc_f(const Conv2dShape& s, int esz)
{
    NhwcFPlan a{};
    NhwcFParams& P = a.P;
    const int64_t PB = (int64_t)s.C_in * esz;
    if (PB % 32 != 0 || PB > (1 << 20)) return a;       // whole K steps of 32 bytes per pixel
    const int RS = s.R * s.S;
    P.H = s.H; P.W = s.W; P.C_out = s.C_out; P.R = s.R; P.S = s.S; P.stride = s.stride;
    P.pad = s.pad; P.dil = s.dil; P.Ho = s.Ho; P.Wo = s.Wo;
    P.PB = (int)PB;
    const int64_t IWp = (int64_t)(s.Wo - 1) * s.stride + (int64_t)(s.S - 1) * s.dil + 1;
    if (IWp > 8192) return a;
    P.IWp = (int)IWp;
    // chunk: the largest of 128, 64, 32 bytes per pixel that divides the pixel and whose filters fit the staging
    // slots; then as many output rows per band as the pixel blocks, the slots and LDS allow
    bool found = false;
    for (int cbytes = 128; cbytes >= 32 && !found; cbytes /= 2) {
        if (PB % cbytes != 0) continue;
        P.CB = cbytes;
        P.chunks = (int)(PB / cbytes);
        P.CP = cbytes + 16;
        const int wrow = RS * cbytes;
        P.WPITCH = wrow + 16 + (128 - wrow % 128) % 128;
        P.c16 = cbytes / 16;
        P.wrow16 = wrow / 16;
        if ((int64_t)64 * P.wrow16 >= 65536) continue;  // (exact fast division of the piece index)
        int TH = (kMaxBlocks * 32) / s.Wo;
        if (TH > s.Ho) TH = s.Ho;
        for (; TH >= 1; --TH) {
            const int64_t IH = (int64_t)(TH - 1) * s.stride + (int64_t)(s.R - 1) * s.dil + 1;
            const int64_t xb = IH * P.IWp * P.CP;
            if (IH * P.IWp * P.c16 <= 256 * kXSlots && xb + (int64_t)64 * P.WPITCH <= kLdsBudget) break;
        }
        if (TH < 1) continue;
        const int bands = (s.Ho + TH - 1) / TH;         // equal bands
        TH = (s.Ho + bands - 1) / bands;
        P.TH = TH;
        P.IH = (TH - 1) * s.stride + (s.R - 1) * s.dil + 1;
        found = true;
    }
    if (!found) return a;
    P.x_bytes = (P.IH * P.IWp * P.CP + 15) & ~15;
    a.lds = (size_t)P.x_bytes + (size_t)64 * P.WPITCH;
    a.bands = (s.Ho + P.TH - 1) / P.TH;
    a.KS = P.CB / 32;
    P.by_c16 = make_fastdiv(P.c16);
    P.by_IWp = make_fastdiv(P.IWp);
    P.by_wrow16 = make_fastdiv(P.wrow16);
    P.by_Wo = make_fastdiv(s.Wo);
    a.ok = a.lds <= (size_t)kLdsBudget && s.N <= 65535 && (s.C_out + 63) / 64 <= 65535 &&
           // 32-bit byte offsets inside one image and inside the filters of 64 channels
           (int64_t)s.H * s.W * PB <= 2147483647LL && (int64_t)64 * RS * PB <= 2147483647LL &&
           (int64_t)P.TH * s.Wo <= kMaxBlocks * 32;
    return a;
}

template <int EK, int KS>
hipError_t launch_nhwc_f(const void* x, const void* w, void* y, const NhwcFPlan& a, const Conv2dShape& s, hipStream_t st)
{
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_nhwc_kernel<EK, KS>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget);
    if (attr != hipSuccess) return attr;
    dim3 grid((unsigned)a.bands, (unsigned)s.N, (unsigned)((s.C_out + 63) / 64));
    SW_NOTED_LAUNCH(note_kernel("mfma_nhwc_kernel", EK, KS), (mfma_nhwc_kernel<EK, KS>), grid, dim3(256), a.lds, st,
                    static_cast<const unsigned char*>(x), static_cast<const unsigned char*>(w), y, a.P);
    return hipGetLastError();
}

}  // namespace

bool mfma_nhwc_supported(const void* x, const void* w, const Conv2dShape& s, int ek)
{
    return reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 && plan_nhwc_f(s, elem_size(ek)).ok;
}

hipError_t launch_mfma_nhwc(const void* x, const void* w, void* y, const Conv2dShape& s, int ek, const Epilogue& ep,
                            hipStream_t st)
{
    NhwcFPlan a = plan_nhwc_f(s, elem_size(ek));
    if (!a.ok) return hipErrorInvalidValue;
    a.P.ep = ep;
#define SW_NHWC(EKC)                                                             \
    do {                                                                         \
        if (a.KS == 4) return launch_nhwc_f<EKC, 4>(x, w, y, a, s, st);          \
        if (a.KS == 2) return launch_nhwc_f<EKC, 2>(x, w, y, a, s, st);          \
        return launch_nhwc_f<EKC, 1>(x, w, y, a, s, st);                         \
    } while (0)
    if (ek == kElemF16) SW_NHWC(kElemF16);
    if (ek == kElemBF16) SW_NHWC(kElemBF16);
    SW_NHWC(kElemF32);
#undef SW_NHWC
}

hipError_t launch_direct_nhwc(const void* x, const void* w, void* y, const Conv2dShape& s, int ek, const Epilogue& ep,
                              hipStream_t st)
{
    const int64_t total = (int64_t)s.N * s.Ho * s.Wo * s.C_out;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    if (ek == kElemF16)
        SW_NOTED_LAUNCH(note_kernel("direct_nhwc_kernel", 2), direct_nhwc_kernel<kElemF16>, dim3((unsigned)blocks), dim3(256), 0, st,
                        x, w, y, s, ep);
    else if (ek == kElemBF16)
        SW_NOTED_LAUNCH(note_kernel("direct_nhwc_kernel", 1), direct_nhwc_kernel<kElemBF16>, dim3((unsigned)blocks), dim3(256), 0, st,
                        x, w, y, s, ep);
    else
        SW_NOTED_LAUNCH(note_kernel("direct_nhwc_kernel", 0), direct_nhwc_kernel<kElemF32>, dim3((unsigned)blocks), dim3(256), 0, st,
                        x, w, y, s, ep);
    return hipGetLastError();
}

}  // namespace swconv
