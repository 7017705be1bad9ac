// Multi-channel fp32 sliding window convolution on the matrix cores for ANY filter extent, stride, padding
// and channel count (paper, section 3: the sliding algorithm re-formulated as small matrix products;
// section 2: every filter size on the unmodified input).
//
// The fixed 3x3 / 5x5 kernel of sw_mfma_f32.hip owns a CU with one large tile; this one trades peak rate for
// reach.  A workgroup of four wavefronts computes 64 output channels x up to 128 output pixels (whole output
// rows of one image).  The input channels are walked in chunks of CK: the chunk's input window (tile + halo,
// zero outside the image and beyond C_in: that is the padding) and the chunk's filters are staged in LDS
// once (filters as they lie in memory, so staging is a row copy); then every tap (r, s) is one small matrix
// product per pixel block,
//     ACC[co, p] += W_rs[co, ci] * X[ci, p shifted by (r, s)],
// on v_mfma_f32_32x32x2_f32, the shift being nothing but an LDS address offset of the B operand (stride is
// a multiplier in the pixel's window address).  No column matrix exists anywhere.  Small LDS footprints let
// several workgroups share a CU, so one's staging hides under another's matrix instructions; that, and
// tiles of 128 pixels, is also why small images (28 x 28 and below), which leave the large-tile kernel
// short of workgroups, run here.
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kTilePx = 128;           // output pixels per workgroup: one 32-pixel block per wavefront
constexpr int kLdsBudget = 64 * 1024;  // keeps at least two workgroups on a CU
constexpr int kLdsLarge = 156 * 1024;  // one workgroup per CU: filters whose 64 x (channels x taps) rows need it
constexpr int kXS = 16;                // register-prefetch slots per thread: input window (floats) ...
constexpr int kWS = 6;                 // ... and filters (16-byte groups)

struct AnyParams {
    Epilogue ep;                       // bias and rectifier applied in the store
    int C_in, C_out, H, W, R, S, stride, pad, Ho, Wo;
    int TH, TW, IH, IW, tiles_x, wpitch, dil;
    FastDiv by_tiles_x, by_TW, by_IW, by_win, by_span, by_span4;
};

// XS > 0: the next chunk travels global memory -> registers while this chunk multiplies (needs 16-byte aligned
// filter rows and at most XS / kWS staging slots per thread); XS == 0: a chunk is staged, then multiplied.
template <int CK, int XS>
__global__ __launch_bounds__(256) void mfma_f32_any_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                           float* __restrict__ y, const AnyParams P)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int RS = P.R * P.S;
    const int WP = P.IH * P.IW;                 // window pixels per channel
    const int span = CK * RS;                   // filter floats per output channel and chunk, contiguous in w
    float* xs = smem;                           // [CK][WP]
    float* ws = smem + ((CK * WP + 3) & ~3);    // [co][CK][RS] as in memory, rows P.wpitch floats apart

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lj = lane & 31, kk = lane >> 5;   // row/column inside a 32 x 32 block, K half

    const int ty = fast_div(blockIdx.x, P.by_tiles_x);
    const int tx = blockIdx.x - ty * P.tiles_x;
    const int n = blockIdx.y;
    const int co0 = blockIdx.z * 64;
    const int row0 = ty * P.TH, col0 = tx * P.TW;               // first output pixel of the tile
    const int grow0 = row0 * P.stride - P.pad, gcol0 = col0 * P.stride - P.pad;   // window origin in the image

    // this lane's output pixel (block = wavefront) and its window offset
    const int tile_px = P.TH * P.TW;
    const int p = wave * 32 + lj;
    const int pi = fast_div(p, P.by_TW), pj = p - pi * P.TW;
    const bool p_ok = p < tile_px && row0 + pi < P.Ho && col0 + pj < P.Wo;
    const int pixoff = p_ok ? (pi * P.stride) * P.IW + pj * P.stride : 0;
    const bool wave_live = __builtin_amdgcn_readfirstlane(wave * 32) < tile_px;

    floatx16 acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }

    const int HW = P.H * P.W;
    const float* xn = x + (int64_t)n * P.C_in * HW;
    const int64_t wrow = (int64_t)P.C_in * RS;                  // floats per output channel in w
    const float* wb = w + (int64_t)co0 * wrow;

    // every tap is a 64 x CK by CK x 32 product per wavefront; the shift is the offset toff
    auto multiply = [&]() {
        if (!wave_live) return;
        const float* bsrc = xs + kk * WP + pixoff;
        const float* asrc = ws + lj * P.wpitch + kk * RS;
        int toff = 0, s = 0;
#pragma unroll 1
        for (int tap = 0; tap < RS; ++tap) {
#pragma unroll
            for (int c2 = 0; c2 < CK / 2; ++c2) {
                const float b = bsrc[2 * c2 * WP + toff];
                const float a0 = asrc[2 * c2 * RS + tap];
                const float a1 = asrc[32 * P.wpitch + 2 * c2 * RS + tap];
                acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b, acc1, 0, 0, 0);
            }
            toff += P.dil;                                   // next tap column, P.dil input positions on
            if (++s == P.S) { s = 0; toff += P.dil * (P.IW - P.S); }
        }
    };

    if constexpr (XS > 0) {
        // staging plan, the same for every chunk: slot u of the window is float tid + 256 u, slot u of the
        // filters is 16-byte group tid + 256 u of the 64 rows
        int xo[XS];           // offset inside channel ci0's plane stack, < 0: padding
        int wo[kWS], wd[kWS], wq[kWS];  // offset from wb + ci0 * RS (< 0: nothing), LDS float index, offset in the row
        const int span4 = span >> 2;
#pragma unroll
        for (int u = 0; u < XS; ++u) {
            const int idx = tid + 256 * u;
            const int c = fast_div(idx, P.by_win);
            const int q = idx - c * WP;
            const int e = fast_div(q, P.by_IW), f = q - e * P.IW;
            const int gr = grow0 + e, gc = gcol0 + f;
            xo[u] = (idx < CK * WP && gr >= 0 && gr < P.H && gc >= 0 && gc < P.W) ? c * HW + gr * P.W + gc : -1;
        }
#pragma unroll
        for (int u = 0; u < kWS; ++u) {
            const int idx = tid + 256 * u;
            const int co_l = fast_div(idx, P.by_span4);
            const int q4 = idx - co_l * span4;
            wo[u] = (idx < 64 * span4 && co0 + co_l < P.C_out) ? co_l * (int)wrow + 4 * q4 : -1;
            wd[u] = co_l * P.wpitch + 4 * q4;
            wq[u] = 4 * q4;
        }
        float xv[XS];
        floatx4 wv[kWS];
        auto fetch = [&](int ci0) {
            const float* xc0 = xn + (int64_t)ci0 * HW;
            const float* wc0 = wb + (int64_t)ci0 * RS;
            const int left = (P.C_in - ci0) * RS;               // filter floats that exist from ci0 on
#pragma unroll
            for (int u = 0; u < XS; ++u) {
                xv[u] = 0.f;
                if (xo[u] >= 0 && ci0 + fast_div(tid + 256 * u, P.by_win) < P.C_in) xv[u] = xc0[xo[u]];
            }
#pragma unroll
            for (int u = 0; u < kWS; ++u) {
                wv[u] = floatx4{0.f, 0.f, 0.f, 0.f};
                // (span and the row length are multiples of 4, so a group lies wholly inside or outside)
                if (wo[u] >= 0 && wq[u] < left)
                    wv[u] = *reinterpret_cast<const floatx4*>(wc0 + wo[u]);
            }
        };
        auto stage = [&]() {
#pragma unroll
            for (int u = 0; u < XS; ++u)
                if (tid + 256 * u < CK * WP) xs[tid + 256 * u] = xv[u];
#pragma unroll
            for (int u = 0; u < kWS; ++u)
                if (tid + 256 * u < 64 * span4) {       // (rows sit an odd number of floats apart: four 4-byte writes)
                    ws[wd[u] + 0] = wv[u].x; ws[wd[u] + 1] = wv[u].y; ws[wd[u] + 2] = wv[u].z; ws[wd[u] + 3] = wv[u].w;
                }
        };
        fetch(0);
        for (int ci0 = 0; ci0 < P.C_in; ci0 += CK) {
            stage();
            __syncthreads();
            if (ci0 + CK < P.C_in) fetch(ci0 + CK);
            multiply();
            __syncthreads();
        }
    } else {
        for (int ci0 = 0; ci0 < P.C_in; ci0 += CK) {
            // input window (coalesced along image rows), zero outside the image and beyond C_in; eight loads go out
            // per thread before the first LDS write, so a batch costs one memory round trip instead of eight
            for (int base = tid; base < CK * WP; base += 256 * 8) {
                float v8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int idx = base + 256 * u;
                    const int c = fast_div(idx, P.by_win);
                    const int q = idx - c * WP;
                    const int e = fast_div(q, P.by_IW), f = q - e * P.IW;
                    const int gr = grow0 + e, gc = gcol0 + f;
                    v8[u] = 0.f;
                    if (idx < CK * WP && ci0 + c < P.C_in && gr >= 0 && gr < P.H && gc >= 0 && gc < P.W)
                        v8[u] = xn[(int64_t)(ci0 + c) * HW + gr * P.W + gc];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (base + 256 * u < CK * WP) xs[base + 256 * u] = v8[u];
            }
            // filters: for one output channel the chunk's span floats are contiguous in memory (batched likewise)
            const int left = (P.C_in - ci0) * RS;
            for (int base = tid; base < 64 * span; base += 256 * 8) {
                float v8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int idx = base + 256 * u;
                    const int co_l = fast_div(idx, P.by_span);
                    const int q = idx - co_l * span;
                    v8[u] = 0.f;
                    if (idx < 64 * span && co0 + co_l < P.C_out && q < left) v8[u] = wb[co_l * wrow + (int64_t)ci0 * RS + q];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int idx = base + 256 * u;
                    if (idx < 64 * span) {
                        const int co_l = fast_div(idx, P.by_span);
                        ws[co_l * P.wpitch + (idx - co_l * span)] = v8[u];
                    }
                }
            }
            __syncthreads();
            multiply();
            __syncthreads();
        }
    }

    // ---- store: register v of a lane is output channel 8*(v/4) + 4*kk + v%4 of the block, pixel lj
    if (!p_ok) return;
    const int HoWo = P.Ho * P.Wo;
    float* yp = y + ((int64_t)n * P.C_out + co0) * HoWo + (row0 + pi) * P.Wo + col0 + pj;
    if (P.ep.bias != nullptr || P.ep.relu != 0) {
        // the lane's biases are read eight at a time (one wait per group, and few registers: the plain path's
        // occupancy must not pay for the epilogue), then added, rectified and stored
#pragma unroll
        for (int h = 0; h < 4; ++h) {                   // h: accumulator (0, 1) x its register halves
            const int cb = h >= 2 ? 32 : 0, v0 = (h & 1) * 8;
            float b[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int v = v0 + i, co = co0 + cb + 8 * (v >> 2) + 4 * kk + (v & 3);
                b[i] = (P.ep.bias && co < P.C_out) ? P.ep.bias[co] : 0.f;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int v = v0 + i, co = cb + 8 * (v >> 2) + 4 * kk + (v & 3);
                const float t = (h >= 2 ? acc1[v] : acc0[v]) + b[i];
                if (co0 + co < P.C_out) yp[(int64_t)co * HoWo] = P.ep.relu ? fmaxf(t, 0.f) : t;
            }
        }
        return;
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int co = 8 * (v >> 2) + 4 * kk + (v & 3);
        if (co0 + co < P.C_out) yp[(int64_t)co * HoWo] = acc0[v];
        if (co0 + 32 + co < P.C_out) yp[(int64_t)(32 + co) * HoWo] = acc1[v];
    }
}

struct AnyPlan {
    int TH, TW, IH, IW, CK, tiles_x, tiles_y, wpitch;
    size_t lds;
    bool ok, prefetch;
};

AnyPlan plan_any(const Conv2dShape& s, const float* w)
{
    AnyPlan a{};
    const int RS = s.R * s.S;
    a.TW = s.Wo < kTilePx ? s.Wo : kTilePx;
    a.TH = kTilePx / a.TW;
    if (a.TH > s.Ho) a.TH = s.Ho;
    if (a.TH < 1) a.TH = 1;
    // channels per chunk: about a hundred (tap, channel) rows of filters per barrier pair, no more than exist
    a.CK = 32;
    while (a.CK > 2 && (a.CK * RS > 96 || a.CK >= 2 * s.C_in)) a.CK /= 2;
    auto bytes = [&]() {
        a.IH = (a.TH - 1) * s.stride + (s.R - 1) * s.dil + 1;
        a.IW = (a.TW - 1) * s.stride + (s.S - 1) * s.dil + 1;
        const int span = a.CK * RS;
        a.wpitch = span | 1;     // odd: the 32 rows an operand read touches fall into 32 banks
        return ((((size_t)a.CK * a.IH * a.IW + 3) & ~(size_t)3) + (size_t)64 * a.wpitch) * sizeof(float);
    };
    // two workgroups per CU if the filters allow it, else one (large filters: 11 x 11 needs 62 KB for the
    // filter rows of two channels alone)
    size_t budget = (size_t)64 * ((2 * RS) | 1) * sizeof(float) + 4096 <= (size_t)kLdsBudget ? kLdsBudget : kLdsLarge;
    while (bytes() > budget) {
        if (a.CK > 2) a.CK /= 2;
        else if (a.TH > 1) a.TH = (a.TH + 1) / 2;
        else if (a.TW > 32) a.TW = (a.TW + 1) / 2;
        else break;
    }
    // with 16-byte aligned filter rows the next chunk can be prefetched into registers, if the window is
    // small enough for the slots a thread has: trade channels per chunk for that
    const bool vec = ((int64_t)s.C_in * RS) % 4 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 && w != nullptr;
    if (vec) {
        bytes();
        while (a.CK > 4 && ((a.CK * RS) % 4 != 0 || (int64_t)a.CK * a.IH * a.IW > 256 * kXS ||
                            64 * (a.CK * RS / 4) > 256 * kWS))
            a.CK /= 2;
    }
    a.lds = bytes();
    a.tiles_x = (s.Wo + a.TW - 1) / a.TW;
    a.tiles_y = (s.Ho + a.TH - 1) / a.TH;
    const int64_t span = (int64_t)a.CK * RS;
    a.ok = a.lds <= budget && (int64_t)a.tiles_x * a.tiles_y * a.tiles_x < 2147483647LL && s.N <= 65535 &&
           (s.C_out + 63) / 64 <= 65535 &&
           // 32-bit index arithmetic inside one image / 64 output channels' filters, and exact fast division
           (int64_t)s.C_in * s.H * s.W <= 2147483647LL && (int64_t)64 * s.C_in * RS <= 2147483647LL &&
           64 * span < 65536 && (int64_t)a.CK * a.IH * a.IW < 65536;
    a.prefetch = span % 4 == 0 && ((int64_t)s.C_in * RS) % 4 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 &&
                 (int64_t)a.CK * a.IH * a.IW <= 256 * kXS && 64 * (span / 4) <= 256 * kWS;
    return a;
}

// Dynamic LDS above 64 KB has to be allowed per kernel, once.
template <int CK, int XS>
hipError_t allow_large_lds()
{
    static const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_f32_any_kernel<CK, XS>),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLarge);
    return e;
}

template <int CK>
hipError_t launch_any(const float* x, const float* w, float* y, const Conv2dShape& s, const AnyPlan& a, hipStream_t st,
                      const Epilogue& ep)
{
    AnyParams P;
    P.ep = ep;
    P.C_in = s.C_in; P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.R = s.R; P.S = s.S; P.stride = s.stride;
    P.pad = s.pad; P.Ho = s.Ho; P.Wo = s.Wo;
    P.TH = a.TH; P.TW = a.TW; P.IH = a.IH; P.IW = a.IW; P.tiles_x = a.tiles_x; P.wpitch = a.wpitch; P.dil = s.dil;
    P.by_tiles_x = make_fastdiv(a.tiles_x);
    P.by_TW = make_fastdiv(a.TW);
    P.by_IW = make_fastdiv(a.IW);
    P.by_win = make_fastdiv(a.IH * a.IW);
    P.by_span = make_fastdiv(CK * s.R * s.S);
    P.by_span4 = make_fastdiv(a.prefetch ? CK * s.R * s.S / 4 : 1);
    dim3 grid((unsigned)(a.tiles_x * a.tiles_y), (unsigned)s.N, (unsigned)((s.C_out + 63) / 64));
    const bool large = a.lds > (size_t)kLdsBudget;
    if (a.prefetch && CK * a.IH * a.IW <= 256 * 8) {
        if (large && allow_large_lds<CK, 8>() != hipSuccess) return hipErrorInvalidValue;
        SW_NOTED_LAUNCH(note_kernel("mfma_f32_any_kernel", (int)(CK), (int)(8)), (mfma_f32_any_kernel<CK, 8>), grid, dim3(256), a.lds, st, x, w, y, P);
    } else if (a.prefetch) {
        if (large && allow_large_lds<CK, kXS>() != hipSuccess) return hipErrorInvalidValue;
        SW_NOTED_LAUNCH(note_kernel("mfma_f32_any_kernel", (int)(CK), (int)(kXS)), (mfma_f32_any_kernel<CK, kXS>), grid, dim3(256), a.lds, st, x, w, y, P);
    } else {
        if (large && allow_large_lds<CK, 0>() != hipSuccess) return hipErrorInvalidValue;
        SW_NOTED_LAUNCH(note_kernel("mfma_f32_any_kernel", (int)(CK), (int)(0)), (mfma_f32_any_kernel<CK, 0>), grid, dim3(256), a.lds, st, x, w, y, P);
    }
    return hipGetLastError();
}

}  // namespace

bool mfma_f32_any_supported(const Conv2dShape& s) { return s.C_in >= 2 && plan_any(s, nullptr).ok; }

hipError_t launch_mfma_f32_any(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st,
                               const Epilogue& ep)
{
    const AnyPlan a = plan_any(s, w);
    if (!a.ok) return hipErrorInvalidValue;
    switch (a.CK) {
        case 32: return launch_any<32>(x, w, y, s, a, st, ep);
        case 16: return launch_any<16>(x, w, y, s, a, st, ep);
        case 8: return launch_any<8>(x, w, y, s, a, st, ep);
        case 4: return launch_any<4>(x, w, y, s, a, st, ep);
        default: return launch_any<2>(x, w, y, s, a, st, ep);
    }
}

}  // namespace swconv
