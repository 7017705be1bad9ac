// Multi-channel fp32 sliding window convolution on the matrix cores for ANY filter extent, stride, padding
// and channel count (paper, section 3: the sliding algorithm re-formulated as small matrix products;
// section 2: every filter size on the unmodified input).
//
// The fixed 3x3 / 5x5 kernel of sw_mfma_f32.hip owns a CU with one large tile; this one trades peak rate for
// reach.  A workgroup of four wavefronts computes 64 output channels x up to 128 output pixels (whole output
// rows of one image).  The input channels are walked in chunks of CK: the chunk's input window (tile + halo,
// zero outside the image and beyond C_in: that is the padding) and the chunk's filters are staged in LDS
// once; then every tap (r, s) is one small matrix product per pixel block,
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

constexpr int kTilePx = 128;           // output pixels per workgroup: one 32-pixel block per wavefront
constexpr int kWPitch = 65;            // floats per (tap, channel) row of the staged filters: 64 channels + 1
constexpr int kLdsBudget = 64 * 1024;  // keeps at least two workgroups on a CU
constexpr int kBatch = 8;              // staging loads in flight per thread

struct AnyParams {
    int C_in, C_out, H, W, R, S, stride, pad, Ho, Wo;
    int TH, TW, IH, IW, tiles_x;
    FastDiv by_tiles_x, by_TW, by_IW, by_win, by_RS, by_CKRS;
};

template <int CK>
__global__ __launch_bounds__(256) void mfma_f32_any_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                           float* __restrict__ y, const AnyParams P)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int RS = P.R * P.S;
    const int WP = P.IH * P.IW;                 // window pixels per channel
    float* xs = smem;                           // [CK][WP]
    float* ws = smem + CK * WP;                 // [RS][CK][kWPitch]

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

    for (int ci0 = 0; ci0 < P.C_in; ci0 += CK) {
        // ---- stage the chunk: input window (coalesced along image rows) ...  Loads go out in batches of
        //      kBatch per thread before the first LDS write, so a batch costs one memory round trip.
        for (int base = tid; base < CK * WP; base += 256 * kBatch) {
            float v[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int idx = base + 256 * u;
                const int c = fast_div(idx, P.by_win);
                const int q = idx - c * WP;
                const int e = fast_div(q, P.by_IW), f = q - e * P.IW;
                const int gr = grow0 + e, gc = gcol0 + f;
                v[u] = 0.f;
                if (idx < CK * WP && ci0 + c < P.C_in && gr >= 0 && gr < P.H && gc >= 0 && gc < P.W)
                    v[u] = xn[(int64_t)(ci0 + c) * HW + gr * P.W + gc];
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
                if (base + 256 * u < CK * WP) xs[base + 256 * u] = v[u];
        }
        // ---- ... and filters: for one output channel the chunk's CK * RS floats are contiguous in memory;
        //      they land transposed, [tap][channel][co], with an odd pitch so that neither these writes nor
        //      the operand reads collide on a bank
        const int span = CK * RS;
        const int left = (P.C_in - ci0) * RS;                   // floats that exist from ci0 on
        for (int base = tid; base < 64 * span; base += 256 * kBatch) {
            float v[kBatch];
            int dst[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int idx = base + 256 * u;
                const int co_l = fast_div(idx, P.by_CKRS);
                const int q = idx - co_l * span;
                const int c = fast_div(q, P.by_RS), tap = q - c * RS;
                v[u] = 0.f;
                dst[u] = idx < 64 * span ? (tap * CK + c) * kWPitch + co_l : -1;
                if (dst[u] >= 0 && co0 + co_l < P.C_out && q < left) v[u] = w[(co0 + co_l) * wrow + (int64_t)ci0 * RS + q];
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
                if (dst[u] >= 0) ws[dst[u]] = v[u];
        }
        __syncthreads();

        // ---- every tap is a 64 x CK by CK x 32 product per wavefront; the shift is the offset toff
        if (wave_live) {
            const float* bsrc = xs + kk * WP + pixoff;
            const float* asrc = ws + kk * kWPitch + lj;
            int toff = 0, s = 0;
#pragma unroll 1
            for (int tap = 0; tap < RS; ++tap) {
#pragma unroll
                for (int c2 = 0; c2 < CK / 2; ++c2) {
                    const float b = bsrc[2 * c2 * WP + toff];
                    const float a0 = asrc[(tap * CK + 2 * c2) * kWPitch];
                    const float a1 = asrc[(tap * CK + 2 * c2) * kWPitch + 32];
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b, acc1, 0, 0, 0);
                }
                ++toff;
                if (++s == P.S) { s = 0; toff += P.IW - P.S; }
            }
        }
        __syncthreads();
    }

    // ---- store: register v of a lane is output channel 8*(v/4) + 4*kk + v%4 of the block, pixel lj
    if (!p_ok) return;
    const int HoWo = P.Ho * P.Wo;
    float* yp = y + ((int64_t)n * P.C_out + co0) * HoWo + (row0 + pi) * P.Wo + col0 + pj;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int co = 8 * (v >> 2) + 4 * kk + (v & 3);
        if (co0 + co < P.C_out) yp[(int64_t)co * HoWo] = acc0[v];
        if (co0 + 32 + co < P.C_out) yp[(int64_t)(32 + co) * HoWo] = acc1[v];
    }
}

struct AnyPlan {
    int TH, TW, IH, IW, CK, tiles_x, tiles_y;
    size_t lds;
    bool ok;
};

AnyPlan plan_any(const Conv2dShape& s)
{
    AnyPlan a{};
    const int RS = s.R * s.S;
    a.TW = s.Wo < kTilePx ? s.Wo : kTilePx;
    a.TH = kTilePx / a.TW;
    if (a.TH > s.Ho) a.TH = s.Ho;
    if (a.TH < 1) a.TH = 1;
    // channels per chunk: about a hundred (tap, channel) rows of filters per barrier pair, no more than exist
    a.CK = 32;
    while (a.CK > 2 && (a.CK * RS > 100 || a.CK >= 2 * s.C_in)) a.CK /= 2;
    auto bytes = [&]() {
        a.IH = (a.TH - 1) * s.stride + s.R;
        a.IW = (a.TW - 1) * s.stride + s.S;
        return ((size_t)a.CK * a.IH * a.IW + (size_t)RS * a.CK * kWPitch) * sizeof(float);
    };
    while (bytes() > (size_t)kLdsBudget) {
        if (a.CK > 2) a.CK /= 2;
        else if (a.TH > 1) a.TH = (a.TH + 1) / 2;
        else if (a.TW > 32) a.TW = (a.TW + 1) / 2;
        else break;
    }
    a.lds = bytes();
    a.tiles_x = (s.Wo + a.TW - 1) / a.TW;
    a.tiles_y = (s.Ho + a.TH - 1) / a.TH;
    a.ok = a.lds <= (size_t)kLdsBudget && (int64_t)a.tiles_x * a.tiles_y * a.tiles_x < 2147483647LL && s.N <= 65535 &&
           (s.C_out + 63) / 64 <= 65535 &&
           // 32-bit index arithmetic inside one image / one output channel's filters, and exact fast division
           (int64_t)s.C_in * s.H * s.W <= 2147483647LL && (int64_t)64 * a.CK * RS < 65536 &&
           (int64_t)a.CK * a.IH * a.IW < 65536;
    return a;
}

template <int CK>
hipError_t launch_any(const float* x, const float* w, float* y, const Conv2dShape& s, const AnyPlan& a, hipStream_t st)
{
    AnyParams P;
    P.C_in = s.C_in; P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.R = s.R; P.S = s.S; P.stride = s.stride;
    P.pad = s.pad; P.Ho = s.Ho; P.Wo = s.Wo;
    P.TH = a.TH; P.TW = a.TW; P.IH = a.IH; P.IW = a.IW; P.tiles_x = a.tiles_x;
    P.by_tiles_x = make_fastdiv(a.tiles_x);
    P.by_TW = make_fastdiv(a.TW);
    P.by_IW = make_fastdiv(a.IW);
    P.by_win = make_fastdiv(a.IH * a.IW);
    P.by_RS = make_fastdiv(s.R * s.S);
    P.by_CKRS = make_fastdiv(CK * s.R * s.S);
    dim3 grid((unsigned)(a.tiles_x * a.tiles_y), (unsigned)s.N, (unsigned)((s.C_out + 63) / 64));
    hipLaunchKernelGGL((mfma_f32_any_kernel<CK>), grid, dim3(256), a.lds, st, x, w, y, P);
    return hipGetLastError();
}

}  // namespace

bool mfma_f32_any_supported(const Conv2dShape& s) { return s.C_in >= 2 && plan_any(s).ok; }

hipError_t launch_mfma_f32_any(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st)
{
    const AnyPlan a = plan_any(s);
    if (!a.ok) return hipErrorInvalidValue;
    switch (a.CK) {
        case 32: return launch_any<32>(x, w, y, s, a, st);
        case 16: return launch_any<16>(x, w, y, s, a, st);
        case 8: return launch_any<8>(x, w, y, s, a, st);
        case 4: return launch_any<4>(x, w, y, s, a, st);
        default: return launch_any<2>(x, w, y, s, a, st);
    }
}

}  // namespace swconv
