// Quantised (int8 -> exact int32) sliding window convolution on the matrix cores for any filter extent,
// stride, padding and channel count (paper, sections 1.1 and 3: quantisation carries over to the sliding
// formulation; every tap is a small matrix product on shifted data).
//
// The resident-K 3x3 kernel of sw_mfma_s8.hip owns a CU with one tile; this one reaches every other shape.
// A workgroup of four wavefronts computes 64 output channels x up to 128 output pixels (whole output rows
// of one image).  Input channels are walked in chunks of CK (32 or 64).  v_mfma_i32_32x32x32_i8 wants 16
// consecutive K bytes per lane while NCHW / OIHW keep the channels of a pixel (of a tap) a plane (a filter)
// apart.  Staging therefore gathers four channels of a pixel with byte loads (coalesced along the image row),
// packs them into a dword and writes [pixel][channel] rows into LDS -- zero outside the image and beyond C_in
// (the padding); the chunk's filters are first copied as they lie in memory (one contiguous run per output
// channel, dword loads) into an LDS staging area and regrouped from there into [tap][co][channel] rows.
// Every tap is then CK / 32 matrix instructions per 32 x 32 block, the shift being an LDS address offset of
// the B operand.  No column matrix exists anywhere.
#include "swconv_internal.h"
#include "sw_s8_perm.h"

#include <cstdlib>

namespace swconv {

namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32;

constexpr int kTilePx = 128;            // output pixels per workgroup: one 32-pixel block per wavefront
constexpr int kLdsTwo = 80 * 1024;      // two workgroups per CU up to here
constexpr int kLdsBudget = 156 * 1024;  // one workgroup per CU up to here

struct S8AnyParams {
    int C_in, C_out, H, W, R, S, stride, pad, Ho, Wo;
    int TH, TW, IH, IW, tiles_x, rawpitch, w_dwords;
    int x_dwords, nq;                  // input rows are read as aligned dwords (four pixels); quads per window row
    FastDiv by_tiles_x, by_TW, by_IW, by_win, by_RS, by_span, by_span4, by_nq, by_rowq;
};

// RQ: the sums leave requantised to int8 (y8) instead of as int32 (y).
template <int CK, bool RQ>
__global__ __launch_bounds__(256) void mfma_s8_any_kernel(const int8_t* __restrict__ x, const int8_t* __restrict__ w,
                                                          int32_t* __restrict__ y, const S8AnyParams P,
                                                          int8_t* __restrict__ y8, const Requant rq)
{
    constexpr int kPitch = CK + 16;             // bytes per pixel row / filter row in LDS (16-byte aligned reads)
    constexpr int G = CK / 4;                   // dwords (groups of four channels) per row
    extern __shared__ __attribute__((aligned(16))) unsigned char smem8[];
    const int RS = P.R * P.S;
    const int WP = P.IH * P.IW;                 // window pixels
    unsigned char* xs = smem8;                  // [WP][kPitch]
    unsigned char* ws = smem8 + WP * kPitch;    // [RS][64][kPitch]
    unsigned char* raw = ws + RS * 64 * kPitch; // [64][P.rawpitch]: the chunk's filters as in memory
    const int span = CK * RS;                   // filter bytes per output channel and chunk

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lj = lane & 31, kg = lane >> 5;   // row/column inside a 32 x 32 block, 16-byte half of a K step

    const int ty = fast_div(blockIdx.x, P.by_tiles_x);
    const int tx = blockIdx.x - ty * P.tiles_x;
    const int n = blockIdx.y;
    const int co0 = blockIdx.z * 64;
    const int row0 = ty * P.TH, col0 = tx * P.TW;
    const int grow0 = row0 * P.stride - P.pad, gcol0 = col0 * P.stride - P.pad;

    const int tile_px = P.TH * P.TW;
    const int p = wave * 32 + lj;
    const int pi = fast_div(p, P.by_TW), pj = p - pi * P.TW;
    const bool p_ok = p < tile_px && row0 + pi < P.Ho && col0 + pj < P.Wo;
    const int pixoff = p_ok ? (pi * P.stride) * P.IW + pj * P.stride : 0;
    const bool wave_live = __builtin_amdgcn_readfirstlane(wave * 32) < tile_px;

    intx16 acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc0[v] = 0; acc1[v] = 0; }

    const int HW = P.H * P.W;
    const int8_t* xn = x + (int64_t)n * P.C_in * HW;
    const int64_t wrow = (int64_t)P.C_in * RS;                  // bytes per output channel in w
    const int8_t* wb = w + (int64_t)co0 * wrow;

    for (int ci0 = 0; ci0 < P.C_in; ci0 += CK) {
        if (P.x_dwords) {
            // ---- input window, rows whose quads of four pixels are aligned dwords (W a multiple of 4): slot =
            //      (group of four channels, window row, quad); four dword loads (one per channel, coalesced along
            //      the image row), a 4 x 4 byte transpose in registers, one dword per pixel into LDS.  A quarter of
            //      the load instructions of the byte path below.
            const int q0 = gcol0 >> 2;                         // first quad that touches the window (floor)
            const int rowq = P.IH * P.nq;
            for (int base = tid; base < G * rowq; base += 256 * 2) {
                u32 r[2][4];
                int e2[2], f2[2], g2[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {                  // the loads of two slots go out together
                    const int idx = base + 256 * u;
                    const int g = fast_div(idx, P.by_rowq);
                    const int t = idx - g * rowq;
                    const int e = fast_div(t, P.by_nq), qd = t - e * P.nq;
                    const int gr = grow0 + e, gc = 4 * (q0 + qd);  // image row, image column of the quad's first pixel
                    r[u][0] = r[u][1] = r[u][2] = r[u][3] = 0u;
                    if (idx < G * rowq && gr >= 0 && gr < P.H && gc >= 0 && gc < P.W) {
                        const int8_t* src = xn + (int64_t)(ci0 + 4 * g) * HW + gr * P.W + gc;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (ci0 + 4 * g + j < P.C_in) r[u][j] = *reinterpret_cast<const u32*>(src + (int64_t)j * HW);
                    }
                    e2[u] = idx < G * rowq ? e : -1;
                    f2[u] = gc - gcol0;                        // window column of the quad's first pixel
                    g2[u] = g;
                }
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    if (e2[u] < 0) continue;
#pragma unroll
                    for (int px = 0; px < 4; ++px) {
                        // byte px of the four channel dwords -> one dword: channels 4g .. 4g+3 of this pixel
                        const u32 t01 = __builtin_amdgcn_perm(r[u][1], r[u][0], (u32)px | ((u32)(4 + px) << 8));
                        const u32 t23 = __builtin_amdgcn_perm(r[u][3], r[u][2], (u32)px | ((u32)(4 + px) << 8));
                        const u32 packed = __builtin_amdgcn_perm(t23, t01, 0x05040100u);
                        const int f = f2[u] + px;
                        if (f >= 0 && f < P.IW)
                            *reinterpret_cast<u32*>(xs + (e2[u] * P.IW + f) * kPitch + 4 * g2[u]) = packed;
                    }
                }
            }
        } else {
        // ---- input window, any alignment: slot = (group of four channels, window pixel); consecutive lanes take
        //      consecutive pixels, so each of the four byte loads is coalesced along the image row
        for (int idx = tid; idx < G * WP; idx += 256) {
            const int g = fast_div(idx, P.by_win);
            const int q = idx - g * WP;
            const int e = fast_div(q, P.by_IW), f = q - e * P.IW;
            const int gr = grow0 + e, gc = gcol0 + f;
            u32 packed = 0;
            if (gr >= 0 && gr < P.H && gc >= 0 && gc < P.W) {
                const int8_t* src = xn + (int64_t)(ci0 + 4 * g) * HW + gr * P.W + gc;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (ci0 + 4 * g + j < P.C_in) packed |= (u32)(unsigned char)src[(int64_t)j * HW] << (8 * j);
            }
            *reinterpret_cast<u32*>(xs + q * kPitch + 4 * g) = packed;
        }
        }
        if (RS == 1 && P.w_dwords) {
            // ---- 1 x 1 filters: four consecutive input channels of an output channel are one aligned dword of w
            //      and one dword of the operand row: copied straight into place, no staging area, no regrouping
            const int left1 = P.C_in - ci0;
            for (int idx = tid; idx < 64 * G; idx += 256) {
                const int co_l = idx / G, g = idx - co_l * G;     // G is a power of two
                u32 v = 0;
                if (co0 + co_l < P.C_out && 4 * g < left1)
                    v = *reinterpret_cast<const u32*>(wb + co_l * wrow + ci0 + 4 * g);
                *reinterpret_cast<u32*>(ws + co_l * kPitch + 4 * g) = v;
            }
            __syncthreads();
        } else {
        // ---- filters, first as they lie in memory: row co_l of the staging area is bytes ci0*RS .. +span of
        //      that output channel's filter (zero beyond C_in and C_out)
        const int left = (P.C_in - ci0) * RS;                 // bytes that exist from ci0 on
        if (P.w_dwords) {
            const int span4 = span >> 2;
            // (eight loads per thread go out before the first LDS write: one memory round trip per batch)
            for (int base = tid; base < 64 * span4; base += 256 * 8) {
                u32 v8[8];
                int dst8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int idx = base + 256 * u;
                    const int co_l = fast_div(idx, P.by_span4);
                    const int q = 4 * (idx - co_l * span4);
                    v8[u] = 0;
                    dst8[u] = idx < 64 * span4 ? co_l * P.rawpitch + q : -1;
                    if (idx < 64 * span4 && co0 + co_l < P.C_out && q < left)   // (row length and span are multiples of 4)
                        v8[u] = *reinterpret_cast<const u32*>(wb + co_l * wrow + (int64_t)ci0 * RS + q);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (dst8[u] >= 0) *reinterpret_cast<u32*>(raw + dst8[u]) = v8[u];
            }
        } else {
            for (int idx = tid; idx < 64 * span; idx += 256) {
                const int co_l = fast_div(idx, P.by_span);
                const int q = idx - co_l * span;
                raw[co_l * P.rawpitch + q] =
                    (co0 + co_l < P.C_out && q < left) ? (unsigned char)wb[co_l * wrow + (int64_t)ci0 * RS + q] : 0;
            }
        }
        __syncthreads();
        // ---- ... then regrouped.  3 x 3 filters: a thread takes the 144 contiguous bytes of (output channel, 16 input
        //      channels) as 36 dwords and permutes them in registers into nine 16-byte operand pieces, one per tap
        if (RS == 9 && P.w_dwords) {
            for (int idx = tid; idx < 64 * (CK / 16); idx += 256) {
                const int co_l = idx / (CK / 16), c16 = idx - co_l * (CK / 16);
                const u32* src = reinterpret_cast<const u32*>(raw + co_l * P.rawpitch + c16 * 144);
                u32 r36[36];
#pragma unroll
                for (int i = 0; i < 36; ++i) r36[i] = src[i];
                unsigned char* dst = ws + co_l * kPitch + 16 * c16;
                *reinterpret_cast<intx4*>(dst + 0 * 64 * kPitch) = s8perm::wgather_tap<0>(r36);
                *reinterpret_cast<intx4*>(dst + 1 * 64 * kPitch) = s8perm::wgather_tap<1>(r36);
                *reinterpret_cast<intx4*>(dst + 2 * 64 * kPitch) = s8perm::wgather_tap<2>(r36);
                *reinterpret_cast<intx4*>(dst + 3 * 64 * kPitch) = s8perm::wgather_tap<3>(r36);
                *reinterpret_cast<intx4*>(dst + 4 * 64 * kPitch) = s8perm::wgather_tap<4>(r36);
                *reinterpret_cast<intx4*>(dst + 5 * 64 * kPitch) = s8perm::wgather_tap<5>(r36);
                *reinterpret_cast<intx4*>(dst + 6 * 64 * kPitch) = s8perm::wgather_tap<6>(r36);
                *reinterpret_cast<intx4*>(dst + 7 * 64 * kPitch) = s8perm::wgather_tap<7>(r36);
                *reinterpret_cast<intx4*>(dst + 8 * 64 * kPitch) = s8perm::wgather_tap<8>(r36);
            }
        } else
        // any other extent: slot = (output channel, group of four input channels, tap)
        for (int idx = tid; idx < 64 * G * RS; idx += 256) {
            const int cg = fast_div(idx, P.by_RS);            // co_l * G + g
            const int tap = idx - cg * RS;
            const int co_l = cg / G, g = cg - co_l * G;       // G is a power of two
            const unsigned char* src = raw + co_l * P.rawpitch + 4 * g * RS + tap;
            const u32 packed = (u32)src[0] | (u32)src[RS] << 8 | (u32)src[2 * RS] << 16 | (u32)src[3 * RS] << 24;
            *reinterpret_cast<u32*>(ws + (tap * 64 + co_l) * kPitch + 4 * g) = packed;
        }
        __syncthreads();

        }
        if (wave_live) {
            const unsigned char* bsrc = xs + pixoff * kPitch + 16 * kg;
            const unsigned char* asrc = ws + lj * kPitch + 16 * kg;
            int toff = 0, s = 0;
#pragma unroll 1
            for (int tap = 0; tap < RS; ++tap) {
#pragma unroll
                for (int ks = 0; ks < CK / 32; ++ks) {
                    const intx4 b = *reinterpret_cast<const intx4*>(bsrc + toff * kPitch + 32 * ks);
                    const intx4 a0 = *reinterpret_cast<const intx4*>(asrc + tap * 64 * kPitch + 32 * ks);
                    const intx4 a1 = *reinterpret_cast<const intx4*>(asrc + (tap * 64 + 32) * kPitch + 32 * ks);
                    acc0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b, acc1, 0, 0, 0);
                }
                ++toff;
                if (++s == P.S) { s = 0; toff += P.IW - P.S; }
            }
        }
        __syncthreads();
    }

    // ---- store: register v of a lane is output channel 8*(v/4) + 4*kg + v%4 of the block, pixel lj
    if (!p_ok) return;
    const int HoWo = P.Ho * P.Wo;
    const int64_t o = ((int64_t)n * P.C_out + co0) * HoWo + (row0 + pi) * P.Wo + col0 + pj;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int co = 8 * (v >> 2) + 4 * kg + (v & 3);
        if constexpr (RQ) {
            if (co0 + co < P.C_out) y8[o + (int64_t)co * HoWo] = requant_s8(acc0[v], co0 + co, rq);
            if (co0 + 32 + co < P.C_out) y8[o + (int64_t)(32 + co) * HoWo] = requant_s8(acc1[v], co0 + 32 + co, rq);
        } else {
            if (co0 + co < P.C_out) y[o + (int64_t)co * HoWo] = acc0[v];
            if (co0 + 32 + co < P.C_out) y[o + (int64_t)(32 + co) * HoWo] = acc1[v];
        }
    }
}

struct S8AnyPlan {
    int TH, TW, IH, IW, CK, tiles_x, tiles_y, rawpitch;
    size_t lds;
    bool ok;
};

S8AnyPlan plan_s8_any(const Conv2dShape& s)
{
    S8AnyPlan a{};
    const int RS = s.R * s.S;
    a.TW = s.Wo < kTilePx ? s.Wo : kTilePx;
    a.TH = kTilePx / a.TW;
    if (a.TH > s.Ho) a.TH = s.Ho;
    if (a.TH < 1) a.TH = 1;
    a.CK = s.C_in > 32 ? 64 : 32;
    auto bytes = [&]() {
        a.IH = (a.TH - 1) * s.stride + s.R;
        a.IW = (a.TW - 1) * s.stride + s.S;
        a.rawpitch = ((a.CK * RS + 3) & ~3) + 4;       // dword aligned rows, off the power-of-two strides
        return ((size_t)a.IH * a.IW + (size_t)RS * 64) * (a.CK + 16) + (size_t)64 * a.rawpitch;
    };
    if (bytes() > (size_t)kLdsTwo) a.CK = 32;            // prefer two workgroups per CU
    while (bytes() > (size_t)kLdsBudget) {
        if (a.CK > 32) a.CK = 32;
        else if (a.TH > 1) a.TH = (a.TH + 1) / 2;
        else if (a.TW > 32) a.TW = (a.TW + 1) / 2;
        else break;
    }
    a.lds = bytes();
    a.tiles_x = (s.Wo + a.TW - 1) / a.TW;
    a.tiles_y = (s.Ho + a.TH - 1) / a.TH;
    a.ok = a.lds <= (size_t)kLdsBudget && (int64_t)a.tiles_x * a.tiles_y * a.tiles_x < 2147483647LL && s.N <= 65535 &&
           (s.C_out + 63) / 64 <= 65535 &&
           // 32-bit index arithmetic inside one image / 64 output channels' filters, and exact fast division
           (int64_t)s.C_in * s.H * s.W <= 2147483647LL && (int64_t)64 * s.C_in * RS <= 2147483647LL &&
           (int64_t)64 * a.CK * RS < 65536 && (int64_t)(a.CK / 4) * a.IH * a.IW < 65536;
    return a;
}

template <int CK, bool RQ>
hipError_t launch_s8_any(const int8_t* x, const int8_t* w, int32_t* y, const Conv2dShape& s, const S8AnyPlan& a,
                         hipStream_t st, int8_t* y8, const Requant& rq)
{
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_s8_any_kernel<CK, RQ>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget);
    if (attr != hipSuccess) return attr;
    S8AnyParams P;
    P.C_in = s.C_in; P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.R = s.R; P.S = s.S; P.stride = s.stride;
    P.pad = s.pad; P.Ho = s.Ho; P.Wo = s.Wo;
    P.TH = a.TH; P.TW = a.TW; P.IH = a.IH; P.IW = a.IW; P.tiles_x = a.tiles_x; P.rawpitch = a.rawpitch;
    // dword copies of the filter rows need every row and every chunk to start on a 4-byte boundary
    const int span = CK * s.R * s.S;
    P.w_dwords = span % 4 == 0 && ((int64_t)s.C_in * s.R * s.S) % 4 == 0 && reinterpret_cast<uintptr_t>(w) % 4 == 0;
    P.by_tiles_x = make_fastdiv(a.tiles_x);
    P.by_TW = make_fastdiv(a.TW);
    P.by_IW = make_fastdiv(a.IW);
    P.by_win = make_fastdiv(a.IH * a.IW);
    P.by_RS = make_fastdiv(s.R * s.S);
    P.by_span = make_fastdiv(span);
    P.by_span4 = make_fastdiv(P.w_dwords ? span / 4 : 1);
    // aligned dword reads of the input rows: every row of every plane starts on a 4-byte boundary
    P.x_dwords = s.W % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 4 == 0;
    P.nq = (a.IW + 3) / 4 + 1;                  // quads that can touch a window row, whatever its alignment
    P.by_nq = make_fastdiv(P.nq);
    P.by_rowq = make_fastdiv(a.IH * P.nq);
    dim3 grid((unsigned)(a.tiles_x * a.tiles_y), (unsigned)s.N, (unsigned)((s.C_out + 63) / 64));
    SW_NOTED_LAUNCH(note_kernel("mfma_s8_any_kernel", (int)(CK), (int)(RQ)), (mfma_s8_any_kernel<CK, RQ>), grid, dim3(256), a.lds, st, x, w, y, P, y8, rq);
    return hipGetLastError();
}

}  // namespace

bool mfma_s8_any_supported(const Conv2dShape& s) { return plan_s8_any(s).ok; }

hipError_t launch_mfma_s8_any(const int8_t* x, const int8_t* w, int32_t* y, const Conv2dShape& s, hipStream_t st)
{
    const S8AnyPlan a = plan_s8_any(s);
    if (!a.ok) return hipErrorInvalidValue;
    const Requant none{nullptr, nullptr, 0};
    if (a.CK == 64) return launch_s8_any<64, false>(x, w, y, s, a, st, nullptr, none);
    return launch_s8_any<32, false>(x, w, y, s, a, st, nullptr, none);
}

hipError_t launch_mfma_s8_any_requant(const int8_t* x, const int8_t* w, int8_t* y8, const Requant& rq,
                                      const Conv2dShape& s, hipStream_t st)
{
    const S8AnyPlan a = plan_s8_any(s);
    if (!a.ok) return hipErrorInvalidValue;
    if (a.CK == 64) return launch_s8_any<64, true>(x, w, nullptr, s, a, st, y8, rq);
    return launch_s8_any<32, true>(x, w, nullptr, s, a, st, y8, rq);
}

}  // namespace swconv
