// Multi-channel fp32 sliding window convolution on the matrix cores for filters of any size, LARGE ones included:
// the compound kernel (paper, section 2: filters wider than one vector are handled as several vectors glued
// together, and the gain of the sliding formulation grows with the filter size; section 3: the taps as small
// matrix products).
//
// A filter of R x S taps over C_in channels is too much to stage at once -- 64 output channels of a 51 x 51
// filter are 666 KB per input channel -- so the reduction is cut into chunks of ONE FILTER ROW of CK input
// channels: chunk (ci0, r) needs the filters w[co][ci0 .. ci0+CK)[r][0 .. S) (64 x CK x S floats) and, per
// input channel, only the input rows that filter row r meets, one per output row of the tile.  Going from r to
// r + 1 the same output tile slides down the input by `dilation` rows: the sliding window sum, one filter row at
// a time.  Inside a chunk every tap column is a 64 x CK by CK x pixels product on v_mfma_f32_32x32x2_f32 whose B
// operand is the window in LDS read at an offset of q * dilation floats: no column matrix, no copy per tap.
// (Whole filters per chunk were tried for small extents: more window rows per chunk, no gain.)
//
// Workgroup = four wavefronts = 64 output channels x a tile of 128 * NBW consecutive output pixels in row-major
// order of one image (so any image width fills the 32-pixel blocks; the window spans the image's width).  Each
// wavefront owns NBW pixel blocks and both 32-channel blocks: 2 * NBW accumulators, every A operand read from
// LDS feeds NBW matrix instructions, every B operand two.  Large tiles are what large filters need: a filter
// float staged in LDS is used by 128 * NBW pixels.  The next chunk travels global memory -> registers (16-byte
// loads) while the current one multiplies out of LDS, so a workgroup overlaps its own staging, and two
// workgroups share a CU on top of that.
//
// Any stride, padding and dilation; C_in and C_out need not be multiples of anything (zero-filled); image rows
// must be whole 16-byte groups (W a multiple of 4, x 16-byte aligned).
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
// a 16-byte load from an address that is only 4-byte aligned (filter rows start anywhere)
typedef float floatx4u __attribute__((ext_vector_type(4), aligned(4)));

constexpr int kLdsHalf = 79 * 1024;    // two workgroups per CU
constexpr int kLdsWhole = 156 * 1024;  // one

// 16-byte groups of the window a thread carries from one chunk's multiplication to the next; those of the filters
// are a template argument (XF): a slot costs instructions in every chunk whether an item lives in it or not, so
// every chunk size comes in variants for short and long filter rows
constexpr int slots_window(int ck) { return ck == 16 ? 6 : ck == 8 ? 4 : 3; }
struct RowsVariant {
    int ck, xf;
};
constexpr RowsVariant kVariants[] = {{16, 4}, {16, 8}, {8, 6}, {8, 8}, {8, 10}, {4, 9}, {4, 11}, {4, 13}, {2, 10}};   // by preference

struct RowsParams {
    Epilogue ep;                       // bias and rectifier applied in the store
    int C_in, C_out, H, W, R, S, stride, pad, dil, Ho, Wo;
    int IH, IW, WP, wpitch;            // window rows / columns, floats per channel in LDS, floats per filter row in LDS
    FastDiv by_Wo, by_W4, by_IH, by_G;
};

template <int CK, int NBW, int XF>
__global__ __launch_bounds__(256, NBW <= 2 ? 2 : 1) void mfma_f32_rows_kernel(const float* __restrict__ x,
                                                                        const float* __restrict__ w,
                                                                        float* __restrict__ y, const RowsParams P)
{
    constexpr int XW = slots_window(CK);
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* xs = smem;                           // [CK][WP]: the window rows of this chunk's filter rows, whole image width
    float* ws = smem + CK * P.WP;               // [64][wpitch]: (channel of the chunk, tap of the chunk) per output channel

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lj = lane & 31, kk = lane >> 5;   // row/column inside a 32 x 32 block, K half
    const int n = blockIdx.y, co0 = blockIdx.z * 64;
    const int HoWo = P.Ho * P.Wo, HW = P.H * P.W, RS = P.R * P.S, S = P.S, T = P.S;
    const int p0 = blockIdx.x * (128 * NBW);            // first output pixel of the tile
    const int row0 = fast_div(p0, P.by_Wo);             // its output row

    // this lane's pixel in each of the wavefront's blocks, and where its window starts in a channel's LDS rows
    int pix[NBW], pixoff[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j) {
        const int p = p0 + (wave * NBW + j) * 32 + lj;
        const int pc = p < HoWo ? p : p0;
        const int pi = fast_div(pc, P.by_Wo), pj = pc - pi * P.Wo;
        pix[j] = p < HoWo ? p : -1;
        pixoff[j] = (pi - row0) * P.IW + pj * P.stride;
    }
    const bool wave_live = __builtin_amdgcn_readfirstlane(p0 + wave * NBW * 32) < HoWo;

    floatx16 acc[2][NBW];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < NBW; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[h][j][v] = 0.f;

    const float* xn = x + (int64_t)n * P.C_in * HW;
    const int64_t wrow = (int64_t)P.C_in * RS;                  // floats per output channel in w
    const float* wb = w + (int64_t)co0 * wrow;

    // ---- staging plan, the same for every chunk.  Window: item = group col4 of four floats of window row (c, e),
    //      i.e. of image row grow + e * stride of channel ci0 + c; it lands pad floats into LDS row (c, e).  The
    //      padding columns are zeroed once; rows above or below the image and channels beyond C_in are written
    //      as zeros chunk by chunk.
    const int W4 = P.W >> 2;
    int xpk[XW];                    // (c, e, col4) in 4 + 14 + 12 bits, < 0: no such item
#pragma unroll
    for (int u = 0; u < XW; ++u) {
        const int idx = tid + 256 * u;
        const int row = fast_div(idx, P.by_W4), col4 = idx - row * W4;
        const int c = fast_div(row, P.by_IH), e = row - c * P.IH;
        xpk[u] = idx < CK * P.IH * W4 ? (c << 26) | (e << 12) | col4 : -1;
    }
    // Filters: item = 16-byte group g of the T floats of (output channel co_l, channel c); the last group of a row
    // starts at T - 4 (it overlaps its neighbour instead of running past the row).  T < 4: one item per row.
    const int G = T >= 4 ? (T + 3) >> 2 : 1;
    int wpk[XF];                    // (co_l, c, q0) in 6 + 4 + 12 bits, < 0: no such item
#pragma unroll
    for (int u = 0; u < XF; ++u) {
        const int idx = tid + 256 * u;
        const int rowid = fast_div(idx, P.by_G), g = idx - rowid * G;
        const int co_l = rowid / CK, c = rowid - co_l * CK;
        const int q0 = T >= 4 ? min(4 * g, T - 4) : 0;
        wpk[u] = idx < 64 * CK * G ? (co_l << 16) | (c << 12) | q0 : -1;
    }
    for (int i = tid; i < CK * P.WP; i += 256) xs[i] = 0.f;
    __syncthreads();

    float xv[XW][4], wv[XF][4];
    auto fetch = [&](int ci0, int r0) __attribute__((always_inline)) {
        const int grow = row0 * P.stride - P.pad + r0 * P.dil;
        const float* xc = xn + (int64_t)ci0 * HW + (int64_t)grow * P.W;
        // (no branch around a load: a clamped address, then a select)
#pragma unroll
        for (int u = 0; u < XW; ++u) {
            const int c = xpk[u] >> 26, e = (xpk[u] >> 12) & 0x3fff, col4 = xpk[u] & 0xfff;
            const int gr = grow + e * P.stride;
            const bool ok = xpk[u] >= 0 && ci0 + c < P.C_in && gr >= 0 && gr < P.H;
            const floatx4 v = *reinterpret_cast<const floatx4*>(ok ? xc + (c * HW + e * P.stride * P.W + 4 * col4) : xn);
            xv[u][0] = ok ? v.x : 0.f; xv[u][1] = ok ? v.y : 0.f; xv[u][2] = ok ? v.z : 0.f; xv[u][3] = ok ? v.w : 0.f;
        }
        const float* wc = wb + (int64_t)ci0 * RS + r0 * S;
        if (T >= 4) {
#pragma unroll
            for (int u = 0; u < XF; ++u) {
                const int co_l = wpk[u] >> 16, c = (wpk[u] >> 12) & 15, q0 = wpk[u] & 0xfff;
                const bool ok = wpk[u] >= 0 && co0 + co_l < P.C_out && ci0 + c < P.C_in;
                const floatx4u v = *reinterpret_cast<const floatx4u*>(ok ? wc + (co_l * (int)wrow + c * RS + q0) : wb);
                wv[u][0] = ok ? v.x : 0.f; wv[u][1] = ok ? v.y : 0.f; wv[u][2] = ok ? v.z : 0.f; wv[u][3] = ok ? v.w : 0.f;
            }
        } else {
#pragma unroll
            for (int u = 0; u < XF; ++u) {
                const int co_l = wpk[u] >> 16, c = (wpk[u] >> 12) & 15;
                const bool ok = wpk[u] >= 0 && co0 + co_l < P.C_out && ci0 + c < P.C_in;
                const float* src = ok ? wc + (co_l * (int)wrow + c * RS) : wb;
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const float v = src[i < T ? i : 0];
                    wv[u][i] = ok ? v : 0.f;
                }
                wv[u][3] = 0.f;
            }
        }
    };
    auto stage = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < XW; ++u)
            if (xpk[u] >= 0) {
                const int c = xpk[u] >> 26, e = (xpk[u] >> 12) & 0x3fff, col4 = xpk[u] & 0xfff;
                float* d = xs + c * P.WP + e * P.IW + P.pad + 4 * col4;
#pragma unroll
                for (int i = 0; i < 4; ++i) d[i] = xv[u][i];
            }
#pragma unroll
        for (int u = 0; u < XF; ++u)
            if (wpk[u] >= 0) {
                const int co_l = wpk[u] >> 16, c = (wpk[u] >> 12) & 15, q0 = wpk[u] & 0xfff;
                float* d = ws + co_l * P.wpitch + c * T + q0;
                if (T >= 4) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) d[i] = wv[u][i];
                } else {
#pragma unroll
                    for (int i = 0; i < 3; ++i)
                        if (i < T) d[i] = wv[u][i];
                }
            }
    };

    // chunk = (channel chunk ci0, filter row r0); the next chunk travels global memory -> registers while this
    // one multiplies out of LDS
    const int chunks = ((P.C_in + CK - 1) / CK) * P.R;
    fetch(0, 0);
    int ci0 = 0, r0 = 0;
    for (int ch = 0; ch < chunks; ++ch) {
        stage();
        __syncthreads();
        if (++r0 == P.R) { r0 = 0; ci0 += CK; }
        if (ch + 1 < chunks) fetch(ci0, r0);
        // ---- every tap of the chunk: 64 x CK by CK x (32 * NBW) per wavefront, the shift is toff
        if (wave_live) {
            const float* bsrc = xs + kk * P.WP;
            const float* asrc = ws + lj * P.wpitch + kk * T;
            int toff = 0;
#pragma unroll 1
            for (int q = 0; q < S; ++q) {
#pragma unroll
                for (int c2 = 0; c2 < CK / 2; ++c2) {
                    const float a0 = asrc[2 * c2 * S + q];
                    const float a1 = asrc[32 * P.wpitch + 2 * c2 * S + q];
#pragma unroll
                    for (int j = 0; j < NBW; ++j) {
                        const float b = bsrc[2 * c2 * P.WP + pixoff[j] + toff];
                        acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b, acc[0][j], 0, 0, 0);
                        acc[1][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b, acc[1][j], 0, 0, 0);
                    }
                }
                toff += P.dil;
            }
        }
        __syncthreads();
    }

    // ---- store: register v of a lane is output channel 8 * (v / 4) + 4 * kk + v % 4 of the block, pixel lj
    float* yn = y + ((int64_t)n * P.C_out + co0) * HoWo;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        float bias[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int co = co0 + 32 * h + 8 * (v >> 2) + 4 * kk + (v & 3);
            bias[v] = (P.ep.bias && co < P.C_out) ? P.ep.bias[co] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
            if (pix[j] < 0) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int co = 32 * h + 8 * (v >> 2) + 4 * kk + (v & 3);
                float t = acc[h][j][v];
                if (P.ep.bias) t += bias[v];
                if (P.ep.relu) t = fmaxf(t, 0.f);
                if (co0 + co < P.C_out) yn[(int64_t)co * HoWo + pix[j]] = t;
            }
        }
    }
}

struct RowsPlan {
    int CK, XF, NBW, IH, IW, WP, wpitch, tiles;
    size_t lds;
    bool ok;
};

RowsPlan plan_rows(const Conv2dShape& s, const float* x)
{
    RowsPlan a{};
    const int64_t HoWo = (int64_t)s.Ho * s.Wo;
    if (s.C_in < 2 || HoWo > (1 << 24) || s.N > 65535 || (s.C_out + 63) / 64 > 65535 || s.W >= 16384 || s.S >= 4096) return a;
    // the window is fetched in 16-byte groups of image rows
    if (s.W % 4 != 0 || reinterpret_cast<uintptr_t>(x) % 16 != 0) return a;
    // 32-bit index arithmetic and exact fast division
    if ((int64_t)s.C_in * s.H * s.W > 2147483647LL || (int64_t)64 * s.C_in * s.R * s.S > 2147483647LL ||
        HoWo * s.Wo >= (1LL << 32))
        return a;
    // tiles of 512 pixels when that still gives every CU two workgroups, else 256
    const int64_t wg512 = ((HoWo + 511) / 512) * s.N * ((s.C_out + 63) / 64);
    a.NBW = wg512 >= 512 ? 4 : 2;
    const int tile = 128 * a.NBW;
    a.tiles = (int)((HoWo + tile - 1) / tile);
    a.IH = (tile + s.Wo - 2) / s.Wo + 1;                 // output rows a tile of `tile` consecutive pixels can touch
    if (a.IH > s.Ho) a.IH = s.Ho;
    // columns the taps reach, and at least the whole image row behind the left padding (rows are staged whole)
    int64_t IW = (int64_t)(s.Wo - 1) * s.stride + (int64_t)(s.S - 1) * s.dil + 1;
    if (IW < (int64_t)s.W + s.pad) IW = (int64_t)s.W + s.pad;
    if (IW > 4096 || a.IH >= 16384) return a;
    a.IW = (int)IW;
    // the two K halves of a B operand read (channels 2 c2 and 2 c2 + 1) should fall into different banks:
    // channel pitch = 32 (mod 64) floats at stride 1, odd otherwise
    const int win = a.IH * a.IW;
    a.WP = s.stride == 1 ? ((win + 31) / 64) * 64 + 32 : (win | 1);
    const int G = s.S >= 4 ? (s.S + 3) / 4 : 1;
    int ck_max = 16;                                       // no more channels per chunk than exist (in steps of 2x)
    while (ck_max > 2 && ck_max >= 2 * s.C_in) ck_max /= 2;
    // measured: per-chunk costs favour many channels for short filter rows, few for long ones
    if (s.S > 20 && ck_max > 4) ck_max = 4;
    else if (s.S > 8 && ck_max > 8) ck_max = 8;
    for (int pass = 0; pass < 2 && !a.ok; ++pass) {        // two workgroups per CU if the chunk allows it, else one
        const size_t budget = pass == 0 ? kLdsHalf : kLdsWhole;
        for (const RowsVariant& v : kVariants) {
            if (a.ok || v.ck > ck_max) continue;
            a.CK = v.ck;
            a.XF = v.xf;
            a.wpitch = (v.ck * s.S) | 1;                   // odd: the 32 rows an operand read touches fall into 32 banks
            a.lds = ((size_t)v.ck * a.WP + (size_t)64 * a.wpitch) * sizeof(float);
            // ... and what a thread carries in registers from one chunk to the next
            a.ok = a.lds <= budget && (int64_t)v.ck * a.IH * (s.W / 4) <= 256 * slots_window(v.ck) &&
                   64 * v.ck * G <= 256 * v.xf;
        }
    }
    // never more than two workgroups on a CU (a third would come out of some other CU's share: 416 tiles on 256 CUs)
    if (a.ok && a.lds < (size_t)55 * 1024) a.lds = (size_t)55 * 1024;
    return a;
}

template <int CK, int NBW, int XF>
hipError_t launch_rows(const float* x, const float* w, float* y, const Conv2dShape& s, const RowsPlan& a, hipStream_t st,
                       const Epilogue& ep)
{
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_f32_rows_kernel<CK, NBW, XF>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsWhole);
    if (attr != hipSuccess) return attr;
    RowsParams P;
    P.ep = ep;
    P.C_in = s.C_in; P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.R = s.R; P.S = s.S; P.stride = s.stride;
    P.pad = s.pad; P.dil = s.dil; P.Ho = s.Ho; P.Wo = s.Wo;
    P.IH = a.IH; P.IW = a.IW; P.WP = a.WP; P.wpitch = a.wpitch;
    P.by_Wo = make_fastdiv(s.Wo);
    P.by_W4 = make_fastdiv(s.W / 4);
    P.by_IH = make_fastdiv(a.IH);
    P.by_G = make_fastdiv(s.S >= 4 ? (s.S + 3) / 4 : 1);
    dim3 grid((unsigned)a.tiles, (unsigned)s.N, (unsigned)((s.C_out + 63) / 64));
    SW_NOTED_LAUNCH(note_kernel("mfma_f32_rows_kernel", CK, NBW, XF), (mfma_f32_rows_kernel<CK, NBW, XF>), grid, dim3(256), a.lds,
                    st, x, w, y, P);
    return hipGetLastError();
}

}  // namespace

bool mfma_f32_rows_supported(const Conv2dShape& s, const float* x) { return plan_rows(s, x).ok; }

hipError_t launch_mfma_f32_rows(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st,
                                const Epilogue& ep)
{
    const RowsPlan a = plan_rows(s, x);
    if (!a.ok) return hipErrorInvalidValue;
#define SW_ROWS(CKC, XFC)                                                                   \
    do {                                                                                    \
        if (a.CK == CKC && a.XF == XFC) {                                                   \
            if (a.NBW == 4) return launch_rows<CKC, 4, XFC>(x, w, y, s, a, st, ep);         \
            return launch_rows<CKC, 2, XFC>(x, w, y, s, a, st, ep);                         \
        }                                                                                   \
    } while (0)
    SW_ROWS(16, 4); SW_ROWS(16, 8); SW_ROWS(8, 6); SW_ROWS(8, 8); SW_ROWS(8, 10); SW_ROWS(4, 9); SW_ROWS(4, 11);
    SW_ROWS(4, 13); SW_ROWS(2, 10);
    return hipErrorInvalidValue;
#undef SW_ROWS
}

}  // namespace swconv
