// A depthwise-separable block in one launch (paper, section 1.2: depthwise separable convolutions; section 1:
// nothing but input, filters and output should move):
//     t = act1(depthwise3x3(x) + b_dw)        stride 1, padding 1, one 3 x 3 filter per channel
//     y = act2(pointwise(t) + b_pw)           1 x 1 convolution over the channels, on the matrix cores
// The intermediate t never exists in memory: a workgroup computes it, 32 channels at a time, for its tile of 128
// output pixels straight into the LDS layout that the matrix instructions read as their B operand
// ([channel quad][pixel], 16 bytes per entry, as in the 128-pixel fp32 kernel), and multiplies it with the chunk's
// pointwise weights.  HBM sees x once per block of up to 256 output channels and y once.
//
// Per chunk: (1) the window of 32 channels (tile + one-pixel frame, zero outside the image) and the chunk's
// depthwise and pointwise weights go to LDS; (2) every thread computes 16 depthwise outputs (one channel-pixel
// pair each: nine LDS reads, nine FMAs, bias, rectifier); (3) four groups of eight channels are multiplied with
// the weights of up to 256 output channels (NB blocks of 64: two 32 x 32 accumulators per block and wavefront),
// so that the depthwise stage is computed once per 256 output channels, not once per 64.  Products and sums are
// fp32 throughout.
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kCK = 32;                // channels per chunk
constexpr int kQ = kCK / 4;            // channel quads per chunk
constexpr int kG = kCK / 8;            // groups of eight channels = four matrix steps
constexpr int kTilePx = 128;           // output pixels per workgroup: one 32-pixel block per wavefront

struct BlockParams {
    const float* b_dw;                 // [C] or null
    const float* b_pw;                 // [C_out] or null
    int relu1, relu2;
    int C, C_out, H, W, TH, TW, IH, IW, tiles_x;
    FastDiv by_tiles_x, by_TW, by_IW, by_win;
};

template <int NB>
__global__ __launch_bounds__(256) void dw_pw_block_kernel(const float* __restrict__ x, const float* __restrict__ w_dw,
                                                          const float* __restrict__ w_pw, float* __restrict__ y,
                                                          const BlockParams P)
{
    extern __shared__ __attribute__((aligned(16))) float smem_blk[];
    const int WP = P.IH * P.IW;                                  // window pixels per channel
    floatx4* xs = reinterpret_cast<floatx4*>(smem_blk);          // [kQ][128]: the depthwise result, B operand
    floatx4* ws = xs + kQ * kTilePx;                             // [NB][kQ][64]: pointwise weights, A operand
    float* wd = reinterpret_cast<float*>(ws + NB * kQ * 64);     // [32][9] depthwise filters, then [32] biases
    float* xw = wd + kCK * 9 + kCK;                              // [32][IH][IW] input window

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lj = lane & 31, kk = lane >> 5;
    const int ty = fast_div(blockIdx.x, P.by_tiles_x);
    const int tx = blockIdx.x - ty * P.tiles_x;
    const int n = blockIdx.y;
    const int co0 = blockIdx.z * (64 * NB);
    const int row0 = ty * P.TH, col0 = tx * P.TW;
    const int tile_px = P.TH * P.TW;
    const int p = wave * 32 + lj;
    const int pi = fast_div(p, P.by_TW), pj = p - pi * P.TW;
    const bool p_ok = p < tile_px && row0 + pi < P.H && col0 + pj < P.W;
    const bool wave_live = __builtin_amdgcn_readfirstlane(wave * 32) < tile_px;

    floatx16 acc[NB][2];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) { acc[b][0][v] = 0.f; acc[b][1][v] = 0.f; }

    const int HW = P.H * P.W;
    const float* xn = x + (int64_t)n * P.C * HW;
    const float* wb = w_pw + (int64_t)co0 * P.C;

    for (int ci0 = 0; ci0 < P.C; ci0 += kCK) {
        // ---- (1) input window of the chunk, zero outside the image and beyond C (coalesced along image rows); eight
        //      loads go out per thread before the first LDS write, so a batch costs one memory round trip
        for (int base = tid; base < kCK * WP; base += 256 * 8) {
            float v8[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + 256 * u;
                const int c = fast_div(idx, P.by_win);
                const int q = idx - c * WP;
                const int e = fast_div(q, P.by_IW), f = q - e * P.IW;
                const int gr = row0 - 1 + e, gc = col0 - 1 + f;
                v8[u] = 0.f;
                if (idx < kCK * WP && ci0 + c < P.C && gr >= 0 && gr < P.H && gc >= 0 && gc < P.W)
                    v8[u] = xn[(int64_t)(ci0 + c) * HW + gr * P.W + gc];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (base + 256 * u < kCK * WP) xw[base + 256 * u] = v8[u];
        }
        // depthwise filters and biases of the chunk
        for (int idx = tid; idx < kCK * 9 + kCK; idx += 256) {
            float v = 0.f;
            if (idx < kCK * 9) {
                const int c = idx / 9;
                if (ci0 + c < P.C) v = w_dw[(int64_t)(ci0 + c) * 9 + (idx - 9 * c)];
            } else {
                const int c = idx - kCK * 9;
                if (P.b_dw && ci0 + c < P.C) v = P.b_dw[ci0 + c];
            }
            wd[idx] = v;
        }
        // pointwise weights of the chunk: entry (quad q, output channel co_l) = channels ci0 + 4q .. + 3
        for (int base = tid; base < NB * 64 * kQ; base += 256 * 2) {       // (two entries = eight loads per turn)
            floatx4 v2[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int idx = base + 256 * u;
                const int co_l = idx >> 3, q = idx & 7;         // co_l: 0 .. 64 * NB - 1
                v2[u] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (idx < NB * 64 * kQ && co0 + co_l < P.C_out) {
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        if (ci0 + 4 * q + t < P.C) v2[u][t] = wb[(int64_t)co_l * P.C + ci0 + 4 * q + t];
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int idx = base + 256 * u;
                if (idx < NB * 64 * kQ) ws[(((idx >> 3) >> 6) * kQ + (idx & 7)) * 64 + ((idx >> 3) & 63)] = v2[u];
            }
        }
        __syncthreads();

        // ---- (2) depthwise 3 x 3 with bias and rectifier, written as the matrix product's B operand
        float* xs_f = reinterpret_cast<float*>(xs);
#pragma unroll 4
        for (int it = tid; it < kCK * kTilePx; it += 256) {
            const int c = it >> 7, pp = it & (kTilePx - 1);
            float v = 0.f;
            if (pp < tile_px) {
                const int pi2 = fast_div(pp, P.by_TW), pj2 = pp - pi2 * P.TW;
                const float* win = xw + c * WP + pi2 * P.IW + pj2;
                const float* f9 = wd + c * 9;
                v = wd[kCK * 9 + c];
#pragma unroll
                for (int r = 0; r < 3; ++r)
#pragma unroll
                    for (int s = 0; s < 3; ++s) v = fmaf(f9[3 * r + s], win[r * P.IW + s], v);
                if (P.relu1) v = fmaxf(v, 0.f);
            }
            xs_f[(((c >> 2) * kTilePx + pp) << 2) + (c & 3)] = v;
        }
        __syncthreads();

        // ---- (3) pointwise: four groups of eight channels, 2 x 4 matrix steps each
        if (wave_live) {
            const floatx4* bp = xs + kk * kTilePx + p;
            const floatx4* ap = ws + kk * 64 + lj;
#pragma unroll
            for (int g = 0; g < kG; ++g) {
                const floatx4 b = bp[2 * g * kTilePx];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const floatx4 a0 = ap[(nb * kQ + 2 * g) * 64], a1 = ap[(nb * kQ + 2 * g) * 64 + 32];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        acc[nb][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[t], b[t], acc[nb][0], 0, 0, 0);
                        acc[nb][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[t], b[t], acc[nb][1], 0, 0, 0);
                    }
                }
            }
        }
        __syncthreads();
    }

    // ---- store: register v of a lane is output channel 8*(v/4) + 4*kk + v%4 of the block, pixel lj
    if (!p_ok) return;
    float* yp = y + ((int64_t)n * P.C_out + co0) * HW + (row0 + pi) * P.W + col0 + pj;
#pragma unroll
    for (int h = 0; h < 4 * NB; ++h) {
        const int nb = h >> 2, half = (h >> 1) & 1, v0 = (h & 1) * 8;
        const int cb = 64 * nb + 32 * half;
        float b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int v = v0 + i, co = co0 + cb + 8 * (v >> 2) + 4 * kk + (v & 3);
            b[i] = (P.b_pw && co < P.C_out) ? P.b_pw[co] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int v = v0 + i, co = cb + 8 * (v >> 2) + 4 * kk + (v & 3);
            const float t = acc[nb][half][v] + b[i];
            if (co0 + co < P.C_out) yp[(int64_t)co * HW] = P.relu2 ? fmaxf(t, 0.f) : t;
        }
    }
}

constexpr size_t kBlockLds = 112 * 1024;

template <int NB>
hipError_t allow_lds()
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(dw_pw_block_kernel<NB>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBlockLds);
}

}  // namespace

bool dw_pw_block_supported(int N, int C, int C_out, int H, int W)
{
    const int TW = W < kTilePx ? W : kTilePx;
    const int TH = kTilePx / TW > H ? H : kTilePx / TW;
    const int64_t tiles = (int64_t)((W + TW - 1) / TW) * ((H + TH - 1) / TH);
    return N <= 65535 && (C_out + 63) / 64 <= 65535 && tiles <= 2147483647LL && (int64_t)C * H * W <= 2147483647LL &&
           (int64_t)kCK * (TH + 2) * (TW + 2) < 65536;
}

hipError_t launch_dw_pw_block(const float* x, const float* w_dw, const float* b_dw, const float* w_pw, const float* b_pw,
                              float* y, int N, int C, int C_out, int H, int W, int relu1, int relu2, hipStream_t st)
{
    BlockParams P;
    P.b_dw = b_dw; P.b_pw = b_pw; P.relu1 = relu1; P.relu2 = relu2;
    P.C = C; P.C_out = C_out; P.H = H; P.W = W;
    P.TW = W < kTilePx ? W : kTilePx;
    P.TH = kTilePx / P.TW;
    if (P.TH > H) P.TH = H;
    if (P.TH < 1) P.TH = 1;
    P.IH = P.TH + 2;
    P.IW = P.TW + 2;
    P.tiles_x = (W + P.TW - 1) / P.TW;
    const int tiles_y = (H + P.TH - 1) / P.TH;
    P.by_tiles_x = make_fastdiv(P.tiles_x);
    P.by_TW = make_fastdiv(P.TW);
    P.by_IW = make_fastdiv(P.IW);
    P.by_win = make_fastdiv(P.IH * P.IW);
    // blocks of 64 output channels per workgroup: as many as the output has, up to four
    const int nb = C_out > 128 ? 4 : C_out > 64 ? 2 : 1;
    const size_t lds = ((size_t)kQ * kTilePx + (size_t)nb * kQ * 64) * 16 +
                       ((size_t)kCK * 9 + kCK + (size_t)kCK * P.IH * P.IW) * sizeof(float);
    if (lds > kBlockLds) return hipErrorInvalidValue;
    dim3 grid((unsigned)(P.tiles_x * tiles_y), (unsigned)N, (unsigned)((C_out + 64 * nb - 1) / (64 * nb)));
    if (nb == 4) {
        static const hipError_t attr = allow_lds<4>();
        if (attr != hipSuccess) return attr;
        SW_NOTED_LAUNCH(note_kernel("dw_pw_block_kernel", (int)(4)), dw_pw_block_kernel<4>, grid, dim3(256), lds, st, x, w_dw, w_pw, y, P);
    } else if (nb == 2) {
        static const hipError_t attr = allow_lds<2>();
        if (attr != hipSuccess) return attr;
        SW_NOTED_LAUNCH(note_kernel("dw_pw_block_kernel", (int)(2)), dw_pw_block_kernel<2>, grid, dim3(256), lds, st, x, w_dw, w_pw, y, P);
    } else {
        static const hipError_t attr = allow_lds<1>();
        if (attr != hipSuccess) return attr;
        SW_NOTED_LAUNCH(note_kernel("dw_pw_block_kernel", (int)(1)), dw_pw_block_kernel<1>, grid, dim3(256), lds, st, x, w_dw, w_pw, y, P);
    }
    return hipGetLastError();
}

}  // namespace swconv
