// Multi-channel fp32 convolution, stride 1, on the matrix cores.
//
// With more than one input channel every filter tap (r, s) is a small matrix, W_rs[co, ci], and the
// output tile is the sum over taps of W_rs times the input tile shifted by (r, s) (paper, section 3:
// sliding sums re-formulated as small matrix multiplications).  The shift is nothing but an address
// offset into the input tile staged in LDS, so no column matrix exists anywhere.
//
// Workgroup = 4 wavefronts = 64 output channels x one tile of TH x TW (<= 400) output pixels of one
// image.  Input channels are consumed in chunks of 16: the chunk's input window (tile + halo,
// zero-filled outside the image) is staged in LDS as [ci/4][pixel][ci%4], so that one 16-byte LDS
// read hands a lane the B operands of four v_mfma_f32_16x16x4_f32 steps.  The K index of those four
// steps is permuted accordingly (step t, lane group q <-> channel 4q + t), which makes the A
// operands of a lane for a whole chunk -- 4 channels x R*S taps of one output channel -- one
// contiguous run of the OIHW weight tensor, loaded straight into registers with 16-byte loads.
// Each wavefront owns 16 output channels and all 25 pixel blocks (16 pixels each) of the tile: 100
// accumulator registers.  The next chunk's input and weights are fetched from HBM/L2 into registers
// while the current chunk is multiplied.
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kCK = 16;        // input channels per chunk
constexpr int kNB = 25;        // 16-pixel blocks per tile
constexpr int kTilePx = kNB * 16;
constexpr int kLdsPx = 576;    // pixels of the staged input window (tile + halo)
constexpr int kItems = 4 * kLdsPx / 256;   // (channel group, pixel) items per thread and chunk
constexpr int kGroup = 5;      // pixel blocks multiplied between LDS read batches

template <int R, int S>
__global__ __launch_bounds__(256, 1) void mfma_f32_kernel(const float* __restrict__ x,
                                                          const float* __restrict__ w,
                                                          float* __restrict__ y, int C_in, int C_out,
                                                          int H, int W, int pad, int Ho, int Wo,
                                                          int TH, int TW, int tiles_x, int tiles_y)
{
    constexpr int RS = R * S;
    __shared__ floatx4 lds[4 * kLdsPx];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lq = lane >> 4, lj = lane & 15;

    int b = blockIdx.x;
    const int tx = b % tiles_x; b /= tiles_x;
    const int ty = b % tiles_y; b /= tiles_y;
    const int mblocks = C_out >> 6;
    const int mb = b % mblocks;
    const int n = b / mblocks;

    const int row0 = ty * TH, col0 = tx * TW;
    const int IH = TH + R - 1, IW = TW + S - 1;
    const int npx = IH * IW;
    const int HW = H * W;
    const float* xn = x + (int64_t)n * C_in * HW;

    // ---- staging plan: item = (channel group q, window pixel); fixed for the whole kernel ----------
    int goff[kItems];      // offset of channel 4q at that pixel inside one image; < 0: zero-fill
    int loff[kItems];      // LDS slot (float4 units); < 0: nothing to write
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        const int idx = tid + 256 * k;
        const int q = idx / npx;
        const int pix = idx - q * npx;
        const int e = pix / IW, c = pix - e * IW;
        const int gr = row0 - pad + e, gc = col0 - pad + c;
        const bool live = idx < 4 * npx;
        const bool inside = live && gr >= 0 && gr < H && gc >= 0 && gc < W;
        goff[k] = inside ? (4 * q * H + gr) * W + gc : -1;
        loff[k] = live ? q * kLdsPx + pix : -1;
    }

    // ---- LDS slots of this lane's B operands, one per pixel block ----------------------------------
    const int tile_px = TH * TW;
    int boff[kNB];
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb) {
        int p = nb * 16 + lj;
        if (p >= tile_px) p = 0;
        const int pi = p / TW, pj = p - pi * TW;
        boff[nb] = lq * kLdsPx + pi * IW + pj;
    }

    // ---- A operands: weights of output channel co, channels c0 + 4*lq .. +3, all taps --------------
    const int co = (mb << 6) + (wave << 4) + lj;
    const float* wl = w + ((int64_t)co * C_in + 4 * lq) * RS;

    floatx4 acc[kNB];
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb) acc[nb] = floatx4{0.f, 0.f, 0.f, 0.f};

    float xr[kItems][4];
    floatx4 ar[RS];        // ar[i] = floats 4i..4i+3 of the run; element t*RS + tap <-> (channel t, tap)

    auto fetch = [&](int c0) {
        const float* xc = xn + (int64_t)c0 * HW;
#pragma unroll
        for (int k = 0; k < kItems; ++k) {
#pragma unroll
            for (int t = 0; t < 4; ++t) xr[k][t] = goff[k] >= 0 ? xc[goff[k] + t * HW] : 0.f;
        }
        const floatx4* wc = reinterpret_cast<const floatx4*>(wl + (int64_t)c0 * RS);
#pragma unroll
        for (int i = 0; i < RS; ++i) ar[i] = wc[i];
    };

    fetch(0);
    const int chunks = C_in / kCK;
    for (int ch = 0; ch < chunks; ++ch) {
#pragma unroll
        for (int k = 0; k < kItems; ++k)
            if (loff[k] >= 0) lds[loff[k]] = floatx4{xr[k][0], xr[k][1], xr[k][2], xr[k][3]};
        float a[4 * RS];
#pragma unroll
        for (int i = 0; i < RS; ++i) {
            a[4 * i + 0] = ar[i].x; a[4 * i + 1] = ar[i].y; a[4 * i + 2] = ar[i].z; a[4 * i + 3] = ar[i].w;
        }
        __syncthreads();
        if (ch + 1 < chunks) fetch((ch + 1) * kCK);

#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const int tap = r * S + s;
                const int toff = r * IW + s;
#pragma unroll
                for (int g = 0; g < kNB; g += kGroup) {
                    floatx4 bv[kGroup];
#pragma unroll
                    for (int i = 0; i < kGroup; ++i) bv[i] = lds[boff[g + i] + toff];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
#pragma unroll
                        for (int i = 0; i < kGroup; ++i)
                            acc[g + i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t * RS + tap], bv[i][t],
                                                                              acc[g + i], 0, 0, 0);
                    }
                }
            }
        }
        __syncthreads();
    }

    // ---- store: lane holds channels co4 .. co4+3 of pixel p for every block --------------------------
    const int co4 = (mb << 6) + (wave << 4) + 4 * lq;
    float* yn = y + ((int64_t)n * C_out + co4) * Ho * Wo;
    const int HoWo = Ho * Wo;
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb) {
        const int p = nb * 16 + lj;
        const int pi = p / TW, pj = p - pi * TW;
        const int oi = row0 + pi, oj = col0 + pj;
        if (p < tile_px && oi < Ho && oj < Wo) {
            float* dst = yn + oi * Wo + oj;
#pragma unroll
            for (int v = 0; v < 4; ++v) dst[v * HoWo] = acc[nb][v];
        }
    }
}

struct Tiling {
    int TH, TW, tiles_x, tiles_y;
};

Tiling pick_tiling(const Conv2dShape& s)
{
    Tiling t;
    const int splits = (s.Wo + 63) / 64;
    t.TW = (s.Wo + splits - 1) / splits;
    t.TH = kTilePx / t.TW;
    if (t.TH > s.Ho) t.TH = s.Ho;
    while (t.TH > 1 && (t.TH + s.R - 1) * (t.TW + s.S - 1) > kLdsPx) --t.TH;
    t.tiles_x = (s.Wo + t.TW - 1) / t.TW;
    t.tiles_y = (s.Ho + t.TH - 1) / t.TH;
    return t;
}

}  // namespace

bool mfma_f32_supported(const Conv2dShape& s)
{
    if (s.stride != 1 || s.C_in % kCK != 0 || s.C_out % 64 != 0) return false;
    if (!((s.R == 3 && s.S == 3) || (s.R == 5 && s.S == 5))) return false;
    if ((int64_t)s.C_in * s.H * s.W > 2147483647LL) return false;
    const Tiling t = pick_tiling(s);
    if ((t.TH + s.R - 1) * (t.TW + s.S - 1) > kLdsPx || t.TH * t.TW > kTilePx) return false;
    const int64_t blocks = (int64_t)s.N * (s.C_out / 64) * t.tiles_x * t.tiles_y;
    return blocks <= 2147483647LL;
}

hipError_t launch_mfma_f32(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st)
{
    if (reinterpret_cast<uintptr_t>(w) % 16 != 0) return launch_direct_conv2d_f32(x, w, y, s, false, st);
    const Tiling t = pick_tiling(s);
    const int64_t blocks = (int64_t)s.N * (s.C_out / 64) * t.tiles_x * t.tiles_y;
    dim3 grid((unsigned)blocks), block(256);
    if (s.R == 3)
        hipLaunchKernelGGL((mfma_f32_kernel<3, 3>), grid, block, 0, st, x, w, y, s.C_in, s.C_out, s.H, s.W,
                           s.pad, s.Ho, s.Wo, t.TH, t.TW, t.tiles_x, t.tiles_y);
    else
        hipLaunchKernelGGL((mfma_f32_kernel<5, 5>), grid, block, 0, st, x, w, y, s.C_in, s.C_out, s.H, s.W,
                           s.pad, s.Ho, s.Wo, t.TH, t.TW, t.tiles_x, t.tiles_y);
    return hipGetLastError();
}

}  // namespace swconv
