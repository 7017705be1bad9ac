// Quantised multi-channel convolution with filters packed once (paper, sections 1.1 and 3: quantised
// inference on the sliding formulation, taps as small matrix products).  The filters of a trained network
// never change between calls, while the channel-first filter tensor has to be byte-transposed into the
// operand order of the matrix instruction by every workgroup of every call that takes it as it is.  Here
// that transposition is done once, by sw_s8_pack_filter, into a caller-owned buffer:
//
//     packed[cb][tap][ks][lane][16 bytes]      cb = co / 32, tap = r * S + s, ks = ci / 32
//         lane l holds w[32 cb + l % 32][32 ks + 16 (l / 32) + 0..15][tap]    (zero beyond C_out, C_in)
//
// which is exactly what a wavefront's 64 lanes load as the A operand of one v_mfma_i32_32x32x32_i8 step:
// one coalesced 16-byte load per lane, straight from L2 into the registers the instruction reads.  The
// input is still the unmodified channel-first tensor: its window (tile + halo, zero outside the image) is
// byte-transposed on its way into LDS as [pixel][ci] and every tap is an address offset into it.
//
// Workgroup = 4 wavefronts = 64 output channels x a tile of at most 256 output pixels of one image;
// wavefront = 32 output channels x up to four blocks of 32 pixels.  A wavefront keeps all its A operands
// (9 taps x C_in / 32 steps) in registers; they arrive from L2 while the input window is being staged, and
// the first multiplications only wait for the operands they use.  Blocks are multiplied two at a time with
// the B operands read from LDS two steps ahead, and the stores of a finished pair drain under the
// multiplications of the next pair.
#include <algorithm>

#include "swconv_internal.h"
#include "sw_s8_perm.h"

namespace swconv {

namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32;
using s8perm::gather4;

constexpr int kNBW = 4;            // 32-pixel blocks per wavefront
constexpr int kTilePx = 2 * kNBW * 32;
constexpr int kWinPx = 320;        // pixels of the staged input window

// 16 channels x 4 pixels (one dword per channel) -> pixel PX's 16 channel bytes
template <int PX>
__device__ __forceinline__ intx4 xgather_px(const u32* in)
{
    intx4 v;
    v.x = (int)gather4<0 * 4 + PX, 1 * 4 + PX, 2 * 4 + PX, 3 * 4 + PX>(in);
    v.y = (int)gather4<4 * 4 + PX, 5 * 4 + PX, 6 * 4 + PX, 7 * 4 + PX>(in);
    v.z = (int)gather4<8 * 4 + PX, 9 * 4 + PX, 10 * 4 + PX, 11 * 4 + PX>(in);
    v.w = (int)gather4<12 * 4 + PX, 13 * 4 + PX, 14 * 4 + PX, 15 * 4 + PX>(in);
    return v;
}

struct PackedParams {
    int C_out, H, W, pad, Ho, Wo, TH, TW, nq_max, wide_store;
    FastDiv by_tiles_x, by_TW, by_IH, by_IW, by_nq_max;
};

// ---- packing: one thread per 16-byte piece -------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_filter_s8_kernel(const int8_t* __restrict__ w, int8_t* __restrict__ packed,
                                                             int C_in, int C_out, int RS, int KSn, int64_t pieces)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= pieces) return;
    const int lane = (int)(idx & 63);
    int64_t t = idx >> 6;
    const int ks = (int)(t % KSn); t /= KSn;
    const int tap = (int)(t % RS);
    const int cb = (int)(t / RS);
    const int co = 32 * cb + (lane & 31);
    const int ci0 = 32 * ks + 16 * (lane >> 5);
    u32 out[4] = {0u, 0u, 0u, 0u};
    if (co < C_out) {
        const int8_t* src = w + ((int64_t)co * C_in + ci0) * RS + tap;
#pragma unroll
        for (int b = 0; b < 16; ++b)
            if (ci0 + b < C_in) out[b >> 2] |= (u32)(unsigned char)src[(int64_t)b * RS] << (8 * (b & 3));
    }
    *reinterpret_cast<intx4*>(packed + idx * 16) = intx4{(int)out[0], (int)out[1], (int)out[2], (int)out[3]};
}

// ---- the convolution ------------------------------------------------------------------------------------
// KS: C_in / 32 (all of K resident: the window in LDS, the A operands in registers).
// XI: input staging items (16 channels x one column quad of a window row) per thread.
// RQ: the sums leave requantised to int8 (y8) instead of as int32 (y).
template <int KS, int XI, bool RQ>
__global__ __launch_bounds__(256, 1) void mfma_s8_packed_kernel(const int8_t* __restrict__ x,
                                                                const int8_t* __restrict__ wp,
                                                                int32_t* __restrict__ y, const PackedParams P,
                                                                int8_t* __restrict__ y8, const Requant rq)
{
    constexpr int C_in = 32 * KS;
    constexpr int kPitch = C_in + 16;          // bytes per window pixel: 16-byte operand reads of 16 consecutive
                                               // pixels fall into distinct banks
    constexpr int NSTEP = 9 * KS;
    const int C_out = P.C_out, H = P.H, W = P.W, pad = P.pad, Ho = P.Ho, Wo = P.Wo;
    const int TH = P.TH, TW = P.TW;
    extern __shared__ __attribute__((aligned(16))) unsigned char lx[];      // [window pixel][ci]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lg = lane >> 5, lj = lane & 31;      // K half and row/column inside a 32 x 32 block
    const int wm = wave >> 1, wn = wave & 1;

    const int ty = fast_div(blockIdx.x, P.by_tiles_x);
    const int tx = blockIdx.x - ty * (int)P.by_tiles_x.d;
    const int n = blockIdx.y;
    const int mb = blockIdx.z;

    const int row0 = ty * TH, col0 = tx * TW;
    const int IH = TH + 2, IW = TW + 2;
    const int HW = H * W;
    const int8_t* xn = x + (int64_t)n * C_in * HW;

    // ---- input staging plan: item = (16-channel group, window row, image column quad) ---------------
    const int wc0 = col0 - pad;                        // image column of window column 0
    const int g_lo = max(wc0 >> 2, 0);                 // first column quad of the image the window touches
    const int nq = min((wc0 + IW - 1) >> 2, (W >> 2) - 1) - g_lo + 1;
    const int nitems = 2 * KS * IH * P.nq_max;
    int xoff[XI];      // byte offset of (channel 16*c16, row, 4g) in the image; < 0: skip item
    int xlds[XI];      // byte address in lx of window column (4g - wc0) of that row, channel 16*c16
    int xc[XI];        // window column of the quad's first pixel (may be < 0)
#pragma unroll
    for (int k = 0; k < XI; ++k) {
        const int idx = tid + 256 * k;
        const int t = fast_div(idx, P.by_nq_max);
        const int g = idx - t * P.nq_max;
        const int c16 = fast_div(t, P.by_IH);
        const int e = t - c16 * IH;
        const int gr = row0 - pad + e;
        const int gc = 4 * (g_lo + g);
        const bool ok = idx < nitems && g < nq && gr >= 0 && gr < H && gc >= 0 && gc + 3 < W;
        xoff[k] = ok ? (16 * c16 * H + gr) * W + gc : -1;
        xc[k] = gc - wc0;
        xlds[k] = (e * IW + xc[k]) * kPitch + 16 * c16;
    }
    u32 xv[XI][16];
#pragma unroll
    for (int k = 0; k < XI; ++k) {
#pragma unroll
        for (int c = 0; c < 16; ++c)      // skipped items read a valid dummy address and are ignored below
            xv[k][c] = *reinterpret_cast<const u32*>(xn + max(xoff[k], 0) + c * HW);
    }

    // ---- this wavefront's A operands: 9 x KS coalesced 16-byte loads, behind the input's loads in the queue
    const intx4* wa = reinterpret_cast<const intx4*>(wp) + ((int64_t)(2 * mb + wm) * NSTEP) * 64 + lane;
    intx4 a[NSTEP];
#pragma unroll
    for (int st = 0; st < NSTEP; ++st) a[st] = wa[st * 64];

    // ---- the padding: window cells outside the image are zeroed once; the staging below writes every cell
    //      inside the image and no other, so no barrier has to separate the two
    {
        const int cells = IH * IW;
        for (int i = tid; i < cells; i += 256) {
            const int e = fast_div(i, P.by_IW), c = i - e * IW;
            const int gr = row0 - pad + e, gc = col0 - pad + c;
            if (gr < 0 || gr >= H || gc < 0 || gc >= W) {
#pragma unroll
                for (int b = 0; b < kPitch; b += 16) *reinterpret_cast<intx4*>(lx + i * kPitch + b) = intx4{0, 0, 0, 0};
            }
        }
    }

    // ---- operand addresses ---------------------------------------------------------------------
    const int tile_px = TH * TW;
    int boff[kNBW];
#pragma unroll
    for (int i = 0; i < kNBW; ++i) {
        int p = (wn * kNBW + i) * 32 + lj;
        if (p >= tile_px) p = 0;
        const int pi = fast_div(p, P.by_TW), pj = p - pi * TW;
        boff[i] = (pi * IW + pj) * kPitch + 16 * lg;
    }
    const int rowoff1 = IW * kPitch, rowoff2 = 2 * IW * kPitch;

    // ---- registers -> LDS with the byte transposes ------------------------------------------------
#pragma unroll
    for (int k = 0; k < XI; ++k) {
        if (xoff[k] >= 0) {
            const int c = xc[k];
            if (c >= 0 && c < IW) *reinterpret_cast<intx4*>(lx + xlds[k]) = xgather_px<0>(xv[k]);
            if (c + 1 >= 0 && c + 1 < IW) *reinterpret_cast<intx4*>(lx + xlds[k] + kPitch) = xgather_px<1>(xv[k]);
            if (c + 2 >= 0 && c + 2 < IW) *reinterpret_cast<intx4*>(lx + xlds[k] + 2 * kPitch) = xgather_px<2>(xv[k]);
            if (c + 3 >= 0 && c + 3 < IW) *reinterpret_cast<intx4*>(lx + xlds[k] + 3 * kPitch) = xgather_px<3>(xv[k]);
        }
    }
    __syncthreads();

    const int HoWo = Ho * Wo;
    const int co_base = (mb << 6) + 32 * wm + 4 * lg;       // this lane's first output channel
    const int64_t ybase = ((int64_t)n * C_out + co_base) * HoWo;
    auto b_at = [&](int i, int st) __attribute__((always_inline)) {
        const int tap = st / KS, kk = st % KS;
        const int r = tap / 3, q = tap - 3 * r;
        const int base = boff[i] + (r == 0 ? 0 : r == 1 ? rowoff1 : rowoff2);
        return *reinterpret_cast<const intx4*>(lx + base + q * kPitch + 32 * kk);
    };
    // offset of this lane's pixel in block i inside a channel plane (-1 when it lies outside the tile/image)
    auto block_dst = [&](int i) -> int {
        const int p = (wn * kNBW + i) * 32 + lj;
        const int pi = fast_div(p, P.by_TW), pj = p - pi * TW;
        const int oi = row0 + pi, oj = col0 + pj;
        return (p < tile_px && oi < Ho && oj < Wo) ? oi * Wo + oj : -1;
    };
    // this lane's sixteen output channels' scales and biases, read once
    float rq_scale[RQ ? 16 : 1];
    int rq_bias[RQ ? 16 : 1];
    if constexpr (RQ) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int co = co_base + 8 * (v >> 2) + (v & 3);
            rq_scale[v] = rq.scale[co];
            rq_bias[v] = rq.bias ? rq.bias[co] : 0;
        }
    }
    auto requant_reg = [&](int acc_v, int v) __attribute__((always_inline)) {
        float r = rintf(__int2float_rn(acc_v + rq_bias[RQ ? v : 0]) * rq_scale[RQ ? v : 0]);
        r = fminf(fmaxf(r, rq.relu ? 0.0f : -128.0f), 127.0f);
        return (int)r;
    };
    // Requantised output, rows whose groups of four pixels are aligned dwords in y8 (P.wide_store): the four
    // lanes of a quad hold four pixels x four consecutive channels; two exchange rounds inside the quad
    // (DPP quad_perm) transpose that, so that lane k ends up with channel k of all four pixels and stores
    // them as one dword instead of four single bytes.
    auto store_quad = [&](int dst, const intx16& c, int g) __attribute__((always_inline)) {
        const int k = lane & 3;
        int r[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) r[t] = requant_reg(c[4 * g + t], 4 * g + t) & 255;
        const bool b0 = k & 1, b1 = k & 2;
        const int keep01 = b0 ? r[1] : r[0], send01 = b0 ? r[0] : r[1];
        const int keep23 = b0 ? r[3] : r[2], send23 = b0 ? r[2] : r[3];
        const int got01 = __builtin_amdgcn_mov_dpp(send01, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
        const int got23 = __builtin_amdgcn_mov_dpp(send23, 0xB1, 0xF, 0xF, true);
        const int own_a = b1 ? keep23 : keep01, own_b = b1 ? got23 : got01;
        const int snd_a = b1 ? keep01 : keep23, snd_b = b1 ? got01 : got23;
        const int far_a = __builtin_amdgcn_mov_dpp(snd_a, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
        const int far_b = __builtin_amdgcn_mov_dpp(snd_b, 0x4E, 0xF, 0xF, true);
        // channel k of pixels k (own_a), k^1 (own_b), k^2 (far_a), k^3 (far_b); byte j of the dword is pixel j
        const unsigned word = (unsigned)own_a << (8 * k) | (unsigned)own_b << (8 * (k ^ 1)) |
                              (unsigned)far_a << (8 * (k ^ 2)) | (unsigned)far_b << (8 * (k ^ 3));
        if (dst >= 0)
            *reinterpret_cast<unsigned*>(y8 + ybase + (int64_t)(8 * g + k) * HoWo + (dst - k)) = word;
    };
    auto store_reg = [&](int dst, const intx16& c, int v) __attribute__((always_inline)) {
        const int ch = 8 * (v >> 2) + (v & 3);
        if constexpr (RQ) {
            if (P.wide_store) {
                if ((v & 3) == 3) store_quad(dst, c, v >> 2);
            } else if (dst >= 0) {
                y8[ybase + (int64_t)ch * HoWo + dst] = (int8_t)requant_reg(c[v], v);
            }
        } else {
            if (dst >= 0) y[ybase + (int64_t)ch * HoWo + dst] = c[v];
        }
    };

    const int live = __builtin_amdgcn_readfirstlane(max(0, min(kNBW, (tile_px - wn * kNBW * 32 + 31) >> 5)));
    if (live == 0) return;
    intx16 c0, c1, d0, d1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { c0[v] = 0; c1[v] = 0; d0[v] = 0; d1[v] = 0; }

    // ---- blocks 0 and 1 (one block: only c0) ---------------------------------------------------------
    if (live >= 2) {
        intx4 b0[3], b1[3];
        b0[0] = b_at(0, 0); b1[0] = b_at(1, 0);
        if (NSTEP > 1) { b0[1] = b_at(0, 1); b1[1] = b_at(1, 1); }
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            if (st + 2 < NSTEP) { b0[(st + 2) % 3] = b_at(0, st + 2); b1[(st + 2) % 3] = b_at(1, st + 2); }
            __builtin_amdgcn_sched_barrier(0);
            c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[st], b0[st % 3], c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[st], b1[st % 3], c1, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        intx4 b0[3];
        b0[0] = b_at(0, 0);
        if (NSTEP > 1) b0[1] = b_at(0, 1);
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            if (st + 2 < NSTEP) b0[(st + 2) % 3] = b_at(0, st + 2);
            __builtin_amdgcn_sched_barrier(0);
            c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[st], b0[st % 3], c0, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    const int dst0 = block_dst(0);
    const int dst1 = live >= 2 ? block_dst(1) : -1;

    // ---- blocks 2 and 3, with the 32 stores of blocks 0 and 1 spread between the matrix instructions ----
    if (live >= 4) {
        intx4 b0[3], b1[3];
        b0[0] = b_at(2, 0); b1[0] = b_at(3, 0);
        if (NSTEP > 1) { b0[1] = b_at(2, 1); b1[1] = b_at(3, 1); }
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            if (st + 2 < NSTEP) { b0[(st + 2) % 3] = b_at(2, st + 2); b1[(st + 2) % 3] = b_at(3, st + 2); }
            // 32 stores over the first 32 of the 9 * KS steps (KS == 1: four per step over the first eight)
            constexpr int PER = NSTEP >= 32 ? 1 : (32 + NSTEP - 2) / (NSTEP - 1);
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int sv = st * PER + u;
                if (sv < 16) store_reg(dst0, c0, sv);
                else if (sv < 32) store_reg(dst1, c1, sv - 16);
            }
            __builtin_amdgcn_sched_barrier(0);
            d0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[st], b0[st % 3], d0, 0, 0, 0);
            d1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[st], b1[st % 3], d1, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        const int dst2 = block_dst(2), dst3 = block_dst(3);
#pragma unroll
        for (int v = 0; v < 16; ++v) store_reg(dst2, d0, v);
#pragma unroll
        for (int v = 0; v < 16; ++v) store_reg(dst3, d1, v);
    } else if (live == 3) {
        intx4 b0[3];
        b0[0] = b_at(2, 0);
        if (NSTEP > 1) b0[1] = b_at(2, 1);
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            if (st + 2 < NSTEP) b0[(st + 2) % 3] = b_at(2, st + 2);
            constexpr int PER = NSTEP >= 32 ? 1 : (32 + NSTEP - 2) / (NSTEP - 1);
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int sv = st * PER + u;
                if (sv < 16) store_reg(dst0, c0, sv);
                else if (sv < 32) store_reg(dst1, c1, sv - 16);
            }
            __builtin_amdgcn_sched_barrier(0);
            d0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[st], b0[st % 3], d0, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        const int dst2 = block_dst(2);
#pragma unroll
        for (int v = 0; v < 16; ++v) store_reg(dst2, d0, v);
    } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) store_reg(dst0, c0, v);
#pragma unroll
        for (int v = 0; v < 16; ++v) store_reg(dst1, c1, v);
    }
}

// Any shape from the packed filters: one thread per output.
template <bool RQ>
__global__ __launch_bounds__(256) void direct_s8_packed_kernel(const int8_t* __restrict__ x, const int8_t* __restrict__ wp,
                                                               int32_t* __restrict__ y, Conv2dShape s, int KSn,
                                                               int8_t* __restrict__ y8, Requant rq)
{
    const int64_t plane_o = (int64_t)s.Ho * s.Wo;
    const int64_t total = (int64_t)s.N * s.C_out * plane_o;
    const int RS = s.R * s.S;
    for (int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (int64_t)gridDim.x * 256) {
        const int64_t nc = o / plane_o;
        const int pix = (int)(o - nc * plane_o);
        const int n = (int)(nc / s.C_out);
        const int co = (int)(nc - (int64_t)n * s.C_out);
        const int i = pix / s.Wo, j = pix - i * s.Wo;
        const int h0 = i * s.stride - s.pad, v0 = j * s.stride - s.pad;
        const int8_t* wco = wp + (int64_t)(co >> 5) * RS * KSn * 1024 + (co & 31) * 16;
        int acc = 0;
        for (int ci = 0; ci < s.C_in; ++ci) {
            const int8_t* xp = x + ((int64_t)n * s.C_in + ci) * s.H * s.W;
            const int8_t* wci = wco + (int64_t)(ci >> 5) * 1024 + ((ci >> 4) & 1) * 512 + (ci & 15);
            for (int r = 0; r < s.R; ++r) {
                const int h = h0 + r;
                if (h < 0 || h >= s.H) continue;
                for (int q = 0; q < s.S; ++q) {
                    const int v = v0 + q;
                    if (v < 0 || v >= s.W) continue;
                    acc += (int)xp[h * s.W + v] * (int)wci[(int64_t)(r * s.S + q) * KSn * 1024];
                }
            }
        }
        if constexpr (RQ) y8[o] = requant_s8(acc, co, rq);
        else y[o] = acc;
    }
}

struct Tiling {
    int TH, TW, tiles_x, tiles_y, nq_max, xi;
};

// Tile = TH rows x TW columns of the output, at most 256 pixels, window at most kWinPx pixels, at most four
// staging items per thread.  xi == 0: no tiling fits.
Tiling pick_tiling(const Conv2dShape& s, int KS)
{
    Tiling t{};
    const int splits = (s.Wo + 63) / 64;
    t.TW = (s.Wo + splits - 1) / splits;
    t.TH = std::min(kTilePx / t.TW, s.Ho);
    auto nq_of = [&](int tw) { return std::min((tw + 2 + 2) / 4 + 1, s.W / 4); };
    auto fits = [&](int th) {
        return (th + 2) * (t.TW + 2) <= kWinPx && 2 * KS * (th + 2) * nq_of(t.TW) <= 4 * 256;
    };
    while (t.TH > 1 && !fits(t.TH)) --t.TH;
    if (t.TH < 1 || !fits(t.TH)) return t;
    const int bands = (s.Ho + t.TH - 1) / t.TH;
    t.TH = (s.Ho + bands - 1) / bands;      // equal row bands: same tile count, no nearly empty last band
    t.tiles_x = (s.Wo + t.TW - 1) / t.TW;
    t.tiles_y = (s.Ho + t.TH - 1) / t.TH;
    t.nq_max = nq_of(t.TW);
    const int items = 2 * KS * (t.TH + 2) * t.nq_max;
    t.xi = items <= 512 ? 2 : 4;
    if ((int64_t)t.tiles_x * t.tiles_y > 65535 || s.N > 65535 || (s.C_out + 63) / 64 > 65535) t.xi = 0;
    return t;
}

bool packed_fast_path(const int8_t* x, const int8_t* wp, const Conv2dShape& s)
{
    if (s.stride != 1 || s.R != 3 || s.S != 3 || s.dil != 1) return false;
    if (s.C_in != 32 && s.C_in != 64 && s.C_in != 128) return false;
    if (s.C_out % 64 != 0 || s.W % 4 != 0) return false;
    if ((int64_t)s.C_in * s.H * s.W > 2147483647LL) return false;
    if (reinterpret_cast<uintptr_t>(x) % 4 != 0 || reinterpret_cast<uintptr_t>(wp) % 16 != 0) return false;
    return pick_tiling(s, s.C_in / 32).xi != 0;
}

template <int KS, int XI, bool RQ>
hipError_t launch_variant(const int8_t* x, const int8_t* wp, int32_t* y, int8_t* y8, const Requant& rq,
                          const PackedParams& P, dim3 grid, size_t lds, hipStream_t st)
{
    hipLaunchKernelGGL((mfma_s8_packed_kernel<KS, XI, RQ>), grid, dim3(256), lds, st, x, wp, y, P, y8, rq);
    return hipGetLastError();
}

template <bool RQ>
hipError_t launch_fast(const int8_t* x, const int8_t* wp, int32_t* y, int8_t* y8, const Requant& rq,
                       const Conv2dShape& s, hipStream_t st)
{
    const int KS = s.C_in / 32;
    const Tiling t = pick_tiling(s, KS);
    PackedParams P;
    P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.pad = s.pad; P.Ho = s.Ho; P.Wo = s.Wo;
    P.TH = t.TH; P.TW = t.TW; P.nq_max = t.nq_max;
    // (requantised output only) dword stores of four pixels: groups of four pixels must be aligned dwords of y8
    P.wide_store = s.Wo % 4 == 0 && t.TW % 4 == 0 && reinterpret_cast<uintptr_t>(y8) % 4 == 0;
    P.by_tiles_x = make_fastdiv(t.tiles_x);
    P.by_TW = make_fastdiv(t.TW);
    P.by_IH = make_fastdiv(t.TH + 2);
    P.by_IW = make_fastdiv(t.TW + 2);
    P.by_nq_max = make_fastdiv(t.nq_max);
    const dim3 grid((unsigned)(t.tiles_x * t.tiles_y), (unsigned)s.N, (unsigned)(s.C_out / 64));
    const size_t lds = (size_t)(t.TH + 2) * (t.TW + 2) * (s.C_in + 16);
    note_kernel("mfma_s8_packed_kernel", KS, t.xi, RQ);
#define SW_PK(KSC, XIC) return launch_variant<KSC, XIC, RQ>(x, wp, y, y8, rq, P, grid, lds, st)
    if (KS == 4) { if (t.xi == 2) SW_PK(4, 2); else SW_PK(4, 4); }
    if (KS == 2) { if (t.xi == 2) SW_PK(2, 2); else SW_PK(2, 4); }
    if (t.xi == 2) SW_PK(1, 2); else SW_PK(1, 4);
#undef SW_PK
}

}  // namespace

int64_t s8_packed_filter_bytes(int C_in, int C_out, int R, int S)
{
    return (int64_t)((C_out + 31) / 32) * R * S * ((C_in + 31) / 32) * 1024;
}

hipError_t launch_pack_filter_s8(const int8_t* w, int8_t* packed, int C_in, int C_out, int R, int S, hipStream_t st)
{
    const int64_t pieces = s8_packed_filter_bytes(C_in, C_out, R, S) / 16;
    note_kernel("pack_filter_s8_kernel");
    hipLaunchKernelGGL(pack_filter_s8_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, w, packed, C_in,
                       C_out, R * S, (C_in + 31) / 32, pieces);
    return hipGetLastError();
}

hipError_t launch_conv2d_s8_packed(const int8_t* x, const int8_t* wp, int32_t* y, int8_t* y8, const Requant* rq,
                                   const Conv2dShape& s, bool allow_fast, hipStream_t st)
{
    const Requant none{nullptr, nullptr, 0};
    if (allow_fast && mfma_s8_band_supported(x, wp, s, false)) return launch_mfma_s8_band(x, wp, y, y8, rq, s, false, st);
    if (allow_fast && packed_fast_path(x, wp, s)) {
        if (rq) return launch_fast<true>(x, wp, nullptr, y8, *rq, s, st);
        return launch_fast<false>(x, wp, y, nullptr, none, s, st);
    }
    const int64_t total = (int64_t)s.N * s.C_out * s.Ho * s.Wo;
    const int64_t blocks = std::min<int64_t>((total + 255) / 256, 256 * 64);
    const int KSn = (s.C_in + 31) / 32;
    note_kernel("direct_s8_packed_kernel", rq != nullptr);
    if (rq)
        hipLaunchKernelGGL(direct_s8_packed_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, x, wp, y, s, KSn, y8, *rq);
    else
        hipLaunchKernelGGL(direct_s8_packed_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, x, wp, y, s, KSn, y8, none);
    return hipGetLastError();
}

}  // namespace swconv
