// Quantised multi-channel convolution: int8 x int8 -> exact int32, 3x3, stride 1, on the matrix cores
// (paper, sections 1.1 and 3: quantisation applied to the sliding formulation; taps as small matrix
// products).  Every tap (r, s) contributes W_rs[co, ci] times the input tile shifted by (r, s); the
// shift is an address offset into the tile staged in LDS, so no column matrix exists.
//
// Workgroup = 4 wavefronts = 64 output channels x a tile of TH x TW (<= 208) output pixels of one
// image; input channels are consumed in chunks of 64, two v_mfma_i32_32x32x32_i8 K steps per tap
// (the 32x32x32 form sustains the matrix cores' peak from one wavefront per SIMD; the 16x16x64 form
// does not).
// The matrix instruction wants 16 consecutive K bytes per lane, i.e. channel-contiguous operands,
// while both tensors arrive channel-strided (NCHW, OIHW).  Both are therefore transposed on their
// way into LDS with byte permutes in registers:
//   input   global [ci][row][col]  -> 16 channels x 4 pixels per lane -> LDS [pixel][ci], 80-byte pitch
//   weights global [co][ci][tap]   -> coalesced copy to an LDS staging area, then 16 channels x 9
//                                     taps per lane -> LDS [tap][co][ci], 80-byte pitch
// The 80-byte pitch spreads the 16-byte operand reads of 16 consecutive pixels (or output channels)
// evenly over the banks.  The wavefronts split the tile 2 x 2: 32 output channels x 4 blocks of 32
// pixels each, 64 accumulator registers.  Two chunks are kept in flight from HBM/L2 into registers,
// so a 128-channel problem issues every global load before its first multiplication.
//
// Resident variant (C_in == 128, the whole K range fits LDS at once: 39 KB of input window, 83 KB of
// transposed weights): both chunks are staged first, each wavefront then keeps its 36 A operands in
// registers and walks over its pixel blocks two at a time, all 36 K steps per pair, and stores a pair
// as soon as it is complete.  The int32 output is 79 % of this problem's memory traffic and the device
// absorbs writes at roughly half the HBM peak, so letting the stores of one pair drain under the
// multiplications of the next is what this order is for; no barrier separates the wavefronts here.
#include <algorithm>

#include "swconv_internal.h"
#include "sw_s8_perm.h"

namespace swconv {

namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32;
using s8perm::gather4;
using s8perm::perm;
using s8perm::wgather_tap;

constexpr int kCK = 64;            // input channels per chunk
constexpr int kPitchChunk = 80;    // bytes per pixel / per weight row in LDS, chunked variant
constexpr int kNBW = 4;            // 32-pixel blocks per wavefront
constexpr int kNB = 2 * kNBW;      // 32-pixel blocks per tile
constexpr int kTilePx = kNB * 32;
constexpr int kLdsPx = 320;        // pixels of the staged input window
constexpr int kXItems = 2;         // (16-channel group, row, column quad) items per thread and chunk
constexpr int kXBytesChunk = kLdsPx * kPitchChunk;  // 25600
constexpr int kWBytesChunk = 9 * 64 * kPitchChunk;  // 46080
constexpr int kRawBytes = 64 * kCK * 9;             // 36864
constexpr int kLdsBytes = kXBytesChunk + kWBytesChunk + kRawBytes;
constexpr int kLdsPxRes = 270;     // window pixels of the resident variant (9 rows x 30)
constexpr int kLdsBytesRes = kLdsPxRes * 144 + 9 * 64 * 144 + kRawBytes;   // 158688 of 163840

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

struct S8Params {
    int C_in, C_out, H, W, pad, Ho, Wo, TH, TW, nq_max, wide_store;
    FastDiv by_tiles_x, by_TW, by_IH, by_nq_max, by_pieces;
};

// RES == 0: input channels in chunks of 64 through LDS.  RES == 128: C_in == 128, all of K resident in LDS.
// XI: input staging items per thread and chunk (1 when 4 * rows * column quads <= 256).
// RQ (resident variant only): the sums leave requantised to int8 (y8) instead of as int32 (y).
template <int RES, int XI, bool RQ = false>
__global__ __launch_bounds__(256, 1) void mfma_s8_kernel(const int8_t* __restrict__ x,
                                                         const int8_t* __restrict__ w,
                                                         int32_t* __restrict__ y, const S8Params P,
                                                         int8_t* __restrict__ y8 = nullptr,
                                                         const Requant rq = Requant{nullptr, nullptr, 0})
{
    static_assert(!RQ || RES != 0, "requantised stores exist in the resident variant only");
    constexpr int kPitch = RES ? RES + 16 : kPitchChunk;            // bytes per pixel / weight row
    constexpr int kXBytes = RES ? kLdsPxRes * kPitch : kXBytesChunk;
    constexpr int kWBytes = 9 * 64 * kPitch;
    const int C_in = P.C_in, C_out = P.C_out, H = P.H, W = P.W, pad = P.pad, Ho = P.Ho, Wo = P.Wo;
    const int TH = P.TH, TW = P.TW;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* lx = smem;                       // [pixel][ci]
    unsigned char* lw = smem + kXBytes;             // [tap][co][ci]
    unsigned char* lraw = smem + kXBytes + kWBytes; // [co][ci][tap]    as in global memory

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lg = lane >> 5, lj = lane & 31;      // K half and row/column inside a 32 x 32 block
    const int wm = wave >> 1, wn = wave & 1;

    const int ty = fast_div(blockIdx.x, P.by_tiles_x);
    const int tx = blockIdx.x - ty * (int)P.by_tiles_x.d;
    // image index before channel block: workgroups that share an input tile get linear ids that are equal
    // modulo 8 when the tile count divides 8, i.e. they land on the same XCD and share its L2
    const int n = blockIdx.y;
    const int mb = blockIdx.z;

    const int row0 = ty * TH, col0 = tx * TW;
    const int IH = TH + 2, IW = TW + 2;
    const int HW = H * W;
    const int8_t* xn = x + (int64_t)n * C_in * HW;

    // zeroes the window cells that lie outside the image (the padding), once: the staging below writes every cell
    // inside the image and no other, so the two never touch the same bytes and no barrier has to separate them.
    // Called after the first global loads have been issued, so that it runs under their latency.
    auto zero_window = [&]() {
        const int IWz = TW + 2, cells = (TH + 2) * IWz;
        for (int i = tid; i < cells; i += 256) {
            const int e = i / IWz, c = i - e * IWz;
            const int gr = row0 - pad + e, gc = col0 - pad + c;
            if (gr < 0 || gr >= H || gc < 0 || gc >= W) {
#pragma unroll
                for (int b = 0; b < kPitch; b += 16) *reinterpret_cast<intx4*>(lx + i * kPitch + b) = intx4{0, 0, 0, 0};
            }
        }
    };

    // ---- weight staging: the workgroup's 64 x 576-byte block is copied in 16-byte pieces (coalesced);
    //      afterwards thread (co = tid/4, 16-channel group tid%4) transposes its 144 bytes = pieces 9*tid .. 9*tid+8.
    //      A wavefront copies exactly the 576 pieces its own lanes transpose (piece wave*576 + i*64 + lane), so the
    //      raw copy needs no workgroup barrier: LDS operations of a wavefront complete in order.
    const int wco = tid >> 2, wc16 = tid & 3;
    const int8_t* wblk = w + (int64_t)(mb << 6) * C_in * 9;
    int woff[9];
#pragma unroll
    for (int i = 0; i < 9; ++i) {
        const int piece = wave * 576 + i * 64 + lane;
        woff[i] = (piece / 36) * C_in * 9 + (piece % 36) * 16;
    }

    intx4 wv0[9], wv1[9];
    if constexpr (RES != 0) {
        // the resident variant's filter loads go out before the index arithmetic of the input plan below
#pragma unroll
        for (int i = 0; i < 9; ++i) wv0[i] = *reinterpret_cast<const intx4*>(wblk + woff[i]);
#pragma unroll
        for (int i = 0; i < 9; ++i) wv1[i] = *reinterpret_cast<const intx4*>(wblk + (int64_t)kCK * 9 + woff[i]);
    }

    // ---- input staging plan: item = (16-channel group, window row, image column quad) ---------------
    const int wc0 = col0 - pad;                        // image column of window column 0
    // column quads of the image that the window touches (quads outside the image stay zero)
    const int g_lo = max(wc0 >> 2, 0);                 // arithmetic shift: floor for negatives
    const int nq = min((wc0 + IW - 1) >> 2, (W >> 2) - 1) - g_lo + 1;
    const int nitems = 4 * IH * P.nq_max;
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

    // two register sets, each holding one chunk on its way from global memory to LDS
    u32 xv0[XI][16], xv1[XI][16];
    auto fetch = [&](u32 (&xv)[XI][16], intx4 (&wv)[9], int c0, bool with_filters = true) {
        const int8_t* xcp = xn + (int64_t)c0 * HW;
#pragma unroll
        for (int k = 0; k < XI; ++k) {
#pragma unroll
            for (int c = 0; c < 16; ++c)      // skipped items read a valid dummy address; stage() ignores them
                xv[k][c] = *reinterpret_cast<const u32*>(xcp + max(xoff[k], 0) + c * HW);
        }
        if (!with_filters) return;
        const int8_t* ws = wblk + (int64_t)c0 * 9;
#pragma unroll
        for (int i = 0; i < 9; ++i) wv[i] = *reinterpret_cast<const intx4*>(ws + woff[i]);
    };

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
    const int aoff = (32 * wm + lj) * kPitch + 16 * lg;

    intx16 acc[kNBW];
#pragma unroll
    for (int i = 0; i < kNBW; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0;

    // registers -> LDS (with the byte transposes), then the chunk's 9 taps x 2 K steps
    // (sync_after: a workgroup barrier after the transposed operands are in place; the resident variant stages two
    // chunks before anybody reads and needs only the second one)
    auto stage = [&](u32 (&xv)[XI][16], intx4 (&wv)[9], int coff, bool sync_after = true) {
#pragma unroll
        for (int k = 0; k < XI; ++k) {
            if (xoff[k] >= 0) {
                const int c = xc[k];
                if (c >= 0 && c < IW) *reinterpret_cast<intx4*>(lx + xlds[k] + coff) = xgather_px<0>(xv[k]);
                if (c + 1 >= 0 && c + 1 < IW) *reinterpret_cast<intx4*>(lx + xlds[k] + coff + kPitch) = xgather_px<1>(xv[k]);
                if (c + 2 >= 0 && c + 2 < IW) *reinterpret_cast<intx4*>(lx + xlds[k] + coff + 2 * kPitch) = xgather_px<2>(xv[k]);
                if (c + 3 >= 0 && c + 3 < IW) *reinterpret_cast<intx4*>(lx + xlds[k] + coff + 3 * kPitch) = xgather_px<3>(xv[k]);
            }
        }
#pragma unroll
        for (int i = 0; i < 9; ++i) *reinterpret_cast<intx4*>(lraw + (wave * 576 + i * 64 + lane) * 16) = wv[i];
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // this wavefront's raw pieces are in LDS
        u32 raw[36];
#pragma unroll
        for (int i = 0; i < 9; ++i) {
            const intx4 v = *reinterpret_cast<const intx4*>(lraw + (wco * 4 + wc16) * 144 + 16 * i);
            raw[4 * i + 0] = (u32)v.x; raw[4 * i + 1] = (u32)v.y; raw[4 * i + 2] = (u32)v.z; raw[4 * i + 3] = (u32)v.w;
        }
        unsigned char* wdst = lw + wco * kPitch + 16 * wc16 + coff;
        *reinterpret_cast<intx4*>(wdst + 0 * 64 * kPitch) = wgather_tap<0>(raw);
        *reinterpret_cast<intx4*>(wdst + 1 * 64 * kPitch) = wgather_tap<1>(raw);
        *reinterpret_cast<intx4*>(wdst + 2 * 64 * kPitch) = wgather_tap<2>(raw);
        *reinterpret_cast<intx4*>(wdst + 3 * 64 * kPitch) = wgather_tap<3>(raw);
        *reinterpret_cast<intx4*>(wdst + 4 * 64 * kPitch) = wgather_tap<4>(raw);
        *reinterpret_cast<intx4*>(wdst + 5 * 64 * kPitch) = wgather_tap<5>(raw);
        *reinterpret_cast<intx4*>(wdst + 6 * 64 * kPitch) = wgather_tap<6>(raw);
        *reinterpret_cast<intx4*>(wdst + 7 * 64 * kPitch) = wgather_tap<7>(raw);
        *reinterpret_cast<intx4*>(wdst + 8 * 64 * kPitch) = wgather_tap<8>(raw);
        if (sync_after) __syncthreads();
    };
    // 18 steps (9 taps x 2 K halves); the operands of step t+1 are read from LDS while step t multiplies
    auto load_step = [&](int step, intx4& a, intx4 (&bv)[kNBW]) {
        const int tap = step >> 1, kk = step & 1;
        const int r = tap / 3, q = tap - 3 * r;
        const int toff = (r * IW + q) * kPitch + 32 * kk;
        a = *reinterpret_cast<const intx4*>(lw + aoff + tap * 64 * kPitch + 32 * kk);
#pragma unroll
        for (int i = 0; i < kNBW; ++i) bv[i] = *reinterpret_cast<const intx4*>(lx + boff[i] + toff);
    };
    auto multiply = [&]() {
        intx4 a[2];
        intx4 bv[2][kNBW];
        load_step(0, a[0], bv[0]);
#pragma unroll
        for (int step = 0; step < 18; ++step) {
            const int cur = step & 1;
            if (step + 1 < 18) load_step(step + 1, a[cur ^ 1], bv[cur ^ 1]);
            __builtin_amdgcn_sched_barrier(0);      // keep the reads ahead of the multiplications
#pragma unroll
            for (int i = 0; i < kNBW; ++i)
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[cur], bv[cur][i], acc[i], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    };

    const int HoWo = Ho * Wo;
    if constexpr (RES != 0) {
        constexpr int KS = RES / 32;            // K steps per tap
        constexpr int NSTEP = 9 * KS;
        fetch(xv0, wv0, 0, false);
        fetch(xv1, wv1, kCK, false);
        zero_window();
        stage(xv0, wv0, 0, false);
        stage(xv1, wv1, kCK);
        intx4 a[NSTEP];    // this wavefront's A operands for the whole K range
#pragma unroll
        for (int st = 0; st < NSTEP; ++st)
            a[st] = *reinterpret_cast<const intx4*>(lw + aoff + (st / KS) * 64 * kPitch + 32 * (st % KS));
        const int co_base = (mb << 6) + 32 * wm + 4 * lg;       // this lane's first output channel
        const int64_t ybase = ((int64_t)n * C_out + co_base) * HoWo;
        auto b_at = [&](int i, int st) {
            const int tap = st / KS, kk = st % KS;
            const int r = tap / 3, q = tap - 3 * r;
            return *reinterpret_cast<const intx4*>(lx + boff[i] + (r * IW + q) * kPitch + 32 * kk);
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
            // exchange 1, partner lane ^ 1: keep the channels whose bit 0 is this lane's bit 0
            const bool b0 = k & 1, b1 = k & 2;
            const int keep01 = b0 ? r[1] : r[0], send01 = b0 ? r[0] : r[1];
            const int keep23 = b0 ? r[3] : r[2], send23 = b0 ? r[2] : r[3];
            const int got01 = __builtin_amdgcn_mov_dpp(send01, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
            const int got23 = __builtin_amdgcn_mov_dpp(send23, 0xB1, 0xF, 0xF, true);
            // now (keep01, got01) = channel b0 of pixels (k, k^1), (keep23, got23) = channel 2 + b0 of the same
            // exchange 2, partner lane ^ 2: keep the pair whose channel has this lane's bit 1
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
        // Pair 0 (blocks 0, 1), then pair 1 (blocks 2, 3) with the 32 stores of pair 0 spread between its
        // matrix instructions, then the stores of pair 1.
        const int live = __builtin_amdgcn_readfirstlane(min(kNBW, (tile_px - wn * kNBW * 32 + 31) >> 5));
        intx16 c0, c1, d0, d1;
#pragma unroll
        for (int v = 0; v < 16; ++v) { c0[v] = 0; c1[v] = 0; d0[v] = 0; d1[v] = 0; }
        if (live >= 1) {
            intx4 b0[2], b1[2];
            b0[0] = b_at(0, 0); b1[0] = b_at(1, 0);
#pragma unroll
            for (int st = 0; st < NSTEP; ++st) {
                const int cur = st & 1;
                if (st + 1 < NSTEP) { b0[cur ^ 1] = b_at(0, st + 1); b1[cur ^ 1] = b_at(1, st + 1); }
                __builtin_amdgcn_sched_barrier(0);
                c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[st], b0[cur], c0, 0, 0, 0);
                c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[st], b1[cur], c1, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        const int dst0 = live >= 1 ? block_dst(0) : -1;
        const int dst1 = live >= 2 ? block_dst(1) : -1;
        if (live >= 3) {
            intx4 b0[2], b1[2];
            b0[0] = b_at(2, 0); b1[0] = b_at(3, 0);
#pragma unroll
            for (int st = 0; st < NSTEP; ++st) {
                const int cur = st & 1;
                if (st + 1 < NSTEP) { b0[cur ^ 1] = b_at(2, st + 1); b1[cur ^ 1] = b_at(3, st + 1); }
                if (st >= 2 && st < 18) store_reg(dst0, c0, st - 2);
                if (st >= 18 && st < 34) store_reg(dst1, c1, st - 18);
                __builtin_amdgcn_sched_barrier(0);
                d0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[st], b0[cur], d0, 0, 0, 0);
                d1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[st], b1[cur], d1, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            const int dst2 = block_dst(2);
            const int dst3 = live >= 4 ? block_dst(3) : -1;
#pragma unroll
            for (int v = 0; v < 16; ++v) store_reg(dst2, d0, v);
#pragma unroll
            for (int v = 0; v < 16; ++v) store_reg(dst3, d1, v);
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) store_reg(dst0, c0, v);
#pragma unroll
            for (int v = 0; v < 16; ++v) store_reg(dst1, c1, v);
        }
        return;
    }

    const int chunks = C_in / kCK;
    fetch(xv0, wv0, 0);
    if (chunks > 1) fetch(xv1, wv1, kCK);
    zero_window();
    for (int ch = 0; ch < chunks; ch += 2) {
        stage(xv0, wv0, 0);
        if (ch + 2 < chunks) fetch(xv0, wv0, (ch + 2) * kCK);
        multiply();
        if (ch + 1 < chunks) {
            stage(xv1, wv1, 0);
            if (ch + 3 < chunks) fetch(xv1, wv1, (ch + 3) * kCK);
            multiply();
        }
    }

    // ---- store: register v of a lane is channel 8*(v/4) + 4*lg + v%4 of the block, pixel lj ---------
    if (P.wide_store) {
        // Full-width tiles: the tile of one channel is one contiguous run of y.  The accumulators go
        // through LDS ([channel][pixel]; the operands are dead by now) and leave as 16-byte stores.
        const int valid_px = min(TH, Ho - row0) * Wo;          // multiple of 4
        const int pitch = tile_px + 4;
        int* lo = reinterpret_cast<int*>(smem);
#pragma unroll
        for (int i = 0; i < kNBW; ++i) {
            const int p = (wn * kNBW + i) * 32 + lj;
            if (p < tile_px) {
#pragma unroll
                for (int v = 0; v < 16; ++v) lo[(32 * wm + 8 * (v >> 2) + 4 * lg + (v & 3)) * pitch + p] = acc[i][v];
            }
        }
        __syncthreads();
        const int pieces = valid_px >> 2;                       // 16-byte pieces per channel
        int32_t* yt = y + ((int64_t)n * C_out + (mb << 6)) * HoWo + row0 * Wo;
        for (int idx = tid; idx < 64 * (int)P.by_pieces.d; idx += 256) {
            const int c = fast_div(idx, P.by_pieces);
            const int q = idx - c * (int)P.by_pieces.d;
            if (q < pieces)
                *reinterpret_cast<intx4*>(yt + (int64_t)c * HoWo + 4 * q) = *reinterpret_cast<const intx4*>(lo + c * pitch + 4 * q);
        }
        return;
    }
    const int co0 = (mb << 6) + 32 * wm + 4 * lg;
    int32_t* yn = y + ((int64_t)n * C_out + co0) * HoWo;
#pragma unroll
    for (int i = 0; i < kNBW; ++i) {
        const int p = (wn * kNBW + i) * 32 + lj;
        const int pi = fast_div(p, P.by_TW), pj = p - pi * TW;
        const int oi = row0 + pi, oj = col0 + pj;
        if (p < tile_px && oi < Ho && oj < Wo) {
            int32_t* dst = yn + oi * Wo + oj;
#pragma unroll
            for (int v = 0; v < 16; ++v) dst[(8 * (v >> 2) + (v & 3)) * HoWo] = acc[i][v];
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
    auto even = [&](int th) { const int bands = (s.Ho + th - 1) / th; return (s.Ho + bands - 1) / bands; };
    auto fits = [&](int th) {
        const int IH = th + 2, IW = t.TW + 2;
        const int nq_max = std::min((IW + 2) / 4 + 1, s.W / 4);   // column quads a window can touch
        return IH * IW <= kLdsPx && 4 * IH * nq_max <= kXItems * 256;
    };
    while (t.TH > 1 && !fits(t.TH)) --t.TH;
    t.TH = even(t.TH);      // equal row bands: same tile count, no nearly empty last band
    t.tiles_x = (s.Wo + t.TW - 1) / t.TW;
    t.tiles_y = (s.Ho + t.TH - 1) / t.TH;
    return t;
}

bool tiling_ok(const Conv2dShape& s, const Tiling& t)
{
    const int IH = t.TH + 2, IW = t.TW + 2;
    const int nq_max = std::min((IW + 2) / 4 + 1, s.W / 4);
    return t.TH >= 1 && t.TH * t.TW <= kTilePx && IH * IW <= kLdsPx && 4 * IH * nq_max <= kXItems * 256 &&
           (int64_t)t.tiles_x * t.tiles_y <= 65535 && s.C_out / 64 <= 65535 && s.N <= 65535;
}

}  // namespace

bool mfma_s8_supported(const Conv2dShape& s)
{
    if (s.stride != 1 || s.R != 3 || s.S != 3) return false;
    if (s.C_in % kCK != 0 || s.C_out % 64 != 0 || s.W % 4 != 0) return false;
    if ((int64_t)s.C_in * s.H * s.W > 2147483647LL) return false;
    return tiling_ok(s, pick_tiling(s));
}

hipError_t launch_mfma_s8(const int8_t* x, const int8_t* w, int32_t* y, const Conv2dShape& s, hipStream_t st)
{
    // the vectorised staging reads 4-byte groups of x and 16-byte groups of w
    if (reinterpret_cast<uintptr_t>(x) % 4 != 0 || reinterpret_cast<uintptr_t>(w) % 16 != 0)
        return launch_direct_conv2d_s8(x, w, y, s, st);
    static const hipError_t attr = [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_s8_kernel<0, 1>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_s8_kernel<0, 2>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_s8_kernel<128, 1>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesRes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_s8_kernel<128, 2>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesRes);
        return e;
    }();
    if (attr != hipSuccess) return attr;
    const Tiling t = pick_tiling(s);
    S8Params P;
    P.C_in = s.C_in; P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.pad = s.pad; P.Ho = s.Ho; P.Wo = s.Wo;
    P.TH = t.TH; P.TW = t.TW;
    P.nq_max = std::min((t.TW + 2 + 2) / 4 + 1, s.W / 4);
    // 16-byte stores need full-width tiles whose runs of y start and end on 16-byte boundaries
    P.wide_store = t.tiles_x == 1 && s.Wo % 4 == 0 && reinterpret_cast<uintptr_t>(y) % 16 == 0 &&
                   64 * (t.TH * t.TW + 4) * 4 <= kLdsBytes;   // (chunked variant only)
    P.by_tiles_x = make_fastdiv(t.tiles_x);
    P.by_TW = make_fastdiv(t.TW);
    P.by_IH = make_fastdiv(t.TH + 2);
    P.by_nq_max = make_fastdiv(P.nq_max);
    P.by_pieces = make_fastdiv(t.TH * s.Wo / 4 > 0 ? t.TH * s.Wo / 4 : 1);
    dim3 grid((unsigned)(t.tiles_x * t.tiles_y), (unsigned)s.N, (unsigned)(s.C_out / 64));
    const bool one_item = 4 * (t.TH + 2) * P.nq_max <= 256;
    const bool resident = s.C_in == 128 && (t.TH + 2) * (t.TW + 2) <= kLdsPxRes;
    if (resident && one_item)
        SW_NOTED_LAUNCH(note_kernel("mfma_s8_kernel", (int)(128), (int)(1)), (mfma_s8_kernel<128, 1>), grid, dim3(256), kLdsBytesRes, st, x, w, y, P);
    else if (resident)
        SW_NOTED_LAUNCH(note_kernel("mfma_s8_kernel", (int)(128), (int)(2)), (mfma_s8_kernel<128, 2>), grid, dim3(256), kLdsBytesRes, st, x, w, y, P);
    else if (one_item)
        SW_NOTED_LAUNCH(note_kernel("mfma_s8_kernel", (int)(0), (int)(1)), (mfma_s8_kernel<0, 1>), grid, dim3(256), kLdsBytes, st, x, w, y, P);
    else
        SW_NOTED_LAUNCH(note_kernel("mfma_s8_kernel", (int)(0), (int)(2)), (mfma_s8_kernel<0, 2>), grid, dim3(256), kLdsBytes, st, x, w, y, P);
    return hipGetLastError();
}

bool mfma_s8_requant_supported(const Conv2dShape& s)
{
    if (!mfma_s8_supported(s) || s.C_in != 128) return false;
    const Tiling t = pick_tiling(s);
    return (t.TH + 2) * (t.TW + 2) <= kLdsPxRes;
}

hipError_t launch_mfma_s8_requant(const int8_t* x, const int8_t* w, int8_t* y8, const Requant& rq, const Conv2dShape& s,
                                  hipStream_t st)
{
    if (reinterpret_cast<uintptr_t>(x) % 4 != 0 || reinterpret_cast<uintptr_t>(w) % 16 != 0)
        return launch_mfma_s8_any_requant(x, w, y8, rq, s, st);
    static const hipError_t attr = [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_s8_kernel<128, 1, true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesRes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_s8_kernel<128, 2, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesRes);
        return e;
    }();
    if (attr != hipSuccess) return attr;
    const Tiling t = pick_tiling(s);
    S8Params P;
    P.C_in = s.C_in; P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.pad = s.pad; P.Ho = s.Ho; P.Wo = s.Wo;
    P.TH = t.TH; P.TW = t.TW;
    P.nq_max = std::min((t.TW + 2 + 2) / 4 + 1, s.W / 4);
    // dword stores of four requantised pixels: groups of four pixels must be aligned dwords of y8
    P.wide_store = s.Wo % 4 == 0 && t.TW % 4 == 0 && reinterpret_cast<uintptr_t>(y8) % 4 == 0;
    P.by_tiles_x = make_fastdiv(t.tiles_x);
    P.by_TW = make_fastdiv(t.TW);
    P.by_IH = make_fastdiv(t.TH + 2);
    P.by_nq_max = make_fastdiv(P.nq_max);
    P.by_pieces = make_fastdiv(1);
    dim3 grid((unsigned)(t.tiles_x * t.tiles_y), (unsigned)s.N, (unsigned)(s.C_out / 64));
    int32_t* none = nullptr;
    if (4 * (t.TH + 2) * P.nq_max <= 256)
        SW_NOTED_LAUNCH(note_kernel("mfma_s8_kernel", (int)(128), (int)(1), (int)(true)), (mfma_s8_kernel<128, 1, true>), grid, dim3(256), kLdsBytesRes, st, x, w, none, P, y8, rq);
    else
        SW_NOTED_LAUNCH(note_kernel("mfma_s8_kernel", (int)(128), (int)(2), (int)(true)), (mfma_s8_kernel<128, 2, true>), grid, dim3(256), kLdsBytesRes, st, x, w, none, P, y8, rq);
    return hipGetLastError();
}

}  // namespace swconv
