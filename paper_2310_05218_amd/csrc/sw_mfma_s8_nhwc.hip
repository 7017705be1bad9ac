// Quantised multi-channel convolution on channel-last tensors: int8 x int8 -> exact int32 (or requantised int8),
// any filter extent and stride, on the matrix cores (paper, sections 1.1 and 3: quantisation applied to the
// sliding formulation; taps as small matrix products).
//
//   x [N, H, W, C_in] int8     w [C_out, R, S, C_in] int8     y [N, H_out, W_out, C_out] int32 / int8
//
// v_mfma_i32_32x32x32_i8 wants 16 consecutive K bytes per lane.  With the channel as the fastest axis of both
// tensors those 16 bytes are 16 consecutive bytes of memory, so nothing is transposed on the way: a workgroup
// copies the rows of the input that its outputs touch and the filters of its 64 output channels into LDS with
// plain 16-byte loads (every load is issued before the first LDS write: one memory round trip), and all of K
// stays resident.  Every tap (r, s) then contributes W_rs[co, ci] times the window shifted by (r, s): the shift is
// an address offset, no column matrix exists.
//
// Workgroup = 4 wavefronts = 64 output channels x a band of TH output rows of one image, taken as up to 8 blocks
// of 32 consecutive output pixels (row-major, so a block may span rows: each lane computes its own pixel's window
// address).  A = pixels (32 x 32 K), B = filters (32 K x 32 channels): a lane of the result holds one output
// channel for 16 pixels, so every store instruction writes runs of 32 consecutive channels, the fastest axis of
// the output.  LDS pitches: a pixel takes C_in + 16 bytes, an output channel's filters R*S*C_in + 16 (+ what makes
// that 16 modulo 128): the 16-byte operand reads of 8 consecutive pixels (channels) then fall into distinct banks.
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx16 __attribute__((ext_vector_type(16)));

constexpr int kMaxBlocks = 8;          // 32-pixel blocks per workgroup
constexpr int kBlocksPerWave = 4;      // a wavefront takes every second block of one 32-channel half
constexpr int kLdsBudgetNhwc = 156 * 1024;
constexpr int kXSlots = 12;            // 16-byte pieces of the window per thread
constexpr int kWSlots = 24;            // 16-byte pieces of the filters per thread

struct NhwcParams {
    int H, W, C_in, C_out, R, S, stride, pad, Ho, Wo;
    int TH, IH, IWp;                   // output rows per band; window rows and columns in LDS
    int CP, WPITCH;                    // bytes per pixel / per output channel's filters in LDS
    int c16;                           // 16-byte pieces per pixel (C_in / 16)
    int wrow16;                        // 16-byte pieces per output channel's filters (R * S * C_in / 16)
    int x_bytes;                       // window bytes in LDS (filters follow)
    FastDiv by_c16, by_IWp, by_wrow16, by_Wo;
};

// RQ: the sums leave requantised to int8 (y8) instead of as int32 (y).
// KS: K steps of 32 channels per tap (C_in / 32) when that is 1, 2 or 4; 0: any multiple of 32, at run time.
template <bool RQ, int KS>
__global__ __launch_bounds__(256, 1) void mfma_s8_nhwc_kernel(const int8_t* __restrict__ x,
                                                              const int8_t* __restrict__ w,
                                                              int32_t* __restrict__ y, int8_t* __restrict__ y8,
                                                              const NhwcParams P, const Requant rq)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* lx = smem;                 // [window row][window column][ci], pitch CP
    unsigned char* lw = smem + P.x_bytes;     // [co][tap][ci], pitch WPITCH
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lg = lane >> 5, lj = lane & 31;          // K half; pixel (A) or channel (B, D) inside a block
    const int band = blockIdx.x, n = blockIdx.y, cb = blockIdx.z;
    const int oi0 = band * P.TH;                        // first output row of the band
    const int rows = min(P.TH, P.Ho - oi0);
    const int npix = rows * P.Wo;                       // output pixels of this band
    const int co0 = cb * 64;

    // ---- global -> registers: every piece of the window and of the filters, before any LDS write ----
    const int gr0 = oi0 * P.stride - P.pad;             // image row / column of window position (0, 0)
    const int gc0 = -P.pad;
    const int n_x = P.IH * P.IWp * P.c16;
    const int8_t* xn = x + (int64_t)n * P.H * P.W * P.C_in;
    intx4 xv[kXSlots];
    int xdst[kXSlots];
#pragma unroll
    for (int u = 0; u < kXSlots; ++u) {
        const int idx = tid + 256 * u;
        const int pix = fast_div(idx, P.by_c16);
        const int c = idx - pix * P.c16;
        const int e = fast_div(pix, P.by_IWp), f = pix - e * P.IWp;
        const int gr = gr0 + e, gc = gc0 + f;
        xdst[u] = idx < n_x ? pix * P.CP + 16 * c : -1;
        xv[u] = intx4{0, 0, 0, 0};                      // outside the image: the zero padding
        if (idx < n_x && gr >= 0 && gr < P.H && gc >= 0 && gc < P.W)
            xv[u] = *reinterpret_cast<const intx4*>(xn + ((int64_t)gr * P.W + gc) * P.C_in + 16 * c);
    }
    const int n_w = 64 * P.wrow16;
    const int8_t* wb = w + (int64_t)co0 * P.wrow16 * 16;
    intx4 wv[kWSlots];
    int wdst[kWSlots];
#pragma unroll
    for (int u = 0; u < kWSlots; ++u) {
        const int idx = tid + 256 * u;
        const int co = fast_div(idx, P.by_wrow16);
        const int q = idx - co * P.wrow16;
        wdst[u] = idx < n_w ? co * P.WPITCH + 16 * q : -1;
        wv[u] = intx4{0, 0, 0, 0};                      // channels beyond C_out: zero filters
        if (idx < n_w && co0 + co < P.C_out) wv[u] = *reinterpret_cast<const intx4*>(wb + (int64_t)idx * 16);
    }
#pragma unroll
    for (int u = 0; u < kXSlots; ++u)
        if (xdst[u] >= 0) *reinterpret_cast<intx4*>(lx + xdst[u]) = xv[u];
#pragma unroll
    for (int u = 0; u < kWSlots; ++u)
        if (wdst[u] >= 0) *reinterpret_cast<intx4*>(lw + wdst[u]) = wv[u];
    __syncthreads();

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
    intx16 acc[kBlocksPerWave];
#pragma unroll
    for (int b = 0; b < kBlocksPerWave; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0;

    // Operands of one tap: KS K steps, the filter block and the wavefront's pixel blocks.  The operands of the
    // next tap are on their way from LDS while the matrix instructions of this one run (two register sets, the
    // tap loop unrolled by two); KS == 0: K steps at run time, read and multiplied one after the other.
    struct Ops {
        intx4 bq[KS > 0 ? KS : 1];
        intx4 aq[KS > 0 ? KS : 1][kBlocksPerWave];
    };
    int tap_x = 0, tap_w = 0, s = 0;                    // byte offsets of the tap in the window / in a filter row
    auto next_tap = [&]() __attribute__((always_inline)) {
        tap_w += P.C_in;
        tap_x += P.CP;
        if (++s == P.S) { s = 0; tap_x += (P.IWp - P.S) * P.CP; }
    };
    auto load_ops = [&](Ops& o) __attribute__((always_inline)) {
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
                if (wp + 2 * b < nblocks)               // (wave-uniform)
                    acc[b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(o.aq[k][b], o.bq[k], acc[b], 0, 0, 0);
    };
    const int RS = P.R * P.S;
    if constexpr (KS > 0) {
        Ops o0, o1;
        load_ops(o0);
        int tap = 0;
#pragma unroll 1
        for (; tap + 2 <= RS; tap += 2) {
            next_tap();
            load_ops(o1);
            __builtin_amdgcn_sched_barrier(0);
            multiply(o0);
            __builtin_amdgcn_sched_barrier(0);
            if (tap + 2 < RS) {
                next_tap();
                load_ops(o0);
            }
            __builtin_amdgcn_sched_barrier(0);
            multiply(o1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (tap < RS) multiply(o0);                     // odd tap count: the last tap is already in o0
    } else {
        const int ksteps = P.C_in >> 5;
#pragma unroll 1
        for (int tap = 0; tap < RS; ++tap) {
#pragma unroll 1
            for (int k = 0; k < ksteps; ++k) {
                const intx4 bq = *reinterpret_cast<const intx4*>(bsrc + tap_w + 32 * k);
                intx4 aq[kBlocksPerWave];
#pragma unroll
                for (int b = 0; b < kBlocksPerWave; ++b)
                    aq[b] = *reinterpret_cast<const intx4*>(lx + aoff[b] + tap_x + 32 * k);
#pragma unroll
                for (int b = 0; b < kBlocksPerWave; ++b)
                    if (wp + 2 * b < nblocks)
                        acc[b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aq[b], bq, acc[b], 0, 0, 0);
            }
            next_tap();
        }
    }

    // ---- store: register v of a lane is pixel 8*(v/4) + 4*lg + v%4 of the block, channel lj ----
    const int co = co0 + 32 * wn + lj;
    const int64_t pix0 = ((int64_t)n * P.Ho + oi0) * P.Wo;
    if constexpr (!RQ) {
        if (co >= P.C_out) return;
#pragma unroll
        for (int b = 0; b < kBlocksPerWave; ++b) {
            if (wp + 2 * b >= nblocks) break;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int p = 32 * (wp + 2 * b) + 8 * (v >> 2) + 4 * lg + (v & 3);
                if (p < npix) y[(pix0 + p) * P.C_out + co] = acc[b][v];
            }
        }
    } else {
        // int8 output: a lane holds one channel of four consecutive pixels in registers 4g .. 4g+3, and its bytes
        // lie a whole pixel apart in memory.  Two exchanges inside each lane quad (DPP quad_perm) transpose the
        // 4 x 4 block, so that lane k ends up with pixel k of the quad's four consecutive channels and stores them
        // as one dword.  (All lanes take part; lanes past C_out or past the band only skip the store.)
        const int cl = co < P.C_out ? co : P.C_out - 1;
        const bool wide = P.C_out % 4 == 0 && reinterpret_cast<uintptr_t>(y8) % 4 == 0;
        const int k = lane & 3;
        const bool b0 = k & 1, b1 = k & 2;
        const int cq = co0 + 32 * wn + (lj & ~3);               // first channel of the quad
#pragma unroll
        for (int b = 0; b < kBlocksPerWave; ++b) {
            if (wp + 2 * b >= nblocks) break;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int p0 = 32 * (wp + 2 * b) + 8 * g + 4 * lg;   // pixel of register 4g
                int r[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) r[t] = (int)requant_s8(acc[b][4 * g + t], cl, rq) & 255;
                if (wide) {
                    const int keep01 = b0 ? r[1] : r[0], send01 = b0 ? r[0] : r[1];
                    const int keep23 = b0 ? r[3] : r[2], send23 = b0 ? r[2] : r[3];
                    const int got01 = __builtin_amdgcn_mov_dpp(send01, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
                    const int got23 = __builtin_amdgcn_mov_dpp(send23, 0xB1, 0xF, 0xF, true);
                    const int own_a = b1 ? keep23 : keep01, own_b = b1 ? got23 : got01;
                    const int snd_a = b1 ? keep01 : keep23, snd_b = b1 ? got01 : got23;
                    const int far_a = __builtin_amdgcn_mov_dpp(snd_a, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
                    const int far_b = __builtin_amdgcn_mov_dpp(snd_b, 0x4E, 0xF, 0xF, true);
                    // pixel k of the channels of lanes k, k^1, k^2, k^3: byte j of the dword is the quad's channel j
                    const unsigned word = (unsigned)own_a << (8 * k) | (unsigned)own_b << (8 * (k ^ 1)) |
                                          (unsigned)far_a << (8 * (k ^ 2)) | (unsigned)far_b << (8 * (k ^ 3));
                    if (p0 + k < npix && cq < P.C_out)
                        *reinterpret_cast<unsigned*>(y8 + (pix0 + p0 + k) * P.C_out + cq) = word;
                } else if (co < P.C_out) {
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        if (p0 + t < npix) y8[(pix0 + p0 + t) * P.C_out + co] = (int8_t)r[t];
                }
            }
        }
    }
}

// One thread per output, any shape: the channel loop runs over contiguous bytes of both tensors.
template <bool RQ>
__global__ __launch_bounds__(256) void direct_s8_nhwc_kernel(const int8_t* __restrict__ x, const int8_t* __restrict__ w,
                                                             int32_t* __restrict__ y, int8_t* __restrict__ y8,
                                                             Conv2dShape s, Requant rq)
{
    const int64_t total = (int64_t)s.N * s.Ho * s.Wo * s.C_out;
    for (int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (int64_t)gridDim.x * 256) {
        const int co = (int)(o % s.C_out);
        int64_t t = o / s.C_out;
        const int oj = (int)(t % s.Wo);
        t /= s.Wo;
        const int oi = (int)(t % s.Ho);
        const int n = (int)(t / s.Ho);
        int acc = 0;
        for (int r = 0; r < s.R; ++r) {
            const int h = oi * s.stride + r - s.pad;
            if (h < 0 || h >= s.H) continue;
            for (int q = 0; q < s.S; ++q) {
                const int v = oj * s.stride + q - s.pad;
                if (v < 0 || v >= s.W) continue;
                const int8_t* xp = x + (((int64_t)n * s.H + h) * s.W + v) * s.C_in;
                const int8_t* wp = w + (((int64_t)co * s.R + r) * s.S + q) * s.C_in;
                for (int ci = 0; ci < s.C_in; ++ci) acc += (int)xp[ci] * (int)wp[ci];
            }
        }
        if (RQ) y8[o] = requant_s8(acc, co, rq);
        else y[o] = acc;
    }
}

struct NhwcPlan {
    NhwcParams P;
    size_t lds;
    int bands;
    bool ok;
};

NhwcPlan plan_nhwc(const Conv2dShape& s)
{
    NhwcPlan a{};
    NhwcParams& P = a.P;
    if (s.C_in % 32 != 0 || s.dil != 1) return a;
    const int RS = s.R * s.S;
    P.H = s.H; P.W = s.W; P.C_in = s.C_in; P.C_out = s.C_out; P.R = s.R; P.S = s.S; P.stride = s.stride;
    P.pad = s.pad; P.Ho = s.Ho; P.Wo = s.Wo;
    P.CP = s.C_in + 16;
    const int wrow = RS * s.C_in;
    P.WPITCH = wrow + 16 + (128 - wrow % 128) % 128;
    P.c16 = s.C_in / 16;
    P.wrow16 = wrow / 16;
    P.IWp = (s.Wo - 1) * s.stride + s.S;
    if ((int64_t)64 * P.wrow16 > 256 * kWSlots) return a;          // the filters of 64 channels in one round trip
    // output rows per band: as many as the pixel blocks, the staging slots and LDS allow
    int TH = (kMaxBlocks * 32) / s.Wo;
    if (TH > s.Ho) TH = s.Ho;
    for (; TH >= 1; --TH) {
        const int IH = (TH - 1) * s.stride + s.R;
        const int64_t xb = (int64_t)IH * P.IWp * P.CP;
        if ((int64_t)IH * P.IWp * P.c16 <= 256 * kXSlots && xb + (int64_t)64 * P.WPITCH <= kLdsBudgetNhwc) break;
    }
    if (TH < 1) return a;
    // equal bands
    const int bands = (s.Ho + TH - 1) / TH;
    TH = (s.Ho + bands - 1) / bands;
    P.TH = TH;
    P.IH = (TH - 1) * s.stride + s.R;
    P.x_bytes = (P.IH * P.IWp * P.CP + 15) & ~15;
    a.lds = (size_t)P.x_bytes + (size_t)64 * P.WPITCH;
    a.bands = (s.Ho + TH - 1) / TH;
    P.by_c16 = make_fastdiv(P.c16);
    P.by_IWp = make_fastdiv(P.IWp);
    P.by_wrow16 = make_fastdiv(P.wrow16);
    P.by_Wo = make_fastdiv(s.Wo);
    a.ok = a.lds <= (size_t)kLdsBudgetNhwc && a.bands <= 2147483647 && s.N <= 65535 && (s.C_out + 63) / 64 <= 65535 &&
           // 32-bit offsets inside one image and inside the filters of 64 channels
           (int64_t)s.H * s.W * s.C_in <= 2147483647LL && (int64_t)TH * s.Wo <= kMaxBlocks * 32;
    return a;
}

template <bool RQ, int KS>
hipError_t launch_nhwc_ks(const int8_t* x, const int8_t* w, int32_t* y, int8_t* y8, const Requant& rq, const NhwcPlan& a,
                          const Conv2dShape& s, hipStream_t st)
{
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_s8_nhwc_kernel<RQ, KS>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudgetNhwc);
    if (attr != hipSuccess) return attr;
    dim3 grid((unsigned)a.bands, (unsigned)s.N, (unsigned)((s.C_out + 63) / 64));
    SW_NOTED_LAUNCH(note_kernel("mfma_s8_nhwc_kernel", (int)(RQ), (int)(KS)), (mfma_s8_nhwc_kernel<RQ, KS>), grid, dim3(256), a.lds, st, x, w, y, y8, a.P, rq);
    return hipGetLastError();
}

template <bool RQ>
hipError_t launch_nhwc(const int8_t* x, const int8_t* w, int32_t* y, int8_t* y8, const Requant& rq, const NhwcPlan& a,
                       const Conv2dShape& s, hipStream_t st)
{
    switch (s.C_in / 32) {
        case 1: return launch_nhwc_ks<RQ, 1>(x, w, y, y8, rq, a, s, st);
        case 2: return launch_nhwc_ks<RQ, 2>(x, w, y, y8, rq, a, s, st);
        case 4: return launch_nhwc_ks<RQ, 4>(x, w, y, y8, rq, a, s, st);
        default: return launch_nhwc_ks<RQ, 0>(x, w, y, y8, rq, a, s, st);
    }
}

}  // namespace

bool mfma_s8_nhwc_supported(const int8_t* x, const int8_t* w, const Conv2dShape& s)
{
    return reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 && plan_nhwc(s).ok;
}

hipError_t launch_mfma_s8_nhwc(const int8_t* x, const int8_t* w, int32_t* y, int8_t* y8, const Requant* rq,
                               const Conv2dShape& s, hipStream_t st)
{
    const NhwcPlan a = plan_nhwc(s);
    if (!a.ok) return hipErrorInvalidValue;
    if (rq) return launch_nhwc<true>(x, w, y, y8, *rq, a, s, st);
    return launch_nhwc<false>(x, w, y, y8, Requant{nullptr, nullptr, 0}, a, s, st);
}

hipError_t launch_direct_s8_nhwc(const int8_t* x, const int8_t* w, int32_t* y, int8_t* y8, const Requant* rq,
                                 const Conv2dShape& s, hipStream_t st)
{
    const int64_t total = (int64_t)s.N * s.Ho * s.Wo * s.C_out;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    if (rq)
        SW_NOTED_LAUNCH(note_kernel("direct_s8_nhwc_kernel", (int)(true)), direct_s8_nhwc_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, x, w, y, y8, s, *rq);
    else
        SW_NOTED_LAUNCH(note_kernel("direct_s8_nhwc_kernel", (int)(false)), direct_s8_nhwc_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, x, w, y, y8, s,
                           Requant{nullptr, nullptr, 0});
    return hipGetLastError();
}

}  // namespace swconv
