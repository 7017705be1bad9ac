// The any-shape fp32 matrix-core kernel for filters of few taps (1x1, 2x2, 3x3, ...: R * S * CK <= 96 with
// channel chunks CK of 8, 16 or 32): same decomposition as sw_mfma_f32_any.hip -- 64 output channels x up to
// 128 output pixels per workgroup, per-tap products on v_mfma_f32_32x32x2_f32, the tap shift and the stride
// as LDS addresses of the B operand (paper, section 3) -- with operands laid out so that ONE 16-byte LDS read
// feeds four matrix steps:
//   input window  [channel quad][pixel]        floatx4 = four channels of one pixel
//   filters       [tap][channel quad][co]      floatx4 = four input channels of one (tap, output channel)
// and the K index of the four steps permuted to match (step t of K lane kk <-> channel 4 kk + t of a group of
// eight), which the matrix instruction allows because both operands use the same map.  A tap costs three LDS
// reads per eight matrix instructions, and the reads of the next tap are issued before this tap's matrix
// instructions.  Staging gathers the four channels of an item with four loads (consecutive lanes: consecutive
// pixels / taps) and writes one 16-byte group; the next chunk is prefetched into registers while this one
// multiplies.  No alignment of x or w is needed; channels beyond C_in and C_out are zero-filled.
#include "swconv_internal.h"

#include <cstdlib>

namespace swconv {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kTilePx = 128;           // output pixels per workgroup: one 32-pixel block per wavefront
constexpr int kLdsBudget = 64 * 1024;
constexpr int kXS = 4;                 // staging items per thread: input window (16-byte groups) ...
constexpr int kWS = 6;                 // ... and filters

struct QuadParams {
    Epilogue ep;                       // bias and rectifier applied in the store
    int C_in, C_out, H, W, R, S, stride, pad, Ho, Wo;
    int TH, TW, IH, IW, tiles_x;
    FastDiv by_tiles_x, by_TW, by_IW, by_win, by_RS, by_QRS;
};

// SPLIT: the workgroup has eight wavefronts, four that only multiply and four that only load.  A wavefront that
// issues the loads of the next chunk sits in their issue until the memory system has taken them (thousands of cycles
// when the launch runs at the HBM rate); in a wavefront of its own that wait holds no matrix instruction back.  The
// loaders copy chunk c + 1 into the second LDS buffer while the others multiply chunk c; one barrier per chunk.
template <int CK, bool SPLIT>
__global__ __launch_bounds__(SPLIT ? 512 : 256, SPLIT ? 4 : 2) void mfma_f32_quad_kernel(const float* __restrict__ x,
                                                                          const float* __restrict__ w,
                                                                          float* __restrict__ y, const QuadParams P)
{
    constexpr int Q = CK / 4;                   // channel quads per chunk
    constexpr int G = CK / 8;                   // groups of eight channels = four matrix steps
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int RS = P.R * P.S;
    const int WP = P.IH * P.IW;                 // window pixels
    const int BUF = Q * WP + RS * Q * 64;                // floatx4 per LDS buffer: window [Q][WP], filters [RS][Q][64]
    floatx4* xs = reinterpret_cast<floatx4*>(smem);
    floatx4* ws = xs + Q * WP;

    const int tid = SPLIT ? (threadIdx.x & 255) : threadIdx.x;   // index among the loading (or all) threads
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool loader = SPLIT && wave >= 4;
    const int lj = lane & 31, kk = lane >> 5;   // row/column inside a 32 x 32 block, K lane

    const int ty = fast_div(blockIdx.x, P.by_tiles_x);
    const int tx = blockIdx.x - ty * P.tiles_x;
    const int n = blockIdx.y;
    const int co0 = blockIdx.z * 64;
    const int row0 = ty * P.TH, col0 = tx * P.TW;
    const int grow0 = row0 * P.stride - P.pad, gcol0 = col0 * P.stride - P.pad;

    const int tile_px = P.TH * P.TW;
    const int p = (wave & 3) * 32 + lj;
    const int pi = fast_div(p, P.by_TW), pj = p - pi * P.TW;
    const bool p_ok = p < tile_px && row0 + pi < P.Ho && col0 + pj < P.Wo;
    const int pixoff = p_ok ? (pi * P.stride) * P.IW + pj * P.stride : 0;
    const bool wave_live = __builtin_amdgcn_readfirstlane((wave & 3) * 32) < tile_px;

    floatx16 acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }

    const int HW = P.H * P.W;
    const float* xn = x + (int64_t)n * P.C_in * HW;
    const int wrow = P.C_in * RS;                               // floats per output channel in w
    const float* wb = w + (int64_t)co0 * wrow;

    // ---- staging plan, the same for every chunk
    int xo[kXS], xq[kXS];      // offset of channel 4q of the item's pixel inside the chunk's planes (< 0: padding), q
    int wo[kWS], wq[kWS], wd[kWS];   // offset of (co, channel 4q, tap) from wb + ci0 * RS (< 0: no such co), q, LDS slot
#pragma unroll
    for (int u = 0; u < kXS; ++u) {
        const int idx = tid + 256 * u;
        const int q = fast_div(idx, P.by_win);
        const int pix = idx - q * WP;
        const int e = fast_div(pix, P.by_IW), f = pix - e * P.IW;
        const int gr = grow0 + e, gc = gcol0 + f;
        xq[u] = q;
        xo[u] = (idx < Q * WP && gr >= 0 && gr < P.H && gc >= 0 && gc < P.W) ? 4 * q * HW + gr * P.W + gc : -1;
    }
#pragma unroll
    for (int u = 0; u < kWS; ++u) {
        const int idx = tid + 256 * u;                          // (co, q, tap), tap fastest: consecutive addresses
        const int co_l = fast_div(idx, P.by_QRS);
        const int rem = idx - co_l * (Q * RS);
        const int q = fast_div(rem, P.by_RS), tap = rem - q * RS;
        wq[u] = q;
        wo[u] = (idx < 64 * Q * RS && co0 + co_l < P.C_out) ? co_l * wrow + 4 * q * RS + tap : -1;
        wd[u] = (tap * Q + q) * 64 + co_l;
    }
    floatx4 xv[kXS], wv[kWS];
    // (always_inline: a lambda left as a call would force everything it captures into scratch memory)
    auto fetch = [&](int ci0) __attribute__((always_inline)) {
        const float* xc0 = xn + (int64_t)ci0 * HW;
        const float* wc0 = wb + (int64_t)ci0 * RS;
#pragma unroll
        for (int u = 0; u < kXS; ++u) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                xv[u][t] = 0.f;
                if (xo[u] >= 0 && ci0 + 4 * xq[u] + t < P.C_in) xv[u][t] = xc0[xo[u] + t * HW];
            }
        }
#pragma unroll
        for (int u = 0; u < kWS; ++u) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                wv[u][t] = 0.f;
                if (wo[u] >= 0 && ci0 + 4 * wq[u] + t < P.C_in) wv[u][t] = wc0[wo[u] + t * RS];
            }
        }
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kXS; ++u)
            if (tid + 256 * u < Q * WP) xs[buf * BUF + tid + 256 * u] = xv[u];
#pragma unroll
        for (int u = 0; u < kWS; ++u)
            if (tid + 256 * u < 64 * Q * RS) ws[buf * BUF + wd[u]] = wv[u];
    };

    // one tap of one group of eight channels: 2 x 4 matrix steps; the operands of the next (tap, group) are read
    // from LDS before these are multiplied
    auto multiply = [&](int buf) __attribute__((always_inline)) {
        if (!wave_live) return;
        const floatx4* bp = xs + buf * BUF + kk * WP + pixoff;
        const floatx4* ap = ws + buf * BUF + kk * 64 + lj;
        floatx4 a0 = ap[0], a1 = ap[32], b = bp[0];
        int toff = 0, s = 0;
#pragma unroll 1
        for (int tap = 0; tap < RS; ++tap) {
            int toff_n = toff + 1, s_n = s + 1;
            if (s_n == P.S) { s_n = 0; toff_n += P.IW - P.S; }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const floatx4 ca0 = a0, ca1 = a1, cb = b;
                if (g + 1 < G) {
                    a0 = ap[(tap * Q + 2 * (g + 1)) * 64];
                    a1 = ap[(tap * Q + 2 * (g + 1)) * 64 + 32];
                    b = bp[2 * (g + 1) * WP + toff];
                } else if (tap + 1 < RS) {
                    a0 = ap[(tap + 1) * Q * 64];
                    a1 = ap[(tap + 1) * Q * 64 + 32];
                    b = bp[toff_n];
                }
                __builtin_amdgcn_sched_barrier(0);      // keep the reads ahead of the matrix instructions
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(ca0[t], cb[t], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(ca1[t], cb[t], acc1, 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            toff = toff_n; s = s_n;
        }
    };

    if constexpr (!SPLIT) {
        fetch(0);
        for (int ci0 = 0; ci0 < P.C_in; ci0 += CK) {
            stage(0);
            __syncthreads();
            if (ci0 + CK < P.C_in) fetch(ci0 + CK);
            multiply(0);
            __syncthreads();
        }
    } else {
        // every wavefront passes 1 + chunks barriers
        const int chunks = (P.C_in + CK - 1) / CK;
        if (loader) {
            fetch(0);
            stage(0);
            __syncthreads();
            for (int c = 0; c < chunks; ++c) {
                if (c + 1 < chunks) {
                    fetch((c + 1) * CK);
                    stage((c + 1) & 1);          // (read by the others in turn c - 1, which the last barrier ended)
                }
                __syncthreads();
            }
            return;
        }
        __syncthreads();
        for (int c = 0; c < chunks; ++c) {
            multiply(c & 1);
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

struct QuadPlan {
    int TH, TW, IH, IW, CK, tiles_x, tiles_y;
    size_t lds;
    bool ok, split;
};

QuadPlan plan_quad(const Conv2dShape& s)
{
    QuadPlan a{};
    const int RS = s.R * s.S;
    a.TW = s.Wo < kTilePx ? s.Wo : kTilePx;
    a.TH = kTilePx / a.TW;
    if (a.TH > s.Ho) a.TH = s.Ho;
    if (a.TH < 1) a.TH = 1;
    a.CK = 32;
    while (a.CK > 8 && (a.CK * RS > 96 || a.CK >= 2 * s.C_in)) a.CK /= 2;
    auto fits = [&]() {
        a.IH = (a.TH - 1) * s.stride + s.R;
        a.IW = (a.TW - 1) * s.stride + s.S;
        return (int64_t)(a.CK / 4) * a.IH * a.IW <= 256 * kXS;
    };
    while (!fits() && a.CK > 8) a.CK /= 2;      // (a window that needs more staging slots goes to the other kernel)
    a.lds = ((size_t)(a.CK / 4) * a.IH * a.IW + (size_t)RS * (a.CK / 4) * 64) * 16;
    // two buffers, loaders a chunk ahead: pays where a chunk has several taps to multiply (14 x 14 x 256 3x3: 143 ->
    // 132 us, 7 x 7 x 512: 280 -> 246 us); with one tap per chunk (1x1) the loaders cannot keep enough bytes in flight
    // from one chunk ahead and the launch is slower (74 -> 103 us at 56 x 56 x 256 -> 64)
    a.split = RS > 1 && 2 * a.lds <= (size_t)kLdsBudget;
    if (a.split) a.lds *= 2;
    a.tiles_x = (s.Wo + a.TW - 1) / a.TW;
    a.tiles_y = (s.Ho + a.TH - 1) / a.TH;
    a.ok = fits() && a.CK * RS <= 96 && a.lds <= (size_t)kLdsBudget &&
           (int64_t)a.tiles_x * a.tiles_y * a.tiles_x < 2147483647LL && s.N <= 65535 && (s.C_out + 63) / 64 <= 65535 &&
           // 32-bit index arithmetic inside one image / 64 output channels' filters
           (int64_t)s.C_in * s.H * s.W <= 2147483647LL && (int64_t)64 * s.C_in * RS <= 2147483647LL;
    return a;
}

template <int CK>
hipError_t launch_quad(const float* x, const float* w, float* y, const Conv2dShape& s, const QuadPlan& a, hipStream_t st,
                       const Epilogue& ep)
{
    QuadParams P;
    P.ep = ep;
    P.C_in = s.C_in; P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.R = s.R; P.S = s.S; P.stride = s.stride;
    P.pad = s.pad; P.Ho = s.Ho; P.Wo = s.Wo;
    P.TH = a.TH; P.TW = a.TW; P.IH = a.IH; P.IW = a.IW; P.tiles_x = a.tiles_x;
    P.by_tiles_x = make_fastdiv(a.tiles_x);
    P.by_TW = make_fastdiv(a.TW);
    P.by_IW = make_fastdiv(a.IW);
    P.by_win = make_fastdiv(a.IH * a.IW);
    P.by_RS = make_fastdiv(s.R * s.S);
    P.by_QRS = make_fastdiv((CK / 4) * s.R * s.S);
    dim3 grid((unsigned)(a.tiles_x * a.tiles_y), (unsigned)s.N, (unsigned)((s.C_out + 63) / 64));
    if (a.split)
        SW_NOTED_LAUNCH(note_kernel("mfma_f32_quad_kernel", (int)(CK), (int)(true)), (mfma_f32_quad_kernel<CK, true>), grid, dim3(512), a.lds, st, x, w, y, P);
    else
        SW_NOTED_LAUNCH(note_kernel("mfma_f32_quad_kernel", (int)(CK), (int)(false)), (mfma_f32_quad_kernel<CK, false>), grid, dim3(256), a.lds, st, x, w, y, P);
    return hipGetLastError();
}

}  // namespace

// (with fewer than five input channels most of an eight-channel group would be zero padding)
bool mfma_f32_quad_supported(const Conv2dShape& s) { return s.dil == 1 && s.C_in >= 5 && plan_quad(s).ok; }

hipError_t launch_mfma_f32_quad(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st,
                                const Epilogue& ep)
{
    const QuadPlan a = plan_quad(s);
    if (!a.ok) return hipErrorInvalidValue;
    if (a.CK == 32) return launch_quad<32>(x, w, y, s, a, st, ep);
    if (a.CK == 16) return launch_quad<16>(x, w, y, s, a, st, ep);
    return launch_quad<8>(x, w, y, s, a, st, ep);
}

}  // namespace swconv
