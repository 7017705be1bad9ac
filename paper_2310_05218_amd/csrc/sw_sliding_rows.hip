// 2-D sliding window sums with one filter per plane (or none: pooling), small fixed windows, stride 1
// or 2, held entirely in registers: no LDS (paper, section 2: the "custom" kernels for small fixed
// sizes; abstract: pooling and convolution are the same sliding sum).
//
// A wavefront owns a strip of 256 input columns (one aligned 16-byte load per lane and input row: 1 KB
// per row, fully coalesced) and a band of TR output rows.  At stride 1 a lane's four outputs of a row
// sit at the same columns as its four inputs, at stride 2 its two outputs sit at half that column, so
// loads and stores are both aligned; the taps that reach across the lane boundary take `pad` values
// from the left neighbour and the rest from the right one, moved with DPP wavefront shifts
// (v_mov_b32_dpp wave_shr:1 / wave_shl:1) -- the row shift of the sliding sum.
// Vertically every input row is loaded once per band and accumulated into each output row it meets
// (choice of accumulator row).  Strips overlap by one lane on each inner side, because the edge lanes
// have no neighbour to take the halo from; at the image border the shifted-in value is the padding
// itself (zero for sums, minus infinity for the maximum, which padding must never win).
// All row loads of a band are issued before the first use, so a band costs one memory round trip: this
// is the kernel for planes that are too few or too ragged for the 56 x 56 tile kernel.
#include "swconv_internal.h"

#include <cmath>

namespace swconv {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int kStripIn = 256;             // input columns per wavefront
constexpr int kStripFirst = 252;          // input columns whose lanes have both neighbours, first strip
constexpr int kStripStep = 248;           // distance between strip origins (lanes 1..62 of later strips)

enum RowsOp { ROWS_CONV = 0, ROWS_AVG = 1, ROWS_MAX = 2 };

// lane i receives lane i-1's value (from_left) or lane i+1's (from_right); the lane without such a
// neighbour receives FILL
template <int OP>
__device__ __forceinline__ float from_left(float v)
{
    if constexpr (OP == ROWS_MAX)
        return __int_as_float(__builtin_amdgcn_update_dpp((int)0xff800000, __float_as_int(v), 0x138, 0xF, 0xF, false));
    else
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x138, 0xF, 0xF, true));
}
template <int OP>
__device__ __forceinline__ float from_right(float v)
{
    if constexpr (OP == ROWS_MAX)
        return __int_as_float(__builtin_amdgcn_update_dpp((int)0xff800000, __float_as_int(v), 0x130, 0xF, 0xF, false));
    else
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x130, 0xF, 0xF, true));
}

// PADC: padding (compile time).  ST: stride, 1 or 2.  OP: weighted sum, average or maximum.
// SEGL: lanes per work item.  64: the wavefront walks strips of a wide plane.  8, 16 or 32: planes narrower
// than 4 * SEGL columns, one (plane, band) item per group of SEGL lanes; the lanes of a group beyond the
// plane's width hold padding, which is exactly what the neighbouring group's edge lane must shift in.
template <int R, int S, int PADC, int TR, int ST, int OP, int SEGL>
__global__ __launch_bounds__(256) void sliding_rows_kernel(const float* __restrict__ x,
                                                           const float* __restrict__ w,
                                                           float* __restrict__ y, int planes_per_x,
                                                           int n_filters, int H, int W, int Ho, int Wo,
                                                           int strips, int bands, int64_t waves, int64_t items,
                                                           int y_vec_ok, const Epilogue ep)
{
    constexpr int NOUT = 4 / ST;                                   // outputs per lane and output row
    constexpr int LEFT = PADC;
    constexpr int RIGHT = ST * (NOUT - 1) + S - 1 - PADC - 3 > 0 ? ST * (NOUT - 1) + S - 1 - PADC - 3 : 0;
    constexpr int NIN = ST * (TR - 1) + R;                         // input rows of a band
    static_assert(LEFT <= 4 && RIGHT <= 4, "halo wider than one neighbour lane");
    const float FILL = OP == ROWS_MAX ? -INFINITY : 0.f;
    const int lane = threadIdx.x & 63;
    const int64_t wv = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wv >= waves) return;
    int c0, col, band, plane;
    bool live = true;
    if constexpr (SEGL == 64) {
        const int strip = (int)(wv % strips);
        const int64_t t = wv / strips;
        band = (int)(t % bands);
        plane = (int)(t / bands);
        c0 = strip * kStripStep;                      // first input column of the strip
        col = c0 + 4 * lane;                          // this lane's input columns
    } else {
        // the last wavefront may hold fewer than 64 / SEGL items: its idle groups load and store nothing
        const int64_t item = wv * (64 / SEGL) + lane / SEGL;
        live = item < items;
        const int64_t it = live ? item : 0;
        band = (int)(it % bands);
        plane = (int)(it / bands);
        c0 = 0;
        col = 4 * (lane % SEGL);
    }
    const int ocol = col / ST;                        // the lane's first output column
    const int i0 = band * TR;                         // first output row of the band
    const float* xp = x + (int64_t)(plane / planes_per_x) * H * W;
    float* yp = y + (int64_t)plane * Ho * Wo;

    float wr[R * S];
    if constexpr (OP == ROWS_CONV) {
        const float* wf = w + (int64_t)(plane % n_filters) * R * S;
#pragma unroll
        for (int k = 0; k < R * S; ++k) wr[k] = wf[k];
    }

    // every input row of the band, one aligned 16-byte load each (padding outside the image)
    floatx4 in[NIN];
#pragma unroll
    for (int e = 0; e < NIN; ++e) {
        const int gr = ST * i0 - PADC + e;
        in[e] = floatx4{FILL, FILL, FILL, FILL};
        if (gr >= 0 && gr < H && col < W && live) in[e] = *reinterpret_cast<const floatx4*>(xp + (int64_t)gr * W + col);
    }

    float acc[TR][NOUT];
#pragma unroll
    for (int i = 0; i < TR; ++i)
#pragma unroll
        for (int p = 0; p < NOUT; ++p) acc[i][p] = FILL;

#pragma unroll
    for (int e = 0; e < NIN; ++e) {
        // v[LEFT + c] = input column col + c, c = -LEFT .. 3 + RIGHT
        float v[LEFT + 4 + RIGHT];
        v[LEFT + 0] = in[e].x; v[LEFT + 1] = in[e].y; v[LEFT + 2] = in[e].z; v[LEFT + 3] = in[e].w;
#pragma unroll
        for (int c = 0; c < LEFT; ++c) v[LEFT - 1 - c] = from_left<OP>(in[e][3 - c]);
#pragma unroll
        for (int c = 0; c < RIGHT; ++c) v[LEFT + 4 + c] = from_right<OP>(in[e][c]);
#pragma unroll
        for (int orow = 0; orow < TR; ++orow) {
            const int r = e - ST * orow;
            if (r < 0 || r >= R) continue;
#pragma unroll
            for (int q = 0; q < S; ++q)
#pragma unroll
                for (int p = 0; p < NOUT; ++p) {
                    const float e_in = v[ST * p + q];
                    if constexpr (OP == ROWS_CONV) acc[orow][p] = fmaf(wr[r * S + q], e_in, acc[orow][p]);
                    else if constexpr (OP == ROWS_AVG) acc[orow][p] += e_in;
                    else acc[orow][p] = fmaxf(acc[orow][p], e_in);
                }
        }
    }

    // lanes without a neighbour inside the strip have no halo: they only feed their neighbours, unless
    // the missing neighbour lies outside the image, where the shifted-in value is the padding itself
    const bool left_ok = SEGL != 64 || lane > 0 || c0 == 0;
    const bool right_ok = SEGL != 64 || lane < 63 || c0 + kStripIn >= W;
    if (!left_ok || !right_ok || ocol >= Wo || !live) return;
    constexpr float kScale = 1.0f / (float)(R * S);
    // convolution only: per-channel bias and rectifier of the fused-epilogue entry point (both off otherwise)
    const bool with_ep = OP == ROWS_CONV && (ep.bias != nullptr || ep.relu != 0);
    const float ep_bias = (OP == ROWS_CONV && ep.bias) ? ep.bias[plane % n_filters] : 0.f;
#pragma unroll
    for (int orow = 0; orow < TR; ++orow) {
        const int oi = i0 + orow;
        if (oi >= Ho) break;
        if constexpr (OP == ROWS_AVG) {
#pragma unroll
            for (int p = 0; p < NOUT; ++p) acc[orow][p] *= kScale;
        }
        if (with_ep) {
#pragma unroll
            for (int p = 0; p < NOUT; ++p) {
                const float t = acc[orow][p] + ep_bias;
                acc[orow][p] = ep.relu ? fmaxf(t, 0.f) : t;
            }
        }
        float* dst = yp + (int64_t)oi * Wo + ocol;
        if (y_vec_ok && ocol + NOUT - 1 < Wo) {
            // (streaming stores: the output is not read again by this kernel)
            if constexpr (NOUT == 4)
                __builtin_nontemporal_store(floatx4{acc[orow][0], acc[orow][1], acc[orow][2], acc[orow][3]},
                                            reinterpret_cast<floatx4*>(dst));
            else
                __builtin_nontemporal_store(floatx2{acc[orow][0], acc[orow][1]}, reinterpret_cast<floatx2*>(dst));
        } else {
#pragma unroll
            for (int p = 0; p < NOUT; ++p)
                if (ocol + p < Wo) dst[p] = acc[orow][p];
        }
    }
}

template <int R, int S, int PADC, int ST, int OP, int SEGL>
hipError_t launch_rows_seg(const float* x, const float* w, float* y, int64_t planes, int planes_per_x, int n_filters,
                           int H, int W, int Ho, int Wo, hipStream_t st, const Epilogue& ep)
{
    constexpr int NOUT = 4 / ST;
    const int y_vec_ok = reinterpret_cast<uintptr_t>(y) % (4 * NOUT) == 0 && Wo % NOUT == 0;
    int strips = 1;
    if (SEGL == 64 && W > kStripIn) {
        // input columns whose lanes produce an output
        const int64_t need = (int64_t)ST * Wo;
        const int Wc = (int)(need < W ? (need + 3) & ~(int64_t)3 : W);
        if (Wc > kStripFirst) strips = 1 + (Wc - kStripFirst + kStripStep - 1) / kStripStep;
    }
    // short bands when the launch would otherwise leave most of the chip idle
    constexpr int TR_BIG = 8 / ST, TR_SMALL = 4 / ST;
    constexpr int PER_WAVE = 64 / SEGL;
    const bool small = (planes * strips * ((Ho + TR_BIG - 1) / TR_BIG) + PER_WAVE - 1) / PER_WAVE < 8192;
    const int TR = small ? TR_SMALL : TR_BIG;
    const int bands = (Ho + TR - 1) / TR;
    const int64_t items = planes * strips * bands;
    const int64_t waves = (items + PER_WAVE - 1) / PER_WAVE;
    const int64_t blocks = (waves + 3) / 4;
    if (blocks > 2147483647LL) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), block(256);
    if (small)
        SW_NOTED_LAUNCH(note_kernel("sliding_rows_kernel", (int)(R), (int)(S), (int)(PADC), (int)(TR_SMALL)), (sliding_rows_kernel<R, S, PADC, TR_SMALL, ST, OP, SEGL>), grid, block, 0, st, x, w, y,
                           planes_per_x, n_filters, H, W, Ho, Wo, strips, bands, waves, items, y_vec_ok, ep);
    else
        SW_NOTED_LAUNCH(note_kernel("sliding_rows_kernel", (int)(R), (int)(S), (int)(PADC), (int)(TR_BIG)), (sliding_rows_kernel<R, S, PADC, TR_BIG, ST, OP, SEGL>), grid, block, 0, st, x, w, y,
                           planes_per_x, n_filters, H, W, Ho, Wo, strips, bands, waves, items, y_vec_ok, ep);
    return hipGetLastError();
}

// Narrow planes share a wavefront: the group must be at least one lane wider than the plane (W / 4 lanes), so
// that the lane between two planes holds padding.
template <int R, int S, int PADC, int ST, int OP>
hipError_t launch_rows(const float* x, const float* w, float* y, int64_t planes, int planes_per_x, int n_filters,
                       int H, int W, int Ho, int Wo, hipStream_t st, const Epilogue& ep)
{
    const int lanes = W / 4 + 1;
#define SW_SEG(L) return launch_rows_seg<R, S, PADC, ST, OP, L>(x, w, y, planes, planes_per_x, n_filters, H, W, Ho, Wo, st, ep)
    if (lanes <= 8) SW_SEG(8);
    if (lanes <= 16) SW_SEG(16);
    if (lanes <= 32) SW_SEG(32);
    SW_SEG(64);
#undef SW_SEG
}

}  // namespace

bool sliding_rows_supported(const float* x, int H, int W, int R, int S, int stride, int pad)
{
    (void)H;
    if ((stride != 1 && stride != 2) || R != S || (R != 3 && R != 5 && R != 7) || pad > (R - 1) / 2 || pad < 0) return false;
    // (padding beyond (R-1)/2 would need more than the compiled halo widths; 7x7 reaches at most four columns into
    // the right neighbour, which rules out the smallest paddings)
    if (R == 7 && pad < (stride == 1 ? 2 : 1)) return false;
    return W % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0;
}

hipError_t launch_sliding_rows(const float* x, const float* w, float* y, int64_t planes, int planes_per_x,
                               int n_filters, int H, int W, int R, int S, int stride, int pad, int Ho, int Wo,
                               hipStream_t st, const Epilogue& ep)
{
    (void)S;
#define SW_ROWS(RC, PC)                                                                                        \
    if (R == RC && pad == PC) {                                                                                \
        if (stride == 1)                                                                                       \
            return launch_rows<RC, RC, PC, 1, ROWS_CONV>(x, w, y, planes, planes_per_x, n_filters, H, W, Ho, Wo, st, ep); \
        return launch_rows<RC, RC, PC, 2, ROWS_CONV>(x, w, y, planes, planes_per_x, n_filters, H, W, Ho, Wo, st, ep);     \
    }
    SW_ROWS(3, 0) SW_ROWS(3, 1) SW_ROWS(5, 0) SW_ROWS(5, 1) SW_ROWS(5, 2)
    if (R == 7 && pad == 3) {
        if (stride == 1) return launch_rows<7, 7, 3, 1, ROWS_CONV>(x, w, y, planes, planes_per_x, n_filters, H, W, Ho, Wo, st, ep);
        return launch_rows<7, 7, 3, 2, ROWS_CONV>(x, w, y, planes, planes_per_x, n_filters, H, W, Ho, Wo, st, ep);
    }
    if (R == 7 && pad == 2) {
        if (stride == 1) return launch_rows<7, 7, 2, 1, ROWS_CONV>(x, w, y, planes, planes_per_x, n_filters, H, W, Ho, Wo, st, ep);
        return launch_rows<7, 7, 2, 2, ROWS_CONV>(x, w, y, planes, planes_per_x, n_filters, H, W, Ho, Wo, st, ep);
    }
    if (R == 7 && pad == 1 && stride == 2)
        return launch_rows<7, 7, 1, 2, ROWS_CONV>(x, w, y, planes, planes_per_x, n_filters, H, W, Ho, Wo, st, ep);
#undef SW_ROWS
    return hipErrorInvalidValue;
}

// Pooling windows with a register-only kernel: 2x2 and 3x3, stride 1 or 2, padding up to half the window.
bool pool_rows_supported(const float* x, int W, int R, int S, int stride, int pad)
{
    if ((stride != 1 && stride != 2) || R != S || (R != 2 && R != 3) || pad < 0 || pad > (R == 3 ? 1 : 0)) return false;
    if (R == 2 && stride == 1) return false;       // (no compiled variant; the direct kernel takes it)
    return W % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0;
}

hipError_t launch_pool_rows(const float* x, float* y, int64_t planes, int H, int W, int R, int stride, int pad,
                            int Ho, int Wo, bool maximum, hipStream_t st)
{
#define SW_POOL(RC, PC, SC)                                                                                    \
    if (R == RC && pad == PC && stride == SC) {                                                                \
        if (maximum) return launch_rows<RC, RC, PC, SC, ROWS_MAX>(x, nullptr, y, planes, 1, 1, H, W, Ho, Wo, st, Epilogue{nullptr, 0}); \
        return launch_rows<RC, RC, PC, SC, ROWS_AVG>(x, nullptr, y, planes, 1, 1, H, W, Ho, Wo, st, Epilogue{nullptr, 0}); \
    }
    SW_POOL(2, 0, 2) SW_POOL(3, 0, 1) SW_POOL(3, 1, 1) SW_POOL(3, 0, 2) SW_POOL(3, 1, 2)
#undef SW_POOL
    return hipErrorInvalidValue;
}

}  // namespace swconv
