// 2-D sliding window sums with one filter per plane, stride 1, small fixed filters (3x3, 5x5), held
// entirely in registers: no LDS (paper, section 2: the "custom" kernels for widths 3 and 5).
//
// A wavefront owns a strip of 256 input columns (one aligned 16-byte load per lane and input row: 1 KB
// per row, fully coalesced) and a band of TR output rows.  A lane's four outputs of a row sit at the
// same columns as its four inputs, so loads and stores are both aligned; the taps that reach across the
// lane boundary take `pad` values from the left neighbour and S - 1 - pad from the right one, moved with
// DPP wavefront shifts (v_mov_b32_dpp wave_shr:1 / wave_shl:1) -- the row shift of the sliding sum.
// Vertically every input row is loaded once per band and accumulated into each output row it meets
// (choice of accumulator row).  Strips overlap by one lane on each inner side, because the edge lanes
// have no neighbour to take the halo from; at the image border the shifted-in zero is the padding.
// All TR + R - 1 row loads of a band are issued before the first use, so a band costs one memory
// round trip: this is the kernel for planes that are too few or too ragged for the 56 x 56 tile kernel.
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kStripIn = 256;             // input columns per wavefront
constexpr int kStripOut0 = 252;           // output columns of the first strip (lanes 0..62)
constexpr int kStripOut = 248;            // ... of the following strips (lanes 1..62)

__device__ __forceinline__ float from_left(float v)   // lane i receives lane i-1's value, lane 0 receives 0
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x138, 0xF, 0xF, true));
}
__device__ __forceinline__ float from_right(float v)  // lane i receives lane i+1's value, lane 63 receives 0
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x130, 0xF, 0xF, true));
}

// PADC: padding (compile time, 0 <= PADC <= S - 1, PADC <= 4, S - 1 - PADC <= 4).
template <int R, int S, int PADC, int TR>
__global__ __launch_bounds__(256) void sliding_rows_kernel(const float* __restrict__ x,
                                                           const float* __restrict__ w,
                                                           float* __restrict__ y, int planes_per_x,
                                                           int n_filters, int H, int W, int Ho, int Wo,
                                                           int strips, int bands, int64_t waves, int y_vec_ok)
{
    constexpr int LEFT = PADC, RIGHT = S - 1 - PADC;
    const int lane = threadIdx.x & 63;
    const int64_t wv = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wv >= waves) return;
    const int strip = (int)(wv % strips);
    const int64_t t = wv / strips;
    const int band = (int)(t % bands);
    const int plane = (int)(t / bands);

    const int c0 = strip * kStripOut;                 // first input column of the strip
    const int col = c0 + 4 * lane;                    // this lane's columns (inputs and outputs)
    const int i0 = band * TR;                         // first output row of the band
    const float* xp = x + (int64_t)(plane / planes_per_x) * H * W;
    const float* wf = w + (int64_t)(plane % n_filters) * R * S;
    float* yp = y + (int64_t)plane * Ho * Wo;

    float wr[R * S];
#pragma unroll
    for (int k = 0; k < R * S; ++k) wr[k] = wf[k];

    // every input row of the band, one aligned 16-byte load each (zero outside the image)
    floatx4 in[TR + R - 1];
#pragma unroll
    for (int e = 0; e < TR + R - 1; ++e) {
        const int gr = i0 - PADC + e;
        in[e] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (gr >= 0 && gr < H && col < W) in[e] = *reinterpret_cast<const floatx4*>(xp + (int64_t)gr * W + col);
    }

    float acc[TR][4];
#pragma unroll
    for (int i = 0; i < TR; ++i)
#pragma unroll
        for (int p = 0; p < 4; ++p) acc[i][p] = 0.f;

#pragma unroll
    for (int e = 0; e < TR + R - 1; ++e) {
        // v[LEFT + c] = input column col + c, c = -LEFT .. 3 + RIGHT
        float v[LEFT + 4 + RIGHT];
        v[LEFT + 0] = in[e].x; v[LEFT + 1] = in[e].y; v[LEFT + 2] = in[e].z; v[LEFT + 3] = in[e].w;
#pragma unroll
        for (int c = 0; c < LEFT; ++c) v[LEFT - 1 - c] = from_left(in[e][3 - c]);
#pragma unroll
        for (int c = 0; c < RIGHT; ++c) v[LEFT + 4 + c] = from_right(in[e][c]);
#pragma unroll
        for (int orow = 0; orow < TR; ++orow) {
            const int r = e - orow;
            if (r < 0 || r >= R) continue;
#pragma unroll
            for (int q = 0; q < S; ++q)
#pragma unroll
                for (int p = 0; p < 4; ++p) acc[orow][p] = fmaf(wr[r * S + q], v[p + q], acc[orow][p]);
        }
    }

    // lanes without a neighbour inside the strip have no halo: they only feed their neighbours, unless
    // the missing neighbour lies outside the image, where the shifted-in zero is the padding itself
    const bool left_ok = LEFT == 0 || lane > 0 || c0 == 0;
    const bool right_ok = RIGHT == 0 || lane < 63 || c0 + kStripIn >= W;
    if (!left_ok || !right_ok || col >= Wo) return;
#pragma unroll
    for (int orow = 0; orow < TR; ++orow) {
        const int oi = i0 + orow;
        if (oi >= Ho) break;
        float* dst = yp + (int64_t)oi * Wo + col;
        if (y_vec_ok && col + 3 < Wo) {
            *reinterpret_cast<floatx4*>(dst) = floatx4{acc[orow][0], acc[orow][1], acc[orow][2], acc[orow][3]};
        } else {
#pragma unroll
            for (int p = 0; p < 4; ++p)
                if (col + p < Wo) dst[p] = acc[orow][p];
        }
    }
}

template <int R, int S, int PADC>
hipError_t launch_rows(const float* x, const float* w, float* y, int64_t planes, int planes_per_x, int n_filters,
                       int H, int W, int Ho, int Wo, hipStream_t st)
{
    const int strips = Wo <= kStripOut0 + 4 && W <= kStripIn ? 1 : 1 + (Wo - kStripOut0 + kStripOut - 1) / kStripOut;
    const int y_vec_ok = reinterpret_cast<uintptr_t>(y) % 16 == 0 && Wo % 4 == 0;
    // short bands when the launch would otherwise leave most of the chip idle
    const bool small = planes * strips * ((Ho + 7) / 8) < 2048;
    const int TR = small ? 4 : 8;
    const int bands = (Ho + TR - 1) / TR;
    const int64_t waves = planes * strips * bands;
    const int64_t blocks = (waves + 3) / 4;
    if (blocks > 2147483647LL) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), block(256);
    if (small)
        hipLaunchKernelGGL((sliding_rows_kernel<R, S, PADC, 4>), grid, block, 0, st, x, w, y, planes_per_x, n_filters,
                           H, W, Ho, Wo, strips, bands, waves, y_vec_ok);
    else
        hipLaunchKernelGGL((sliding_rows_kernel<R, S, PADC, 8>), grid, block, 0, st, x, w, y, planes_per_x, n_filters,
                           H, W, Ho, Wo, strips, bands, waves, y_vec_ok);
    return hipGetLastError();
}

}  // namespace

bool sliding_rows_supported(const float* x, int H, int W, int R, int S, int stride, int pad)
{
    (void)H;
    if (stride != 1 || R != S || (R != 3 && R != 5) || pad > (R - 1) / 2 || pad < 0) return false;
    // (padding beyond (R-1)/2 would need more than the compiled halo widths)
    return W % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0;
}

hipError_t launch_sliding_rows(const float* x, const float* w, float* y, int64_t planes, int planes_per_x,
                               int n_filters, int H, int W, int R, int S, int pad, int Ho, int Wo, hipStream_t st)
{
    (void)S;
#define SW_ROWS(RC, PC) return launch_rows<RC, RC, PC>(x, w, y, planes, planes_per_x, n_filters, H, W, Ho, Wo, st)
    if (R == 3 && pad == 0) SW_ROWS(3, 0);
    if (R == 3 && pad == 1) SW_ROWS(3, 1);
    if (R == 5 && pad == 0) SW_ROWS(5, 0);
    if (R == 5 && pad == 1) SW_ROWS(5, 1);
    if (R == 5 && pad == 2) SW_ROWS(5, 2);
#undef SW_ROWS
    return hipErrorInvalidValue;
}

}  // namespace swconv
