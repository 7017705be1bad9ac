// 2-D sliding window sums with one filter per plane, stride 1: single-channel convolution and
// depthwise convolution (paper, section 2: 2-D sliding convolution, fixed-size "custom" kernels
// beside a generic one; section 1.2: depthwise stage of separable convolutions).
//
// One wavefront owns a 56 x 56 output tile of one plane.  It brings the tile's input window
// (tile + filter halo, zero-filled outside the image: that is the padding) from HBM into LDS once
// with coalesced 16-byte loads.  The 64 lanes form an 8 x 8 grid; each lane owns a 7 x 7 block of
// outputs held in 49 registers.  For every input row of its window the lane reads 7 + S - 1
// values from LDS once and accumulates them into every output row and tap column they belong to:
// the horizontal shift of the window is a register rename, the vertical shift is the choice of
// accumulator row.  Filter taps are wave-uniform and sit in scalar registers.  The finished tile
// goes back through LDS so that it leaves as coalesced 16-byte stores.
//
// LDS pitches are chosen so that the 8 x 4 lanes served together hit 32 distinct banks:
// lane (bx, by) reads float 7*bx + 7*pitch*by + const, and 7*pitch = 8 or 24 (mod 32) makes the four
// by-translates of {0,7,14,21,28,3,10,17} disjoint.  72 and 104 (= 8 mod 32) serve the input
// window, 56 (= 24 mod 32) the output tile.
#include "swconv_internal.h"

namespace swconv {

namespace {

constexpr int kB = 7;            // outputs per lane per axis
constexpr int kTile = 8 * kB;    // 56 outputs per tile per axis
constexpr int kMaxRS = 17;       // largest filter extent this kernel takes
constexpr int kOutPitch = kTile;

constexpr int in_pitch(int S) { return (3 + kTile + S - 1) <= 72 ? 72 : 104; }
constexpr int in_rows(int R) { return kTile + R - 1; }

// RC, SC > 0: filter extent known at compile time.  RC == 0: extent (R, S) at run time, up to kMaxRS.
template <int RC, int SC>
__global__ __launch_bounds__(64) void sliding_plane_kernel(const float* __restrict__ x,
                                                           const float* __restrict__ w,
                                                           float* __restrict__ y, int planes_per_x,
                                                           int n_filters, int H, int W, int R_rt,
                                                           int S_rt, int pad, int Ho, int Wo,
                                                           int tiles_x, int tiles_y, int x_vec_ok,
                                                           int y_vec_ok)
{
    constexpr int RMAX = RC > 0 ? RC : kMaxRS;
    constexpr int SMAX = RC > 0 ? SC : kMaxRS;
    constexpr int P = in_pitch(SMAX);
    constexpr int F4_PER_ROW = (3 + kTile + SMAX - 1 + 3) / 4;   // 16-byte groups loaded per row
    static_assert(F4_PER_ROW * 4 <= P, "pitch too small");
    constexpr int LDS_FLOATS = in_rows(RMAX) * P > kTile * kOutPitch ? in_rows(RMAX) * P : kTile * kOutPitch;
    __shared__ __attribute__((aligned(16))) float lds[LDS_FLOATS];

    const int R = RC > 0 ? RC : R_rt;
    const int S = RC > 0 ? SC : S_rt;
    const int lane = threadIdx.x;
    int b = blockIdx.x;
    const int tx = b % tiles_x; b /= tiles_x;
    const int ty = b % tiles_y; b /= tiles_y;
    const int plane = b;
    const int row0 = ty * kTile, col0 = tx * kTile;          // first output of the tile
    const float* xp = x + (int64_t)(plane / planes_per_x) * H * W;
    const float* wf = w + (int64_t)(plane % n_filters) * R * S;
    float* yp = y + (int64_t)plane * Ho * Wo;

    // LDS (row e, column c) holds input (row0 - pad + e, gcol0 + c); gcol0 is a multiple of 4.
    const int pad_up = (pad + 3) & ~3;
    const int shift = pad_up - pad;
    const int gcol0 = col0 - pad_up;
    const int grow0 = row0 - pad;
    const int rows_in = kTile + R - 1;

    for (int idx = lane; idx < rows_in * F4_PER_ROW; idx += 64) {
        const int e = idx / F4_PER_ROW;
        const int c4 = idx - e * F4_PER_ROW;
        const int gr = grow0 + e;
        const int gc = gcol0 + 4 * c4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gr >= 0 && gr < H && gc + 3 >= 0 && gc < W) {
            const float* src = xp + (int64_t)gr * W + gc;
            if (x_vec_ok && gc >= 0 && gc + 3 < W) {
                v = *reinterpret_cast<const float4*>(src);
            } else {
                if (gc >= 0) v.x = src[0];
                if (gc + 1 >= 0 && gc + 1 < W) v.y = src[1];
                if (gc + 2 >= 0 && gc + 2 < W) v.z = src[2];
                if (gc + 3 < W) v.w = src[3];
            }
        }
        *reinterpret_cast<float4*>(lds + e * P + 4 * c4) = v;
    }
    __syncthreads();

    const int bx = lane & 7, by = lane >> 3;
    float acc[kB][kB];
#pragma unroll
    for (int i = 0; i < kB; ++i)
#pragma unroll
        for (int j = 0; j < kB; ++j) acc[i][j] = 0.f;

    const float* win = lds + (kB * by) * P + shift + kB * bx;   // the lane's window origin

    if (RC > 0) {
        float wr[RMAX * SMAX];
#pragma unroll
        for (int t = 0; t < RMAX * SMAX; ++t) wr[t] = wf[t];
#pragma unroll
        for (int ir = 0; ir < kB + RMAX - 1; ++ir) {
            float in[kB + SMAX - 1];
#pragma unroll
            for (int c = 0; c < kB + SMAX - 1; ++c) in[c] = win[ir * P + c];
#pragma unroll
            for (int orow = 0; orow < kB; ++orow) {
                const int r = ir - orow;
                if (r < 0 || r >= RMAX) continue;
#pragma unroll
                for (int s = 0; s < SMAX; ++s)
#pragma unroll
                    for (int oc = 0; oc < kB; ++oc)
                        acc[orow][oc] = fmaf(wr[r * SMAX + s], in[oc + s], acc[orow][oc]);
            }
        }
    } else {
        for (int r = 0; r < R; ++r) {
            for (int s = 0; s < S; ++s) {
                const float wv = wf[r * S + s];
                const float* src = win + r * P + s;
#pragma unroll
                for (int orow = 0; orow < kB; ++orow)
#pragma unroll
                    for (int oc = 0; oc < kB; ++oc)
                        acc[orow][oc] = fmaf(wv, src[orow * P + oc], acc[orow][oc]);
            }
        }
    }

    __syncthreads();   // every lane has finished reading the window; reuse LDS for the output tile
#pragma unroll
    for (int i = 0; i < kB; ++i)
#pragma unroll
        for (int j = 0; j < kB; ++j) lds[(kB * by + i) * kOutPitch + kB * bx + j] = acc[i][j];
    __syncthreads();

    const int rows_out = min(kTile, Ho - row0);
    const int cols_out = min(kTile, Wo - col0);
    for (int idx = lane; idx < rows_out * (kTile / 4); idx += 64) {
        const int e = idx / (kTile / 4);
        const int c = 4 * (idx - e * (kTile / 4));
        if (c >= cols_out) continue;
        const float4 v = *reinterpret_cast<const float4*>(lds + e * kOutPitch + c);
        float* dst = yp + (int64_t)(row0 + e) * Wo + col0 + c;
        if (y_vec_ok && c + 3 < cols_out) {
            *reinterpret_cast<float4*>(dst) = v;
        } else {
            dst[0] = v.x;
            if (c + 1 < cols_out) dst[1] = v.y;
            if (c + 2 < cols_out) dst[2] = v.z;
            if (c + 3 < cols_out) dst[3] = v.w;
        }
    }
}

}  // namespace

bool sliding_plane_supported(int H, int W, int R, int S, int stride, int pad)
{
    (void)H; (void)W;
    return stride == 1 && R <= kMaxRS && S <= kMaxRS && pad >= 0 && pad <= 2 * kMaxRS;
}

hipError_t launch_sliding_plane(const float* x, const float* w, float* y, int64_t planes, int planes_per_x,
                                int n_filters, int H, int W, int R, int S, int pad, int Ho, int Wo,
                                hipStream_t st)
{
    const int tiles_x = (Wo + kTile - 1) / kTile, tiles_y = (Ho + kTile - 1) / kTile;
    const int64_t blocks = planes * tiles_x * tiles_y;
    if (blocks > 2147483647LL) return hipErrorInvalidValue;
    const int x_vec_ok = reinterpret_cast<uintptr_t>(x) % 16 == 0 && W % 4 == 0;
    const int y_vec_ok = reinterpret_cast<uintptr_t>(y) % 16 == 0 && Wo % 4 == 0;
    dim3 grid((unsigned)blocks), block(64);
#define SW_PLANE(RC, SC)                                                                                  \
    hipLaunchKernelGGL((sliding_plane_kernel<RC, SC>), grid, block, 0, st, x, w, y, planes_per_x, n_filters, \
                       H, W, R, S, pad, Ho, Wo, tiles_x, tiles_y, x_vec_ok, y_vec_ok)
    if (R == 3 && S == 3) SW_PLANE(3, 3);
    else if (R == 5 && S == 5) SW_PLANE(5, 5);
    else if (R == 7 && S == 7) SW_PLANE(7, 7);
    else SW_PLANE(0, 0);
#undef SW_PLANE
    return hipGetLastError();
}

}  // namespace swconv
