// 1-D sliding window sums, stride 1: convolution, average and maximum share one kernel and differ
// only in the accumulate operator (paper, abstract: pooling and convolution as sliding sums
// evaluated by kernels with a shared structure).
//
// A workgroup owns TILE consecutive outputs of one row.  It loads the TILE + k - 1 inputs they
// depend on from HBM once, with coalesced 16-byte loads, into LDS (zero-filled outside the row:
// that is the padding).  Each lane then owns four consecutive outputs.  It keeps an 8-float window
// of the input in registers; the four taps j..j+3 are accumulated against the window shifted by
// 0..3 elements (a register rename, no data movement), then the window slides on by four elements
// with one 16-byte LDS read.  Outputs leave as 16-byte stores that are aligned in memory whatever the row
// length: the groups of four are laid out from the row's own alignment, and that offset, like the padding,
// becomes a compile-time register offset inside the window (so LDS reads stay aligned 16-byte reads too).
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Inputs are read once and outputs written once: both bypass the caches' retention (nontemporal).
__device__ __forceinline__ floatx4 stream_load4(const float* p) { return __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(p)); }
__device__ __forceinline__ void stream_store4(float* p, floatx4 v) { __builtin_nontemporal_store(v, reinterpret_cast<floatx4*>(p)); }

constexpr int kThreads = 256;
constexpr int kSub = kThreads * 4;      // outputs per pass over the workgroup
constexpr int kPasses = 2;
constexpr int kTile = kSub * kPasses;   // outputs per workgroup
constexpr int kMaxK = 64;
constexpr int kLdsIn = kTile + kMaxK + 16;  // tile + halo + alignment offset + read-ahead, multiple of 4

template <int OP>
__device__ __forceinline__ float accumulate(float acc, float wj, float xv)
{
    if (OP == OP_CONV) return fmaf(wj, xv, acc);
    if (OP == OP_AVG) return acc + xv;
    return fmaxf(acc, xv);
}

// The lane's four outputs from LDS.  src is 16-byte aligned; the first input the lane needs sits SH
// floats further on (SH = 0..3 folds the padding and the misalignment of the output row into a register
// offset, so every LDS read stays an aligned 16-byte read).  buf holds 8 or 12 consecutive floats; taps
// j..j+3 are accumulated against buf[SH + p + jj], then buf slides on by four with one more read.
template <int OP, int KC, int SH>
__device__ __forceinline__ void slide4(const float* __restrict__ src, const float* __restrict__ w, int k,
                                       float (&acc)[4])
{
    constexpr int N = SH <= 1 ? 8 : 12;      // SH + 3 + 3 is the largest index a group of four taps touches
    float buf[N];
#pragma unroll
    for (int c = 0; c < N / 4; ++c) {
        const floatx4 v = *reinterpret_cast<const floatx4*>(src + 4 * c);
        buf[4 * c + 0] = v.x; buf[4 * c + 1] = v.y; buf[4 * c + 2] = v.z; buf[4 * c + 3] = v.w;
    }
    int j = 0;
#pragma unroll
    for (; j + 4 <= k; j += 4) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const float wj = (OP == OP_CONV) ? w[j + jj] : 0.f;
#pragma unroll
            for (int p = 0; p < 4; ++p) acc[p] = accumulate<OP>(acc[p], wj, buf[SH + p + jj]);
        }
#pragma unroll
        for (int e = 0; e < N - 4; ++e) buf[e] = buf[e + 4];
        if (j + 4 < k) {
            const floatx4 v = *reinterpret_cast<const floatx4*>(src + j + N);
            buf[N - 4] = v.x; buf[N - 3] = v.y; buf[N - 2] = v.z; buf[N - 1] = v.w;
        }
    }
#pragma unroll
    for (int jj = 0; jj < 3; ++jj) {
        if (j + jj < k) {
            const float wj = (OP == OP_CONV) ? w[j + jj] : 0.f;
#pragma unroll
            for (int p = 0; p < 4; ++p) acc[p] = accumulate<OP>(acc[p], wj, buf[SH + p + jj]);
        }
    }
}

// Both passes of a lane over the staged tile, for one register offset SH.
template <int OP, int KC, int SH>
__device__ __forceinline__ void tile_outputs(const float* __restrict__ s_in, const float* __restrict__ w, int k,
                                             float* __restrict__ yrow, int o0, int o_end, int tid)
{
    const float inv_k = 1.0f / (float)k;
#pragma unroll
    for (int pass = 0; pass < kPasses; ++pass) {
        const int q = pass * kSub + 4 * tid;           // first of this lane's four outputs, tile-relative
        const int o = o0 + q;                          // ... and row-relative (may be < 0 in the first tile)
        if (o + 3 < 0 || o >= o_end) continue;
        float acc[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) acc[p] = (OP == OP_MAX) ? -__builtin_inff() : 0.f;
        slide4<OP, KC, SH>(s_in + q, w, k, acc);
        if (OP == OP_AVG) {
#pragma unroll
            for (int p = 0; p < 4; ++p) acc[p] *= inv_k;
        }
        if (o >= 0 && o + 3 < o_end) {
            stream_store4(yrow + o, floatx4{acc[0], acc[1], acc[2], acc[3]});
        } else {
#pragma unroll
            for (int p = 0; p < 4; ++p)
                if (o + p >= 0 && o + p < o_end) yrow[o + p] = acc[p];
        }
    }
}

// KC > 0: tap count known at compile time (fully unrolled, taps in scalar registers).
// KC == 0: tap count k at run time.
template <int OP, int KC>
__global__ __launch_bounds__(kThreads) void sliding_1d_kernel(const float* __restrict__ x,
                                                              const float* __restrict__ w,
                                                              float* __restrict__ y, int len,
                                                              int len_out, int k_rt, int pad,
                                                              int tiles_per_row, int x_vec_ok)
{
    __shared__ __attribute__((aligned(16))) float s_in[kLdsIn];

    const int k = KC > 0 ? KC : k_rt;
    const int tid = threadIdx.x;
    const int row = blockIdx.x / tiles_per_row;
    const int tile = blockIdx.x - row * tiles_per_row;
    const float* xr = x + (int64_t)row * len;
    float* yrow = y + (int64_t)row * len_out;

    // Outputs are grouped so that every group of four starts on a 16-byte boundary in memory: with `a` the
    // misalignment (in floats) of the row's first output, the tile owns outputs o0 .. o0 + kTile - 1 with
    // o0 = tile * kTile - a (the first tile of a misaligned row starts before output 0).
    const int a = (int)((reinterpret_cast<uintptr_t>(yrow) >> 2) & 3);
    const int o0 = tile * kTile - a;
    // LDS element e holds input position t0 + e; t0 is a multiple of 4 so that 16-byte global loads stay
    // aligned.  Output o0 + q reads inputs from position o0 + q - pad, i.e. LDS element q + sh.
    const int lead = (a + pad + 3) & ~3;
    const int sh = lead - a - pad;                     // 0..3
    const int t0 = tile * kTile - lead;
    const int o_end = min(o0 + kTile, len_out);        // one past the tile's last real output
    const int n_in = (o_end - o0) + k - 1 + sh;        // LDS elements the outputs read
    const int n_in4 = (n_in + 3) >> 2;

    if (x_vec_ok) {
        for (int f = tid; f < n_in4; f += kThreads) {
            const int t = t0 + 4 * f;
            floatx4 v;
            if (t >= 0 && t + 3 < len) {
                v = stream_load4(xr + t);
            } else {
                v.x = (t >= 0 && t < len) ? xr[t] : 0.f;
                v.y = (t + 1 >= 0 && t + 1 < len) ? xr[t + 1] : 0.f;
                v.z = (t + 2 >= 0 && t + 2 < len) ? xr[t + 2] : 0.f;
                v.w = (t + 3 >= 0 && t + 3 < len) ? xr[t + 3] : 0.f;
            }
            *reinterpret_cast<floatx4*>(s_in + 4 * f) = v;
        }
    } else {
        for (int e = tid; e < 4 * n_in4; e += kThreads) {
            const int t = t0 + e;
            s_in[e] = (t >= 0 && t < len) ? xr[t] : 0.f;
        }
    }
    __syncthreads();

    switch (sh) {
        case 0: tile_outputs<OP, KC, 0>(s_in, w, k, yrow, o0, o_end, tid); break;
        case 1: tile_outputs<OP, KC, 1>(s_in, w, k, yrow, o0, o_end, tid); break;
        case 2: tile_outputs<OP, KC, 2>(s_in, w, k, yrow, o0, o_end, tid); break;
        default: tile_outputs<OP, KC, 3>(s_in, w, k, yrow, o0, o_end, tid); break;
    }
}

template <int OP>
hipError_t launch_op(const float* x, const float* w, float* y, int64_t rows, int len, int len_out, int k,
                     int pad, hipStream_t st)
{
    // up to three outputs of misalignment per row are absorbed by the first tile
    const int tiles_per_row = (len_out + 3 + kTile - 1) / kTile;
    const int64_t blocks = rows * tiles_per_row;
    const int x_vec_ok = (reinterpret_cast<uintptr_t>(x) % 16 == 0) && (len % 4 == 0 || rows == 1);
    dim3 grid((unsigned)blocks), block(kThreads);
#define SW_CASE(KC)                                                                                      \
    case KC:                                                                                             \
        hipLaunchKernelGGL((sliding_1d_kernel<OP, KC>), grid, block, 0, st, x, w, y, len, len_out, k,    \
                           pad, tiles_per_row, x_vec_ok);                                                \
        break;
    switch (k) {
        SW_CASE(2) SW_CASE(3) SW_CASE(4) SW_CASE(5) SW_CASE(6) SW_CASE(7) SW_CASE(8) SW_CASE(9)
        SW_CASE(11) SW_CASE(13) SW_CASE(15) SW_CASE(16) SW_CASE(17)
        default:
            hipLaunchKernelGGL((sliding_1d_kernel<OP, 0>), grid, block, 0, st, x, w, y, len, len_out, k, pad,
                               tiles_per_row, x_vec_ok);
    }
#undef SW_CASE
    return hipGetLastError();
}

}  // namespace

bool sliding_1d_supported(int64_t len, int k, int stride, int pad)
{
    return stride == 1 && k >= 1 && k <= kMaxK && pad >= 0 && pad < k && len <= 2147483647LL - 4096;
}

hipError_t launch_sliding_1d(const float* x, const float* w, float* y, int64_t rows, int64_t len,
                             int64_t len_out, int k, int pad, Op1D op, hipStream_t st)
{
    const int64_t tiles = (len_out + 3 + kTile - 1) / kTile;
    if (rows * tiles > 2147483647LL) return hipErrorInvalidValue;
    switch (op) {
        case OP_CONV: return launch_op<OP_CONV>(x, w, y, rows, (int)len, (int)len_out, k, pad, st);
        case OP_AVG: return launch_op<OP_AVG>(x, w, y, rows, (int)len, (int)len_out, k, pad, st);
        case OP_MAX: return launch_op<OP_MAX>(x, w, y, rows, (int)len, (int)len_out, k, pad, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace swconv
