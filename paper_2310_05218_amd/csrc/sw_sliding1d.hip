// 1-D sliding window sums, stride 1: convolution, average and maximum share one kernel and differ
// only in the accumulate operator (paper, abstract: pooling and convolution as sliding sums
// evaluated by kernels with a shared structure).
//
// A workgroup owns TILE consecutive outputs of one row.  It loads the TILE + k - 1 inputs they
// depend on from HBM once, with coalesced 16-byte loads, into LDS (zero-filled outside the row:
// that is the padding).  Each lane then owns four consecutive outputs.  It keeps an 8-float window
// of the input in registers; the four taps j..j+3 are accumulated against the window shifted by
// 0..3 elements (a register rename, no data movement), then the window slides on by four elements
// with one 16-byte LDS read.  Outputs leave through 16-byte stores: directly when every output row is
// 16-byte aligned, otherwise through LDS, re-grouped so that each store is aligned in memory.
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
constexpr int kLdsIn = kTile + kMaxK + 8;  // tile + halo + alignment shift, multiple of 4

template <int OP>
__device__ __forceinline__ float accumulate(float acc, float wj, float xv)
{
    if (OP == OP_CONV) return fmaf(wj, xv, acc);
    if (OP == OP_AVG) return acc + xv;
    return fmaxf(acc, xv);
}

// KC > 0: tap count known at compile time (fully unrolled, taps in scalar registers).
// KC == 0: tap count k at run time.
template <int OP, int KC>
__global__ __launch_bounds__(kThreads) void sliding_1d_kernel(const float* __restrict__ x,
                                                              const float* __restrict__ w,
                                                              float* __restrict__ y, int len,
                                                              int len_out, int k_rt, int pad,
                                                              int tiles_per_row, int x_vec_ok,
                                                              int y_vec_ok)
{
    __shared__ __attribute__((aligned(16))) float s_in[kLdsIn];
    __shared__ __attribute__((aligned(16))) float s_out[kTile];

    const int k = KC > 0 ? KC : k_rt;
    const int tid = threadIdx.x;
    const int row = blockIdx.x / tiles_per_row;
    const int tile = blockIdx.x - row * tiles_per_row;
    const int o0 = tile * kTile;                       // first output of this tile
    const int n_out = min(kTile, len_out - o0);
    const float* xr = x + (int64_t)row * len;
    float* yr = y + (int64_t)row * len_out + o0;

    // LDS element e holds input position t0 + e; t0 is a multiple of 4 so that 16-byte global
    // loads stay aligned whatever the padding is.
    const int pad_up = (pad + 3) & ~3;
    const int shift = pad_up - pad;                    // first needed input sits at LDS element shift
    const int t0 = o0 - pad_up;
    const int n_in = n_out + k - 1 + shift;            // LDS elements the outputs read
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

    const float inv_k = 1.0f / (float)k;
#pragma unroll
    for (int pass = 0; pass < kPasses; ++pass) {
        const int base = pass * kSub + 4 * tid;        // first of this lane's four outputs
        float acc[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) acc[p] = (OP == OP_MAX) ? -__builtin_inff() : 0.f;
        if (base < n_out) {
            // window[0..7] = inputs base+j .. base+j+7 (relative to the first needed input)
            float win[8];
            const float* src = s_in + shift + base;
            if (shift == 0) {
                const float4 a = *reinterpret_cast<const float4*>(src);
                const float4 b = *reinterpret_cast<const float4*>(src + 4);
                win[0] = a.x; win[1] = a.y; win[2] = a.z; win[3] = a.w;
                win[4] = b.x; win[5] = b.y; win[6] = b.z; win[7] = b.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) win[e] = src[e];
            }
            int j = 0;
#pragma unroll
            for (; j + 4 <= k; j += 4) {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const float wj = (OP == OP_CONV) ? w[j + jj] : 0.f;
#pragma unroll
                    for (int p = 0; p < 4; ++p) acc[p] = accumulate<OP>(acc[p], wj, win[p + jj]);
                }
                // slide by four
#pragma unroll
                for (int e = 0; e < 4; ++e) win[e] = win[e + 4];
                if (j + 4 < k) {
                    if (shift == 0) {
                        const float4 b = *reinterpret_cast<const float4*>(src + j + 8);
                        win[4] = b.x; win[5] = b.y; win[6] = b.z; win[7] = b.w;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) win[4 + e] = src[j + 8 + e];
                    }
                }
            }
#pragma unroll
            for (int jj = 0; jj < 3; ++jj) {
                if (j + jj < k) {
                    const float wj = (OP == OP_CONV) ? w[j + jj] : 0.f;
#pragma unroll
                    for (int p = 0; p < 4; ++p) acc[p] = accumulate<OP>(acc[p], wj, win[p + jj]);
                }
            }
            if (OP == OP_AVG) {
#pragma unroll
                for (int p = 0; p < 4; ++p) acc[p] *= inv_k;
            }
            if (y_vec_ok) {
                if (base + 3 < n_out) {
                    stream_store4(yr + base, floatx4{acc[0], acc[1], acc[2], acc[3]});
                } else {
#pragma unroll
                    for (int p = 0; p < 4; ++p)
                        if (base + p < n_out) yr[base + p] = acc[p];
                }
            }
        }
        if (!y_vec_ok) *reinterpret_cast<float4*>(s_out + base) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    }
    if (!y_vec_ok) {
        // The output row does not start on a 16-byte boundary: peel up to three elements, then store
        // 16-byte groups that are aligned in memory (read from LDS at the matching odd offset).
        __syncthreads();
        const int head = min(n_out, (int)(((16u - (unsigned)(reinterpret_cast<uintptr_t>(yr) & 15u)) & 15u) >> 2));
        const int body4 = (n_out - head) >> 2;
        const int tail0 = head + 4 * body4;
        if (tid < head) yr[tid] = s_out[tid];
        for (int f = tid; f < body4; f += kThreads) {
            const int e = head + 4 * f;
            stream_store4(yr + e, floatx4{s_out[e], s_out[e + 1], s_out[e + 2], s_out[e + 3]});
        }
        if (tid < n_out - tail0) yr[tail0 + tid] = s_out[tail0 + tid];
    }
}

template <int OP>
hipError_t launch_op(const float* x, const float* w, float* y, int64_t rows, int len, int len_out, int k,
                     int pad, hipStream_t st)
{
    const int tiles_per_row = (len_out + kTile - 1) / kTile;
    const int64_t blocks = rows * tiles_per_row;
    const int x_vec_ok = (reinterpret_cast<uintptr_t>(x) % 16 == 0) && (len % 4 == 0 || rows == 1);
    const int y_vec_ok = (reinterpret_cast<uintptr_t>(y) % 16 == 0) && (len_out % 4 == 0 || rows == 1);
    dim3 grid((unsigned)blocks), block(kThreads);
#define SW_CASE(KC)                                                                                      \
    case KC:                                                                                             \
        hipLaunchKernelGGL((sliding_1d_kernel<OP, KC>), grid, block, 0, st, x, w, y, len, len_out, k,    \
                           pad, tiles_per_row, x_vec_ok, y_vec_ok);                                      \
        break;
    switch (k) {
        SW_CASE(2) SW_CASE(3) SW_CASE(4) SW_CASE(5) SW_CASE(6) SW_CASE(7) SW_CASE(8) SW_CASE(9)
        SW_CASE(11) SW_CASE(13) SW_CASE(15) SW_CASE(16) SW_CASE(17)
        default:
            hipLaunchKernelGGL((sliding_1d_kernel<OP, 0>), grid, block, 0, st, x, w, y, len, len_out, k, pad,
                               tiles_per_row, x_vec_ok, y_vec_ok);
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
    const int64_t tiles = (len_out + kTile - 1) / kTile;
    if (rows * tiles > 2147483647LL) return hipErrorInvalidValue;
    switch (op) {
        case OP_CONV: return launch_op<OP_CONV>(x, w, y, rows, (int)len, (int)len_out, k, pad, st);
        case OP_AVG: return launch_op<OP_AVG>(x, w, y, rows, (int)len, (int)len_out, k, pad, st);
        case OP_MAX: return launch_op<OP_MAX>(x, w, y, rows, (int)len, (int)len_out, k, pad, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace swconv
