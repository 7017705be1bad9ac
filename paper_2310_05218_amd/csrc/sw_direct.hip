// Direct kernels: one thread per output element, taps accumulated straight from global memory.
// They cover every valid shape (any stride, padding, filter extent) and serve the shapes the
// tiled sliding kernels do not specialise; they also read the unmodified input and write
// nothing but the output (paper, section 2).
#include "swconv_internal.h"

#include <cmath>

namespace swconv {

namespace {

constexpr int kThreads = 256;

inline int grid_for(int64_t total)
{
    int64_t g = (total + kThreads - 1) / kThreads;
    const int64_t cap = 256 * 64;  // grid-stride beyond this
    return (int)(g < cap ? g : cap);
}

template <int OP>
__global__ __launch_bounds__(kThreads) void direct_1d_kernel(const float* __restrict__ x,
                                                             const float* __restrict__ w,
                                                             float* __restrict__ y, int64_t rows,
                                                             int64_t len, int64_t len_out, int k,
                                                             int stride, int pad)
{
    const int64_t total = rows * len_out;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * kThreads) {
        const int64_t row = o / len_out;
        const int64_t i = o - row * len_out;
        const float* xr = x + row * len;
        const int64_t t0 = i * stride - pad;
        float acc;
        if (OP == OP_MAX) {
            acc = xr[t0];
            for (int j = 1; j < k; ++j) acc = fmaxf(acc, xr[t0 + j]);
        } else {
            acc = 0.f;
            for (int j = 0; j < k; ++j) {
                const int64_t t = t0 + j;
                if (t >= 0 && t < len) acc = (OP == OP_CONV) ? fmaf(w[j], xr[t], acc) : acc + xr[t];
            }
            if (OP == OP_AVG) acc = acc / (float)k;
        }
        y[o] = acc;
    }
}

// RQ: the int32 sum is requantised to int8 on its way out (y8), see requant_s8.
template <typename TI, typename TA, bool DW, bool RQ = false>
__global__ __launch_bounds__(kThreads) void direct_conv2d_kernel(const TI* __restrict__ x,
                                                                 const TI* __restrict__ w,
                                                                 TA* __restrict__ y, Conv2dShape s,
                                                                 int8_t* __restrict__ y8 = nullptr,
                                                                 Requant rq = Requant{nullptr, nullptr, 0},
                                                                 Epilogue ep = Epilogue{nullptr, 0})
{
    const int64_t plane_o = (int64_t)s.Ho * s.Wo;
    const int64_t total = (int64_t)s.N * s.C_out * plane_o;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * kThreads) {
        const int64_t nc = o / plane_o;
        const int pix = (int)(o - nc * plane_o);
        const int n = (int)(nc / s.C_out);
        const int co = (int)(nc - (int64_t)n * s.C_out);
        const int i = pix / s.Wo, j = pix - i * s.Wo;
        const int h0 = i * s.stride - s.pad, v0 = j * s.stride - s.pad;
        const int ci_lo = DW ? co : 0;
        const int ci_hi = DW ? co + 1 : s.C_in;
        TA acc = 0;
        for (int ci = ci_lo; ci < ci_hi; ++ci) {
            const TI* xp = x + ((int64_t)n * s.C_in + ci) * s.H * s.W;
            const TI* wp = w + ((int64_t)co * (DW ? 1 : s.C_in) + (DW ? 0 : ci)) * s.R * s.S;
            for (int r = 0; r < s.R; ++r) {
                const int h = h0 + r * s.dil;
                if (h < 0 || h >= s.H) continue;
                for (int q = 0; q < s.S; ++q) {
                    const int v = v0 + q * s.dil;
                    if (v < 0 || v >= s.W) continue;
                    acc += (TA)xp[h * s.W + v] * (TA)wp[r * s.S + q];
                }
            }
        }
        if constexpr (RQ) y8[o] = requant_s8((int)acc, co, rq);
        else if constexpr (sizeof(TI) == 4) y[o] = apply_epilogue(acc, co, ep);
        else y[o] = acc;
    }
}

// Depthwise convolution on bf16 planes, one thread per output: bf16 in, fp32 products and sums, bf16 out
// (nearest, ties to even).
__global__ __launch_bounds__(kThreads) void direct_depthwise_bf16_kernel(const unsigned short* __restrict__ x,
                                                                         const float* __restrict__ w,
                                                                         unsigned short* __restrict__ y, Conv2dShape s)
{
    const int64_t plane_o = (int64_t)s.Ho * s.Wo;
    const int64_t total = (int64_t)s.N * s.C_out * plane_o;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += (int64_t)gridDim.x * kThreads) {
        const int64_t nc = o / plane_o;
        const int pix = (int)(o - nc * plane_o);
        const int c = (int)(nc % s.C_out);
        const int i = pix / s.Wo, j = pix - i * s.Wo;
        const int h0 = i * s.stride - s.pad, v0 = j * s.stride - s.pad;
        const unsigned short* xp = x + nc * s.H * s.W;
        const float* wp = w + (int64_t)c * s.R * s.S;
        float acc = 0.f;
        for (int r = 0; r < s.R; ++r) {
            const int h = h0 + r;
            if (h < 0 || h >= s.H) continue;
            for (int q = 0; q < s.S; ++q) {
                const int v = v0 + q;
                if (v < 0 || v >= s.W) continue;
                acc = fmaf(__uint_as_float((unsigned)xp[h * s.W + v] << 16), wp[r * s.S + q], acc);
            }
        }
        const unsigned u = __float_as_uint(acc);
        unsigned b = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) b = (u >> 16) | 0x40u;
        y[o] = (unsigned short)b;
    }
}

// 2-D pooling, one thread per output: the average sums the zero-padded window and scales by 1/(R*S),
// the maximum runs over the window positions inside the plane.
template <bool MAXIMUM>
__global__ __launch_bounds__(kThreads) void direct_pool2d_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                                 int64_t planes, int H, int W, int R, int S,
                                                                 int stride, int pad, int Ho, int Wo)
{
    const int64_t plane_o = (int64_t)Ho * Wo;
    const int64_t total = planes * plane_o;
    const float scale = 1.0f / (float)(R * S);
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * kThreads) {
        const int64_t p = o / plane_o;
        const int pix = (int)(o - p * plane_o);
        const int i = pix / Wo, j = pix - i * Wo;
        const float* xp = x + p * H * W;
        const int h0 = i * stride - pad, v0 = j * stride - pad;
        const int r_lo = h0 < 0 ? -h0 : 0, r_hi = H - h0 < R ? H - h0 : R;
        const int s_lo = v0 < 0 ? -v0 : 0, s_hi = W - v0 < S ? W - v0 : S;
        float acc = MAXIMUM ? -INFINITY : 0.f;
        for (int r = r_lo; r < r_hi; ++r)
            for (int q = s_lo; q < s_hi; ++q) {
                const float e = xp[(int64_t)(h0 + r) * W + v0 + q];
                acc = MAXIMUM ? fmaxf(acc, e) : acc + e;
            }
        y[o] = MAXIMUM ? acc : acc * scale;
    }
}

// Pooling with large windows (global pooling above all), one wavefront per output: the lanes stride over
// the window positions, which lie in runs of S consecutive addresses, and a butterfly of lane exchanges
// folds the 64 partial results.
template <bool MAXIMUM>
__global__ __launch_bounds__(kThreads) void wave_pool2d_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                               int64_t planes, int H, int W, int R, int S,
                                                               int stride, int pad, int Ho, int Wo)
{
    const int lane = threadIdx.x & 63;
    const int64_t plane_o = (int64_t)Ho * Wo;
    const int64_t total = planes * plane_o;
    const float scale = 1.0f / (float)(R * S);
    for (int64_t o = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6); o < total;
         o += (int64_t)gridDim.x * (kThreads / 64)) {
        const int64_t p = o / plane_o;
        const int pix = (int)(o - p * plane_o);
        const int i = pix / Wo, j = pix - i * Wo;
        const float* xp = x + p * H * W;
        const int h0 = i * stride - pad, v0 = j * stride - pad;
        float acc = MAXIMUM ? -INFINITY : 0.f;
        for (int t = lane; t < R * S; t += 64) {
            const int r = t / S, q = t - r * S;
            const int h = h0 + r, v = v0 + q;
            if (h >= 0 && h < H && v >= 0 && v < W) {
                const float e = xp[(int64_t)h * W + v];
                acc = MAXIMUM ? fmaxf(acc, e) : acc + e;
            }
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            const float other = __shfl_xor(acc, m, 64);
            acc = MAXIMUM ? fmaxf(acc, other) : acc + other;
        }
        if (lane == 0) y[o] = MAXIMUM ? acc : acc * scale;
    }
}

}  // namespace

hipError_t launch_direct_1d(const float* x, const float* w, float* y, int64_t rows, int64_t len,
                            int64_t len_out, int k, int stride, int pad, Op1D op, hipStream_t st)
{
    const int grid = grid_for(rows * len_out);
    switch (op) {
        case OP_CONV:
            SW_NOTED_LAUNCH(note_kernel("direct_1d_kernel", (int)(OP_CONV)), direct_1d_kernel<OP_CONV>, dim3(grid), dim3(kThreads), 0, st, x, w, y, rows,
                               len, len_out, k, stride, pad);
            break;
        case OP_AVG:
            SW_NOTED_LAUNCH(note_kernel("direct_1d_kernel", (int)(OP_AVG)), direct_1d_kernel<OP_AVG>, dim3(grid), dim3(kThreads), 0, st, x, w, y, rows,
                               len, len_out, k, stride, pad);
            break;
        case OP_MAX:
            SW_NOTED_LAUNCH(note_kernel("direct_1d_kernel", (int)(OP_MAX)), direct_1d_kernel<OP_MAX>, dim3(grid), dim3(kThreads), 0, st, x, w, y, rows,
                               len, len_out, k, stride, pad);
            break;
    }
    return hipGetLastError();
}

hipError_t launch_direct_conv2d_f32(const float* x, const float* w, float* y, const Conv2dShape& s,
                                    bool depthwise, hipStream_t st, const Epilogue* ep)
{
    const int grid = grid_for((int64_t)s.N * s.C_out * s.Ho * s.Wo);
    const Epilogue e = ep ? *ep : Epilogue{nullptr, 0};
    const Requant none{nullptr, nullptr, 0};
    if (depthwise)
        SW_NOTED_LAUNCH(note_kernel("direct_conv2d_kernel", (int)(true)), (direct_conv2d_kernel<float, float, true>), dim3(grid), dim3(kThreads), 0, st, x,
                           w, y, s, static_cast<int8_t*>(nullptr), none, e);
    else
        SW_NOTED_LAUNCH(note_kernel("direct_conv2d_kernel", (int)(false)), (direct_conv2d_kernel<float, float, false>), dim3(grid), dim3(kThreads), 0, st, x,
                           w, y, s, static_cast<int8_t*>(nullptr), none, e);
    return hipGetLastError();
}

hipError_t launch_direct_conv2d_s8(const int8_t* x, const int8_t* w, int32_t* y, const Conv2dShape& s,
                                   hipStream_t st)
{
    const int grid = grid_for((int64_t)s.N * s.C_out * s.Ho * s.Wo);
    SW_NOTED_LAUNCH(note_kernel("direct_conv2d_kernel", (int)(false)), (direct_conv2d_kernel<int8_t, int32_t, false>), dim3(grid), dim3(kThreads), 0, st, x,
                       w, y, s);
    return hipGetLastError();
}

hipError_t launch_direct_conv2d_s8_requant(const int8_t* x, const int8_t* w, int8_t* y8, const Requant& rq,
                                           const Conv2dShape& s, hipStream_t st)
{
    const int grid = grid_for((int64_t)s.N * s.C_out * s.Ho * s.Wo);
    SW_NOTED_LAUNCH(note_kernel("direct_conv2d_kernel", (int)(false), (int)(true)), (direct_conv2d_kernel<int8_t, int32_t, false, true>), dim3(grid), dim3(kThreads), 0, st, x,
                       w, static_cast<int32_t*>(nullptr), s, y8, rq);
    return hipGetLastError();
}

hipError_t launch_direct_pool2d(const float* x, float* y, int64_t planes, int H, int W, int R, int S, int stride,
                                int pad, int Ho, int Wo, bool maximum, hipStream_t st)
{
    if (R * S >= 32) {      // large windows: a wavefront per output
        const int64_t waves = planes * Ho * Wo;
        const int64_t g = (waves + kThreads / 64 - 1) / (kThreads / 64);
        const int grid = (int)(g < 256 * 256 ? g : 256 * 256);
        if (maximum)
            SW_NOTED_LAUNCH(note_kernel("wave_pool2d_kernel", (int)(true)), wave_pool2d_kernel<true>, dim3(grid), dim3(kThreads), 0, st, x, y, planes, H, W, R, S,
                               stride, pad, Ho, Wo);
        else
            SW_NOTED_LAUNCH(note_kernel("wave_pool2d_kernel", (int)(false)), wave_pool2d_kernel<false>, dim3(grid), dim3(kThreads), 0, st, x, y, planes, H, W, R, S,
                               stride, pad, Ho, Wo);
        return hipGetLastError();
    }
    const int grid = grid_for(planes * Ho * Wo);
    if (maximum)
        SW_NOTED_LAUNCH(note_kernel("direct_pool2d_kernel", (int)(true)), direct_pool2d_kernel<true>, dim3(grid), dim3(kThreads), 0, st, x, y, planes, H, W, R, S,
                           stride, pad, Ho, Wo);
    else
        SW_NOTED_LAUNCH(note_kernel("direct_pool2d_kernel", (int)(false)), direct_pool2d_kernel<false>, dim3(grid), dim3(kThreads), 0, st, x, y, planes, H, W, R, S,
                           stride, pad, Ho, Wo);
    return hipGetLastError();
}

hipError_t launch_direct_depthwise_bf16(const unsigned short* x, const float* w, unsigned short* y,
                                        const Conv2dShape& s, hipStream_t st)
{
    const int grid = grid_for((int64_t)s.N * s.C_out * s.Ho * s.Wo);
    SW_NOTED_LAUNCH(note_kernel("direct_depthwise_bf16_kernel"), direct_depthwise_bf16_kernel, dim3(grid), dim3(kThreads), 0, st, x, w, y, s);
    return hipGetLastError();
}

}  // namespace swconv
