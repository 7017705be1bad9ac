// 1-D sliding window sums with a stride above 1: convolution, average and maximum (paper, abstract: pooling
// and convolution share one kernel structure; the common pooling step is the window itself).
//
// A workgroup owns kTileOut consecutive outputs of one row.  The (kTileOut - 1) * stride + k inputs they depend
// on are one contiguous run of the row: it is brought into LDS once with coalesced loads (16 bytes per lane
// from a start rounded down to an aligned address; zero outside the row: that is the padding).  Consecutive
// lanes own consecutive outputs, whose windows start `stride` floats apart in LDS, and outputs leave as they
// are computed: consecutive lanes, consecutive addresses.  Inputs are read once, outputs written once.
#include "swconv_internal.h"

#include <cmath>

namespace swconv {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kPer = 4;                       // outputs per thread
constexpr int kTileOut = kThreads * kPer;     // outputs per workgroup
constexpr int kMaxStride = 8;
constexpr int kMaxK = 64;
constexpr int kLdsFloats = (kTileOut - 1) * kMaxStride + kMaxK + 8;   // tile + halo + alignment slack

template <int OP>
__global__ __launch_bounds__(kThreads) void strided_1d_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                              float* __restrict__ y, int len, int len_out, int k,
                                                              int stride, int pad, int tiles_per_row, FastDiv by_tiles,
                                                              int x_vec_ok)
{
    __shared__ __attribute__((aligned(16))) float lds[kLdsFloats];
    const int tid = threadIdx.x;
    const int row = fast_div(blockIdx.x, by_tiles);
    const int tile = blockIdx.x - row * tiles_per_row;
    const int o0 = tile * kTileOut;                                  // first output of the tile
    const int n_out = len_out - o0 < kTileOut ? len_out - o0 : kTileOut;
    const int64_t rbase = (int64_t)row * len;                        // first element of the row in x
    const int start = o0 * stride - pad;                             // row position of the tile's first input
    const int span = (n_out - 1) * stride + k;                       // inputs the tile touches
    // LDS slot 0 holds row position `a0`: start rounded down so that its global address is 16-byte aligned
    const int mis = (int)((rbase + start) & 3);
    const int a0 = x_vec_ok ? start - mis : start;
    const int n_lds = start - a0 + span;
    const float* xr = x + rbase;
    if (x_vec_ok) {
        for (int i = 4 * tid; i < n_lds; i += 4 * kThreads) {
            const int pos = a0 + i;                                  // row position of the group's first float
            floatx4 v = floatx4{0.f, 0.f, 0.f, 0.f};
            if (pos >= 0 && pos + 3 < len) {
                v = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(xr + pos));
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (pos + j >= 0 && pos + j < len) v[j] = xr[pos + j];
            }
            *reinterpret_cast<floatx4*>(lds + i) = v;
        }
    } else {
        for (int i = tid; i < n_lds; i += kThreads) {
            const int pos = a0 + i;
            lds[i] = (pos >= 0 && pos < len) ? xr[pos] : 0.f;
        }
    }
    __syncthreads();

    const float* win0 = lds + (start - a0);
    float* yr = y + (int64_t)row * len_out + o0;
    const float scale = 1.0f / (float)k;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int o = tid + kThreads * j;
        if (o >= n_out) break;
        const float* win = win0 + o * stride;
        float acc = OP == OP_MAX ? -INFINITY : 0.f;
        for (int t = 0; t < k; ++t) {
            const float e = win[t];
            if (OP == OP_CONV) acc = fmaf(w[t], e, acc);
            else if (OP == OP_AVG) acc += e;
            else acc = fmaxf(acc, e);
        }
        __builtin_nontemporal_store(OP == OP_AVG ? acc * scale : acc, yr + o);
    }
}

// Pooling whose windows tile the rows exactly (stride == window in {2, 4, 8}, row length a multiple of the
// window and of 4): rows follow each other without a gap, so the whole tensor is one flat sequence of windows
// and every window lies inside one or two aligned 16-byte groups.  Registers only: a lane loads its groups
// (coalesced), folds them and stores; four groups per thread are in flight.
template <int OP, int WIN>
__global__ __launch_bounds__(kThreads) void pool_tiles_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                              int64_t n_groups)
{
    constexpr int U = 4;
    constexpr float kScale = 1.0f / (float)WIN;
    auto fold = [](float a, float b) { return OP == OP_MAX ? fmaxf(a, b) : a + b; };
    const floatx4* src = reinterpret_cast<const floatx4*>(x);
    for (int64_t base = (int64_t)blockIdx.x * (kThreads * U) + threadIdx.x; base < n_groups;
         base += (int64_t)gridDim.x * (kThreads * U)) {
        floatx4 v[U][WIN == 8 ? 2 : 1];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t g = base + kThreads * u;
            if (g < n_groups) {
                if (WIN == 8) {
                    v[u][0] = __builtin_nontemporal_load(src + 2 * g);
                    v[u][WIN == 8 ? 1 : 0] = __builtin_nontemporal_load(src + 2 * g + 1);
                } else {
                    v[u][0] = __builtin_nontemporal_load(src + g);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t g = base + kThreads * u;
            if (g >= n_groups) break;
            const floatx4 a = v[u][0];
            if (WIN == 2) {
                float lo = fold(a.x, a.y), hi = fold(a.z, a.w);
                if (OP == OP_AVG) { lo *= kScale; hi *= kScale; }
                typedef float floatx2 __attribute__((ext_vector_type(2)));
                __builtin_nontemporal_store(floatx2{lo, hi}, reinterpret_cast<floatx2*>(y) + g);
            } else {
                float r = fold(fold(a.x, a.y), fold(a.z, a.w));
                if (WIN == 8) {
                    const floatx4 b = v[u][WIN == 8 ? 1 : 0];
                    r = fold(r, fold(fold(b.x, b.y), fold(b.z, b.w)));
                }
                __builtin_nontemporal_store(OP == OP_AVG ? r * kScale : r, y + g);
            }
        }
    }
}

}  // namespace

bool pool_tiles_supported(const float* x, const float* y, int64_t len, int window, int stride)
{
    if (stride != window || (window != 2 && window != 4 && window != 8)) return false;
    return len % window == 0 && len % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0 &&
           reinterpret_cast<uintptr_t>(y) % 8 == 0;
}

hipError_t launch_pool_tiles(const float* x, float* y, int64_t rows, int64_t len, int window, bool maximum,
                             hipStream_t st)
{
    const int64_t n_groups = window == 8 ? rows * len / 8 : rows * len / 4;
    int64_t blocks = (n_groups + kThreads * 4 - 1) / (kThreads * 4);
    if (blocks > 256 * 64) blocks = 256 * 64;
    dim3 grid((unsigned)blocks), block(kThreads);
#define SW_TILES(OPC, WINC) SW_NOTED_LAUNCH(note_kernel("pool_tiles_kernel", (int)(OPC), (int)(WINC)), (pool_tiles_kernel<OPC, WINC>), grid, block, 0, st, x, y, n_groups)
    if (maximum) {
        if (window == 2) SW_TILES(OP_MAX, 2); else if (window == 4) SW_TILES(OP_MAX, 4); else SW_TILES(OP_MAX, 8);
    } else {
        if (window == 2) SW_TILES(OP_AVG, 2); else if (window == 4) SW_TILES(OP_AVG, 4); else SW_TILES(OP_AVG, 8);
    }
#undef SW_TILES
    return hipGetLastError();
}

bool strided_1d_supported(int64_t rows, int64_t len, int64_t len_out, int k, int stride, int pad)
{
    if (stride < 2 || stride > kMaxStride || k < 1 || k > kMaxK || pad < 0 || pad >= k) return false;
    const int64_t tiles = (len_out + kTileOut - 1) / kTileOut;
    // 32-bit positions inside a row, a grid of at most 2^31 - 1 workgroups, exact fast division
    return len <= 2147483647LL - 4096 && rows * tiles <= 2147483647LL && rows * tiles * tiles < 4294967296LL;
}

hipError_t launch_strided_1d(const float* x, const float* w, float* y, int64_t rows, int64_t len, int64_t len_out,
                             int k, int stride, int pad, Op1D op, hipStream_t st)
{
    const int tiles = (int)((len_out + kTileOut - 1) / kTileOut);
    const int x_vec_ok = reinterpret_cast<uintptr_t>(x) % 16 == 0;
    dim3 grid((unsigned)(rows * tiles)), block(kThreads);
    const FastDiv by_tiles = make_fastdiv(tiles);
#define SW_STRIDED(OPC)                                                                                        \
    SW_NOTED_LAUNCH(note_kernel("strided_1d_kernel", (int)(OPC)), strided_1d_kernel<OPC>, grid, block, 0, st, x, w, y, (int)len, (int)len_out, k, stride, pad, \
                       tiles, by_tiles, x_vec_ok)
    if (op == OP_CONV) SW_STRIDED(OP_CONV);
    else if (op == OP_AVG) SW_STRIDED(OP_AVG);
    else SW_STRIDED(OP_MAX);
#undef SW_STRIDED
    return hipGetLastError();
}

}  // namespace swconv
