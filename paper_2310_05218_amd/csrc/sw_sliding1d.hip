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
constexpr int kPasses = 4;
constexpr int kTile = kSub * kPasses;   // outputs per workgroup
constexpr int kMaxK = 64;
constexpr int kMaxBlocks = 256 * 32;     // workgroups per launch; beyond that a workgroup walks over several tiles
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

// Geometry of one tile (all wave-uniform).
struct Tile1D {
    const float* xr;   // the row's input
    float* yrow;       // the row's output
    int o0;            // first output of the tile, row-relative (may be < 0 in the first tile of a row)
    int o_end;         // one past its last real output
    int t0;            // input position held by LDS element 0 (multiple of 4)
    int sh;            // register offset 0..3 (padding and output misalignment)
    int n_in4;         // 16-byte groups of input the tile reads
};

__device__ __forceinline__ Tile1D tile_geometry(const float* x, float* y, int tile_id, int tiles_per_row,
                                                int len, int len_out, int k, int pad)
{
    Tile1D g;
    const int row = tile_id / tiles_per_row;          // (tile counts are checked to fit 31 bits on the host)
    const int tile = tile_id - row * tiles_per_row;
    g.xr = x + (int64_t)row * len;
    g.yrow = y + (int64_t)row * len_out;
    // Outputs are grouped so that every group of four starts on a 16-byte boundary in memory: with `a` the
    // misalignment (in floats) of the row's first output, the tile owns outputs o0 .. o0 + kTile - 1 with
    // o0 = tile * kTile - a.
    const int a = (int)((reinterpret_cast<uintptr_t>(g.yrow) >> 2) & 3);
    g.o0 = tile * kTile - a;
    // LDS element e holds input position t0 + e; t0 is a multiple of 4 so that 16-byte global loads stay
    // aligned.  Output o0 + q reads inputs from position o0 + q - pad, i.e. LDS element q + sh.
    const int lead = (a + pad + 3) & ~3;
    g.sh = lead - a - pad;
    g.t0 = tile * kTile - lead;
    g.o_end = min(g.o0 + kTile, len_out);
    g.n_in4 = ((g.o_end - g.o0) + k - 1 + g.sh + 3) >> 2;
    return g;
}

// One 16-byte group of a row's input, zero outside the row.
__device__ __forceinline__ floatx4 load_group(const float* __restrict__ xr, int t, int len)
{
    if (t >= 0 && t + 3 < len) return stream_load4(xr + t);
    floatx4 v;
    v.x = (t >= 0 && t < len) ? xr[t] : 0.f;
    v.y = (t + 1 >= 0 && t + 1 < len) ? xr[t + 1] : 0.f;
    v.z = (t + 2 >= 0 && t + 2 < len) ? xr[t + 2] : 0.f;
    v.w = (t + 3 >= 0 && t + 3 < len) ? xr[t + 3] : 0.f;
    return v;
}

// Workgroup barrier that orders LDS traffic only: unlike __syncthreads() it does not wait for global loads
// in flight, which is what lets the next tile's fetch overlap this tile's arithmetic and stores.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

constexpr int kPre = (kLdsIn / 4 + kThreads - 1) / kThreads;    // 16-byte groups a lane prefetches per tile

// KC > 0: tap count known at compile time (fully unrolled, taps in scalar registers).
// KC == 0: tap count k at run time.
// A workgroup walks over tiles blockIdx.x, blockIdx.x + gridDim.x, ...; the next tile's input is on its way
// from HBM into registers while the current tile is accumulated and stored.
template <int OP, int KC>
__global__ __launch_bounds__(kThreads) void sliding_1d_kernel(const float* __restrict__ x,
                                                              const float* __restrict__ w,
                                                              float* __restrict__ y, int len,
                                                              int len_out, int k_rt, int pad,
                                                              int tiles_per_row, int tiles, int x_vec_ok)
{
    __shared__ __attribute__((aligned(16))) float s_in[kLdsIn];

    const int k = KC > 0 ? KC : k_rt;
    const int tid = threadIdx.x;
    int tile_id = blockIdx.x;
    Tile1D g = tile_geometry(x, y, tile_id, tiles_per_row, len, len_out, k, pad);

    floatx4 pre[kPre];
    if (x_vec_ok) {
#pragma unroll
        for (int i = 0; i < kPre; ++i)
            if (tid + i * kThreads < g.n_in4) pre[i] = load_group(g.xr, g.t0 + 4 * (tid + i * kThreads), len);
    }
    while (true) {
        if (x_vec_ok) {
#pragma unroll
            for (int i = 0; i < kPre; ++i)
                if (tid + i * kThreads < g.n_in4) *reinterpret_cast<floatx4*>(s_in + 4 * (tid + i * kThreads)) = pre[i];
        } else {
            for (int e = tid; e < 4 * g.n_in4; e += kThreads) {
                const int t = g.t0 + e;
                s_in[e] = (t >= 0 && t < len) ? g.xr[t] : 0.f;
            }
        }
        lds_barrier();

        const int next_id = tile_id + (int)gridDim.x;
        const bool more = next_id < tiles;
        Tile1D gn = g;
        if (more) {
            gn = tile_geometry(x, y, next_id, tiles_per_row, len, len_out, k, pad);
            if (x_vec_ok) {
#pragma unroll
                for (int i = 0; i < kPre; ++i)
                    if (tid + i * kThreads < gn.n_in4) pre[i] = load_group(gn.xr, gn.t0 + 4 * (tid + i * kThreads), len);
            }
        }

        switch (g.sh) {
            case 0: tile_outputs<OP, KC, 0>(s_in, w, k, g.yrow, g.o0, g.o_end, tid); break;
            case 1: tile_outputs<OP, KC, 1>(s_in, w, k, g.yrow, g.o0, g.o_end, tid); break;
            case 2: tile_outputs<OP, KC, 2>(s_in, w, k, g.yrow, g.o0, g.o_end, tid); break;
            default: tile_outputs<OP, KC, 3>(s_in, w, k, g.yrow, g.o0, g.o_end, tid); break;
        }
        if (!more) break;
        lds_barrier();      // every lane is done reading this tile before the next one is written
        tile_id = next_id;
        g = gn;
    }
}

template <int OP>
hipError_t launch_op(const float* x, const float* w, float* y, int64_t rows, int len, int len_out, int k,
                     int pad, hipStream_t st)
{
    // up to three outputs of misalignment per row are absorbed by the first tile
    const int tiles_per_row = (len_out + 3 + kTile - 1) / kTile;
    const int64_t tiles = rows * tiles_per_row;
    // enough workgroups to fill the chip several times over in flight, each walking over >= 1 tiles
    const int64_t blocks = tiles < kMaxBlocks ? tiles : kMaxBlocks;
    const int x_vec_ok = (reinterpret_cast<uintptr_t>(x) % 16 == 0) && (len % 4 == 0 || rows == 1);
    dim3 grid((unsigned)blocks), block(kThreads);
#define SW_CASE(KC)                                                                                      \
    case KC:                                                                                             \
        SW_NOTED_LAUNCH(note_kernel("sliding_1d_kernel", (int)(OP), (int)(KC)), (sliding_1d_kernel<OP, KC>), grid, block, 0, st, x, w, y, len, len_out, k,    \
                           pad, tiles_per_row, (int)tiles, x_vec_ok);                                    \
        break;
    switch (k) {
        SW_CASE(2) SW_CASE(3) SW_CASE(4) SW_CASE(5) SW_CASE(6) SW_CASE(7) SW_CASE(8) SW_CASE(9)
        SW_CASE(11) SW_CASE(13) SW_CASE(15) SW_CASE(16) SW_CASE(17)
        SW_CASE(25) SW_CASE(32) SW_CASE(33) SW_CASE(49) SW_CASE(64)
        default:
            SW_NOTED_LAUNCH(note_kernel("sliding_1d_kernel", (int)(OP), (int)(0)), (sliding_1d_kernel<OP, 0>), grid, block, 0, st, x, w, y, len, len_out, k, pad,
                               tiles_per_row, (int)tiles, x_vec_ok);
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
