// Depthwise sliding window sums over SMALL planes (14 x 14, 7 x 7, ... -- the tail of a CNN), any filter
// extent, stride and padding (paper, section 1.2: depthwise convolutions; section 2: the input is used as it
// lies in memory).
//
// A 56 x 56 tile per wavefront wastes most of its lanes on such planes, and one thread per output reads them
// with scattered accesses.  Here a workgroup takes a run of consecutive planes -- which is one contiguous run
// of memory, whatever the plane's width -- and brings it into LDS once with coalesced loads, each plane framed
// by its zero padding, together with the planes' filters.  A thread then owns four consecutive outputs of a
// column: for every filter column it reads the R + 3 inputs they depend on once and slides them under the
// taps (register rename), exactly the 1-D sliding sum turned upright; no position needs a bounds test because
// the padding is in LDS.  Consecutive threads own consecutive columns, so LDS reads fall into distinct banks
// and every store instruction writes a run of consecutive outputs.
#include "swconv_internal.h"

namespace swconv {

namespace {

constexpr int kThreads = 256;
constexpr int kLdsFloats = 12 * 1024;      // 48 KB per workgroup: three workgroups per CU

struct SmallParams {
    Epilogue ep;                           // per-channel bias and rectifier of the fused-epilogue entry point
    int H, W, R, S, stride, pad, Ho, Wo, n_filters, G;
    int Hp, Wp, QH;                        // framed plane in LDS, groups of four output rows
    int64_t planes;
    int vec;                               // the run of planes starts on a 16-byte boundary in every workgroup: 16-byte loads
    FastDiv by_frame, by_Wp, by_items, by_Wo, by_HW, by_W;
};

// RC, SC, STC > 0: filter extent and stride at compile time (taps unrolled); 0: at run time.
template <int RC, int SC, int STC>
__global__ __launch_bounds__(kThreads) void small_planes_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                                float* __restrict__ y, const SmallParams P)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int R = RC > 0 ? RC : P.R, S = RC > 0 ? SC : P.S, ST = RC > 0 ? STC : P.stride;
    const int HW = P.H * P.W, RS = R * S, HoWo = P.Ho * P.Wo;
    const int frame = P.Hp * P.Wp;
    const int tid = threadIdx.x;
    const int64_t p0 = (int64_t)blockIdx.x * P.G;
    const int np = P.planes - p0 < P.G ? (int)(P.planes - p0) : P.G;
    float* xs = lds;                               // [np][Hp][Wp]
    float* ws = lds + P.G * frame;                 // [np][RS]

    const float* src = x + p0 * HW;
    if (P.vec) {
        // The run of planes is one contiguous, 16-byte aligned piece of memory: it comes in with 16-byte loads (four
        // in flight per thread: one or two memory round trips for the whole run) and is scattered element by element
        // into the frames, whose padding has been zeroed before.
        typedef float floatx4 __attribute__((ext_vector_type(4)));
        const int cells = np * frame;
        for (int i = tid; i < cells / 4; i += kThreads) reinterpret_cast<floatx4*>(xs)[i] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (tid < cells % 4) xs[cells - 1 - tid] = 0.f;
        __syncthreads();
        const int n = np * HW, n4 = n / 4;
        auto place = [&](int i, float v) __attribute__((always_inline)) {
            const int g = fast_div(i, P.by_HW), c = i - g * HW;
            const int h = fast_div(c, P.by_W), col = c - h * P.W;
            if (h + P.pad < P.Hp && col + P.pad < P.Wp) xs[g * frame + (h + P.pad) * P.Wp + col + P.pad] = v;
        };
        for (int base = tid; base < n4; base += kThreads * 4) {
            floatx4 v4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = base + kThreads * u;
                v4[u] = reinterpret_cast<const floatx4*>(src)[q < n4 ? q : n4 - 1];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = base + kThreads * u;
                if (q < n4) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) place(4 * q + e, v4[u][e]);
                }
            }
        }
        if (tid < n % 4) place(n - 1 - tid, src[n - 1 - tid]);
    } else {
        // every cell of the framed planes: the image where there is one, zero (the padding) around it; loads go
        // out eight per thread before the first LDS write, so a batch costs one memory round trip
        for (int base = tid; base < np * frame; base += kThreads * 8) {
            float v8[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = base + kThreads * u;
                const int g = fast_div(i, P.by_frame);
                const int c = i - g * frame;
                const int hp = fast_div(c, P.by_Wp), vp = c - hp * P.Wp;
                const int h = hp - P.pad, v = vp - P.pad;
                v8[u] = 0.f;
                if (i < np * frame && (unsigned)h < (unsigned)P.H && (unsigned)v < (unsigned)P.W) v8[u] = src[g * HW + h * P.W + v];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (base + kThreads * u < np * frame) xs[base + kThreads * u] = v8[u];
        }
    }
    // the filters of these planes (plane p uses filter p % n_filters)
    for (int i = tid; i < np * RS; i += kThreads) {
        const int g = i / RS;
        ws[i] = w[(int64_t)((p0 + g) % P.n_filters) * RS + (i - g * RS)];
    }
    __syncthreads();

    float* dst = y + p0 * HoWo;
    const int items = P.QH * P.Wo;                 // groups of four outputs (one column, four rows) per plane
    for (int idx = tid; idx < np * items; idx += kThreads) {
        const int g = fast_div(idx, P.by_items);
        const int it = idx - g * items;
        const int qi = fast_div(it, P.by_Wo), oj = it - qi * P.Wo;
        const int oi = 4 * qi;
        const float* xp = xs + g * frame + (oi * ST) * P.Wp + oj * ST;
        const float* wf = ws + g * RS;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        if constexpr (RC > 0) {
            constexpr int N = 3 * STC + RC;        // inputs of a filter column that the four outputs touch
#pragma unroll
            for (int q = 0; q < SC; ++q) {
                float in[N];
#pragma unroll
                for (int c = 0; c < N; ++c) in[c] = xp[c * P.Wp + q];
#pragma unroll
                for (int r = 0; r < RC; ++r) {
                    const float tap = wf[r * SC + q];
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[j] = fmaf(tap, in[j * STC + r], acc[j]);
                }
            }
        } else {
            for (int r = 0; r < R; ++r)
                for (int q = 0; q < S; ++q) {
                    const float tap = wf[r * S + q];
                    const float* col = xp + r * P.Wp + q;
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[j] = fmaf(tap, col[j * ST * P.Wp], acc[j]);
                }
        }
        if (P.ep.bias != nullptr || P.ep.relu != 0) {
            const float eb = P.ep.bias ? P.ep.bias[(p0 + g) % P.n_filters] : 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float t = acc[j] + eb;
                acc[j] = P.ep.relu ? fmaxf(t, 0.f) : t;
            }
        }
        float* o = dst + g * HoWo + oi * P.Wo + oj;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (oi + j < P.Ho) o[j * P.Wo] = acc[j];
    }
}

// Frame of a plane in LDS: the rows and columns that outputs (with their four-wide groups) can touch.
void frame_of(int R, int S, int stride, int Ho, int Wo, int* Hp, int* Wp, int* QH)
{
    *QH = (Ho + 3) / 4;
    *Hp = (4 * *QH - 1) * stride + R;
    *Wp = (Wo - 1) * stride + S;
}

}  // namespace

// Planes of at most 1024 elements, at least 4 of them per workgroup's LDS, one input plane per output plane.
bool small_planes_supported(int64_t planes, int planes_per_x, int H, int W, int R, int S, int stride, int Ho, int Wo)
{
    if (planes_per_x != 1 || (int64_t)H * W > 1024 || planes < 64 || R * S > 1024 || stride > 8) return false;
    int Hp, Wp, QH;
    frame_of(R, S, stride, Ho, Wo, &Hp, &Wp, &QH);
    const int64_t per = (int64_t)Hp * Wp + R * S;
    if (per > kLdsFloats / 4) return false;
    const int64_t G = kLdsFloats / per;
    return G * Hp * Wp < 65536;
}

hipError_t launch_small_planes(const float* x, const float* w, float* y, int64_t planes, int n_filters, int H, int W,
                               int R, int S, int stride, int pad, int Ho, int Wo, hipStream_t st, const Epilogue& ep)
{
    SmallParams P;
    P.ep = ep;
    P.H = H; P.W = W; P.R = R; P.S = S; P.stride = stride; P.pad = pad; P.Ho = Ho; P.Wo = Wo;
    P.n_filters = n_filters; P.planes = planes;
    frame_of(R, S, stride, Ho, Wo, &P.Hp, &P.Wp, &P.QH);
    const int per = P.Hp * P.Wp + R * S;
    int G = kLdsFloats / per;
    // enough workgroups to fill the chip three times over before the groups grow to the LDS limit
    while (G > 4 && (planes + G - 1) / G < 3 * 256) G = (G + 1) / 2;
    if (G > 64) G = 64;
    P.G = G;
    P.by_frame = make_fastdiv(P.Hp * P.Wp);
    P.by_Wp = make_fastdiv(P.Wp);
    P.by_items = make_fastdiv(P.QH * Wo);
    P.by_Wo = make_fastdiv(Wo);
    P.by_HW = make_fastdiv(H * W);
    P.by_W = make_fastdiv(W);
    // every workgroup's run starts at plane k * G: a multiple of 16 bytes when G * H * W is a multiple of four floats
    if ((H * W) % 4 != 0 && G >= 4) G &= ~3;
    P.G = G;
    P.vec = reinterpret_cast<uintptr_t>(x) % 16 == 0 && ((int64_t)G * H * W) % 4 == 0;
    const int64_t groups = (planes + G - 1) / G;
    if (groups > 2147483647LL) return hipErrorInvalidValue;
    const size_t lds = (size_t)G * per * sizeof(float);
    dim3 grid((unsigned)groups), block(kThreads);
#define SW_SMALL(RC, STC)                                                                                     \
    if (R == RC && S == RC && stride == STC) {                                                                \
        SW_NOTED_LAUNCH(note_kernel("small_planes_kernel", (int)(RC), (int)(RC), (int)(STC)), (small_planes_kernel<RC, RC, STC>), grid, block, lds, st, x, w, y, P);             \
        return hipGetLastError();                                                                             \
    }
    SW_SMALL(3, 1) SW_SMALL(3, 2) SW_SMALL(5, 1) SW_SMALL(5, 2) SW_SMALL(7, 1)
#undef SW_SMALL
    SW_NOTED_LAUNCH(note_kernel("small_planes_kernel", (int)(0), (int)(0), (int)(0)), (small_planes_kernel<0, 0, 0>), grid, block, lds, st, x, w, y, P);
    return hipGetLastError();
}

}  // namespace swconv
