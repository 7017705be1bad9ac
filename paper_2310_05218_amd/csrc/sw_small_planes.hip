// Depthwise sliding window sums over SMALL planes (14 x 14, 7 x 7, ... -- the tail of a CNN), any filter
// extent, stride and padding (paper, section 1.2: depthwise convolutions; section 2: the input is used as it
// lies in memory).
//
// A 56 x 56 tile per wavefront wastes most of its lanes on such planes, and one thread per output reads them
// with scattered accesses.  Here a workgroup takes a run of consecutive planes -- which is one contiguous run
// of memory, whatever the plane's width -- and brings it into LDS once with coalesced loads (16 bytes per lane
// when the run is aligned), together with the planes' filters.  Every thread then produces outputs idx,
// idx + 256, ... of the run: the window of an output is read from LDS at shifted addresses (positions outside
// the plane are the zero padding and are skipped), and since consecutive outputs are consecutive in memory
// the stores are coalesced as they are.
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kLdsFloats = 12 * 1024;      // 48 KB per workgroup: three workgroups per CU

struct SmallParams {
    int H, W, R, S, stride, pad, Ho, Wo, n_filters, G;
    int64_t planes;
    FastDiv by_HoWo, by_Wo;
};

// RC, SC > 0: filter extent at compile time (taps unrolled); 0: at run time.
template <int RC, int SC>
__global__ __launch_bounds__(kThreads) void small_planes_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                                float* __restrict__ y, const SmallParams P, int x_vec_ok)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int R = RC > 0 ? RC : P.R, S = RC > 0 ? SC : P.S;
    const int HW = P.H * P.W, RS = R * S, HoWo = P.Ho * P.Wo;
    const int tid = threadIdx.x;
    const int64_t p0 = (int64_t)blockIdx.x * P.G;
    const int np = P.planes - p0 < P.G ? (int)(P.planes - p0) : P.G;
    float* xs = lds;                               // [np][HW]
    float* ws = lds + ((P.G * HW + 3) & ~3);       // [np][RS]

    // the run of planes, as it lies in memory
    const int n = np * HW;
    const float* src = x + p0 * HW;
    const int n4 = (x_vec_ok && ((p0 * HW) & 3) == 0) ? n >> 2 : 0;
    for (int i = tid; i < n4; i += kThreads)
        reinterpret_cast<floatx4*>(xs)[i] = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(src) + i);
    for (int i = 4 * n4 + tid; i < n; i += kThreads) xs[i] = src[i];
    // the filters of these planes (plane p uses filter p % n_filters)
    for (int i = tid; i < np * RS; i += kThreads) {
        const int g = i / RS;
        ws[i] = w[(int64_t)((p0 + g) % P.n_filters) * RS + (i - g * RS)];
    }
    __syncthreads();

    float* dst = y + p0 * HoWo;
    for (int idx = tid; idx < np * HoWo; idx += kThreads) {
        const int g = fast_div(idx, P.by_HoWo);
        const int pix = idx - g * HoWo;
        const int oi = fast_div(pix, P.by_Wo), oj = pix - oi * P.Wo;
        const int h0 = oi * P.stride - P.pad, v0 = oj * P.stride - P.pad;
        const float* xg = xs + g * HW;
        const float* wf = ws + g * RS;
        float acc = 0.f;
        if (RC > 0) {
#pragma unroll
            for (int r = 0; r < (RC > 0 ? RC : 1); ++r)
#pragma unroll
                for (int q = 0; q < (SC > 0 ? SC : 1); ++q) {
                    // (positions outside the plane read element 0 and count as zero: no address leaves the plane)
                    const bool in = (unsigned)(h0 + r) < (unsigned)P.H && (unsigned)(v0 + q) < (unsigned)P.W;
                    const float e = xg[in ? (h0 + r) * P.W + v0 + q : 0];
                    acc = fmaf(wf[r * SC + q], in ? e : 0.f, acc);
                }
        } else {
            const int r_lo = h0 < 0 ? -h0 : 0, r_hi = P.H - h0 < R ? P.H - h0 : R;
            const int q_lo = v0 < 0 ? -v0 : 0, q_hi = P.W - v0 < S ? P.W - v0 : S;
            for (int r = r_lo; r < r_hi; ++r)
                for (int q = q_lo; q < q_hi; ++q) acc = fmaf(wf[r * S + q], xg[(h0 + r) * P.W + v0 + q], acc);
        }
        dst[idx] = acc;
    }
}

}  // namespace

// Planes of at most 1024 elements, at least 8 of them per workgroup's LDS, one input plane per output plane.
bool small_planes_supported(int64_t planes, int planes_per_x, int H, int W, int R, int S, int Ho, int Wo)
{
    if (planes_per_x != 1 || (int64_t)H * W > 1024 || planes < 64) return false;
    const int G = kLdsFloats / (H * W + R * S + 1);
    return G >= 8 && (int64_t)G * Ho * Wo < 65536 && R * S <= 1024;
}

hipError_t launch_small_planes(const float* x, const float* w, float* y, int64_t planes, int n_filters, int H, int W,
                               int R, int S, int stride, int pad, int Ho, int Wo, hipStream_t st)
{
    SmallParams P;
    P.H = H; P.W = W; P.R = R; P.S = S; P.stride = stride; P.pad = pad; P.Ho = Ho; P.Wo = Wo;
    P.n_filters = n_filters; P.planes = planes;
    int G = kLdsFloats / (H * W + R * S + 1);
    // enough workgroups to fill the chip three times over before the groups grow to the LDS limit
    while (G > 8 && (planes + G - 1) / G < 3 * 256) G = (G + 1) / 2;
    if (G > 64) G = 64;
    P.G = G;
    P.by_HoWo = make_fastdiv(Ho * Wo);
    P.by_Wo = make_fastdiv(Wo);
    const int64_t groups = (planes + G - 1) / G;
    if (groups > 2147483647LL) return hipErrorInvalidValue;
    const size_t lds = (size_t)(((G * H * W + 3) & ~3) + G * R * S) * sizeof(float);
    const int x_vec_ok = reinterpret_cast<uintptr_t>(x) % 16 == 0;
    dim3 grid((unsigned)groups), block(kThreads);
    if (R == 3 && S == 3)
        hipLaunchKernelGGL((small_planes_kernel<3, 3>), grid, block, lds, st, x, w, y, P, x_vec_ok);
    else if (R == 5 && S == 5)
        hipLaunchKernelGGL((small_planes_kernel<5, 5>), grid, block, lds, st, x, w, y, P, x_vec_ok);
    else
        hipLaunchKernelGGL((small_planes_kernel<0, 0>), grid, block, lds, st, x, w, y, P, x_vec_ok);
    return hipGetLastError();
}

}  // namespace swconv
