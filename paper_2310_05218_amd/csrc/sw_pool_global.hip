// Global pooling of small planes (the window is the whole plane, e.g. the 7 x 7 average that ends a CNN).
// One thread per output would read 64 planes at 64 scattered addresses per load.  Here a wavefront takes 64
// consecutive planes, which are one contiguous run of 64 * H * W floats: it copies the run into LDS with
// coalesced 16-byte loads, then every lane folds its own plane out of LDS and the 64 results leave as one
// coalesced store.  The sliding sum degenerates to a single window position, so nothing slides; what is
// kept of the method is that the input is read once, in place (paper, section 2).
#include "swconv_internal.h"

#include <cmath>

namespace swconv {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

template <bool MAXIMUM>
__global__ __launch_bounds__(64) void global_pool_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                         int64_t planes, int HW, int vec_ok)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int lane = threadIdx.x;
    const int64_t p0 = (int64_t)blockIdx.x * 64;
    const int np = planes - p0 < 64 ? (int)(planes - p0) : 64;
    const int n = np * HW;                           // floats of this group's run
    const float* src = x + p0 * HW;                  // 256-byte aligned relative to x
    const int n4 = vec_ok ? n >> 2 : 0;
    for (int i = lane; i < n4; i += 64)
        reinterpret_cast<floatx4*>(lds)[i] = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(src) + i);
    for (int i = 4 * n4 + lane; i < n; i += 64) lds[i] = src[i];
    __syncthreads();
    if (lane >= np) return;
    // lane's plane starts HW floats after its neighbour's: with an even HW the lanes start their walk at
    // different offsets, so that the 64 addresses of a step fall into different banks
    const float* mine = lds + lane * HW;
    const int rot = (HW & 1) ? 0 : lane % HW;
    float acc = MAXIMUM ? -INFINITY : 0.f;
    int t = rot;
    for (int k = 0; k < HW; ++k) {
        const float e = mine[t];
        acc = MAXIMUM ? fmaxf(acc, e) : acc + e;
        t = t + 1 == HW ? 0 : t + 1;
    }
    y[p0 + lane] = MAXIMUM ? acc : acc * (1.0f / (float)HW);
}

}  // namespace

bool global_pool_supported(int H, int W, int R, int S, int pad)
{
    return R == H && S == W && pad == 0 && (int64_t)H * W <= 256;     // 64 planes of 256 floats fill 64 KB of LDS
}

hipError_t launch_global_pool(const float* x, float* y, int64_t planes, int HW, bool maximum, hipStream_t st)
{
    const int64_t groups = (planes + 63) / 64;
    if (groups > 2147483647LL) return hipErrorInvalidValue;
    const int vec_ok = reinterpret_cast<uintptr_t>(x) % 16 == 0;
    const size_t lds = (size_t)64 * HW * sizeof(float);
    if (maximum)
        SW_NOTED_LAUNCH(note_kernel("global_pool_kernel", (int)(true)), global_pool_kernel<true>, dim3((unsigned)groups), dim3(64), lds, st, x, y, planes, HW, vec_ok);
    else
        SW_NOTED_LAUNCH(note_kernel("global_pool_kernel", (int)(false)), global_pool_kernel<false>, dim3((unsigned)groups), dim3(64), lds, st, x, y, planes, HW, vec_ok);
    return hipGetLastError();
}

}  // namespace swconv
