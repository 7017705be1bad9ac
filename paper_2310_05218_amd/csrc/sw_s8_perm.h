// Byte permutations shared by the int8 kernels: the matrix instruction wants 16 consecutive K bytes per lane,
// the channel-first tensors keep the channels of a pixel (of a tap) a plane (a filter) apart, so operands are
// byte-transposed in registers with v_perm_b32 on their way into LDS.
#pragma once

#include <hip/hip_runtime.h>

namespace swconv {
namespace s8perm {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32;

// byte k of the result = byte sel_k of the 8-byte value {hi, lo} (lo = bytes 0..3)
__device__ __forceinline__ u32 perm(u32 hi, u32 lo, u32 sel) { return __builtin_amdgcn_perm(hi, lo, sel); }

// Gathers bytes P0..P3 (byte positions in the dword array r) into one dword.
template <int P0, int P1, int P2, int P3>
__device__ __forceinline__ u32 gather4(const u32* r)
{
    const u32 t01 = perm(r[P1 >> 2], r[P0 >> 2], (u32)(P0 & 3) | ((u32)(4 + (P1 & 3)) << 8));
    const u32 t23 = perm(r[P3 >> 2], r[P2 >> 2], (u32)(P2 & 3) | ((u32)(4 + (P3 & 3)) << 8));
    return perm(t23, t01, 0x05040100u);
}

// out[tap][a] = channels 4a..4a+3 of tap `tap`, from raw = 16 channels x 9 taps (tap fastest)
template <int TAP, int A>
__device__ __forceinline__ u32 wgather(const u32* raw)
{
    return gather4<(4 * A) * 9 + TAP, (4 * A + 1) * 9 + TAP, (4 * A + 2) * 9 + TAP, (4 * A + 3) * 9 + TAP>(raw);
}

template <int TAP>
__device__ __forceinline__ intx4 wgather_tap(const u32* raw)
{
    intx4 v;
    v.x = (int)wgather<TAP, 0>(raw);
    v.y = (int)wgather<TAP, 1>(raw);
    v.z = (int)wgather<TAP, 2>(raw);
    v.w = (int)wgather<TAP, 3>(raw);
    return v;
}

}  // namespace s8perm
}  // namespace swconv
