// 16-bit (bf16 or IEEE half) multi-channel convolution on channel-last tensors with the pixel operand read straight
// from global memory (paper, section 3: every tap a small matrix product; section 1.1: reduced precision on the same
// sliding sums).
//
//   x [N, H, W, C]     w [C_out, R, S, C]     y [N, H_out, W_out, C_out]     16-bit patterns, fp32 sums
//
// The two formats differ in the matrix instruction (v_mfma_f32_32x32x16_bf16 / _f16; a product of two 16-bit values
// is exact in fp32 in both) and in the one rounding of the finished value (nearest even in both; half precision
// overflows to infinity beyond 65504 and keeps its denormals).
//
// With the channel as the fastest axis, the operand of v_mfma_f32_32x32x16_bf16 for (pixel, tap, 16 channels) is, per
// lane, 16 consecutive and 16-byte aligned bytes of x: eight channels of the pixel the tap shifts the lane's output
// pixel to.  A lane loads them itself with one buffer load; a tap that falls into the padding is an offset beyond the
// buffer's extent, for which the load returns zeros.  No window is staged, no barrier sits in the loop, and the address
// arithmetic of the loads runs on the vector pipe beside the bf16 matrix instructions (measured: the two overlap, unlike
// fp32 matrix instructions).  The filters of the workgroup's CB * 32 output channels (all taps, all channels; rows of w
// as they lie in memory) are copied to LDS once.
//
// A wavefront owns PB blocks of 32 consecutive output pixels (counted through all images) and CB blocks of 32 output
// channels.  Filters are the A operand, pixels the B operand, so a lane of the result holds, for its own pixel, groups
// of four consecutive output channels: 8-byte stores.  One iteration is (tap, 16 channels): PB loads, CB LDS reads,
// PB * CB matrix instructions; the loads run two iterations ahead in a ring of three register sets.
//
// What bounds it: a load instruction touches 32 pixels, 32 bytes of each pixel's 128-byte line, so the vector memory
// path looks up four times as many lines as it moves whole ones.  32 x 56 x 56 x 64 -> 64, 3 x 3: 113 k loads x 32
// lines on 256 CUs, 29 us (the kernel that stages a window in LDS: 42 us); 1 x 1 256 -> 64: 21 us (52), 64 -> 256:
// 31 us (105), 3 x 3 stride 2 64 -> 128: 19 us (48), 3 x 3 32 -> 32 at 112 x 112: 32 us (122).
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

constexpr size_t kLdsMax = 150 * 1024;
constexpr int kRing = 3;                        // register sets of pixel operands (4, 6 and 8 measured no faster)
constexpr unsigned kBeyond = 0x80000000u;      // a byte offset no tensor of less than 2 GiB reaches

struct NdParams {
    Epilogue ep;
    int H, W, C, C_out, R, S, stride, pad, dil, Ho, Wo;
    int total_px;      // N * Ho * Wo
    int tiles;         // of 32 * PB pixels
    int KS;            // steps of 16 channels per tap
    int IT;            // R * S * KS iterations
    int wpitch;        // bytes between output channels' filters in LDS
    int w16;           // 16-byte pieces of an output channel's filters
    unsigned x_bytes;
    FastDiv by_KS, by_S, by_w16;
};

__device__ __forceinline__ unsigned bf16_rne_bits(float f)
{
    unsigned u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ unsigned f16_rne_bits(float f)
{
    return (unsigned)__builtin_bit_cast(unsigned short, (_Float16)f);      // v_cvt_f16_f32: nearest even
}

// wavefronts per SIMD the register file holds: accumulators, the ring of pixel operands, two sets of filter operands,
// per-block bookkeeping and about 30 more
constexpr int waves_per_simd(int cb, int pb, int nb)
{
    const int regs = 16 * cb * pb + 4 * nb * pb + 8 * cb + 4 * pb + 30;
    return 512 / regs > 4 ? 4 : 512 / regs < 1 ? 1 : 512 / regs;
}

// F16: IEEE half precision (else bf16)
template <int CB, int PB, int NB, bool F16>
__global__ __launch_bounds__(256, waves_per_simd(CB, PB, NB)) void mfma_bf16_nhwc_direct_kernel(const unsigned char* __restrict__ x,
                                                                       const unsigned char* __restrict__ w,
                                                                       unsigned short* __restrict__ y, const NdParams P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lw[];     // [CB * 32][wpitch]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lj = lane & 31, kq = lane >> 5;
    const int co0 = blockIdx.y * (CB * 32);

    // filters: rows co0 .. co0 + CB * 32 - 1 (zero beyond C_out), 16 bytes at a time, eight loads in flight per thread
    {
        const int total = CB * 32 * P.w16;
        const int64_t row_bytes = (int64_t)P.w16 * 16;
#pragma unroll 1
        for (int i0 = tid; i0 < total; i0 += 8 * 256) {
            intx4 v[8];
            int at[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + 256 * u, ic = i < total ? i : total - 1;
                const int row = fast_div(ic, P.by_w16), g = ic - row * P.w16;
                at[u] = i < total ? row * P.wpitch + 16 * g : -1;
                const int rc = co0 + row < P.C_out ? co0 + row : P.C_out - 1;
                v[u] = *reinterpret_cast<const intx4*>(w + rc * row_bytes + 16 * g);
                if (co0 + row >= P.C_out) v[u] = intx4{0, 0, 0, 0};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (at[u] >= 0) *reinterpret_cast<intx4*>(lw + at[u]) = v[u];
        }
    }
    __syncthreads();

    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(x), 0, P.x_bytes, 0x00020000);
    const unsigned char* arow = lw + lj * P.wpitch + 16 * kq;      // + cb * 32 * wpitch + 32 it
    const int IT = P.IT, IT3 = IT - IT % NB;
    const int HoWo = P.Ho * P.Wo;
    const int nwaves = (int)gridDim.x * 4;
#pragma unroll 1
    for (int tile = (int)blockIdx.x * 4 + wave; tile < P.tiles; tile += nwaves) {
        // the lane's pixel in each block: byte offset of (tap (0, 0), its half of the first 16 channels), and which
        // filter rows / columns fall inside the image for it (bit r / bit s)
        int base[PB];
        unsigned rows_in[PB], cols_in[PB];
        int ypix[PB];                                       // flat output pixel, -1: none
#pragma unroll
        for (int b = 0; b < PB; ++b) {
            const int p = tile * (32 * PB) + 32 * b + lj;
            const bool live = p < P.total_px;
            const int pc = live ? p : 0;
            const int n = pc / HoWo, rem = pc - n * HoWo;
            const int oh = rem / P.Wo, ow = rem - oh * P.Wo;
            const int ih0 = oh * P.stride - P.pad, iw0 = ow * P.stride - P.pad;
            base[b] = ((n * P.H + ih0) * P.W + iw0) * (2 * P.C) + 16 * kq;
            unsigned rm = 0, cm = 0;
            for (int r = 0; r < P.R; ++r) rm |= (unsigned)((unsigned)(ih0 + r * P.dil) < (unsigned)P.H) << r;
            for (int s = 0; s < P.S; ++s) cm |= (unsigned)((unsigned)(iw0 + s * P.dil) < (unsigned)P.W) << s;
            rows_in[b] = rm;
            cols_in[b] = cm;
            ypix[b] = live ? p : -1;
        }

        floatx16 acc[CB][PB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int b = 0; b < PB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[cb][b][v] = 0.f;

        intx4 bq[NB][PB];
        // iteration it = (tap, step of 16 channels) into register set `buf`; past the last iteration the last one again
        auto fetch = [&](int buf, int it) __attribute__((always_inline)) {
            const int itc = it < IT ? it : IT - 1;
            const int tap = fast_div(itc, P.by_KS), ks = itc - tap * P.KS;
            const int r = fast_div(tap, P.by_S), s = tap - r * P.S;
            const int toff = ((r * P.dil) * P.W + s * P.dil) * (2 * P.C) + 32 * ks;        // (wave-uniform)
#pragma unroll
            for (int b = 0; b < PB; ++b) {
                const bool in = ((rows_in[b] >> r) & (cols_in[b] >> s) & 1u) != 0;
                const unsigned off = in ? (unsigned)(base[b] + toff) : kBeyond;
                bq[buf][b] = __builtin_amdgcn_raw_buffer_load_b128(xr, off, 0, 0);
            }
        };
        auto read_a = [&](intx4 (&a)[CB], int it) __attribute__((always_inline)) {
            const int itc = it < IT ? it : IT - 1;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) a[cb] = *reinterpret_cast<const intx4*>(arow + cb * 32 * P.wpitch + 32 * itc);
        };
        auto multiply = [&](const intx4 (&a)[CB], int buf) __attribute__((always_inline)) {
#pragma unroll
            for (int b = 0; b < PB; ++b)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    if constexpr (F16)
                        acc[cb][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, a[cb]),
                                                                            __builtin_bit_cast(halfx8, bq[buf][b]), acc[cb][b], 0, 0, 0);
                    else
                        acc[cb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[cb]),
                                                                             __builtin_bit_cast(bf16x8, bq[buf][b]), acc[cb][b], 0, 0, 0);
                }
        };

#pragma unroll
        for (int i = 0; i < NB; ++i) fetch(i, i);
        intx4 a[2][CB];
        read_a(a[0], 0);
#pragma unroll 1
        for (int it = 0; it < IT3; it += NB) {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                read_a(a[(i + 1) & 1], it + i + 1);
                multiply(a[i & 1], i);
                __builtin_amdgcn_sched_barrier(0);
                fetch(i, it + NB + i);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (NB & 1) {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) a[0][cb] = a[1][cb];
            }
        }
#pragma unroll
        for (int i = 0; i < NB - 1; ++i) {
            if (IT3 + i < IT) {
                read_a(a[(i + 1) & 1], IT3 + i + 1);
                multiply(a[i & 1], i);
            }
        }

        // register v of a lane is output channel 8 (v / 4) + 4 kq + v % 4 of the block, for the lane's pixel
#pragma unroll
        for (int b = 0; b < PB; ++b) {
            if (ypix[b] < 0) continue;
            unsigned short* yp = y + (int64_t)ypix[b] * P.C_out;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int co = co0 + cb * 32 + 8 * i + 4 * kq;
                    if (co < P.C_out) {
                        unsigned h[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const float t = apply_epilogue(acc[cb][b][4 * i + j], co + j, P.ep);
                            h[j] = F16 ? f16_rne_bits(t) : bf16_rne_bits(t);
                        }
                        *reinterpret_cast<intx2*>(yp + co) = intx2{(int)(h[0] | (h[1] << 16)), (int)(h[2] | (h[3] << 16))};
                    }
                }
        }
    }
}

struct NdPlan {
    bool ok = false;
    int CB = 0, PB = 0;
    size_t lds = 0;
    NdParams P;
};

NdPlan plan_direct(const Conv2dShape& s, const void* x, const void* w, const void* y)
{
    NdPlan a;
    const int RS = s.R * s.S;
    const int64_t x_bytes = (int64_t)s.N * s.H * s.W * s.C_in * 2, px = (int64_t)s.N * s.Ho * s.Wo;
    if (s.C_in % 16 != 0 || s.C_out % 4 != 0 || s.R > 32 || s.S > 32) return a;
    if (x_bytes >= (1LL << 31) || px >= (1LL << 31) - (1 << 20) || (int64_t)RS * s.C_in * 2 >= (1 << 20)) return a;
    if (reinterpret_cast<uintptr_t>(x) % 16 != 0 || reinterpret_cast<uintptr_t>(w) % 16 != 0 || reinterpret_cast<uintptr_t>(y) % 8 != 0) return a;
    const int row = RS * s.C_in * 2;                                   // bytes of an output channel's filters
    const int wpitch = row + 16 + (128 - row % 128) % 128;              // 16 modulo 128: 32 rows, 32 different 16-byte banks
    const auto fits = [&](int cb) { return (size_t)cb * 32 * wpitch <= kLdsMax; };
    const auto units = [&](int cb, int pb) { return ((px + 32 * pb - 1) / (32 * pb)) * ((s.C_out + 32 * cb - 1) / (32 * cb)); };
    // (channel blocks, pixel blocks) per wavefront: 2 x 2 measured best of 2 x 4, 4 x 2, 1 x 4, 2 x 2, 1 x 2, 2 x 1, 4 x 1 on
    // every layer tried but one; 1 x 2 when two blocks' filters do not fit LDS or would leave SIMDs without a tile
    static const int kVariants[][2] = {{2, 2}, {1, 2}};
    for (const auto& v : kVariants) {
        if (!fits(v[0])) continue;
        a.CB = v[0];
        a.PB = v[1];
        a.ok = true;
        if (units(v[0], v[1]) >= 700) break;
    }
    if (!a.ok) return a;
    a.lds = (size_t)a.CB * 32 * wpitch;
    NdParams& P = a.P;
    P.H = s.H; P.W = s.W; P.C = s.C_in; P.C_out = s.C_out; P.R = s.R; P.S = s.S; P.stride = s.stride; P.pad = s.pad;
    P.dil = s.dil; P.Ho = s.Ho; P.Wo = s.Wo;
    P.total_px = (int)px;
    P.tiles = (int)((px + 32 * a.PB - 1) / (32 * a.PB));
    P.KS = s.C_in / 16;
    P.IT = RS * P.KS;
    P.wpitch = wpitch;
    P.w16 = row / 16;
    P.x_bytes = (unsigned)x_bytes;
    P.by_KS = make_fastdiv(P.KS);
    P.by_S = make_fastdiv(s.S);
    P.by_w16 = make_fastdiv(P.w16);
    return a;
}

template <int CB, int PB, int NB, bool F16>
hipError_t launch_direct(const void* x, const void* w, void* y, const Conv2dShape& s, NdPlan& a, const Epilogue& ep, hipStream_t st)
{
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_bf16_nhwc_direct_kernel<CB, PB, NB, F16>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax);
    if (attr != hipSuccess) return attr;
    a.P.ep = ep;
    const int gy = (s.C_out + CB * 32 - 1) / (CB * 32);
    int per_cu = (int)((160 * 1024) / (a.lds + 512));
    if (per_cu > 4) per_cu = 4;
    if (per_cu < 1) per_cu = 1;
    int gx = (a.P.tiles + 3) / 4;
    const int cap = (256 * per_cu + gy - 1) / gy;
    if (gx > cap) gx = cap;
    SW_NOTED_LAUNCH(note_kernel(F16 ? "mfma_f16_nhwc_direct_kernel" : "mfma_bf16_nhwc_direct_kernel", CB, PB),
                    (mfma_bf16_nhwc_direct_kernel<CB, PB, NB, F16>),
                    dim3((unsigned)gx, (unsigned)gy), dim3(256), a.lds, st, static_cast<const unsigned char*>(x),
                    static_cast<const unsigned char*>(w), static_cast<unsigned short*>(y), a.P);
    return hipGetLastError();
}

}  // namespace

bool mfma_bf16_nhwc_direct_supported(const void* x, const void* w, const void* y, const Conv2dShape& s)
{
    return plan_direct(s, x, w, y).ok;
}

hipError_t launch_mfma_bf16_nhwc_direct(const void* x, const void* w, void* y, const Conv2dShape& s, bool f16, const Epilogue& ep,
                                        hipStream_t st)
{
    NdPlan a = plan_direct(s, x, w, y);
    if (!a.ok) return hipErrorInvalidValue;
#define SW_ND(CBC, PBC)                                                                                  \
    if (a.CB == CBC && a.PB == PBC)                                                                      \
        return f16 ? launch_direct<CBC, PBC, kRing, true>(x, w, y, s, a, ep, st)                         \
                   : launch_direct<CBC, PBC, kRing, false>(x, w, y, s, a, ep, st)
    SW_ND(2, 2); SW_ND(1, 2);
#undef SW_ND
    return hipErrorInvalidValue;
}

}  // namespace swconv
