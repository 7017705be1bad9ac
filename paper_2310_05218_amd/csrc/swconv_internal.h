// Internal declarations shared by the translation units of libswconv.so.
// Launchers take validated arguments, enqueue on the given stream and return
// the HIP error of the launch.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swconv {

enum Op1D { OP_CONV = 0, OP_AVG = 1, OP_MAX = 2 };

// Division by a run-time constant without the integer divide sequence: exact while n * d < 2^32.
struct FastDiv {
    uint32_t d, magic;
};
inline FastDiv make_fastdiv(int d)
{
    return FastDiv{(uint32_t)d, d == 1 ? 0u : (uint32_t)(0x100000000ULL / (uint32_t)d) + 1u};
}
__device__ __forceinline__ int fast_div(int n, FastDiv f) { return f.magic ? (int)__umulhi((uint32_t)n, f.magic) : n; }

struct Conv2dShape {
    int N, C_in, C_out, H, W, R, S, stride, pad, Ho, Wo;
    int dil = 1;      // input positions between neighbouring taps (the any-shape fp32, run-time-extent tile and direct kernels take > 1)
};

// A launch plan found by a search over tilings costs host time that a small layer cannot hide behind its own run time.
// Each host thread keeps the plans of the shapes it saw last.  A plan may depend on the shape and on the low four address
// bits of up to three buffers, on nothing else.
template <class Plan>
struct PlanCache {
    struct Entry {
        bool used = false;
        Conv2dShape s;
        unsigned align = 0;
        Plan plan;
    };
    static constexpr int kEntries = 16;
    Entry e[kEntries];
    int next = 0;
    static unsigned low_bits(const void* a, const void* b, const void* c)
    {
        return (unsigned)(reinterpret_cast<uintptr_t>(a) & 15) | (unsigned)(reinterpret_cast<uintptr_t>(b) & 15) << 4 |
               (unsigned)(reinterpret_cast<uintptr_t>(c) & 15) << 8;
    }
    static bool same(const Conv2dShape& a, const Conv2dShape& b)
    {
        return a.N == b.N && a.C_in == b.C_in && a.C_out == b.C_out && a.H == b.H && a.W == b.W && a.R == b.R && a.S == b.S &&
               a.stride == b.stride && a.pad == b.pad && a.Ho == b.Ho && a.Wo == b.Wo && a.dil == b.dil;
    }
    template <class Search>
    const Plan& get(const Conv2dShape& s, unsigned align, Search&& search)
    {
        for (int i = 0; i < kEntries; ++i)
            if (e[i].used && e[i].align == align && same(e[i].s, s)) return e[i].plan;
        Entry& n = e[next];
        next = (next + 1) % kEntries;
        n.used = true; n.s = s; n.align = align; n.plan = search();
        return n.plan;
    }
};

// Per-channel bias and rectifier on an fp32 sum on its way out: y = relu ? max(acc + bias[co], 0) : acc + bias[co]
// (one fp32 addition).  bias may be null.
struct Epilogue {
    const float* bias;
    int relu;
};
__device__ __forceinline__ float apply_epilogue(float acc, int co, const Epilogue& e)
{
    float t = acc;
    if (e.bias) t += e.bias[co];
    if (e.relu) t = fmaxf(t, 0.0f);
    return t;
}

// Requantisation of an exact int32 sum to int8, per output channel:
//     q = clamp(rne(scale[co] * float(acc + bias[co])), relu ? 0 : -128, 127)
// with the conversion, the product and the rounding in fp32 (v_cvt_f32_i32, v_mul_f32, v_rndne_f32: the
// same IEEE operations as the definition).  bias may be null.
struct Requant {
    const int32_t* bias;
    const float* scale;
    int relu;
};
__device__ __forceinline__ int8_t requant_s8(int acc, int co, const Requant& rq)
{
    const int t = acc + (rq.bias ? rq.bias[co] : 0);
    float r = rintf(__int2float_rn(t) * rq.scale[co]);
    r = fmaxf(r, rq.relu ? 0.0f : -128.0f);
    r = fminf(r, 127.0f);
    return (int8_t)(int)r;
}

// Records the kernel a launcher is about to enqueue (name and up to four template arguments) for the calling
// thread; sw_last_kernel() reports it.  Costs a few stores per launch.
void note_kernel(const char* name, int a = -1, int b = -1, int c = -1, int d = -1);
// A launch with its note, as one statement.
#define SW_NOTED_LAUNCH(note_call, ...)      \
    do {                                     \
        note_call;                           \
        hipLaunchKernelGGL(__VA_ARGS__);     \
    } while (0)

// ---- direct (one thread per output) kernels: any valid shape -------------------------------
hipError_t launch_direct_1d(const float* x, const float* w, float* y, int64_t rows, int64_t len,
                            int64_t len_out, int k, int stride, int pad, Op1D op, hipStream_t st);
hipError_t launch_direct_conv2d_f32(const float* x, const float* w, float* y, const Conv2dShape& s,
                                    bool depthwise, hipStream_t st, const Epilogue* ep = nullptr);
hipError_t launch_direct_conv2d_s8(const int8_t* x, const int8_t* w, int32_t* y, const Conv2dShape& s,
                                   hipStream_t st);
hipError_t launch_direct_pool2d(const float* x, float* y, int64_t planes, int H, int W, int R, int S, int stride,
                                int pad, int Ho, int Wo, bool maximum, hipStream_t st);

// ---- sliding 1-D kernel (stride 1): LDS tile + halo, register window ---------------------------
bool       sliding_1d_supported(int64_t len, int k, int stride, int pad);
hipError_t launch_sliding_1d(const float* x, const float* w, float* y, int64_t rows, int64_t len,
                             int64_t len_out, int k, int pad, Op1D op, hipStream_t st);

// ---- 1-D kernel for strides 2..8: contiguous input run per tile through LDS ---------------------------------
bool       strided_1d_supported(int64_t rows, int64_t len, int64_t len_out, int k, int stride, int pad);
hipError_t launch_strided_1d(const float* x, const float* w, float* y, int64_t rows, int64_t len, int64_t len_out,
                             int k, int stride, int pad, Op1D op, hipStream_t st);

// ---- pooling whose windows tile the rows (stride == window in {2, 4, 8}): registers only --------------------
bool       pool_tiles_supported(const float* x, const float* y, int64_t len, int window, int stride);
hipError_t launch_pool_tiles(const float* x, float* y, int64_t rows, int64_t len, int window, bool maximum,
                             hipStream_t st);

// ---- sliding plane kernel (stride 1): one filter per plane (single channel, depthwise) --------
// x plane index for output plane p is p / planes_per_x (conv2d with C_in == 1: C_out filters share
// one input plane; depthwise: 1); filter index is p % n_filters.
bool       sliding_plane_supported(int H, int W, int R, int S, int stride, int pad, int dil = 1);
bool       sliding_plane_worthwhile(int64_t planes, int Ho, int Wo, int R, int S);
bool       sliding_plane_whole(const float* x, const float* y, int H, int W, int R, int S, int pad, int Ho, int Wo);

// ---- sliding rows kernel (stride 1 or 2; 3x3 / 5x5 filters, 2x2 / 3x3 pooling windows): registers only,
// DPP wavefront shifts for the halo ---------------------------------------------------------------
bool       sliding_rows_supported(const float* x, int H, int W, int R, int S, int stride, int pad);
hipError_t launch_sliding_rows(const float* x, const float* w, float* y, int64_t planes, int planes_per_x,
                               int n_filters, int H, int W, int R, int S, int stride, int pad, int Ho, int Wo,
                               hipStream_t st, const Epilogue& ep = Epilogue{nullptr, 0});
bool       pool_rows_supported(const float* x, int W, int R, int S, int stride, int pad);
hipError_t launch_pool_rows(const float* x, float* y, int64_t planes, int H, int W, int R, int stride, int pad,
                            int Ho, int Wo, bool maximum, hipStream_t st);
hipError_t launch_sliding_plane(const float* x, const float* w, float* y, int64_t planes,
                                int planes_per_x, int n_filters, int H, int W, int R, int S, int pad,
                                int Ho, int Wo, hipStream_t st, const Epilogue& ep = Epilogue{nullptr, 0}, int dil = 1);

// ---- multi-channel fp32, few taps (1x1 ... 4x4), C_in % 8 == 0, any stride / padding / dilation: both operands
// brought into LDS by direct-to-LDS loads, two stages (16-byte aligned w, tensors below 2 GiB)
bool       mfma_f32_dma_supported(const Conv2dShape& s, const float* x, const float* w);
hipError_t launch_mfma_f32_dma(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st,
                               const Epilogue& ep = Epilogue{nullptr, 0});

// ---- fp32 / bf16 / half multi-channel convolution on channel-last tensors ------------------------------------
enum Elem { kElemF32 = 0, kElemBF16 = 1, kElemF16 = 2 };      // element format of x, w and y
constexpr int elem_size(int ek) { return ek == kElemF32 ? 4 : 2; }
bool       mfma_nhwc_supported(const void* x, const void* w, const Conv2dShape& s, int ek);
hipError_t launch_mfma_nhwc(const void* x, const void* w, void* y, const Conv2dShape& s, int ek, const Epilogue& ep,
                            hipStream_t st);
// 16-bit formats with the pixel operand read straight from global memory (C_in % 16 == 0, C_out % 4 == 0, filters of
// the channel block resident in LDS)
bool       mfma_bf16_nhwc_direct_supported(const void* x, const void* w, const void* y, const Conv2dShape& s);
hipError_t launch_mfma_bf16_nhwc_direct(const void* x, const void* w, void* y, const Conv2dShape& s, bool f16, const Epilogue& ep,
                                        hipStream_t st);
// fp32 and the 16-bit formats (ek: Elem) with both operands in LDS, the window by direct-to-LDS loads (pixels of whole
// 32 bytes, C_out % 4 == 0, tiles of output rows at most 256 outputs wide whose windows fit LDS)
bool       mfma_nhwc_lds_supported(const void* x, const void* w, const void* y, const Conv2dShape& s, int ek);
hipError_t launch_mfma_nhwc_lds(const void* x, const void* w, void* y, const Conv2dShape& s, int ek, const Epilogue& ep, hipStream_t st);
// the same kernel on int8 tensors: exact int32 sums, leaving as int32 (rq null) or requantised to int8 (C_in % 32 == 0)
bool       mfma_s8_nhwc_lds_supported(const int8_t* x, const int8_t* w, const void* y, bool requant, const Conv2dShape& s);
hipError_t launch_mfma_s8_nhwc_lds(const int8_t* x, const int8_t* w, void* y, const Requant* rq, const Conv2dShape& s, hipStream_t st);
hipError_t launch_direct_nhwc(const void* x, const void* w, void* y, const Conv2dShape& s, int ek, const Epilogue& ep,
                              hipStream_t st);

// ---- depthwise 3x3 (stride 1, padding 1) -> pointwise 1x1 in one launch, the intermediate only in LDS
bool       dw_pw_block_supported(int N, int C, int C_out, int H, int W);
hipError_t launch_dw_pw_block(const float* x, const float* w_dw, const float* b_dw, const float* w_pw, const float* b_pw,
                              float* y, int N, int C, int C_out, int H, int W, int relu1, int relu2, hipStream_t st);

// ---- int8 on channel-last tensors (x [N,H,W,C_in], w [C_out,R,S,C_in], y [N,Ho,Wo,C_out]); rq == nullptr: int32 out
bool       mfma_s8_nhwc_supported(const int8_t* x, const int8_t* w, const Conv2dShape& s);
hipError_t launch_mfma_s8_nhwc(const int8_t* x, const int8_t* w, int32_t* y, int8_t* y8, const Requant* rq,
                               const Conv2dShape& s, hipStream_t st);
hipError_t launch_direct_s8_nhwc(const int8_t* x, const int8_t* w, int32_t* y, int8_t* y8, const Requant* rq,
                                 const Conv2dShape& s, hipStream_t st);

// ---- bf16 activations (bit patterns in unsigned short), fp32 filters and accumulation --------------------
bool       sliding_plane_bf16_supported(const void* x, const void* y, int H, int W, int R, int S, int stride, int pad, int Ho,
                                        int Wo);
hipError_t launch_sliding_plane_bf16(const unsigned short* x, const float* w, unsigned short* y, int64_t planes,
                                     int n_filters, int H, int W, int R, int pad, int Ho, int Wo, hipStream_t st);
hipError_t launch_direct_depthwise_bf16(const unsigned short* x, const float* w, unsigned short* y,
                                        const Conv2dShape& s, hipStream_t st);

// ---- sw_jit.hip: one-filter-per-plane kernels compiled at run time, one per geometry (status codes) ------
bool       jit_plane_supported(const float* x, const float* y, int H, int W, int R, int S, int stride, int pad, int dil = 1);
int        jit_prepare_plane(int H, int W, int R, int S, int stride, int pad, int dil = 1);
int        jit_compile_only(int H, int W, int R, int S, int stride, int pad, int dil = 1);
int        jit_cached_kernels();
int        jit_launch_plane(const float* x, const float* w, float* y, int64_t planes, int planes_per_x, int n_filters,
                            int H, int W, int R, int S, int stride, int pad, int dil, hipStream_t st);

// ---- depthwise on small planes (at most 1024 elements): a run of planes per workgroup through LDS --------
bool       small_planes_supported(int64_t planes, int planes_per_x, int H, int W, int R, int S, int stride, int Ho,
                                  int Wo);
hipError_t launch_small_planes(const float* x, const float* w, float* y, int64_t planes, int n_filters, int H, int W,
                               int R, int S, int stride, int pad, int Ho, int Wo, hipStream_t st,
                               const Epilogue& ep = Epilogue{nullptr, 0});

// ---- global pooling of planes of at most 256 elements: 64 planes per wavefront through LDS ----------------
bool       global_pool_supported(int H, int W, int R, int S, int pad);
hipError_t launch_global_pool(const float* x, float* y, int64_t planes, int HW, bool maximum, hipStream_t st);

// ---- multi-channel kernels on the matrix cores (stride 1) --------------------------------------
bool       mfma_f32_supported(const Conv2dShape& s);
hipError_t launch_mfma_f32(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st,
                           const Epilogue& ep = Epilogue{nullptr, 0});
int64_t    mfma_f32_workgroups(const Conv2dShape& s);     // of the fixed 3x3 / 5x5 kernel, one per CU at a time; 0: tiles half empty
bool       mfma_f32_any_supported(const Conv2dShape& s);  // any extent, stride and channel count (C_in >= 2)
hipError_t launch_mfma_f32_any(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st,
                               const Epilogue& ep = Epilogue{nullptr, 0});
bool       mfma_f32_rows_supported(const Conv2dShape& s, const float* x); // large filters: one filter row of a channel chunk at a time
hipError_t launch_mfma_f32_rows(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st,
                                const Epilogue& ep = Epilogue{nullptr, 0});
// 1 x 1, stride 1, no padding, C_in a multiple of 8: B operands straight from global memory, filters resident in LDS
bool       mfma_f32_pointwise_supported(const Conv2dShape& s, const float* x, const float* w, const float* y);
hipError_t launch_mfma_f32_pointwise(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st,
                                     const Epilogue& ep = Epilogue{nullptr, 0});
bool       mfma_f32_quad_supported(const Conv2dShape& s); // the same for few taps (R * S <= 12): 16-byte operand reads
hipError_t launch_mfma_f32_quad(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st,
                                const Epilogue& ep = Epilogue{nullptr, 0});
bool       mfma_s8_supported(const Conv2dShape& s);
hipError_t launch_mfma_s8(const int8_t* x, const int8_t* w, int32_t* y, const Conv2dShape& s, hipStream_t st);
// the same with the requantisation fused into the store (y8: int8 output)
bool       mfma_s8_requant_supported(const Conv2dShape& s);
hipError_t launch_mfma_s8_requant(const int8_t* x, const int8_t* w, int8_t* y8, const Requant& rq, const Conv2dShape& s,
                                  hipStream_t st);
hipError_t launch_mfma_s8_any_requant(const int8_t* x, const int8_t* w, int8_t* y8, const Requant& rq,
                                      const Conv2dShape& s, hipStream_t st);
hipError_t launch_direct_conv2d_s8_requant(const int8_t* x, const int8_t* w, int8_t* y8, const Requant& rq,
                                           const Conv2dShape& s, hipStream_t st);
// ---- int8 with filters packed once into the matrix instruction's operand order (sw_mfma_s8_packed.hip);
// rq == nullptr: int32 out (y), else int8 out (y8); allow_fast == false: one thread per output
int64_t    s8_packed_filter_bytes(int C_in, int C_out, int R, int S);
hipError_t launch_pack_filter_s8(const int8_t* w, int8_t* packed, int C_in, int C_out, int R, int S, hipStream_t st);
hipError_t launch_conv2d_s8_packed(const int8_t* x, const int8_t* wp, int32_t* y, int8_t* y8, const Requant* rq,
                                   const Conv2dShape& s, bool allow_fast, hipStream_t st);
// ... the same for full-width row bands of narrow images (sw_mfma_s8_band.hip)
// (raw_filters: w is the caller's channel-first filter tensor, transposed by every workgroup on its way into LDS)
bool       mfma_s8_band_supported(const int8_t* x, const int8_t* w, const Conv2dShape& s, bool raw_filters);
hipError_t launch_mfma_s8_band(const int8_t* x, const int8_t* w, int32_t* y, int8_t* y8, const Requant* rq,
                               const Conv2dShape& s, bool raw_filters, hipStream_t st);
bool       mfma_s8_any_supported(const Conv2dShape& s);   // any extent, stride and channel count
hipError_t launch_mfma_s8_any(const int8_t* x, const int8_t* w, int32_t* y, const Conv2dShape& s, hipStream_t st);

}  // namespace swconv
