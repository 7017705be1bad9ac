// C ABI of libswconv.so: host-side validation and kernel selection.  Every argument error is
// reported before anything is enqueued; nothing here allocates or synchronises.
#include "../../include/swconv.h"

#include <cstdio>
#include <cstdlib>

#include "swconv_internal.h"

using namespace swconv;

namespace swconv {

namespace {
struct LastKernel {
    const char* name;
    int arg[4];
};
thread_local LastKernel g_last_kernel{nullptr, {-1, -1, -1, -1}};
}  // namespace

void note_kernel(const char* name, int a, int b, int c, int d) { g_last_kernel = LastKernel{name, {a, b, c, d}}; }

}  // namespace swconv

namespace {

constexpr int64_t kMaxElems = 2147483647LL;  // element count per tensor
constexpr int kMaxTaps1D = 64;
constexpr int kMaxFilter2D = 64;

bool force_direct()
{
    static const bool v = [] {
        const char* e = std::getenv("SWCONV_FORCE_DIRECT");
        return e && e[0] == '1';
    }();
    return v;
}

bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; }

bool overlaps(const void* a, int64_t abytes, const void* b, int64_t bbytes)
{
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + (uintptr_t)bbytes && b0 < a0 + (uintptr_t)abytes;
}

int launch_status(hipError_t e) { return e == hipSuccess ? SW_OK : SW_ERR_LAUNCH; }

// One filter per plane (single input channel, depthwise): picks among the whole-plane kernel (many planes
// that fit a 56 x 56 tile), the register-only rows kernel (3x3 / 5x5), the tile kernel and the direct kernel.
int run_plane(const float* x, const float* w, float* y, int64_t planes, int planes_per_x, int n_filters,
              const Conv2dShape& s, bool depthwise, hipStream_t st, const Epilogue& ep = Epilogue{nullptr, 0})
{
    if (!force_direct() && s.dil != 1) {
        // dilated taps: the run-time-extent tile kernel, whose window holds the filter's span
        if (sliding_plane_supported(s.H, s.W, s.R, s.S, s.stride, s.pad, s.dil) &&
            sliding_plane_worthwhile(planes, s.Ho, s.Wo, s.R, s.S))
            return launch_status(launch_sliding_plane(x, w, y, planes, planes_per_x, n_filters, s.H, s.W, s.R, s.S,
                                                      s.pad, s.Ho, s.Wo, st, ep, s.dil));
    } else if (!force_direct()) {
        // planes up to 20 x 20, and larger ragged ones (width not a multiple of 4) that the register-only and
        // whole-plane kernels do not take: a run of planes per workgroup
        if ((s.H * s.W <= 400 || s.W % 4 != 0 || s.R * s.S >= 25) &&
            small_planes_supported(planes, planes_per_x, s.H, s.W, s.R, s.S, s.stride, s.Ho, s.Wo))
            return launch_status(launch_small_planes(x, w, y, planes, n_filters, s.H, s.W, s.R, s.S, s.stride, s.pad,
                                                     s.Ho, s.Wo, st, ep));
        const bool rows = sliding_rows_supported(x, s.H, s.W, s.R, s.S, s.stride, s.pad);
        // the whole-plane kernel spends a 56 x 56 tile per plane: planes up to 32 wide leave most of its lanes
        // idle and go to the rows kernel (lane groups) when that has a variant
        const bool whole = s.stride == 1 && sliding_plane_whole(x, y, s.H, s.W, s.R, s.S, s.pad, s.Ho, s.Wo) &&
                           planes >= 512 && !(rows && s.W <= 32);
        if (!whole && rows)
            return launch_status(launch_sliding_rows(x, w, y, planes, planes_per_x, n_filters, s.H, s.W, s.R, s.S,
                                                     s.stride, s.pad, s.Ho, s.Wo, st, ep));
        if (sliding_plane_supported(s.H, s.W, s.R, s.S, s.stride, s.pad) &&
            sliding_plane_worthwhile(planes, s.Ho, s.Wo, s.R, s.S))
            return launch_status(launch_sliding_plane(x, w, y, planes, planes_per_x, n_filters, s.H, s.W, s.R, s.S,
                                                      s.pad, s.Ho, s.Wo, st, ep));
    }
    return launch_status(launch_direct_conv2d_f32(x, w, y, s, depthwise, st, &ep));
}

// Shared validation of the 2-D calls.  esz_in / esz_out are element sizes in bytes.
int check_conv2d(const void* x, const void* w, const void* y, int N, int C_in, int C_out, int H, int W,
                 int R, int S, int stride, int pad, bool depthwise, size_t esz_in, size_t esz_out,
                 Conv2dShape* out, int dil = 1)
{
    if (!x || !w || !y) return SW_ERR_NULL;
    if (N <= 0 || C_in <= 0 || C_out <= 0 || H <= 0 || W <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0 ||
        dil <= 0)
        return SW_ERR_SHAPE;
    // a dilated filter spans dil * (k - 1) + 1 input positions
    const int64_t span_r = (int64_t)dil * (R - 1) + 1, span_s = (int64_t)dil * (S - 1) + 1;
    if (span_r > kMaxElems || span_s > kMaxElems) return SW_ERR_SHAPE;
    const int64_t Ho = sw_out_dim(H, (int)span_r, stride, pad), Wo = sw_out_dim(W, (int)span_s, stride, pad);
    if (Ho <= 0 || Wo <= 0) return SW_ERR_SHAPE;
    const int64_t nx = (int64_t)N * C_in * H * W;
    const int64_t nw = (int64_t)C_out * (depthwise ? 1 : C_in) * R * S;
    const int64_t ny = (int64_t)N * C_out * Ho * Wo;
    if (nx > kMaxElems || nw > kMaxElems || ny > kMaxElems) return SW_ERR_SHAPE;
    if ((int64_t)H + 2 * (int64_t)pad > kMaxElems || (int64_t)W + 2 * (int64_t)pad > kMaxElems)
        return SW_ERR_SHAPE;
    if (R > kMaxFilter2D || S > kMaxFilter2D) return SW_ERR_UNSUPPORTED;
    if (misaligned(x, esz_in) || misaligned(w, esz_in) || misaligned(y, esz_out)) return SW_ERR_ALIGN;
    if (overlaps(y, ny * (int64_t)esz_out, x, nx * (int64_t)esz_in) ||
        overlaps(y, ny * (int64_t)esz_out, w, nw * (int64_t)esz_in))
        return SW_ERR_ALIAS;
    *out = Conv2dShape{N, C_in, C_out, H, W, R, S, stride, pad, (int)Ho, (int)Wo, dil};
    return SW_OK;
}

int run_1d(const float* x, const float* w, float* y, int64_t rows, int64_t len, int k, int stride, int pad,
           Op1D op, void* hip_stream)
{
    if (!x || !y || (op == OP_CONV && !w)) return SW_ERR_NULL;
    if (rows <= 0 || len <= 0 || k <= 0 || stride <= 0 || pad < 0) return SW_ERR_SHAPE;
    const int64_t len_out = sw_out_dim(len, k, stride, pad);
    if (len_out <= 0) return SW_ERR_SHAPE;
    if (len > kMaxElems / rows || len_out > kMaxElems / rows) return SW_ERR_SHAPE;
    if (k > kMaxTaps1D || pad >= k) return SW_ERR_UNSUPPORTED;
    if (misaligned(x, 4) || misaligned(y, 4) || (w && misaligned(w, 4))) return SW_ERR_ALIGN;
    if (overlaps(y, rows * len_out * 4, x, rows * len * 4) || (w && overlaps(y, rows * len_out * 4, w, k * 4)))
        return SW_ERR_ALIAS;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (!force_direct() && sliding_1d_supported(len, k, stride, pad))
        return launch_status(launch_sliding_1d(x, w, y, rows, len, len_out, k, pad, op, st));
    if (!force_direct() && op != OP_CONV && pool_tiles_supported(x, y, len, k, stride))
        return launch_status(launch_pool_tiles(x, y, rows, len, k, op == OP_MAX, st));
    if (!force_direct() && strided_1d_supported(rows, len, len_out, k, stride, pad))
        return launch_status(launch_strided_1d(x, w, y, rows, len, len_out, k, stride, pad, op, st));
    return launch_status(launch_direct_1d(x, w, y, rows, len, len_out, k, stride, pad, op, st));
}

}  // namespace

extern "C" {

int64_t sw_out_dim(int64_t in, int k, int stride, int pad)
{
    if (in <= 0 || k <= 0 || stride <= 0 || pad < 0) return 0;
    const int64_t span = in + 2 * (int64_t)pad - k;
    if (span < 0) return 0;
    return span / stride + 1;
}

int64_t sw_out_dim_dilated(int64_t in, int k, int stride, int pad, int dilation)
{
    if (k <= 0 || dilation <= 0) return 0;
    const int64_t span = (int64_t)dilation * (k - 1) + 1;      // input positions a dilated filter covers
    if (span > kMaxElems) return 0;
    return sw_out_dim(in, (int)span, stride, pad);
}

size_t sw_workspace_bytes(void) { return 0; }

const char* sw_status_string(int status)
{
    switch (status) {
        case SW_OK: return "ok";
        case SW_ERR_NULL: return "a required pointer is NULL";
        case SW_ERR_SHAPE: return "invalid shape, stride or padding";
        case SW_ERR_UNSUPPORTED: return "valid problem without a kernel in this library";
        case SW_ERR_ALIGN: return "pointer not aligned to its element size";
        case SW_ERR_ALIAS: return "output overlaps an input";
        case SW_ERR_LAUNCH: return "HIP launch failed";
        case SW_ERR_JIT: return "run-time compilation of a generated kernel failed";
        default: return "unknown status";
    }
}

int sw_version(void) { return 200; }

const char* sw_last_kernel(void)
{
    thread_local char text[160];
    const auto& k = g_last_kernel;
    if (!k.name) return "";
    int n = std::snprintf(text, sizeof text, "%s", k.name);
    for (int i = 0; i < 4 && k.arg[i] >= 0 && n > 0 && n < (int)sizeof text; ++i)
        n += std::snprintf(text + n, sizeof text - n, "%s%d", i == 0 ? "<" : ",", k.arg[i]);
    if (k.arg[0] >= 0 && n > 0 && n < (int)sizeof text - 1) std::snprintf(text + n, sizeof text - n, ">");
    return text;
}

int sw_conv1d(const float* x, const float* w, float* y, int64_t rows, int64_t len, int k, int stride,
              int pad, void* hip_stream)
{
    return run_1d(x, w, y, rows, len, k, stride, pad, OP_CONV, hip_stream);
}

int sw_pool1d(const float* x, float* y, int64_t rows, int64_t len, int window, int stride, int mode,
              void* hip_stream)
{
    if (mode != SW_POOL_AVG && mode != SW_POOL_MAX) return x && y ? SW_ERR_UNSUPPORTED : SW_ERR_NULL;
    return run_1d(x, nullptr, y, rows, len, window, stride, 0, mode == SW_POOL_AVG ? OP_AVG : OP_MAX,
                  hip_stream);
}

int sw_pool2d(const float* x, float* y, int N, int C, int H, int W, int R, int S, int stride, int pad, int mode,
              void* hip_stream)
{
    if (!x || !y) return SW_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return SW_ERR_SHAPE;
    const int64_t Ho = sw_out_dim(H, R, stride, pad), Wo = sw_out_dim(W, S, stride, pad);
    if (Ho <= 0 || Wo <= 0) return SW_ERR_SHAPE;
    const int64_t planes = (int64_t)N * C;
    const int64_t nx = planes * H * W, ny = planes * Ho * Wo;
    if (nx > kMaxElems || ny > kMaxElems) return SW_ERR_SHAPE;
    if (mode != SW_POOL_AVG && mode != SW_POOL_MAX) return SW_ERR_UNSUPPORTED;
    if (R > kMaxFilter2D || S > kMaxFilter2D) return SW_ERR_UNSUPPORTED;
    if (2 * pad > (R < S ? R : S)) return SW_ERR_UNSUPPORTED;   // a window could lie wholly in the padding
    if (misaligned(x, 4) || misaligned(y, 4)) return SW_ERR_ALIGN;
    if (overlaps(y, ny * 4, x, nx * 4)) return SW_ERR_ALIAS;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const bool maximum = mode == SW_POOL_MAX;
    if (!force_direct() && global_pool_supported(H, W, R, S, pad))
        return launch_status(launch_global_pool(x, y, planes, H * W, maximum, st));
    if (!force_direct() && pool_rows_supported(x, W, R, S, stride, pad))
        return launch_status(launch_pool_rows(x, y, planes, H, W, R, stride, pad, (int)Ho, (int)Wo, maximum, st));
    return launch_status(launch_direct_pool2d(x, y, planes, H, W, R, S, stride, pad, (int)Ho, (int)Wo, maximum, st));
}

// The multi-channel fp32 convolution with the store's epilogue (none for sw_conv2d).
static int run_conv2d(const float* x, const float* w, float* y, const Conv2dShape& s, const Epilogue& ep, hipStream_t st)
{
    const bool plain = !ep.bias && !ep.relu;
    (void)plain;
    if (s.C_in == 1)
        return run_plane(x, w, y, (int64_t)s.N * s.C_out, s.C_out, s.C_out, s, false, st, ep);
    if (!force_direct() && s.C_in > 1) {
        // The fixed 3x3 / 5x5 kernel holds a CU with one large tile: it needs enough of them to fill the chip
        // (28 x 28 images and below at batch 32 leave it at 128 or fewer); the any-shape kernel's 128-pixel
        // tiles take over there, and everywhere the fixed kernel has no variant.
        // Filters of 25 taps and more over at least 8 channels: the compound kernel (one filter row of a channel
        // chunk at a time, 256-pixel tiles), measured faster than the kernels below from 5 x 5 upward and the only
        // matrix-core kernel beyond 13 x 13.
        // One tap, stride 1, no padding: the input is the B operand as it lies in memory (nothing staged); measured
        // faster than the window kernels on every such layer tried.
        if (mfma_f32_pointwise_supported(s, x, w, y))
            return launch_status(launch_mfma_f32_pointwise(x, w, y, s, st, ep));
        if (s.R * s.S >= 25 && s.C_in >= 8 && mfma_f32_rows_supported(s, x))
            return launch_status(launch_mfma_f32_rows(x, w, y, s, st, ep));
        const bool quad_ok = mfma_f32_quad_supported(s);
        const bool any_ok = quad_ok || mfma_f32_any_supported(s);
        if (mfma_f32_supported(s) && (mfma_f32_workgroups(s) >= 160 || !any_ok))
            return launch_status(launch_mfma_f32(x, w, y, s, st, ep));
        // few taps over whole groups of eight channels: operands by direct-to-LDS loads, the next chunk in flight
        // while this one multiplies
        if (mfma_f32_dma_supported(s, x, w)) return launch_status(launch_mfma_f32_dma(x, w, y, s, st, ep));
        if (quad_ok) return launch_status(launch_mfma_f32_quad(x, w, y, s, st, ep));
        if (any_ok) return launch_status(launch_mfma_f32_any(x, w, y, s, st, ep));
        if (mfma_f32_rows_supported(s, x)) return launch_status(launch_mfma_f32_rows(x, w, y, s, st, ep));
    }
    return launch_status(launch_direct_conv2d_f32(x, w, y, s, false, st, &ep));
}

int sw_conv2d(const float* x, const float* w, float* y, int N, int C_in, int C_out, int H, int W, int R,
              int S, int stride, int pad, void* hip_stream)
{
    Conv2dShape s;
    const int rc = check_conv2d(x, w, y, N, C_in, C_out, H, W, R, S, stride, pad, false, 4, 4, &s);
    if (rc != SW_OK) return rc;
    return run_conv2d(x, w, y, s, Epilogue{nullptr, 0}, static_cast<hipStream_t>(hip_stream));
}

int sw_conv2d_bias_relu(const float* x, const float* w, const float* bias, float* y, int N, int C_in, int C_out, int H,
                        int W, int R, int S, int stride, int pad, int relu, void* hip_stream)
{
    Conv2dShape s;
    const int rc = check_conv2d(x, w, y, N, C_in, C_out, H, W, R, S, stride, pad, false, 4, 4, &s);
    if (rc != SW_OK) return rc;
    if (bias && misaligned(bias, 4)) return SW_ERR_ALIGN;
    if (bias && overlaps(y, (int64_t)N * C_out * s.Ho * s.Wo * 4, bias, (int64_t)C_out * 4)) return SW_ERR_ALIAS;
    return run_conv2d(x, w, y, s, Epilogue{bias, relu != 0}, static_cast<hipStream_t>(hip_stream));
}

int sw_conv2d_dilated(const float* x, const float* w, float* y, int N, int C_in, int C_out, int H, int W, int R,
                      int S, int stride, int pad, int dilation, void* hip_stream)
{
    Conv2dShape s;
    const int rc = check_conv2d(x, w, y, N, C_in, C_out, H, W, R, S, stride, pad, false, 4, 4, &s, dilation);
    if (rc != SW_OK) return rc;
    return run_conv2d(x, w, y, s, Epilogue{nullptr, 0}, static_cast<hipStream_t>(hip_stream));
}

int sw_conv2d_depthwise_dilated(const float* x, const float* w, float* y, int N, int C, int H, int W, int R, int S,
                                int stride, int pad, int dilation, void* hip_stream)
{
    Conv2dShape s;
    const int rc = check_conv2d(x, w, y, N, C, C, H, W, R, S, stride, pad, true, 4, 4, &s, dilation);
    if (rc != SW_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return run_plane(x, w, y, (int64_t)N * C, 1, C, s, true, st);
}

int sw_conv2d_depthwise(const float* x, const float* w, float* y, int N, int C, int H, int W, int R, int S,
                        int stride, int pad, void* hip_stream)
{
    Conv2dShape s;
    const int rc = check_conv2d(x, w, y, N, C, C, H, W, R, S, stride, pad, true, 4, 4, &s);
    if (rc != SW_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return run_plane(x, w, y, (int64_t)N * C, 1, C, s, true, st);
}

// fp32 / bf16 / half (ek: Elem) convolution on channel-last tensors with the store's epilogue
static int run_nhwc(const void* x, const void* w, const float* bias, void* y, int N, int H, int W, int C_in, int C_out,
                    int R, int S, int stride, int pad, int dilation, int relu, int ek, void* hip_stream)
{
    const int esz = elem_size(ek);
    Conv2dShape s;
    const int rc = check_conv2d(x, w, y, N, C_in, C_out, H, W, R, S, stride, pad, false, (size_t)esz, (size_t)esz, &s,
                                dilation);
    if (rc != SW_OK) return rc;
    if (bias && misaligned(bias, 4)) return SW_ERR_ALIGN;
    if (bias && overlaps(y, (int64_t)N * C_out * s.Ho * s.Wo * esz, bias, (int64_t)C_out * 4)) return SW_ERR_ALIAS;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const Epilogue ep{bias, relu != 0};
    if (!force_direct() && mfma_nhwc_lds_supported(x, w, y, s, ek))
        return launch_status(launch_mfma_nhwc_lds(x, w, y, s, ek, ep, st));
    if (!force_direct() && esz == 2 && mfma_bf16_nhwc_direct_supported(x, w, y, s))
        return launch_status(launch_mfma_bf16_nhwc_direct(x, w, y, s, ek == kElemF16, ep, st));
    if (!force_direct() && mfma_nhwc_supported(x, w, s, ek)) return launch_status(launch_mfma_nhwc(x, w, y, s, ek, ep, st));
    return launch_status(launch_direct_nhwc(x, w, y, s, ek, ep, st));
}

int sw_conv2d_nhwc(const float* x, const float* w, const float* bias, float* y, int N, int H, int W, int C_in, int C_out,
                   int R, int S, int stride, int pad, int dilation, int relu, void* hip_stream)
{
    return run_nhwc(x, w, bias, y, N, H, W, C_in, C_out, R, S, stride, pad, dilation, relu, kElemF32, hip_stream);
}

int sw_conv2d_bf16_nhwc(const void* x, const void* w, const float* bias, void* y, int N, int H, int W, int C_in, int C_out,
                        int R, int S, int stride, int pad, int dilation, int relu, void* hip_stream)
{
    return run_nhwc(x, w, bias, y, N, H, W, C_in, C_out, R, S, stride, pad, dilation, relu, kElemBF16, hip_stream);
}

int sw_conv2d_f16_nhwc(const void* x, const void* w, const float* bias, void* y, int N, int H, int W, int C_in, int C_out,
                       int R, int S, int stride, int pad, int dilation, int relu, void* hip_stream)
{
    return run_nhwc(x, w, bias, y, N, H, W, C_in, C_out, R, S, stride, pad, dilation, relu, kElemF16, hip_stream);
}

// int8 convolution on channel-last tensors; bias/scale == nullptr and y8 == nullptr: int32 sums
static int run_s8_nhwc(const int8_t* x, const int8_t* w, const int32_t* bias, const float* scale, int32_t* y, int8_t* y8,
                       int N, int H, int W, int C_in, int C_out, int R, int S, int stride, int pad, int relu,
                       void* hip_stream)
{
    Conv2dShape s;
    const void* out = y8 ? static_cast<const void*>(y8) : static_cast<const void*>(y);
    const int rc = check_conv2d(x, w, out, N, C_in, C_out, H, W, R, S, stride, pad, false, 1, y8 ? 1 : 4, &s);
    if (rc != SW_OK) return rc;
    if ((int64_t)C_in * R * S > 131071) return SW_ERR_SHAPE;  // 131072 * 2^14 = 2^31 leaves int32
    Requant rq{bias, scale, relu != 0};
    if (y8) {
        if (misaligned(scale, 4) || (bias && misaligned(bias, 4))) return SW_ERR_ALIGN;
        const int64_t ny = (int64_t)N * C_out * s.Ho * s.Wo;
        if (overlaps(y8, ny, scale, (int64_t)C_out * 4) || (bias && overlaps(y8, ny, bias, (int64_t)C_out * 4)))
            return SW_ERR_ALIAS;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (!force_direct() && mfma_s8_nhwc_lds_supported(x, w, y8 ? static_cast<const void*>(y8) : static_cast<const void*>(y), y8 != nullptr, s))
        return launch_status(launch_mfma_s8_nhwc_lds(x, w, y8 ? static_cast<void*>(y8) : static_cast<void*>(y), y8 ? &rq : nullptr, s, st));
    if (!force_direct() && mfma_s8_nhwc_supported(x, w, s))
        return launch_status(launch_mfma_s8_nhwc(x, w, y, y8, y8 ? &rq : nullptr, s, st));
    return launch_status(launch_direct_s8_nhwc(x, w, y, y8, y8 ? &rq : nullptr, s, st));
}

int sw_conv2d_s8_nhwc(const int8_t* x, const int8_t* w, int32_t* y, int N, int H, int W, int C_in, int C_out, int R,
                      int S, int stride, int pad, void* hip_stream)
{
    return run_s8_nhwc(x, w, nullptr, nullptr, y, nullptr, N, H, W, C_in, C_out, R, S, stride, pad, 0, hip_stream);
}

int sw_conv2d_s8_nhwc_requant(const int8_t* x, const int8_t* w, const int32_t* bias, const float* scale, int8_t* y,
                              int N, int H, int W, int C_in, int C_out, int R, int S, int stride, int pad, int relu,
                              void* hip_stream)
{
    if (!scale || !y) return SW_ERR_NULL;
    return run_s8_nhwc(x, w, bias, scale, nullptr, y, N, H, W, C_in, C_out, R, S, stride, pad, relu, hip_stream);
}

int sw_dw_pw_block(const float* x, const float* w_dw, const float* b_dw, const float* w_pw, const float* b_pw, float* y,
                   int N, int C, int C_out, int H, int W, int relu_dw, int relu_pw, void* hip_stream)
{
    if (!x || !w_dw || !w_pw || !y) return SW_ERR_NULL;
    if (N <= 0 || C <= 0 || C_out <= 0 || H <= 0 || W <= 0) return SW_ERR_SHAPE;
    const int64_t nx = (int64_t)N * C * H * W, ny = (int64_t)N * C_out * H * W, npw = (int64_t)C_out * C;
    if (nx > kMaxElems || ny > kMaxElems || npw > kMaxElems) return SW_ERR_SHAPE;
    if (misaligned(x, 4) || misaligned(w_dw, 4) || misaligned(w_pw, 4) || misaligned(y, 4) ||
        (b_dw && misaligned(b_dw, 4)) || (b_pw && misaligned(b_pw, 4)))
        return SW_ERR_ALIGN;
    if (overlaps(y, ny * 4, x, nx * 4) || overlaps(y, ny * 4, w_dw, (int64_t)C * 9 * 4) || overlaps(y, ny * 4, w_pw, npw * 4) ||
        (b_dw && overlaps(y, ny * 4, b_dw, (int64_t)C * 4)) || (b_pw && overlaps(y, ny * 4, b_pw, (int64_t)C_out * 4)))
        return SW_ERR_ALIAS;
    if (!dw_pw_block_supported(N, C, C_out, H, W)) return SW_ERR_UNSUPPORTED;
    return launch_status(launch_dw_pw_block(x, w_dw, b_dw, w_pw, b_pw, y, N, C, C_out, H, W, relu_dw != 0, relu_pw != 0,
                                            static_cast<hipStream_t>(hip_stream)));
}

int sw_conv2d_depthwise_bias_relu(const float* x, const float* w, const float* bias, float* y, int N, int C, int H,
                                  int W, int R, int S, int stride, int pad, int relu, void* hip_stream)
{
    Conv2dShape s;
    const int rc = check_conv2d(x, w, y, N, C, C, H, W, R, S, stride, pad, true, 4, 4, &s);
    if (rc != SW_OK) return rc;
    if (bias && misaligned(bias, 4)) return SW_ERR_ALIGN;
    if (bias && overlaps(y, (int64_t)N * C * s.Ho * s.Wo * 4, bias, (int64_t)C * 4)) return SW_ERR_ALIAS;
    return run_plane(x, w, y, (int64_t)N * C, 1, C, s, true, static_cast<hipStream_t>(hip_stream),
                     Epilogue{bias, relu != 0});
}

int sw_conv2d_depthwise_bf16(const uint16_t* x, const float* w, uint16_t* y, int N, int C, int H, int W, int R, int S,
                             int stride, int pad, void* hip_stream)
{
    Conv2dShape s;
    // (element sizes: activations 2 bytes; the filter is checked as fp32 below)
    const int rc = check_conv2d(x, w, y, N, C, C, H, W, R, S, stride, pad, true, 2, 2, &s);
    if (rc != SW_OK) return rc;
    if (misaligned(w, 4)) return SW_ERR_ALIGN;
    if (overlaps(y, (int64_t)N * C * s.Ho * s.Wo * 2, w, (int64_t)C * R * S * 4)) return SW_ERR_ALIAS;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (!force_direct() && sliding_plane_bf16_supported(x, y, H, W, R, S, stride, pad, s.Ho, s.Wo))
        return launch_status(launch_sliding_plane_bf16(x, w, y, (int64_t)N * C, C, H, W, R, pad, s.Ho, s.Wo, st));
    return launch_status(launch_direct_depthwise_bf16(x, w, y, s, st));
}

int sw_conv2d_depthwise_dilated_jit(const float* x, const float* w, float* y, int N, int C, int H, int W, int R, int S,
                                    int stride, int pad, int dilation, void* hip_stream)
{
    Conv2dShape s;
    const int rc = check_conv2d(x, w, y, N, C, C, H, W, R, S, stride, pad, true, 4, 4, &s, dilation);
    if (rc != SW_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (!force_direct() && jit_plane_supported(x, y, H, W, R, S, stride, pad, dilation)) {
        // a geometry whose generated kernel cannot be compiled or loaded is served by the precompiled kernels
        if (jit_launch_plane(x, w, y, (int64_t)N * C, 1, C, H, W, R, S, stride, pad, dilation, st) == SW_OK) return SW_OK;
    }
    return run_plane(x, w, y, (int64_t)N * C, 1, C, s, true, st);
}

int sw_conv2d_depthwise_jit(const float* x, const float* w, float* y, int N, int C, int H, int W, int R, int S,
                            int stride, int pad, void* hip_stream)
{
    return sw_conv2d_depthwise_dilated_jit(x, w, y, N, C, H, W, R, S, stride, pad, 1, hip_stream);
}

static int jit_geometry_ok(int H, int W, int R, int S, int stride, int pad, int dilation)
{
    if (H <= 0 || W <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0 || dilation <= 0) return SW_ERR_SHAPE;
    if (sw_out_dim_dilated(H, R, stride, pad, dilation) <= 0 || sw_out_dim_dilated(W, S, stride, pad, dilation) <= 0)
        return SW_ERR_SHAPE;
    return SW_OK;
}

int sw_jit_prepare_depthwise_dilated(int H, int W, int R, int S, int stride, int pad, int dilation)
{
    const int rc = jit_geometry_ok(H, W, R, S, stride, pad, dilation);
    return rc != SW_OK ? rc : jit_prepare_plane(H, W, R, S, stride, pad, dilation);
}

int sw_jit_prepare_depthwise(int H, int W, int R, int S, int stride, int pad)
{
    return sw_jit_prepare_depthwise_dilated(H, W, R, S, stride, pad, 1);
}

int sw_jit_compile_check_dilated(int H, int W, int R, int S, int stride, int pad, int dilation)
{
    const int rc = jit_geometry_ok(H, W, R, S, stride, pad, dilation);
    return rc != SW_OK ? rc : jit_compile_only(H, W, R, S, stride, pad, dilation);
}

int sw_jit_compile_check(int H, int W, int R, int S, int stride, int pad)
{
    return sw_jit_compile_check_dilated(H, W, R, S, stride, pad, 1);
}

int sw_jit_cached_kernels(void) { return jit_cached_kernels(); }

int sw_conv2d_s8(const int8_t* x, const int8_t* w, int32_t* y, int N, int C_in, int C_out, int H, int W,
                 int R, int S, int stride, int pad, void* hip_stream)
{
    Conv2dShape s;
    const int rc = check_conv2d(x, w, y, N, C_in, C_out, H, W, R, S, stride, pad, false, 1, 4, &s);
    if (rc != SW_OK) return rc;
    if ((int64_t)C_in * R * S > 131071) return SW_ERR_SHAPE;  // 131072 * 2^14 = 2^31 leaves int32
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (!force_direct()) {
        if (mfma_s8_band_supported(x, w, s, true))
            return launch_status(launch_mfma_s8_band(x, w, y, nullptr, nullptr, s, true, st));
        if (mfma_s8_supported(s)) return launch_status(launch_mfma_s8(x, w, y, s, st));
        if (mfma_s8_any_supported(s)) return launch_status(launch_mfma_s8_any(x, w, y, s, st));
    }
    return launch_status(launch_direct_conv2d_s8(x, w, y, s, st));
}

int sw_conv2d_s8_requant(const int8_t* x, const int8_t* w, const int32_t* bias, const float* scale, int8_t* y, int N,
                         int C_in, int C_out, int H, int W, int R, int S, int stride, int pad, int relu,
                         void* hip_stream)
{
    if (!scale) return SW_ERR_NULL;
    Conv2dShape s;
    const int rc = check_conv2d(x, w, y, N, C_in, C_out, H, W, R, S, stride, pad, false, 1, 1, &s);
    if (rc != SW_OK) return rc;
    if ((int64_t)C_in * R * S > 131071) return SW_ERR_SHAPE;  // 131072 * 2^14 = 2^31 leaves int32
    if (misaligned(scale, 4) || (bias && misaligned(bias, 4))) return SW_ERR_ALIGN;
    const int64_t ny = (int64_t)N * C_out * s.Ho * s.Wo;
    if (overlaps(y, ny, scale, (int64_t)C_out * 4) || (bias && overlaps(y, ny, bias, (int64_t)C_out * 4)))
        return SW_ERR_ALIAS;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const Requant rq{bias, scale, relu != 0};
    if (!force_direct()) {
        if (mfma_s8_band_supported(x, w, s, true))
            return launch_status(launch_mfma_s8_band(x, w, nullptr, y, &rq, s, true, st));
        if (mfma_s8_requant_supported(s))
            return launch_status(launch_mfma_s8_requant(x, w, y, rq, s, st));
        if (mfma_s8_any_supported(s)) return launch_status(launch_mfma_s8_any_requant(x, w, y, rq, s, st));
    }
    return launch_status(launch_direct_conv2d_s8_requant(x, w, y, rq, s, st));
}

int64_t sw_s8_packed_filter_bytes(int C_in, int C_out, int R, int S)
{
    if (C_in <= 0 || C_out <= 0 || R <= 0 || S <= 0 || R > kMaxFilter2D || S > kMaxFilter2D) return 0;
    if ((int64_t)C_out * C_in * R * S > kMaxElems) return 0;
    const int64_t bytes = s8_packed_filter_bytes(C_in, C_out, R, S);
    return bytes > kMaxElems ? 0 : bytes;
}

int sw_s8_pack_filter(const int8_t* w, int8_t* packed, int C_in, int C_out, int R, int S, void* hip_stream)
{
    if (!w || !packed) return SW_ERR_NULL;
    if (C_in <= 0 || C_out <= 0 || R <= 0 || S <= 0) return SW_ERR_SHAPE;
    if (R > kMaxFilter2D || S > kMaxFilter2D) return SW_ERR_UNSUPPORTED;
    const int64_t nw = (int64_t)C_out * C_in * R * S;
    if (nw > kMaxElems) return SW_ERR_SHAPE;
    const int64_t bytes = sw_s8_packed_filter_bytes(C_in, C_out, R, S);
    if (bytes <= 0) return SW_ERR_SHAPE;
    if (misaligned(packed, 16)) return SW_ERR_ALIGN;
    if (overlaps(packed, bytes, w, nw)) return SW_ERR_ALIAS;
    return launch_status(launch_pack_filter_s8(w, packed, C_in, C_out, R, S, static_cast<hipStream_t>(hip_stream)));
}

// Shared by the two packed-filter calls; bias/scale/y8 == nullptr: int32 sums.
static int run_s8_packed(const int8_t* x, const int8_t* packed, const int32_t* bias, const float* scale, int32_t* y,
                         int8_t* y8, int N, int C_in, int C_out, int H, int W, int R, int S, int stride, int pad, int relu,
                         void* hip_stream)
{
    Conv2dShape s;
    const void* out = y8 ? static_cast<const void*>(y8) : static_cast<const void*>(y);
    // (check_conv2d sees the packed buffer as the filter: it is at least as large as the filter tensor)
    const int rc = check_conv2d(x, packed, out, N, C_in, C_out, H, W, R, S, stride, pad, false, 1, y8 ? 1 : 4, &s);
    if (rc != SW_OK) return rc;
    if ((int64_t)C_in * R * S > 131071) return SW_ERR_SHAPE;  // 131072 * 2^14 = 2^31 leaves int32
    const int64_t bytes = sw_s8_packed_filter_bytes(C_in, C_out, R, S);
    if (bytes <= 0) return SW_ERR_SHAPE;
    if (misaligned(packed, 16)) return SW_ERR_ALIGN;
    const int64_t ny = (int64_t)N * C_out * s.Ho * s.Wo * (y8 ? 1 : 4);
    if (overlaps(out, ny, packed, bytes)) return SW_ERR_ALIAS;
    Requant rq{bias, scale, relu != 0};
    if (y8) {
        if (misaligned(scale, 4) || (bias && misaligned(bias, 4))) return SW_ERR_ALIGN;
        if (overlaps(y8, ny, scale, (int64_t)C_out * 4) || (bias && overlaps(y8, ny, bias, (int64_t)C_out * 4)))
            return SW_ERR_ALIAS;
    }
    return launch_status(launch_conv2d_s8_packed(x, packed, y, y8, y8 ? &rq : nullptr, s, !force_direct(),
                                                 static_cast<hipStream_t>(hip_stream)));
}

int sw_conv2d_s8_packed(const int8_t* x, const int8_t* packed, int32_t* y, int N, int C_in, int C_out, int H, int W,
                        int R, int S, int stride, int pad, void* hip_stream)
{
    return run_s8_packed(x, packed, nullptr, nullptr, y, nullptr, N, C_in, C_out, H, W, R, S, stride, pad, 0, hip_stream);
}

int sw_conv2d_s8_packed_requant(const int8_t* x, const int8_t* packed, const int32_t* bias, const float* scale,
                                int8_t* y, int N, int C_in, int C_out, int H, int W, int R, int S, int stride, int pad,
                                int relu, void* hip_stream)
{
    if (!scale || !y) return SW_ERR_NULL;
    return run_s8_packed(x, packed, bias, scale, nullptr, y, N, C_in, C_out, H, W, R, S, stride, pad, relu, hip_stream);
}

}  // extern "C"
