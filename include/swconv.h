/*
 * swconv -- Sliding Window Sum convolution and pooling for AMD Instinct MI355X (gfx950).
 *
 * C ABI of libswconv.so.  Every entry point evaluates a DNN convolution or a
 * pooling directly on the unmodified input: a tile of the input plus its halo
 * is brought on chip once and the filter taps are accumulated over shifted
 * windows of that tile.  No column matrix (im2col) and no other workspace is
 * ever written (paper, section 1: the column matrix is k times the input;
 * section 2: the sliding kernel works on the unmodified input).
 *
 * Conventions common to all calls
 * -------------------------------
 *  - "Convolution" is the DNN one: cross-correlation, the filter is not flipped.
 *  - Layout: dense row-major NCHW activations, OIHW weights.
 *  - Padding is symmetric zero padding; output extent per axis is
 *        out = floor((in + 2*pad - k) / stride) + 1        (see sw_out_dim).
 *  - Every pointer is a DEVICE pointer owned by the caller.  The library never
 *    allocates, frees or keeps device memory.  x and w are only read; y is
 *    only written, and every element of y is written.
 *  - Alignment: fp32 / int32 pointers must be 4-byte aligned (SW_ERR_ALIGN
 *    otherwise).  16-byte alignment of x and y selects the vectorised paths;
 *    anything less aligned still computes the same values.
 *  - y must not overlap x or w (SW_ERR_ALIAS when the byte ranges intersect).
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *    A call validates its arguments on the host, enqueues its kernel on that
 *    stream and returns; it never synchronises.  Argument errors are detected
 *    before anything is enqueued.
 *  - Return value: an sw_status.  No exceptions, no abort.
 *  - fp32 results are accumulated in fp32 (order unspecified); int8 results
 *    are the exact int32 sums.
 */
#ifndef SWCONV_H
#define SWCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SW_OK = 0,
    SW_ERR_NULL = 1,        /* a required pointer is NULL                             */
    SW_ERR_SHAPE = 2,       /* dim <= 0, stride <= 0, pad < 0, filter > padded input,  */
                            /* or an element count beyond 2^31-1 per tensor            */
    SW_ERR_UNSUPPORTED = 3, /* a valid problem the library has no kernel for           */
    SW_ERR_ALIGN = 4,       /* pointer not aligned to its element size                 */
    SW_ERR_ALIAS = 5,       /* y overlaps x or w                                       */
    SW_ERR_LAUNCH = 6,      /* the HIP runtime refused the launch (or no device)       */
    SW_ERR_JIT = 7          /* the run-time compiler refused a generated kernel        */
} sw_status;

typedef enum { SW_POOL_AVG = 0, SW_POOL_MAX = 1 } sw_pool_mode;

/*
 * 1-D convolution as a sliding window sum (paper, abstract and section 2).
 *     y[row, i] = sum_{j<k} w[j] * xz[row, i*stride + j - pad]
 * x: [rows, len] fp32;  w: [k] fp32, one tap vector shared by all rows;
 * y: [rows, len_out] fp32, len_out = sw_out_dim(len, k, stride, pad).
 * Supported: 1 <= k <= 64, pad < k.  Otherwise SW_ERR_UNSUPPORTED.
 * Stride 1 runs the sliding kernel, strides 2..8 a tiled kernel that reads each
 * input once through LDS, larger strides one thread per output.
 */
int sw_conv1d(const float* x, const float* w, float* y,
              int64_t rows, int64_t len, int k, int stride, int pad, void* hip_stream);

/*
 * 1-D pooling with the same kernel structure (paper, abstract).
 *     avg: y[row, i] = (1/window) * sum_{j<window} x[row, i*stride + j]
 *     max: y[row, i] = max_{j<window} x[row, i*stride + j]
 * No padding, so the average always divides by window.  The maximum is
 * bit-exact; NaN inputs are outside the contract.
 * x: [rows, len];  y: [rows, sw_out_dim(len, window, stride, 0)].
 * Supported: 1 <= window <= 64.  mode is an sw_pool_mode (else SW_ERR_UNSUPPORTED).
 * Kernels as for sw_conv1d; windows that tile the rows (stride == window in
 * {2, 4, 8}, len a multiple of 4 and of the window, 16-byte aligned x, 8-byte
 * aligned y) run a register-only kernel.
 */
int sw_pool1d(const float* x, float* y, int64_t rows, int64_t len,
              int window, int stride, int mode, void* hip_stream);

/*
 * 2-D pooling over R x S windows of every plane, again as a sliding window sum
 * (paper, abstract: pooling and convolution share the kernel structure).
 *     avg: y[n,c,i,j] = (1/(R*S)) * sum_{r,s} xz[n,c,i*stride+r-pad, j*stride+s-pad]
 *     max: y[n,c,i,j] = max over the (r,s) whose position lies inside the plane
 * The average is the sliding sum of the zero-padded plane with the constant
 * divisor R*S (padded positions count as zeros); padding never wins a maximum.
 * x: [N,C,H,W];  y: [N,C,H_out,W_out], extents by sw_out_dim.
 * Supported: R,S <= 64 and 2*pad <= min(R,S) (so that no window lies wholly in
 * the padding), else SW_ERR_UNSUPPORTED; mode as in sw_pool1d.  2x2 stride 2 and
 * 3x3 stride 1 or 2 with W % 4 == 0 and 16-byte aligned x run in the register-only
 * kernel, every other case in the one-thread-per-output kernel.
 * The maximum is bit-exact; NaN inputs are outside the contract.
 */
int sw_pool2d(const float* x, float* y, int N, int C, int H, int W, int R, int S,
              int stride, int pad, int mode, void* hip_stream);

/*
 * 2-D convolution (paper, section 2: the 2-D sliding window convolution; for
 * C_in > 1 every tap is a small C_out x C_in matrix product accumulated into
 * the output tile, the re-formulation section 3 asks for).
 *     y[n,co,i,j] = sum_{ci,r,s} w[co,ci,r,s] * xz[n,ci,i*stride+r-pad, j*stride+s-pad]
 * x: [N,C_in,H,W] fp32;  w: [C_out,C_in,R,S] fp32;  y: [N,C_out,H_out,W_out] fp32.
 * Supported: any shape with R,S <= 64 (SW_ERR_UNSUPPORTED beyond).  C_in >= 2
 * runs on the matrix cores: 3x3 and 5x5 at stride 1 with C_in % 16 == 0,
 * C_out % 64 == 0 and 16-byte aligned w in a large-tile kernel when the problem
 * fills the chip with such tiles, 1x1 at stride 1 without padding (C_in % 8 == 0,
 * an even number of pixels per plane, x and y aligned to 8 bytes, w to 16) in a
 * kernel that reads its operands straight from x, every other extent, stride,
 * padding and channel count in an any-shape kernel (one thread per output only
 * when its window or filter does not fit 64 KB of LDS).  C_in == 1 runs the
 * one-filter-per-plane kernels of sw_conv2d_depthwise.
 */
int sw_conv2d(const float* x, const float* w, float* y,
              int N, int C_in, int C_out, int H, int W, int R, int S,
              int stride, int pad, void* hip_stream);

/*
 * sw_conv2d with a per-channel bias and an optional rectifier applied in the
 * store (paper, section 1: the layers these kernels serve; the output is
 * still written once and nothing else is):
 *     y[n,co,i,j] = act(conv + bias[co]),  act(t) = relu ? max(t, 0) : t
 * bias: [C_out] fp32 device pointer or NULL (no bias); relu: 0 or non-zero.
 * One more fp32 addition than sw_conv2d.  Shapes, support and errors as
 * sw_conv2d; bias must be 4-byte aligned and must not overlap y.
 * sw_conv2d_depthwise_bias_relu: the same for sw_conv2d_depthwise (bias: [C]).
 */
int sw_conv2d_bias_relu(const float* x, const float* w, const float* bias, float* y,
                        int N, int C_in, int C_out, int H, int W, int R, int S,
                        int stride, int pad, int relu, void* hip_stream);
int sw_conv2d_depthwise_bias_relu(const float* x, const float* w, const float* bias, float* y,
                                  int N, int C, int H, int W, int R, int S,
                                  int stride, int pad, int relu, void* hip_stream);

/*
 * Depthwise 2-D convolution: one R x S filter per channel (paper, section 1.2,
 * depthwise separable convolutions) -- a pure sliding sum, no C_in reduction.
 *     y[n,c,i,j] = sum_{r,s} w[c,0,r,s] * xz[n,c,i*stride+r-pad, j*stride+s-pad]
 * x: [N,C,H,W];  w: [C,1,R,S];  y: [N,C,H_out,W_out].
 * Supported: any shape with R,S <= 64 (SW_ERR_UNSUPPORTED beyond).  3x3, 5x5
 * and 7x7 at stride 1, and 3x3 and 5x5 at stride 2, have fixed-size kernels (the
 * paper's "custom" kernels, section 2); other extents up to 51 x 51 at stride 1
 * run the generic sliding kernel; every other case one thread per output.
 */
int sw_conv2d_depthwise(const float* x, const float* w, float* y,
                        int N, int C, int H, int W, int R, int S,
                        int stride, int pad, void* hip_stream);

/*
 * Quantised 2-D convolution (paper, sections 1.1 and 3: quantisation applies to
 * the sliding formulation as it does to GEMM).  int8 activations and weights,
 * exact int32 sums, no requantisation.  Shapes as sw_conv2d.
 * The caller guarantees C_in*R*S <= 131071 so that no sum can leave int32
 * (SW_ERR_SHAPE otherwise).  x and w need no alignment; y is 4-byte aligned.
 * All shapes run on the matrix cores: 3x3 at stride 1 with C_in % 64 == 0,
 * C_out % 64 == 0, W % 4 == 0, 4-byte aligned x and 16-byte aligned w in a
 * large-tile kernel, every other extent, stride, padding and channel count in an
 * any-shape kernel (one thread per output only when the filter does not fit the
 * LDS, about R*S > 40).
 */
int sw_conv2d_s8(const int8_t* x, const int8_t* w, int32_t* y,
                 int N, int C_in, int C_out, int H, int W, int R, int S,
                 int stride, int pad, void* hip_stream);

/*
 * The same convolution with the requantisation of a quantised pipeline fused into the store (paper, section
 * 1.1: quantised inference keeps activations in 8 bits): the int32 sums never reach memory, the output is int8.
 *     q[n,co,i,j] = clamp(rne(scale[co] * float(acc[n,co,i,j] + bias[co])), relu ? 0 : -128, 127)
 * acc is the exact sum of sw_conv2d_s8; acc + bias must fit int32 (caller's guarantee); the conversion to
 * fp32, the product and the rounding (to nearest, ties to even) are fp32 operations, so the result is the
 * same bits on every IEEE machine.  bias: [C_out] int32 or NULL (zeros); scale: [C_out] fp32, finite;
 * y: [N,C_out,H_out,W_out] int8.  Errors as sw_conv2d_s8; scale == NULL is SW_ERR_NULL.
 */
int sw_conv2d_s8_requant(const int8_t* x, const int8_t* w, const int32_t* bias, const float* scale, int8_t* y,
                         int N, int C_in, int C_out, int H, int W, int R, int S,
                         int stride, int pad, int relu, void* hip_stream);

/*
 * The quantised convolution with filters packed once (paper, section 1.1: the weights of a
 * quantised network are fixed at inference time; section 3: taps as small matrix products).
 * sw_s8_pack_filter rewrites w [C_out,C_in,R,S] int8 into the operand order of the int8
 * matrix instruction; sw_conv2d_s8_packed / _requant then compute exactly the sums of
 * sw_conv2d_s8 / sw_conv2d_s8_requant (bit for bit) without transposing the filters in every
 * workgroup of every call.  The input and the output are the same unmodified channel-first
 * tensors as before.
 *     packed: caller-owned device buffer of sw_s8_packed_filter_bytes(C_in, C_out, R, S) bytes,
 *             16-byte aligned (SW_ERR_ALIGN), not overlapping w or y (SW_ERR_ALIAS).  Its
 *             contents are private to this library version (sw_version) and depend on
 *             (C_in, C_out, R, S) only; pack once, use for any N, H, W, stride and padding.
 * sw_s8_packed_filter_bytes returns 0 for invalid extents (<= 0, R or S > 64, more than
 * 2^31-1 filter elements).  sw_s8_pack_filter enqueues one small kernel on hip_stream; the
 * convolution calls must be ordered after it (same stream, or an event).
 * Errors of the convolution calls as sw_conv2d_s8 / sw_conv2d_s8_requant.  3x3 at stride 1
 * with C_in in {32, 64, 128}, C_out % 64 == 0, W % 4 == 0 and 4-byte aligned x runs on the
 * matrix cores with every A operand loaded straight into registers; every other valid shape
 * one thread per output.
 */
int64_t sw_s8_packed_filter_bytes(int C_in, int C_out, int R, int S);
int sw_s8_pack_filter(const int8_t* w, int8_t* packed, int C_in, int C_out, int R, int S, void* hip_stream);
int sw_conv2d_s8_packed(const int8_t* x, const int8_t* packed, int32_t* y,
                        int N, int C_in, int C_out, int H, int W, int R, int S,
                        int stride, int pad, void* hip_stream);
int sw_conv2d_s8_packed_requant(const int8_t* x, const int8_t* packed, const int32_t* bias, const float* scale,
                                int8_t* y, int N, int C_in, int C_out, int H, int W, int R, int S,
                                int stride, int pad, int relu, void* hip_stream);

/*
 * A depthwise-separable block in one launch (paper, section 1.2: depthwise
 * separable convolutions; sections 1 and 2: nothing but input, filters and output
 * moves): depthwise 3 x 3 (stride 1, padding 1) with bias and optional rectifier,
 * then a pointwise 1 x 1 convolution with bias and optional rectifier,
 *     t[n,c,i,j]  = act_dw( sum_{r,s} w_dw[c,0,r,s] * xz[n,c,i+r-1,j+s-1] + b_dw[c] )
 *     y[n,co,i,j] = act_pw( sum_c w_pw[co,c,0,0] * t[n,c,i,j] + b_pw[co] )
 * with t kept in LDS: it is never written to device memory.
 * x: [N,C,H,W];  w_dw: [C,1,3,3];  b_dw: [C] or NULL;  w_pw: [C_out,C,1,1];
 * b_pw: [C_out] or NULL;  y: [N,C_out,H,W].  All fp32, products and sums fp32.
 * Errors as sw_conv2d (SW_ERR_NULL, _SHAPE, _ALIGN, _ALIAS); any N, C, C_out, H, W
 * within the 2^31-1 element bound is supported.  What it saves is the memory and
 * the traffic of the intermediate (N*C*H*W floats written and read back); as it
 * stands it is 2-4 x slower than sw_conv2d_depthwise_bias_relu followed by
 * sw_conv2d_bias_relu (its stages run one after the other inside a workgroup, and
 * on this chip fp32 vector arithmetic does not overlap with fp32 matrix
 * instructions): call those two unless the intermediate's memory is what matters.
 */
int sw_dw_pw_block(const float* x, const float* w_dw, const float* b_dw,
                   const float* w_pw, const float* b_pw, float* y,
                   int N, int C, int C_out, int H, int W,
                   int relu_dw, int relu_pw, void* hip_stream);

/*
 * Depthwise 2-D convolution on bf16 activations with fp32 accumulation (paper,
 * section 1.1: reduced-precision inference; the sliding kernels are bound by the
 * bytes of the planes, which this halves).  x and y hold bf16 bit patterns (the
 * upper 16 bits of an IEEE fp32); the filter stays fp32.  Every product and sum
 * is fp32, exactly as in sw_conv2d_depthwise on the widened input; the finished
 * sum is rounded to bf16 once (nearest, ties to even; NaN stays NaN).
 * x: [N,C,H,W] bf16;  w: [C,1,R,S] fp32;  y: [N,C,H_out,W_out] bf16.
 * x and y must be 2-byte aligned, w 4-byte aligned; errors as sw_conv2d_depthwise.
 * 3x3, 5x5, 7x7 at stride 1 on planes up to 56 x 56 with W and W_out multiples of
 * 8 and 16-byte aligned x, y run the sliding whole-plane kernel; every other
 * valid shape one thread per output.
 */
int sw_conv2d_depthwise_bf16(const uint16_t* x, const float* w, uint16_t* y,
                             int N, int C, int H, int W, int R, int S,
                             int stride, int pad, void* hip_stream);

/*
 * Dilated (a trous) variants of sw_conv2d and sw_conv2d_depthwise (paper, figure 2
 * names dilated variants among the 2-D kernels): neighbouring taps are `dilation`
 * input positions apart,
 *     y[n,co,i,j] = sum_{ci,r,s} w[co,ci,r,s] * xz[n,ci,i*stride+r*dilation-pad, j*stride+s*dilation-pad]
 * so the filter spans dilation*(R-1)+1 rows and H_out = sw_out_dim(H, dilation*(R-1)+1, stride, pad)
 * (columns alike).  dilation >= 1 (else SW_ERR_SHAPE); dilation == 1 is the undilated call.
 * Other arguments, layouts and errors as the undilated calls.  With C_in >= 2 the
 * matrix-core kernel runs (the window in LDS grows, the taps step through it
 * `dilation` apart); depthwise and C_in == 1 at stride 1 run the sliding tile
 * kernel while the filter's span is at most 51 (3x3 at dilation 2 and 4 unrolled,
 * other extents and dilations with run-time loops), else one thread per output.
 */
int sw_conv2d_dilated(const float* x, const float* w, float* y,
                      int N, int C_in, int C_out, int H, int W, int R, int S,
                      int stride, int pad, int dilation, void* hip_stream);
int sw_conv2d_depthwise_dilated(const float* x, const float* w, float* y,
                                int N, int C, int H, int W, int R, int S,
                                int stride, int pad, int dilation, void* hip_stream);

/*
 * Depthwise 2-D convolution through a kernel generated at run time (paper, section 2:
 * custom kernels generated at run time for every filter size).  Arguments, layouts,
 * result and errors as sw_conv2d_depthwise.  For stride 1 or 2, an output plane of at
 * most 56 x 56 (at least 9 x 9, and at least half of the 8 x 8 lane grid's share), W and W_out
 * multiples of 4, H*W <= 4096, H_out <= H and W_out <= W, an LDS window of at most 37 KB
 * (33 x 33 at 56 x 56)
 * and x, y 16-byte aligned, the first
 * call for a geometry (H, W, R, S, pad) compiles a kernel specialised on it (about a
 * second on the calling thread, host-synchronous; do not make that first call inside
 * a stream capture -- use sw_jit_prepare_depthwise beforehand), keeps it for the life
 * of the process and launches it; later calls only launch.  That first call is the one
 * place where this library allocates: loading the compiled module takes host and device
 * memory from the HIP runtime, so callers that must not allocate (stream capture, serving
 * loops) call sw_jit_prepare_depthwise for their geometries at set-up.  Every other valid
 * shape, and a geometry whose generated kernel cannot be compiled or loaded (the compiler's
 * log goes to stderr; sw_jit_prepare_depthwise reports SW_ERR_JIT), runs
 * sw_conv2d_depthwise's precompiled kernels.  Thread-safe.
 */
int sw_conv2d_depthwise_jit(const float* x, const float* w, float* y,
                            int N, int C, int H, int W, int R, int S,
                            int stride, int pad, void* hip_stream);

/*
 * Compiles and loads the generated kernel of a geometry ahead of its first use.
 * SW_OK; SW_ERR_UNSUPPORTED if sw_conv2d_depthwise_jit would run a precompiled
 * kernel for it; SW_ERR_SHAPE for invalid extents; SW_ERR_JIT; SW_ERR_LAUNCH
 * (no device, or the module did not load).
 */
int sw_jit_prepare_depthwise(int H, int W, int R, int S, int stride, int pad);

/*
 * As sw_jit_prepare_depthwise, but only compiles (needs no device, caches
 * nothing): tells whether the generated source builds for a geometry.
 */
int sw_jit_compile_check(int H, int W, int R, int S, int stride, int pad);

/*
 * The generated kernels with strides and dilations (paper, section 2: a custom kernel
 * for every filter; figure 2 names strided and dilated variants): as the three calls
 * above with taps `dilation` input positions apart (dilation == 1: the same calls).
 * Generated for stride 1 and 2 and any dilation whose span (R-1)*dilation+1 is at most
 * 64: the 8 x 8 lanes of a wavefront own ceil(max(H_out, W_out) / 8)^2 outputs each, the
 * stride and the dilation are constants of the register slide.  The other limits are
 * those of sw_conv2d_depthwise_jit (output plane at most 56 x 56 and at least 9 x 9,
 * H*W <= 4096, W and W_out multiples of 4, LDS window at most 37 KB).
 */
int sw_conv2d_depthwise_dilated_jit(const float* x, const float* w, float* y,
                                    int N, int C, int H, int W, int R, int S,
                                    int stride, int pad, int dilation, void* hip_stream);
int sw_jit_prepare_depthwise_dilated(int H, int W, int R, int S, int stride, int pad, int dilation);
int sw_jit_compile_check_dilated(int H, int W, int R, int S, int stride, int pad, int dilation);

/* Number of generated kernels this process holds. */
int sw_jit_cached_kernels(void);

/*
 * The quantised convolution on channel-last tensors (paper, sections 1.1 and 3; the
 * layout quantised inference engines keep their activations in):
 *     x: [N,H,W,C_in] int8;  w: [C_out,R,S,C_in] int8;
 *     y: [N,H_out,W_out,C_out] int32 (sw_conv2d_s8_nhwc) or int8 (…_requant),
 * the same sums as sw_conv2d_s8 / sw_conv2d_s8_requant on the transposed tensors, bit
 * for bit.  The matrix instruction reads 16 consecutive channels per lane, which in
 * this layout are 16 consecutive bytes: nothing is transposed on the way.  Note the
 * argument order (H, W before the channel counts).  Errors as the channel-first
 * calls.  C_in a multiple of 32 and 16-byte aligned x and w run on the matrix cores:
 * with C_out % 4 == 0, y aligned to four elements, tensors below 2 GiB and tiles of
 * output rows (at most 256 outputs wide) whose windows fit LDS, on the kernel that
 * brings the windows in by direct-to-LDS loads a tile ahead (the one the channel-last
 * fp32 / bf16 / half calls run on); else, with the filters of 64 output channels within
 * 96 KB, on one that copies them through registers (any extent and stride, C_out any);
 * every other valid shape one thread per output.
 */
int sw_conv2d_s8_nhwc(const int8_t* x, const int8_t* w, int32_t* y,
                      int N, int H, int W, int C_in, int C_out, int R, int S,
                      int stride, int pad, void* hip_stream);
int sw_conv2d_s8_nhwc_requant(const int8_t* x, const int8_t* w, const int32_t* bias, const float* scale, int8_t* y,
                              int N, int H, int W, int C_in, int C_out, int R, int S,
                              int stride, int pad, int relu, void* hip_stream);

/*
 * The multi-channel convolution on channel-last tensors in fp32, bf16 and IEEE half (paper,
 * section 3: the taps as small matrix products; section 1.1: reduced precision):
 *     x: [N,H,W,C_in];  w: [C_out,R,S,C_in];  y: [N,H_out,W_out,C_out];
 *     y[n,i,j,co] = act(sum_{r,s,ci} w[co,r,s,ci] * xz[n, i*stride+r*dilation-pad, j*stride+s*dilation-pad, ci] + bias[co])
 * with act(t) = relu ? max(t, 0) : t, bias: [C_out] fp32 device pointer or NULL,
 * dilation >= 1, H_out = sw_out_dim_dilated(H, R, stride, pad, dilation).
 * sw_conv2d_nhwc: fp32 tensors, fp32 products and sums (any order), one fp32 addition
 * of the bias.  sw_conv2d_bf16_nhwc: x, w and y hold bf16 bit patterns (2-byte
 * aligned); products and sums are fp32 (a product of two bf16 values is exact in
 * fp32: bf16 matrix instructions with fp32 accumulators), the bias is added in fp32,
 * and the finished value is rounded once to bf16, to nearest, ties to even.
 * sw_conv2d_f16_nhwc: the same with IEEE half-precision bit patterns (a product of two
 * halves is exact in fp32 as well; the one rounding to half is to nearest, ties to
 * even, beyond 65504 to infinity, denormal results kept; denormal inputs count).
 * Note the argument order (H, W before the channel counts).  Errors as sw_conv2d.
 * Pixels of a multiple of 32 bytes (C_in % 8 == 0 in fp32, % 16 in bf16 / half) and 16-byte
 * aligned x and w run on the matrix cores, the channels in chunks of up to 128 bytes
 * per pixel (any extent, stride, dilation and C_out); every other valid shape one
 * thread per output.  With C_out % 4 == 0, y aligned to four elements and tensors below
 * 2 GiB there are faster kernels.  Where a tile of output rows (at most 256 outputs wide)
 * and its window fit LDS (all three formats), the windows are brought in by
 * direct-to-LDS loads a tile ahead, the filters resident in LDS (those of 32 output
 * channels within 76 KB) or, larger, fetched chunk by chunk with the windows; otherwise,
 * bf16 / half with R, S <= 32 and the filters of 32 output channels within 150 KB read
 * the pixel operands straight from x (no window in LDS).
 */
int sw_conv2d_nhwc(const float* x, const float* w, const float* bias, float* y,
                   int N, int H, int W, int C_in, int C_out, int R, int S,
                   int stride, int pad, int dilation, int relu, void* hip_stream);
int sw_conv2d_bf16_nhwc(const void* x, const void* w, const float* bias, void* y,
                        int N, int H, int W, int C_in, int C_out, int R, int S,
                        int stride, int pad, int dilation, int relu, void* hip_stream);
int sw_conv2d_f16_nhwc(const void* x, const void* w, const float* bias, void* y,
                       int N, int H, int W, int C_in, int C_out, int R, int S,
                       int stride, int pad, int dilation, int relu, void* hip_stream);

/* Output extent of one axis; <= 0 means the filter does not fit (or bad arguments). */
int64_t sw_out_dim(int64_t in, int k, int stride, int pad);

/* The same for a filter whose taps are `dilation` input positions apart (span dilation*(k-1)+1). */
int64_t sw_out_dim_dilated(int64_t in, int k, int stride, int pad, int dilation);

/* Device workspace the library needs: always 0 (paper, sections 1 and 2). */
size_t sw_workspace_bytes(void);

/* Static, NUL-terminated description of an sw_status value. */
const char* sw_status_string(int status);

/* major*10000 + minor*100 + patch */
int sw_version(void);

/*
 * Measurement aids (no part of the convolution path): sw_probe enqueues a kernel that issues `iters` loop
 * turns of one kind of arithmetic instruction on every SIMD of the device and touches no memory (the two
 * "fed" kinds read their operands from LDS, one workgroup of one or two wavefronts per SIMD on every CU);
 * sw_probe_ops(kind, iters) is the number of arithmetic operations (2 per multiply-add) that launch performs.
 * Timing the launch gives the rate the chip sustains for that instruction, to quote beside the datasheet peak.
 * SW_ERR_SHAPE for iters <= 0, SW_ERR_UNSUPPORTED for an unknown kind.
 */
typedef enum {
    SW_PROBE_MFMA_F32 = 0,  /* v_mfma_f32_32x32x2_f32                                  */
    SW_PROBE_MFMA_I8 = 1,   /* v_mfma_i32_32x32x32_i8                                  */
    SW_PROBE_FMA_F32 = 2,   /* v_fma_f32, wave-uniform multiplicand (no packed forms)  */
    SW_PROBE_FMA_MFMA_F32 = 3, /* nine v_fma_f32, one v_mfma_f32_16x16x4_f32, ... in one stream: do the two pipes overlap? */
    SW_PROBE_MFMA_F32_FED = 4, /* v_mfma_f32_32x32x2_f32 with one 4-byte LDS operand read behind each, one wavefront per SIMD */
    SW_PROBE_MFMA_F32_FED2 = 5, /* the same with two wavefronts per SIMD */
    SW_PROBE_MFMA_BF16 = 6     /* v_mfma_f32_32x32x16_bf16 */
} sw_probe_kind;
int sw_probe(int kind, int iters, void* hip_stream);
int64_t sw_probe_ops(int kind, int iters);

/*
 * Diagnostics: the name (with template arguments) of the kernel that the calling thread's most
 * recent convolution, pooling or packing call enqueued; "" before the first call.  The string
 * lives in thread-local storage and is overwritten by the next sw_last_kernel call of the thread.
 * Tests use it to check that a small case runs the same kernel as the large launch it stands for.
 */
const char* sw_last_kernel(void);

#ifdef __cplusplus
}
#endif
#endif /* SWCONV_H */
