/*
 * CPU oracle for sliding-window-sum convolution and pooling.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU path and
 * the GPU path never calls it.
 *
 * What it computes.  The paper (section 2, "Experiments") states that the
 * sliding-window kernels perform the same arithmetic operations as the naive
 * algorithm and are a drop-in for the ONNX convolution call, and its abstract
 * states that 1-D pooling and convolution are both sliding sums.  The result
 * therefore has a plain definition, which is written out here:
 *
 *   conv2d     y[n,co,i,j] = sum_{ci,r,s} w[co,ci,r,s] * xz[n,ci,i*st+r-pad,j*st+s-pad]
 *   depthwise  y[n,c,i,j]  = sum_{r,s}    w[c,0,r,s]   * xz[n,c,i*st+r-pad,j*st+s-pad]
 *   conv1d     y[row,i]    = sum_{j<k}    w[j]         * xz[row,i*st+j-pad]
 *   avg pool   y[row,i]    = (1/window) * sum_{j<window} x[row,i*st+j]
 *   max pool   y[row,i]    = max_{j<window} x[row,i*st+j]
 *   avg pool2d y[p,i,j]    = (1/(R*S)) * sum_{r,s} xz[p,i*st+r-pad,j*st+s-pad]
 *   max pool2d y[p,i,j]    = max over the (r,s) whose position lies inside the plane
 *   requantise q[n,co,p]   = clamp(rne(scale[co] * float(acc[n,co,p] + bias[co])), lo, 127),  lo = relu ? 0 : -128
 *   bias, relu y[n,co,p]   = act(y[n,co,p] + bias[co]),  act(t) = relu ? max(t, 0) : t
 *   dilated    y[n,co,i,j] = sum_{ci,r,s} w[co,ci,r,s] * xz[n,ci,i*st+r*dil-pad,j*st+s*dil-pad]
 *
 * xz is x inside the tensor and 0 outside (zero padding); no filter flip
 * (cross-correlation, as DNN frameworks define "convolution"); output extent
 * floor((in + 2*pad - k)/st) + 1; NCHW activations, OIHW weights, dense.
 *
 * Arithmetic: fp32 inputs are widened exactly to fp64, every product and sum
 * is taken in fp64 in the fixed order (ci, r, s); the int8 path accumulates
 * in int64 and refuses a sum that does not fit int32.  Beside each
 * floating-point output the magnitude sum D = sum |x*w| is returned; the
 * parity tolerance is stated relative to it.
 *
 * OpenMP only splits independent outputs, so threading cannot change a value.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Output extent of a strided, zero-padded window of size k; <= 0 if none fits. */
int64_t oracle_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad)
{
    if (in <= 0 || k <= 0 || stride <= 0 || pad < 0) return 0;
    int64_t span = in + 2 * pad - k;
    if (span < 0) return 0;
    return span / stride + 1;
}

/* conv2d by its definition.  y and d hold N*C_out*H_out*W_out doubles; d may be NULL. */
int oracle_conv2d(const float *x, const float *w, double *y, double *d,
                  int64_t N, int64_t C_in, int64_t C_out, int64_t H, int64_t W,
                  int64_t R, int64_t S, int64_t stride, int64_t pad)
{
    const int64_t Ho = oracle_out_dim(H, R, stride, pad);
    const int64_t Wo = oracle_out_dim(W, S, stride, pad);
    if (N <= 0 || C_in <= 0 || C_out <= 0 || Ho <= 0 || Wo <= 0) return 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t co = 0; co < C_out; ++co) {
            for (int64_t i = 0; i < Ho; ++i) {
                for (int64_t j = 0; j < Wo; ++j) {
                    double acc = 0.0, mag = 0.0;
                    for (int64_t ci = 0; ci < C_in; ++ci) {
                        for (int64_t r = 0; r < R; ++r) {
                            const int64_t h = i * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int64_t s = 0; s < S; ++s) {
                                const int64_t v = j * stride + s - pad;
                                if (v < 0 || v >= W) continue;
                                const double xv = (double)x[((n * C_in + ci) * H + h) * W + v];
                                const double wv = (double)w[((co * C_in + ci) * R + r) * S + s];
                                const double p = xv * wv;
                                acc += p;
                                mag += fabs(p);
                            }
                        }
                    }
                    const int64_t o = ((n * C_out + co) * Ho + i) * Wo + j;
                    y[o] = acc;
                    if (d) d[o] = mag;
                }
            }
        }
    }
    return 0;
}

/* One R x S filter per channel: w is [C,1,R,S]. */
int oracle_conv2d_depthwise(const float *x, const float *w, double *y, double *d,
                            int64_t N, int64_t C, int64_t H, int64_t W,
                            int64_t R, int64_t S, int64_t stride, int64_t pad)
{
    const int64_t Ho = oracle_out_dim(H, R, stride, pad);
    const int64_t Wo = oracle_out_dim(W, S, stride, pad);
    if (N <= 0 || C <= 0 || Ho <= 0 || Wo <= 0) return 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t c = 0; c < C; ++c) {
            for (int64_t i = 0; i < Ho; ++i) {
                for (int64_t j = 0; j < Wo; ++j) {
                    double acc = 0.0, mag = 0.0;
                    for (int64_t r = 0; r < R; ++r) {
                        const int64_t h = i * stride + r - pad;
                        if (h < 0 || h >= H) continue;
                        for (int64_t s = 0; s < S; ++s) {
                            const int64_t v = j * stride + s - pad;
                            if (v < 0 || v >= W) continue;
                            const double p = (double)x[((n * C + c) * H + h) * W + v] *
                                             (double)w[(c * R + r) * S + s];
                            acc += p;
                            mag += fabs(p);
                        }
                    }
                    const int64_t o = ((n * C + c) * Ho + i) * Wo + j;
                    y[o] = acc;
                    if (d) d[o] = mag;
                }
            }
        }
    }
    return 0;
}

/* One tap vector w[k] shared by every row. */
int oracle_conv1d(const float *x, const float *w, double *y, double *d,
                  int64_t rows, int64_t len, int64_t k, int64_t stride, int64_t pad)
{
    const int64_t Lo = oracle_out_dim(len, k, stride, pad);
    if (rows <= 0 || Lo <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t row = 0; row < rows; ++row) {
        for (int64_t i = 0; i < Lo; ++i) {
            double acc = 0.0, mag = 0.0;
            for (int64_t j = 0; j < k; ++j) {
                const int64_t t = i * stride + j - pad;
                if (t < 0 || t >= len) continue;
                const double p = (double)w[j] * (double)x[row * len + t];
                acc += p;
                mag += fabs(p);
            }
            y[row * Lo + i] = acc;
            if (d) d[row * Lo + i] = mag;
        }
    }
    return 0;
}

/* mode 0 = average (divisor is always window: there is no padding), 1 = maximum.
 * For the maximum d is set to |y| (the maximum never rounds; d is unused there). */
int oracle_pool1d(const float *x, double *y, double *d,
                  int64_t rows, int64_t len, int64_t window, int64_t stride, int mode)
{
    const int64_t Lo = oracle_out_dim(len, window, stride, 0);
    if (rows <= 0 || Lo <= 0 || (mode != 0 && mode != 1)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t row = 0; row < rows; ++row) {
        for (int64_t i = 0; i < Lo; ++i) {
            const float *p = x + row * len + i * stride;
            if (mode == 0) {
                double acc = 0.0, mag = 0.0;
                for (int64_t j = 0; j < window; ++j) {
                    acc += (double)p[j];
                    mag += fabs((double)p[j]);
                }
                y[row * Lo + i] = acc / (double)window;
                if (d) d[row * Lo + i] = mag / (double)window;
            } else {
                double m = (double)p[0];
                for (int64_t j = 1; j < window; ++j)
                    if ((double)p[j] > m) m = (double)p[j];
                y[row * Lo + i] = m;
                if (d) d[row * Lo + i] = fabs(m);
            }
        }
    }
    return 0;
}

/* Pooling over R x S windows of each of `planes` H x W planes (abstract: pooling is a sliding sum).
 * mode 0 = average: the sliding sum of the zero-padded plane times 1/(R*S); the divisor is R*S
 * everywhere, padded positions count as zeros.  mode 1 = maximum over the window positions that
 * lie inside the plane (padding never wins); a window with no position inside is an error (3).
 * d: average -> sum |x| / (R*S); maximum -> |y|. */
int oracle_pool2d(const float *x, double *y, double *d, int64_t planes, int64_t H, int64_t W,
                  int64_t R, int64_t S, int64_t stride, int64_t pad, int mode)
{
    const int64_t Ho = oracle_out_dim(H, R, stride, pad);
    const int64_t Wo = oracle_out_dim(W, S, stride, pad);
    if (planes <= 0 || Ho <= 0 || Wo <= 0 || (mode != 0 && mode != 1)) return 1;
    int empty = 0;
#pragma omp parallel for schedule(static) reduction(| : empty)
    for (int64_t p = 0; p < planes; ++p) {
        const float *xp = x + p * H * W;
        for (int64_t i = 0; i < Ho; ++i) {
            for (int64_t j = 0; j < Wo; ++j) {
                double acc = 0.0, mag = 0.0, m = 0.0;
                int64_t inside = 0;
                for (int64_t r = 0; r < R; ++r) {
                    const int64_t h = i * stride + r - pad;
                    if (h < 0 || h >= H) continue;
                    for (int64_t s = 0; s < S; ++s) {
                        const int64_t v = j * stride + s - pad;
                        if (v < 0 || v >= W) continue;
                        const double e = (double)xp[h * W + v];
                        acc += e;
                        mag += fabs(e);
                        if (inside == 0 || e > m) m = e;
                        ++inside;
                    }
                }
                const int64_t o = (p * Ho + i) * Wo + j;
                if (mode == 0) {
                    y[o] = acc / (double)(R * S);
                    if (d) d[o] = mag / (double)(R * S);
                } else {
                    if (inside == 0) empty = 1;
                    y[o] = m;
                    if (d) d[o] = fabs(m);
                }
            }
        }
    }
    return empty ? 3 : 0;
}

/* int8 x int8 -> exact integer sum; returns 2 if any sum leaves the int32 range. */
int oracle_conv2d_s8(const int8_t *x, const int8_t *w, int32_t *y,
                     int64_t N, int64_t C_in, int64_t C_out, int64_t H, int64_t W,
                     int64_t R, int64_t S, int64_t stride, int64_t pad)
{
    const int64_t Ho = oracle_out_dim(H, R, stride, pad);
    const int64_t Wo = oracle_out_dim(W, S, stride, pad);
    if (N <= 0 || C_in <= 0 || C_out <= 0 || Ho <= 0 || Wo <= 0) return 1;
    int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : overflow)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t co = 0; co < C_out; ++co) {
            for (int64_t i = 0; i < Ho; ++i) {
                for (int64_t j = 0; j < Wo; ++j) {
                    int64_t acc = 0;
                    for (int64_t ci = 0; ci < C_in; ++ci) {
                        for (int64_t r = 0; r < R; ++r) {
                            const int64_t h = i * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int64_t s = 0; s < S; ++s) {
                                const int64_t v = j * stride + s - pad;
                                if (v < 0 || v >= W) continue;
                                acc += (int64_t)x[((n * C_in + ci) * H + h) * W + v] *
                                       (int64_t)w[((co * C_in + ci) * R + r) * S + s];
                            }
                        }
                    }
                    if (acc > INT32_MAX || acc < INT32_MIN) overflow |= 1;
                    y[((n * C_out + co) * Ho + i) * Wo + j] = (int32_t)acc;
                }
            }
        }
    }
    return overflow ? 2 : 0;
}

/* Requantisation of exact int32 sums to int8 (section 1.1 of the paper: quantised inference keeps activations
 * in 8 bits; the paper gives no formula, this is the common per-channel one).  The sum plus the channel's bias is
 * taken exactly (int64; 2 is returned if it leaves int32), converted to fp32 (round to nearest even), multiplied
 * by the channel's fp32 scale in fp32, rounded to the nearest integer (ties to even) and clamped to
 * [relu ? 0 : -128, 127].  The precision of every step is part of the definition: the same steps in the same
 * precision give the same bits on any IEEE machine.  bias may be NULL (zeros). */
int oracle_requant_s8(const int32_t *acc, const int32_t *bias, const float *scale, int8_t *q,
                      int64_t N, int64_t C_out, int64_t pixels, int relu)
{
    if (N <= 0 || C_out <= 0 || pixels <= 0) return 1;
    int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : overflow)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t co = 0; co < C_out; ++co) {
            const int64_t b = bias ? (int64_t)bias[co] : 0;
            const float sc = scale[co];
            for (int64_t p = 0; p < pixels; ++p) {
                const int64_t t = (int64_t)acc[(n * C_out + co) * pixels + p] + b;
                if (t > INT32_MAX || t < INT32_MIN) overflow |= 1;
                const float v = (float)(int32_t)t;
                const float prod = v * sc;
                float r = nearbyintf(prod);
                const float lo = relu ? 0.0f : -128.0f;
                if (r < lo) r = lo;
                if (r > 127.0f) r = 127.0f;
                q[(n * C_out + co) * pixels + p] = (int8_t)r;
            }
        }
    }
    return overflow ? 2 : 0;
}

/* Per-channel bias and rectifier on a finished fp64 convolution result (section 1 of the paper: the layers these
 * kernels serve are followed by a bias and an activation; the paper gives no formula, this is the usual one):
 * y <- y + bias[co], the magnitude sum D <- D + |bias[co]| (the bias is one more term of the sum), then
 * y <- max(y, 0) if relu.  bias may be NULL (zeros).  In place. */
int oracle_bias_relu(double *y, double *d, const float *bias, int64_t N, int64_t C_out, int64_t pixels, int relu)
{
    if (N <= 0 || C_out <= 0 || pixels <= 0) return 1;
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t co = 0; co < C_out; ++co) {
            const double b = bias ? (double)bias[co] : 0.0;
            for (int64_t p = 0; p < pixels; ++p) {
                const int64_t o = (n * C_out + co) * pixels + p;
                double t = y[o] + b;
                if (relu && t < 0.0) t = 0.0;
                y[o] = t;
                d[o] += fabs(b);
            }
        }
    }
    return 0;
}

/* Dilated (a trous) convolution by its definition: the taps of the filter are `dil` input positions apart, so
 * the filter spans dil*(k-1)+1 inputs per axis and the output extent is that of a filter of this span (figure 2
 * of the paper names dilated variants among the 2-D kernels).  depthwise != 0: one filter per channel,
 * w is [C,1,R,S] and C_in == C_out is required; else w is [C_out,C_in,R,S].  d may be NULL. */
int64_t oracle_out_dim_dilated(int64_t in, int64_t k, int64_t stride, int64_t pad, int64_t dil)
{
    if (k <= 0 || dil <= 0) return 0;
    return oracle_out_dim(in, dil * (k - 1) + 1, stride, pad);
}

int oracle_conv2d_dilated(const float *x, const float *w, double *y, double *d,
                          int64_t N, int64_t C_in, int64_t C_out, int64_t H, int64_t W,
                          int64_t R, int64_t S, int64_t stride, int64_t pad, int64_t dil, int depthwise)
{
    if (dil <= 0 || R <= 0 || S <= 0) return 1;
    const int64_t Ho = oracle_out_dim_dilated(H, R, stride, pad, dil);
    const int64_t Wo = oracle_out_dim_dilated(W, S, stride, pad, dil);
    if (N <= 0 || C_in <= 0 || C_out <= 0 || Ho <= 0 || Wo <= 0) return 1;
    if (depthwise && C_in != C_out) return 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t co = 0; co < C_out; ++co) {
            const int64_t ci_first = depthwise ? co : 0, ci_end = depthwise ? co + 1 : C_in;
            for (int64_t i = 0; i < Ho; ++i) {
                for (int64_t j = 0; j < Wo; ++j) {
                    double acc = 0.0, mag = 0.0;
                    for (int64_t ci = ci_first; ci < ci_end; ++ci) {
                        const float *wf = depthwise ? w + co * R * S : w + (co * C_in + ci) * R * S;
                        for (int64_t r = 0; r < R; ++r) {
                            const int64_t hd = i * stride + r * dil - pad;
                            if (hd < 0 || hd >= H) continue;
                            for (int64_t s = 0; s < S; ++s) {
                                const int64_t vd = j * stride + s * dil - pad;
                                if (vd < 0 || vd >= W) continue;
                                const double t = (double)x[((n * C_in + ci) * H + hd) * W + vd] * (double)wf[r * S + s];
                                acc += t;
                                mag += fabs(t);
                            }
                        }
                    }
                    const int64_t o = ((n * C_out + co) * Ho + i) * Wo + j;
                    y[o] = acc;
                    if (d) d[o] = mag;
                }
            }
        }
    }
    return 0;
}
