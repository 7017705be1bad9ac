/* Runs every function of sw_oracle.c on small deterministic inputs held in exactly-sized heap buffers, and prints
 * one line per call: "<function> <parameters> : <FNV-1a hash of the outputs>".  Built with
 * -fsanitize=address,undefined by tests/test_oracle_sanitized.py (an out-of-bounds access, a signed overflow or a
 * misaligned access in the oracle aborts the run); the test also recomputes every line through the ordinary build.
 * Test infrastructure, like the oracle itself. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int64_t oracle_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad);
int64_t oracle_out_dim_dilated(int64_t in, int64_t k, int64_t stride, int64_t pad, int64_t dil);
int oracle_conv2d(const float *, const float *, double *, double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                  int64_t, int64_t, int64_t);
int oracle_conv2d_depthwise(const float *, const float *, double *, double *, int64_t, int64_t, int64_t, int64_t, int64_t,
                            int64_t, int64_t, int64_t);
int oracle_conv1d(const float *, const float *, double *, double *, int64_t, int64_t, int64_t, int64_t, int64_t);
int oracle_pool1d(const float *, double *, double *, int64_t, int64_t, int64_t, int64_t, int);
int oracle_pool2d(const float *, double *, double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int);
int oracle_conv2d_s8(const int8_t *, const int8_t *, int32_t *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                     int64_t, int64_t);
int oracle_requant_s8(const int32_t *, const int32_t *, const float *, int8_t *, int64_t, int64_t, int64_t, int);
int oracle_bias_relu(double *, double *, const float *, int64_t, int64_t, int64_t, int);
int oracle_conv2d_dilated(const float *, const float *, double *, double *, int64_t, int64_t, int64_t, int64_t, int64_t,
                          int64_t, int64_t, int64_t, int64_t, int64_t, int);

static uint32_t mix(uint64_t i, uint32_t salt) { return (uint32_t)((i + salt) * 2654435761u); }
static float *floats(int64_t n, uint32_t salt)
{
    float *p = malloc((size_t)n * sizeof *p);
    for (int64_t i = 0; i < n; ++i) p[i] = (float)((mix((uint64_t)i, salt) >> 8) & 0xFFFF) / 32768.0f - 1.0f;
    return p;
}
static int8_t *bytes(int64_t n, uint32_t salt)
{
    int8_t *p = malloc((size_t)n);
    for (int64_t i = 0; i < n; ++i) p[i] = (int8_t)(mix((uint64_t)i, salt) >> 11);
    return p;
}
static uint64_t fnv(uint64_t h, const void *data, size_t n)
{
    const unsigned char *b = data;
    for (size_t i = 0; i < n; ++i) h = (h ^ b[i]) * 1099511628211ull;
    return h;
}
#define FNV0 1469598103934665603ull

int main(void)
{
    /* N, C_in, C_out, H, W, R, S, stride, pad */
    static const int64_t conv[][9] = {{1, 1, 1, 3, 3, 3, 3, 1, 0}, {2, 3, 4, 7, 9, 3, 3, 1, 1}, {1, 2, 3, 8, 6, 5, 2, 2, 2},
                                      {1, 4, 2, 5, 5, 1, 1, 1, 0}, {1, 1, 2, 4, 4, 7, 7, 1, 3}, {2, 5, 5, 6, 6, 3, 3, 3, 1}};
    for (size_t c = 0; c < sizeof conv / sizeof conv[0]; ++c) {
        const int64_t *p = conv[c], Ho = oracle_out_dim(p[3], p[5], p[7], p[8]), Wo = oracle_out_dim(p[4], p[6], p[7], p[8]);
        const int64_t ny = p[0] * p[2] * Ho * Wo;
        float *x = floats(p[0] * p[1] * p[3] * p[4], 1), *w = floats(p[2] * p[1] * p[5] * p[6], 2);
        double *y = malloc((size_t)ny * 8), *d = malloc((size_t)ny * 8);
        if (oracle_conv2d(x, w, y, d, p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7], p[8])) return 2;
        printf("conv2d %ld %ld %ld %ld %ld %ld %ld %ld %ld : %016llx\n", (long)p[0], (long)p[1], (long)p[2], (long)p[3], (long)p[4],
               (long)p[5], (long)p[6], (long)p[7], (long)p[8], (unsigned long long)fnv(fnv(FNV0, y, (size_t)ny * 8), d, (size_t)ny * 8));
        /* the same shapes through the int8 path and, with a dilation of 2, through the dilated one */
        int8_t *x8 = bytes(p[0] * p[1] * p[3] * p[4], 3), *w8 = bytes(p[2] * p[1] * p[5] * p[6], 4);
        int32_t *y32 = malloc((size_t)ny * 4);
        if (oracle_conv2d_s8(x8, w8, y32, p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7], p[8])) return 2;
        printf("conv2d_s8 %ld %ld %ld %ld %ld %ld %ld %ld %ld : %016llx\n", (long)p[0], (long)p[1], (long)p[2], (long)p[3], (long)p[4],
               (long)p[5], (long)p[6], (long)p[7], (long)p[8], (unsigned long long)fnv(FNV0, y32, (size_t)ny * 4));
        float *scale = floats(p[2], 5);
        for (int64_t i = 0; i < p[2]; ++i) scale[i] = 0.001f * (2.0f + scale[i]);
        int32_t *bias = malloc((size_t)p[2] * 4);
        for (int64_t i = 0; i < p[2]; ++i) bias[i] = (int32_t)(mix((uint64_t)i, 6) >> 18) - 8192;
        int8_t *q = malloc((size_t)ny);
        if (oracle_requant_s8(y32, bias, scale, q, p[0], p[2], Ho * Wo, (int)(c & 1))) return 2;
        printf("requant_s8 %ld %ld %ld %ld %ld %ld %ld %ld %ld %d : %016llx\n", (long)p[0], (long)p[1], (long)p[2], (long)p[3],
               (long)p[4], (long)p[5], (long)p[6], (long)p[7], (long)p[8], (int)(c & 1), (unsigned long long)fnv(FNV0, q, (size_t)ny));
        float *fb = floats(p[2], 7);
        if (oracle_bias_relu(y, d, fb, p[0], p[2], Ho * Wo, (int)(c & 1))) return 2;
        printf("bias_relu %ld %ld %ld %ld %ld %ld %ld %ld %ld %d : %016llx\n", (long)p[0], (long)p[1], (long)p[2], (long)p[3],
               (long)p[4], (long)p[5], (long)p[6], (long)p[7], (long)p[8], (int)(c & 1),
               (unsigned long long)fnv(fnv(FNV0, y, (size_t)ny * 8), d, (size_t)ny * 8));
        const int64_t Hd = oracle_out_dim_dilated(p[3], p[5], p[7], p[8] + 1, 2), Wd = oracle_out_dim_dilated(p[4], p[6], p[7], p[8] + 1, 2);
        if (Hd > 0 && Wd > 0) {
            const int64_t nd = p[0] * p[2] * Hd * Wd;
            double *yd = malloc((size_t)nd * 8), *dd = malloc((size_t)nd * 8);
            if (oracle_conv2d_dilated(x, w, yd, dd, p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7], p[8] + 1, 2, 0)) return 2;
            printf("conv2d_dilated %ld %ld %ld %ld %ld %ld %ld %ld %ld 2 : %016llx\n", (long)p[0], (long)p[1], (long)p[2], (long)p[3],
                   (long)p[4], (long)p[5], (long)p[6], (long)p[7], (long)(p[8] + 1),
                   (unsigned long long)fnv(fnv(FNV0, yd, (size_t)nd * 8), dd, (size_t)nd * 8));
            free(yd); free(dd);
        }
        free(x); free(w); free(y); free(d); free(x8); free(w8); free(y32); free(scale); free(bias); free(q); free(fb);
    }
    /* N, C, H, W, R, S, stride, pad: depthwise, and 2-D pooling in both modes (2 * pad <= min(R, S)) */
    static const int64_t dw[][8] = {{1, 1, 3, 3, 3, 3, 1, 0}, {2, 3, 7, 9, 3, 3, 1, 1}, {1, 4, 8, 6, 5, 2, 2, 1}, {1, 2, 9, 9, 7, 7, 1, 3},
                                    {3, 2, 6, 10, 2, 2, 2, 0}};
    for (size_t c = 0; c < sizeof dw / sizeof dw[0]; ++c) {
        const int64_t *p = dw[c], Ho = oracle_out_dim(p[2], p[4], p[6], p[7]), Wo = oracle_out_dim(p[3], p[5], p[6], p[7]);
        const int64_t ny = p[0] * p[1] * Ho * Wo;
        float *x = floats(p[0] * p[1] * p[2] * p[3], 8), *w = floats(p[1] * p[4] * p[5], 9);
        double *y = malloc((size_t)ny * 8), *d = malloc((size_t)ny * 8);
        if (oracle_conv2d_depthwise(x, w, y, d, p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7])) return 2;
        printf("depthwise %ld %ld %ld %ld %ld %ld %ld %ld : %016llx\n", (long)p[0], (long)p[1], (long)p[2], (long)p[3], (long)p[4],
               (long)p[5], (long)p[6], (long)p[7], (unsigned long long)fnv(fnv(FNV0, y, (size_t)ny * 8), d, (size_t)ny * 8));
        for (int mode = 0; mode < 2; ++mode) {
            if (oracle_pool2d(x, y, d, p[0] * p[1], p[2], p[3], p[4], p[5], p[6], p[7], mode)) return 2;
            printf("pool2d %ld %ld %ld %ld %ld %ld %ld %ld %d : %016llx\n", (long)p[0], (long)p[1], (long)p[2], (long)p[3], (long)p[4],
                   (long)p[5], (long)p[6], (long)p[7], mode, (unsigned long long)fnv(fnv(FNV0, y, (size_t)ny * 8), d, (size_t)ny * 8));
        }
        free(x); free(w); free(y); free(d);
    }
    /* rows, len, k, stride, pad */
    static const int64_t one_d[][5] = {{1, 9, 9, 1, 0}, {3, 40, 5, 1, 4}, {2, 33, 4, 3, 2}, {2, 64, 64, 1, 0}, {4, 17, 1, 2, 0}};
    for (size_t c = 0; c < sizeof one_d / sizeof one_d[0]; ++c) {
        const int64_t *p = one_d[c], Lo = oracle_out_dim(p[1], p[2], p[3], p[4]), ny = p[0] * Lo;
        float *x = floats(p[0] * p[1], 10), *w = floats(p[2], 11);
        double *y = malloc((size_t)ny * 8), *d = malloc((size_t)ny * 8);
        if (oracle_conv1d(x, w, y, d, p[0], p[1], p[2], p[3], p[4])) return 2;
        printf("conv1d %ld %ld %ld %ld %ld : %016llx\n", (long)p[0], (long)p[1], (long)p[2], (long)p[3], (long)p[4],
               (unsigned long long)fnv(fnv(FNV0, y, (size_t)ny * 8), d, (size_t)ny * 8));
        const int64_t Lp = oracle_out_dim(p[1], p[2], p[3], 0), np_ = p[0] * Lp;
        double *yp = malloc((size_t)np_ * 8), *dp = malloc((size_t)np_ * 8);
        for (int mode = 0; mode < 2; ++mode) {
            if (oracle_pool1d(x, yp, dp, p[0], p[1], p[2], p[3], mode)) return 2;
            printf("pool1d %ld %ld %ld %ld %d : %016llx\n", (long)p[0], (long)p[1], (long)p[2], (long)p[3], mode,
                   (unsigned long long)fnv(fnv(FNV0, yp, (size_t)np_ * 8), dp, (size_t)np_ * 8));
        }
        free(x); free(w); free(y); free(d); free(yp); free(dp);
    }
    printf("done\n");
    return 0;
}
