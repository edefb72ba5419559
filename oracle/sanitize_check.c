/*
 * Host-side sanitizer run of the CPU oracle (test infrastructure only): every routine of xnor_oracle.c on small
 * shapes with padding, strides, even filters and channel counts around the word size, every buffer allocated
 * with exactly the size the routine's contract names, so that AddressSanitizer sees any access outside it and
 * UndefinedBehaviorSanitizer any overflow, bad shift or misaligned access.  Built and run by
 * tests/test_sanitizers.py:  gcc -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -fopenmp
 * -ffp-contract=off sanitize_check.c xnor_oracle.c -lm.  Prints "sanitize_check ok <checksum>" and returns 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void xo_batchnorm(const float *x, const float *scale, const float *shift, float *y, int n, int c, int h, int w);
void xo_sign(const float *v, int8_t *s, size_t count);
void xo_alpha(const float *W, double *alpha, int k_out, int c, int kh, int kw);
void xo_A(const float *I, double *A, int n, int c, int h, int w);
void xo_K(const double *A, double *K, int n, int h, int w, int kh, int kw, int stride_h, int stride_w, int pad_h,
          int pad_w);
void xo_dot(const int8_t *sI, const int8_t *sW, int32_t *dot, int n, int c, int h, int w, int k_out, int kh, int kw,
            int stride_h, int stride_w, int pad_h, int pad_w);
void xo_scale(const int32_t *dot, const double *K, const double *alpha, float *out, int n, int k_out, int ho, int wo);
void xo_bwn(const float *I, const int8_t *sW, const double *alpha, float *out, int n, int c, int h, int w, int k_out,
            int kh, int kw, int stride_h, int stride_w, int pad_h, int pad_w);
void xo_bingrad(const float *g, const float *K, const float *alpha, const int8_t *sW, int8_t *sg, float *gmax,
                int32_t *dot_t, float *gin, int n, int c, int h, int w, int k_out, int kh, int kw, int stride_h,
                int stride_w, int pad_h, int pad_w);
void xo_qk_levels(const float *x, int32_t *a, size_t count, int k);
void xo_kbit_dot(const int32_t *ax, const int32_t *aw, int64_t *num, int n, int c, int h, int w, int k_out, int kh,
                 int kw, int stride_h, int stride_w, int pad_h, int pad_w);

static uint32_t rng_state = 12345u;
static float frand(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return (float)((int32_t)(rng_state >> 8) % 2001 - 1000) / 500.0f;     /* [-2, 2], includes exact zeros */
}

static double run_case(int n, int c, int h, int w, int k, int kh, int kw, int sh, int sw, int ph, int pw)
{
    const int ho = (h + 2 * ph - kh) / sh + 1, wo = (w + 2 * pw - kw) / sw + 1;
    const size_t xin = (size_t)n * c * h * w, wn = (size_t)k * c * kh * kw, on = (size_t)n * k * ho * wo;
    float *x = malloc(xin * sizeof(float)), *y = malloc(xin * sizeof(float)), *W = malloc(wn * sizeof(float));
    float *scale = malloc(c * sizeof(float)), *shift = malloc(c * sizeof(float));
    int8_t *sI = malloc(xin), *sW = malloc(wn), *sg = malloc(on);
    double *alpha = malloc(k * sizeof(double)), *A = malloc((size_t)n * h * w * sizeof(double));
    double *K = malloc((size_t)n * ho * wo * sizeof(double));
    int32_t *dot = malloc(on * sizeof(int32_t)), *dot_t = malloc(xin * sizeof(int32_t));
    float *out = malloc(on * sizeof(float)), *g = malloc(on * sizeof(float)), *gin = malloc(xin * sizeof(float));
    float *Kf = malloc((size_t)n * ho * wo * sizeof(float)), *af = malloc(k * sizeof(float)), *gmax = malloc(n * sizeof(float));
    int32_t *ax = malloc(xin * sizeof(int32_t)), *aw = malloc(wn * sizeof(int32_t));
    int64_t *num = malloc(on * sizeof(int64_t));
    for (size_t i = 0; i < xin; ++i) x[i] = frand();
    for (size_t i = 0; i < wn; ++i) W[i] = frand() * 0.05f;
    for (int i = 0; i < c; ++i) { scale[i] = 1.0f + 0.25f * frand(); shift[i] = 0.1f * frand(); }
    for (size_t i = 0; i < on; ++i) g[i] = frand();
    xo_batchnorm(x, scale, shift, y, n, c, h, w);
    xo_batchnorm(x, NULL, NULL, y, n, c, h, w);
    xo_sign(y, sI, xin);
    xo_sign(W, sW, wn);
    xo_alpha(W, alpha, k, c, kh, kw);
    xo_A(y, A, n, c, h, w);
    xo_K(A, K, n, h, w, kh, kw, sh, sw, ph, pw);
    xo_dot(sI, sW, dot, n, c, h, w, k, kh, kw, sh, sw, ph, pw);
    xo_scale(dot, K, alpha, out, n, k, ho, wo);
    xo_bwn(y, sW, alpha, out, n, c, h, w, k, kh, kw, sh, sw, ph, pw);
    for (size_t i = 0; i < (size_t)n * ho * wo; ++i) Kf[i] = (float)K[i];
    for (int i = 0; i < k; ++i) af[i] = (float)alpha[i];
    xo_bingrad(g, Kf, af, sW, sg, gmax, dot_t, gin, n, c, h, w, k, kh, kw, sh, sw, ph, pw);
    xo_bingrad(g, NULL, NULL, sW, sg, gmax, dot_t, gin, n, c, h, w, k, kh, kw, sh, sw, ph, pw);
    double sum = 0.0;
    for (int bits = 1; bits <= 8; bits += 3) {
        xo_qk_levels(x, ax, xin, bits);
        xo_qk_levels(W, aw, wn, bits);
        xo_kbit_dot(ax, aw, num, n, c, h, w, k, kh, kw, sh, sw, ph, pw);
        for (size_t i = 0; i < on; ++i) sum += (double)num[i];
    }
    for (size_t i = 0; i < on; ++i) sum += out[i] + dot[i];
    for (size_t i = 0; i < xin; ++i) sum += gin[i] + dot_t[i];
    free(x); free(y); free(W); free(scale); free(shift); free(sI); free(sW); free(sg); free(alpha); free(A); free(K);
    free(dot); free(dot_t); free(out); free(g); free(gin); free(Kf); free(af); free(gmax); free(ax); free(aw); free(num);
    return sum;
}

int main(void)
{
    double s = 0.0;
    /*            n  c   h   w   k  kh kw sh sw ph pw */
    s += run_case(1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0);
    s += run_case(2, 3, 5, 7, 2, 3, 3, 1, 1, 1, 1);
    s += run_case(2, 31, 9, 8, 5, 3, 2, 1, 1, 1, 0);
    s += run_case(3, 33, 11, 13, 33, 3, 3, 2, 2, 1, 1);
    s += run_case(1, 64, 14, 14, 64, 3, 3, 1, 1, 1, 1);
    s += run_case(2, 40, 12, 10, 9, 4, 2, 2, 1, 1, 1);
    s += run_case(1, 8, 20, 3, 4, 5, 3, 1, 1, 2, 1);
    s += run_case(2, 96, 9, 9, 7, 5, 5, 1, 1, 2, 2);
    printf("sanitize_check ok %.6e\n", s);
    return isnan(s) ? 1 : 0;
}
