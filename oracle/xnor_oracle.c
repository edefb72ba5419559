/*
 * CPU oracle for the XNOR-Net forward binary convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path, and nothing in the product path may call it.
 *
 * What it evaluates (paper section 3.2 "Binary Convolution", the equation
 * I * W ~ (sign(I) (*) sign(W)) . K alpha):
 *   sign(v)  = +1 if v >= 0, -1 otherwise        (sec. 3.1, rule given with B* = sign(W))
 *   alpha_k  = (1/n) sum |W_k|, n = c*kh*kw      (sec. 3.1, optimal scaling factor)
 *   A        = (1/c) sum_c |I[c]|                (sec. 3.2, matrix A)
 *   K        = A conv k, k_ij = 1/(kh*kw)        (sec. 3.2, matrix K)
 *   dot      = sum over the window of sign(I)*sign(W)   (what XNOR+bitcount reaches)
 *   out      = dot * K * alpha
 *
 * The fast method (XNOR + bitcount) reaches exactly the integer that the plain
 * +-1 correlation defines, so the oracle is that definition written out: a
 * direct correlation over +-1 tensors with exact integer accumulation.  All
 * real-valued quantities are accumulated in double and rounded to float once.
 *
 * Readings of points on which the paper is silent:
 *   - padding: a padded position contributes 0 to the dot product and 0 to A;
 *   - the divisor of K is always kh*kw (the box filter has fixed taps 1/(kh*kw));
 *   - correlation, not flipped convolution; NCHW storage; K indexed [oy][ox];
 *   - A and K are per image, alpha is shared by the batch;
 *   - sign uses a comparison, so sign(-0.0f) = +1 and NaN -> -1;
 *   - batch normalisation (block order BatchNorm -> BinActiv -> BinConv) is the
 *     inference affine map y = fmaf(x, scale_c, shift_c) evaluated in float,
 *     because that float value decides the sign bit.
 *
 * Pins (tests/test_oracle_pins.py): brute-force least squares for alpha and B,
 * per-window beta = |X|_1/n against K, exhaustive +-1 dot vs bitcount identity,
 * all-ones input closed form, constant-magnitude special case against a library
 * float convolution, sign flip antisymmetry, parity/bound invariants, the FC =
 * whole-input-filter equivalence; for the later functions: xo_bwn against a library
 * float convolution with weights alpha*sign(W); xo_bingrad against autograd of a
 * library convolution and the adjoint identity with xo_dot; xo_qk_levels against the
 * formula in rational arithmetic and q_1 = sign; xo_kbit_dot against a library
 * convolution of the dequantised tensors.  Every function below is pinned by at least one.
 *
 * Build: gcc -O3 -fopenmp -ffp-contract=off -shared -fPIC
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

/* y = x*scale_c + shift_c in float with one rounding (fmaf); scale==NULL copies x.
 * Block order of sec. 3.2 "Training XNOR-Networks": normalise before binarising. */
void xo_batchnorm(const float *x, const float *scale, const float *shift, float *y,
                  int n, int c, int h, int w)
{
    const size_t hw = (size_t)h * w;
    for (int b = 0; b < n; ++b)
        for (int ch = 0; ch < c; ++ch) {
            const float *src = x + ((size_t)b * c + ch) * hw;
            float *dst = y + ((size_t)b * c + ch) * hw;
            for (size_t i = 0; i < hw; ++i)
                dst[i] = scale ? fmaf(src[i], scale[ch], shift[ch]) : src[i];
        }
}

/* sign of sec. 3.1: +1 when v >= 0, -1 when v < 0 (also applied to inputs). */
void xo_sign(const float *v, int8_t *s, size_t count)
{
    for (size_t i = 0; i < count; ++i)
        s[i] = (v[i] >= 0.0f) ? (int8_t)1 : (int8_t)-1;
}

/* alpha_k = ||W_k||_1 / n  (sec. 3.1, closed form of the optimal scale). */
void xo_alpha(const float *W, double *alpha, int k_out, int c, int kh, int kw)
{
    const size_t n = (size_t)c * kh * kw;
    for (int k = 0; k < k_out; ++k) {
        double s = 0.0;
        for (size_t i = 0; i < n; ++i)
            s += fabs((double)W[(size_t)k * n + i]);
        alpha[k] = s / (double)n;
    }
}

/* A[b][y][x] = (1/c) sum_ch |I[b][ch][y][x]|  (sec. 3.2). */
void xo_A(const float *I, double *A, int n, int c, int h, int w)
{
    const size_t hw = (size_t)h * w;
    for (int b = 0; b < n; ++b)
        for (size_t p = 0; p < hw; ++p) {
            double s = 0.0;
            for (int ch = 0; ch < c; ++ch)
                s += fabs((double)I[((size_t)b * c + ch) * hw + p]);
            A[(size_t)b * hw + p] = s / (double)c;
        }
}

/* K = A correlated with the constant filter 1/(kh*kw), evaluated at the output
 * positions of the convolution; out-of-range A counts as 0 (sec. 3.2). */
void xo_K(const double *A, double *K, int n, int h, int w, int kh, int kw,
          int stride_h, int stride_w, int pad_h, int pad_w)
{
    const int ho = (h + 2 * pad_h - kh) / stride_h + 1;
    const int wo = (w + 2 * pad_w - kw) / stride_w + 1;
    for (int b = 0; b < n; ++b)
        for (int oy = 0; oy < ho; ++oy)
            for (int ox = 0; ox < wo; ++ox) {
                double s = 0.0;
                for (int dy = 0; dy < kh; ++dy)
                    for (int dx = 0; dx < kw; ++dx) {
                        const int iy = oy * stride_h - pad_h + dy;
                        const int ix = ox * stride_w - pad_w + dx;
                        if (iy >= 0 && iy < h && ix >= 0 && ix < w)
                            s += A[((size_t)b * h + iy) * w + ix];
                    }
                K[((size_t)b * ho + oy) * wo + ox] = s / (double)(kh * kw);
            }
}

/* dot[b][k][oy][ox] = sum_{ch,dy,dx in bounds} sI[b][ch][iy][ix] * sW[k][ch][dy][dx]
 * over +-1 tensors: the value XNOR + bitcount computes (sec. 3.2).  Exact in int32. */
void xo_dot(const int8_t *sI, const int8_t *sW, int32_t *dot,
            int n, int c, int h, int w, int k_out, int kh, int kw,
            int stride_h, int stride_w, int pad_h, int pad_w)
{
    const int ho = (h + 2 * pad_h - kh) / stride_h + 1;
    const int wo = (w + 2 * pad_w - kw) / stride_w + 1;
    const long jobs = (long)n * k_out;
#pragma omp parallel for schedule(static)
    for (long job = 0; job < jobs; ++job) {
        const int b = (int)(job / k_out), k = (int)(job % k_out);
        int32_t *acc = dot + (size_t)job * ho * wo;
        for (int i = 0; i < ho * wo; ++i)
            acc[i] = 0;
        for (int ch = 0; ch < c; ++ch)
            for (int dy = 0; dy < kh; ++dy)
                for (int dx = 0; dx < kw; ++dx) {
                    const int32_t sw = sW[(((size_t)k * c + ch) * kh + dy) * kw + dx];
                    const int8_t *plane = sI + ((size_t)b * c + ch) * h * w;
                    for (int oy = 0; oy < ho; ++oy) {
                        const int iy = oy * stride_h - pad_h + dy;
                        if (iy < 0 || iy >= h)
                            continue;
                        for (int ox = 0; ox < wo; ++ox) {
                            const int ix = ox * stride_w - pad_w + dx;
                            if (ix < 0 || ix >= w)
                                continue;
                            acc[oy * wo + ox] += (int32_t)plane[(size_t)iy * w + ix] * sw;
                        }
                    }
                }
    }
}

/* out = (float)(dot * K * alpha), the right-hand side of the binary-convolution
 * equation; product formed in double, rounded once. */
void xo_scale(const int32_t *dot, const double *K, const double *alpha, float *out,
              int n, int k_out, int ho, int wo)
{
    const size_t px = (size_t)ho * wo;
    for (int b = 0; b < n; ++b)
        for (int k = 0; k < k_out; ++k)
            for (size_t p = 0; p < px; ++p) {
                const size_t o = ((size_t)b * k_out + k) * px + p;
                out[o] = (float)((double)dot[o] * K[(size_t)b * px + p] * alpha[k]);
            }
}

/* Binary-Weight-Network convolution (sec. 3.1, I * W ~ (I (+) B) alpha): real input, weights
 * alpha_k * sign(W_k).  out[b][k][oy][ox] = alpha_k * sum_{ch,dy,dx in bounds} I * sign(W): only
 * additions and subtractions of the inputs, accumulated in double, scaled and rounded once. */
void xo_bwn(const float *I, const int8_t *sW, const double *alpha, float *out,
            int n, int c, int h, int w, int k_out, int kh, int kw,
            int stride_h, int stride_w, int pad_h, int pad_w)
{
    const int ho = (h + 2 * pad_h - kh) / stride_h + 1;
    const int wo = (w + 2 * pad_w - kw) / stride_w + 1;
    const long jobs = (long)n * k_out;
#pragma omp parallel for schedule(static)
    for (long job = 0; job < jobs; ++job) {
        const int b = (int)(job / k_out), k = (int)(job % k_out);
        double *acc = (double *)malloc(sizeof(double) * (size_t)ho * wo);
        for (int i = 0; i < ho * wo; ++i)
            acc[i] = 0.0;
        for (int ch = 0; ch < c; ++ch)
            for (int dy = 0; dy < kh; ++dy)
                for (int dx = 0; dx < kw; ++dx) {
                    const int sw = sW[(((size_t)k * c + ch) * kh + dy) * kw + dx];
                    const float *plane = I + ((size_t)b * c + ch) * h * w;
                    for (int oy = 0; oy < ho; ++oy) {
                        const int iy = oy * stride_h - pad_h + dy;
                        if (iy < 0 || iy >= h)
                            continue;
                        for (int ox = 0; ox < wo; ++ox) {
                            const int ix = ox * stride_w - pad_w + dx;
                            if (ix < 0 || ix >= w)
                                continue;
                            const double v = (double)plane[(size_t)iy * w + ix];
                            acc[oy * wo + ox] += sw > 0 ? v : -v;      /* add or subtract, no multiply */
                        }
                    }
                }
        for (int i = 0; i < ho * wo; ++i)
            out[(size_t)job * ho * wo + i] = (float)(acc[i] * alpha[k]);
        free(acc);
    }
}

/* Binary gradient (sec. 3.2, paragraph "Binary Gradient"): in the backward pass the gradient
 * that meets the weight filters in a convolution is binarised like the forward input, with the
 * largest magnitude of the tensor as its scaling factor (not the mean of eq. alpha = |W|_1/n).
 * The forward layer is out = dot * K * alpha_k with dot = sign(I) (*) sign(W), so the gradient
 * that reaches the binary convolution is gd = g_out * alpha_k * K (two float multiplies in this
 * order: the float value decides the sign bit).  Readings: one scaling factor per image,
 * m_b = max |gd[b]|; sign(gd) by the comparison rule of sec. 3.1; K and alpha may be absent (= 1).
 * The data-gradient convolution is the transpose of the forward correlation, written out as
 * the scatter it is: every output position adds sign(gd) * sign(W) to the input positions its
 * window covered (padded positions receive nothing).  Exact integers; g_in = m_b * dot_t.
 *   sg [n][k][ho][wo] int8, gmax [n], dot_t [n][c][h][w] int32, gin [n][c][h][w] float. */
void xo_bingrad(const float *g, const float *K, const float *alpha, const int8_t *sW,
                int8_t *sg, float *gmax, int32_t *dot_t, float *gin,
                int n, int c, int h, int w, int k_out, int kh, int kw,
                int stride_h, int stride_w, int pad_h, int pad_w)
{
    const int ho = (h + 2 * pad_h - kh) / stride_h + 1;
    const int wo = (w + 2 * pad_w - kw) / stride_w + 1;
    const size_t plane = (size_t)ho * wo;
    for (int b = 0; b < n; ++b) {
        float m = 0.0f;
        for (int k = 0; k < k_out; ++k)
            for (size_t p = 0; p < plane; ++p) {
                const size_t i = ((size_t)b * k_out + k) * plane + p;
                float gd = g[i];
                if (alpha)
                    gd = gd * alpha[k];
                if (K)
                    gd = gd * K[(size_t)b * plane + p];
                sg[i] = gd >= 0.0f ? 1 : -1;
                if (fabsf(gd) > m)
                    m = fabsf(gd);
            }
        gmax[b] = m;
    }
    const long jobs = (long)n * c;
#pragma omp parallel for schedule(static)
    for (long job = 0; job < jobs; ++job) {
        const int b = (int)(job / c), ch = (int)(job % c);
        int32_t *dst = dot_t + (size_t)job * h * w;
        for (int i = 0; i < h * w; ++i)
            dst[i] = 0;
        for (int k = 0; k < k_out; ++k)
            for (int oy = 0; oy < ho; ++oy)
                for (int ox = 0; ox < wo; ++ox) {
                    const int s = sg[((size_t)b * k_out + k) * plane + (size_t)oy * wo + ox];
                    for (int dy = 0; dy < kh; ++dy) {
                        const int iy = oy * stride_h - pad_h + dy;
                        if (iy < 0 || iy >= h)
                            continue;
                        for (int dx = 0; dx < kw; ++dx) {
                            const int ix = ox * stride_w - pad_w + dx;
                            if (ix < 0 || ix >= w)
                                continue;
                            dst[iy * w + ix] += s * sW[(((size_t)k * c + ch) * kh + dy) * kw + dx];
                        }
                    }
                }
        for (int i = 0; i < h * w; ++i)
            gin[(size_t)job * h * w + i] = (float)((double)gmax[b] * (double)dst[i]);
    }
}

/* k-bit quantisation (sec. 3.2, paragraph "k-bit Quantization"): q_k(x) = 2*([(2^k - 1)(x+1)/2]/(2^k - 1) - 1/2)
 * for x in [-1, 1], in place of sign().  With L = 2^k - 1 the level index is u = [L*(x+1)/2] in 0..L and
 * q_k = (2u - L)/L: the odd integer a = 2u - L in [-L, L] over L.  Readings: inputs outside [-1, 1] are
 * clamped (NaN -> -1); [.] rounds halves up (u = floor(v + 1/2)), so that q_1 = sign with sign(0) = +1;
 * the level index is decided in float arithmetic in this order of operations, each rounded to float:
 * v = ((x + 1) * 0.5) * L + 0.5, u = floor(v), clamped to 0..L.  k in 1..8.
 * k = 1 is decided by the comparison x >= 0 instead: the formula evaluated exactly gives -1 for every
 * negative x, but in float x + 1 rounds to 1 for -2^-25 < x < 0 and would give +1; with the comparison
 * q_1 is the sign function of sec. 3.1 for every float. */
void xo_qk_levels(const float *x, int32_t *a, size_t count, int k)
{
    const int L = (1 << k) - 1;
    for (size_t i = 0; i < count; ++i) {
        float t = x[i];
        t = t >= -1.0f ? t : -1.0f;                 /* NaN -> -1 */
        t = t <= 1.0f ? t : 1.0f;
        const float h = (t + 1.0f) * 0.5f;
        const float v = h * (float)L + 0.5f;
        int u = (int)floorf(v);
        u = u < 0 ? 0 : (u > L ? L : u);
        if (k == 1) u = x[i] >= 0.0f ? 1 : 0;
        a[i] = 2 * u - L;
    }
}

/* Convolution of k-bit quantised inputs with k-bit quantised weights: the plain correlation of
 * q_ka(x) and q_kw(w), zero padding, evaluated exactly: num = sum a_x * a_w over the in-bounds window
 * (odd-integer numerators, 64-bit accumulation), out = num / (La * Lw).
 *   ax [n][c][h][w], aw [k_out][c][kh][kw] int32 numerators; num [n][k_out][ho][wo] int64. */
void xo_kbit_dot(const int32_t *ax, const int32_t *aw, int64_t *num,
                 int n, int c, int h, int w, int k_out, int kh, int kw,
                 int stride_h, int stride_w, int pad_h, int pad_w)
{
    const int ho = (h + 2 * pad_h - kh) / stride_h + 1;
    const int wo = (w + 2 * pad_w - kw) / stride_w + 1;
    const long jobs = (long)n * k_out;
#pragma omp parallel for schedule(static)
    for (long job = 0; job < jobs; ++job) {
        const int b = (int)(job / k_out), k = (int)(job % k_out);
        for (int oy = 0; oy < ho; ++oy)
            for (int ox = 0; ox < wo; ++ox) {
                int64_t s = 0;
                for (int ch = 0; ch < c; ++ch)
                    for (int dy = 0; dy < kh; ++dy) {
                        const int iy = oy * stride_h - pad_h + dy;
                        if (iy < 0 || iy >= h)
                            continue;
                        for (int dx = 0; dx < kw; ++dx) {
                            const int ix = ox * stride_w - pad_w + dx;
                            if (ix < 0 || ix >= w)
                                continue;
                            s += (int64_t)ax[(((size_t)b * c + ch) * h + iy) * w + ix] *
                                 (int64_t)aw[(((size_t)k * c + ch) * kh + dy) * kw + dx];
                        }
                    }
                num[((size_t)job * ho + oy) * wo + ox] = s;
            }
    }
}
