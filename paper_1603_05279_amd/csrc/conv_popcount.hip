// Binary convolution on the vector ALU (sec. 3.2): dot = n_valid - 2*bitcount(x XOR w), then the
// fused scaling by K and alpha.
//
// Lanes run along output pixels; a wave shares one filter group, so every weight word is
// wave-uniform and is fetched through the scalar path (it reaches the XOR as a scalar operand),
// while each lane holds the words of its own pixel for the current tap.  Out-of-bounds taps are
// skipped per lane, which is exactly "padding contributes 0".
#include "xnor_internal.h"

namespace xnor {

template <int F, int CH>   // F filters per thread, CH channel words per inner chunk (divides cw)
__global__ __launch_bounds__(256) void conv_popcount_kernel(
    const uint32_t *__restrict__ xbits, const uint32_t *__restrict__ wbits,
    const float *__restrict__ K, const float *__restrict__ A, const float *__restrict__ alpha,
    float *__restrict__ out, int32_t *__restrict__ dot_out, ConvGeom g)
{
    const uint32_t m = blockIdx.x * 256u + threadIdx.x;
    const bool live = m < (uint32_t)g.m_total;
    const uint32_t mm = live ? m : (uint32_t)g.m_total - 1u;
    const uint32_t img = g.div_howo.div(mm);
    const uint32_t pix = mm - img * (uint32_t)(g.ho * g.wo);
    const uint32_t oy = g.div_wo.div(pix);
    const uint32_t ox = pix - oy * (uint32_t)g.wo;
    const int k0 = blockIdx.y * F;

    uint32_t acc[F];
#pragma unroll
    for (int f = 0; f < F; ++f) acc[f] = 0;
    int valid_taps = 0;

    for (int dy = 0; dy < g.kh; ++dy) {
        const int iy = (int)oy * g.sh - g.ph + dy;
        for (int dx = 0; dx < g.kw; ++dx) {
            const int ix = (int)ox * g.sw - g.pw + dx;
            const bool ok = live && iy >= 0 && iy < g.h && ix >= 0 && ix < g.w;
            if (!ok) continue;
            ++valid_taps;
            const int t = dy * g.kw + dx;
            const uint32_t *xp = xbits + (((size_t)img * g.h + iy) * g.w + ix) * g.cw;
            for (int w0 = 0; w0 < g.cw; w0 += CH) {
                uint32_t a[CH];
#pragma unroll
                for (int i = 0; i < CH; ++i) a[i] = xp[w0 + i];
#pragma unroll
                for (int f = 0; f < F; ++f) {
                    const int k = min(k0 + f, g.k_out - 1);
                    const uint32_t *wp = wbits + ((size_t)k * g.taps + t) * g.cw + w0;
#pragma unroll
                    for (int i = 0; i < CH; ++i) acc[f] += __builtin_popcount(a[i] ^ wp[i]);
                }
            }
        }
    }
    if (!live) return;
    const int n_valid = g.c * valid_taps;
    const float Km = K ? K[m] : box_K(A, g, m);
    const size_t plane = (size_t)g.ho * g.wo;
#pragma unroll
    for (int f = 0; f < F; ++f) {
        const int k = k0 + f;
        if (k < g.k_out) {
            const int dot = n_valid - 2 * (int)acc[f];
            const size_t o = ((size_t)img * g.k_out + k) * plane + pix;
            out[o] = (float)dot * Km * alpha[k];
            if (dot_out) dot_out[o] = dot;
        }
    }
}

// Same loop over weights in scalar-path order: for one (tap, channel word) the 32 filters' words are
// one aligned 128-byte run, fetched with wide scalar loads that overlap the vector work, instead of
// one dependent scalar load per filter.
template <int CH>   // channel words per inner chunk (divides cw)
__global__ __launch_bounds__(256) void conv_popcount_t_kernel(
    const uint32_t *__restrict__ xbits, const uint32_t *__restrict__ wpop,
    const float *__restrict__ K, const float *__restrict__ A, const float *__restrict__ alpha,
    float *__restrict__ out, int32_t *__restrict__ dot_out, ConvGeom g)
{
    constexpr int F = 32;
    const uint32_t m = blockIdx.x * 256u + threadIdx.x;
    const bool live = m < (uint32_t)g.m_total;
    const uint32_t mm = live ? m : (uint32_t)g.m_total - 1u;
    const uint32_t img = g.div_howo.div(mm);
    const uint32_t pix = mm - img * (uint32_t)(g.ho * g.wo);
    const uint32_t oy = g.div_wo.div(pix);
    const uint32_t ox = pix - oy * (uint32_t)g.wo;
    const int kb = blockIdx.y;
    const uint32_t *wblk = wpop + (size_t)kb * g.taps * g.cw * 32;

    uint32_t acc[F];
#pragma unroll
    for (int f = 0; f < F; ++f) acc[f] = 0;
    int valid_taps = 0;
    for (int dy = 0; dy < g.kh; ++dy) {
        const int iy = (int)oy * g.sh - g.ph + dy;
        for (int dx = 0; dx < g.kw; ++dx) {
            const int ix = (int)ox * g.sw - g.pw + dx;
            const bool ok = live && iy >= 0 && iy < g.h && ix >= 0 && ix < g.w;
            if (!ok) continue;
            ++valid_taps;
            const int t = dy * g.kw + dx;
            const uint32_t *xp = xbits + (((size_t)img * g.h + iy) * g.w + ix) * g.cw;
            const uint32_t *wt = wblk + (size_t)t * g.cw * 32;
            for (int w0 = 0; w0 < g.cw; w0 += CH) {
                uint32_t a[CH];
#pragma unroll
                for (int i = 0; i < CH; ++i) a[i] = xp[w0 + i];
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    const uint32_t *wr = wt + (size_t)(w0 + i) * 32;
#pragma unroll
                    for (int f = 0; f < F; ++f) acc[f] += __builtin_popcount(a[i] ^ wr[f]);
                }
            }
        }
    }
    if (!live) return;
    const int n_valid = g.c * valid_taps;
    const float Km = K ? K[m] : box_K(A, g, m);
    const size_t plane = (size_t)g.ho * g.wo;
#pragma unroll
    for (int f = 0; f < F; ++f) {
        const int k = kb * F + f;
        if (k < g.k_out) {
            const int dot = n_valid - 2 * (int)acc[f];
            const size_t o = ((size_t)img * g.k_out + k) * plane + pix;
            out[o] = (float)dot * Km * alpha[k];
            if (dot_out) dot_out[o] = dot;
        }
    }
}

template <int F>
static xnor_status launch_f(const uint32_t *xbits, const uint32_t *wbits, const float *K, const float *A,
                            const float *alpha, float *out, int32_t *dot_out, const ConvGeom &g,
                            hipStream_t stream)
{
    dim3 grid((unsigned)((g.m_total + 255) / 256), (unsigned)((g.k_out + F - 1) / F)), block(256);
    if (grid.y > 65535u) return XNOR_ERR_UNSUPPORTED;
#define XNOR_GO(CH) conv_popcount_kernel<F, CH><<<grid, block, 0, stream>>>(xbits, wbits, K, A, alpha, out, dot_out, g)
    if (g.cw % 8 == 0) XNOR_GO(8);
    else if (g.cw % 4 == 0) XNOR_GO(4);
    else if (g.cw % 3 == 0) XNOR_GO(3);
    else if (g.cw % 2 == 0) XNOR_GO(2);
    else XNOR_GO(1);
#undef XNOR_GO
    return hip_status(hipGetLastError());
}

xnor_status launch_conv_popcount(const uint32_t *xbits, const uint32_t *wbits, const void *wmfma, const float *K,
                                 const float *A, const float *alpha, float *out, int32_t *dot_out,
                                 const ConvGeom &g, hipStream_t stream)
{
    if (wmfma) {
        const uint32_t *wpop = reinterpret_cast<const uint32_t *>(
            static_cast<const uint8_t *>(wmfma) + wimg_i8_bytes(g.k_out, g.c, g.taps) + wimg_f4_bytes(g.k_out, g.c, g.taps));
        dim3 grid((unsigned)((g.m_total + 255) / 256), (unsigned)g.fblocks), block(256);
        if (grid.y > 65535u) return XNOR_ERR_UNSUPPORTED;
#define XNOR_GO(CH) conv_popcount_t_kernel<CH><<<grid, block, 0, stream>>>(xbits, wpop, K, A, alpha, out, dot_out, g)
        if (g.cw % 2 == 0) XNOR_GO(2);
        else XNOR_GO(1);
#undef XNOR_GO
        return hip_status(hipGetLastError());
    }
    return launch_f<32>(xbits, wbits, K, A, alpha, out, dot_out, g, stream);
}

}  // namespace xnor
