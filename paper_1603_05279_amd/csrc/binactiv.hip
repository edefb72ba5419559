// BinActiv layer (sec. 3.2): sign(I) packed to bits, A = channel mean of |I|, K = box filter of A.
// Optional batch normalisation folded in front (block order BatchNorm -> BinActiv).
#include "xnor_internal.h"

namespace xnor {

// One workgroup = 64 consecutive pixels of one image x all channels.  Lanes run along the
// pixels (contiguous in NCHW, so every channel row is read as 256-byte coalesced segments);
// the 4 waves split the channel words.  Each lane builds its pixel's words bit by bit and
// accumulates |y| in float; the 4 partial sums per pixel meet in LDS in a fixed order.
template <bool WRITE_BITS, bool WRITE_A>
__global__ __launch_bounds__(256) void binactiv_kernel(
    const float *__restrict__ x, const float *__restrict__ bn_scale,
    const float *__restrict__ bn_shift, uint32_t *__restrict__ xbits, float *__restrict__ A,
    int c, int hw, int cw, int tiles_per_image)
{
    __shared__ float part[4][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int img = blockIdx.x / tiles_per_image;
    const int tile = blockIdx.x - img * tiles_per_image;
    const int p = tile * 64 + lane;
    const bool live = p < hw;
    const float *xi = x + (size_t)img * c * hw + (live ? p : 0);
    const bool bn = bn_scale != nullptr;
    float asum = 0.0f;
    for (int wd = wave; wd < cw; wd += 4) {
        const int ch0 = wd * 32;
        const int nch = min(32, c - ch0);
        uint32_t word = 0;
        if (nch == 32) {
#pragma unroll 16
            for (int j = 0; j < 32; ++j) {
                float v = live ? xi[(size_t)(ch0 + j) * hw] : 0.0f;
                if (bn) v = __builtin_fmaf(v, bn_scale[ch0 + j], bn_shift[ch0 + j]);
                word |= (v >= 0.0f ? 1u : 0u) << j;
                asum += __builtin_fabsf(v);
            }
        } else {
            for (int j = 0; j < nch; ++j) {
                float v = live ? xi[(size_t)(ch0 + j) * hw] : 0.0f;
                if (bn) v = __builtin_fmaf(v, bn_scale[ch0 + j], bn_shift[ch0 + j]);
                word |= (v >= 0.0f ? 1u : 0u) << j;
                asum += __builtin_fabsf(v);
            }
        }
        if (WRITE_BITS && live) xbits[((size_t)img * hw + p) * cw + wd] = word;
    }
    if (WRITE_A) {
        part[wave][lane] = asum;
        __syncthreads();
        if (wave == 0 && live) {
            const float s = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
            A[(size_t)img * hw + p] = s / (float)c;
        }
    }
}

xnor_status launch_binactiv(const float *x, const float *bn_scale, const float *bn_shift,
                            uint32_t *xbits, float *A, int n, int c, int hw, hipStream_t stream)
{
    const int cw = (c + 31) / 32;
    const int tiles = (hw + 63) / 64;
    const long long blocks = (long long)n * tiles;
    if (blocks > 0x7fffffffLL) return XNOR_ERR_SHAPE;
    dim3 grid((unsigned)blocks), block(256);
    if (xbits && A)
        binactiv_kernel<true, true><<<grid, block, 0, stream>>>(x, bn_scale, bn_shift, xbits, A, c, hw, cw, tiles);
    else if (xbits)
        binactiv_kernel<true, false><<<grid, block, 0, stream>>>(x, bn_scale, bn_shift, xbits, A, c, hw, cw, tiles);
    else
        binactiv_kernel<false, true><<<grid, block, 0, stream>>>(x, bn_scale, bn_shift, xbits, A, c, hw, cw, tiles);
    return hip_status(hipGetLastError());
}

// K[n][oy][ox] = (1/(kh*kw)) * sum over in-bounds taps of A (sec. 3.2).  One thread per output;
// A is 1/c of the input volume and stays in L2, taps are summed in row-major order.
__global__ __launch_bounds__(256) void boxfilter_kernel(const float *__restrict__ A,
                                                        float *__restrict__ K, ConvGeom g)
{
    const uint32_t m = blockIdx.x * 256u + threadIdx.x;
    if (m >= (uint32_t)g.m_total) return;
    const uint32_t img = g.div_howo.div(m);
    const uint32_t rem = m - img * (uint32_t)(g.ho * g.wo);
    const uint32_t oy = g.div_wo.div(rem);
    const uint32_t ox = rem - oy * (uint32_t)g.wo;
    const float *Ai = A + (size_t)img * g.h * g.w;
    float s = 0.0f;
    for (int dy = 0; dy < g.kh; ++dy) {
        const int iy = (int)oy * g.sh - g.ph + dy;
        if (iy < 0 || iy >= g.h) continue;
        for (int dx = 0; dx < g.kw; ++dx) {
            const int ix = (int)ox * g.sw - g.pw + dx;
            if (ix < 0 || ix >= g.w) continue;
            s += Ai[iy * g.w + ix];
        }
    }
    K[m] = s / (float)(g.kh * g.kw);
}

xnor_status launch_boxfilter(const float *A, float *K, const ConvGeom &g, hipStream_t stream)
{
    dim3 grid((unsigned)((g.m_total + 255) / 256)), block(256);
    boxfilter_kernel<<<grid, block, 0, stream>>>(A, K, g);
    return hip_status(hipGetLastError());
}

}  // namespace xnor
