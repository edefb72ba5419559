// Internal declarations shared by the translation units of libxnor (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "xnor.h"
#include "xnor_tuning.h"
#include "fastdiv.h"

namespace xnor {

// Geometry handed to the convolution kernels (derived from xnor_conv_desc on the host).
struct ConvGeom {
    int n, c, h, w, k_out, kh, kw, sh, sw, ph, pw;
    int ho, wo;        // output extent
    int cw;            // words per pixel
    int taps;          // kh*kw
    int hp, wp;        // padded input extent h+2ph, w+2pw
    int m_total;       // n*ho*wo output pixels
    int fblocks;       // ceil(k_out/32) filter blocks in the matrix-core weight image
    FastDiv div_wo, div_howo, div_kw;
    // Input dilation (transposed convolutions of strided layers): the h x w input above is a virtual image
    // whose pixel (y, x) is pixel (y / dil_h, x / dil_w) of the real real_h x real_w tensor when both
    // divisions are exact and in range, and zero otherwise.  1 / h / w for ordinary convolutions.
    int dil_h, dil_w, real_h, real_w;
    FastDiv div_dil_h, div_dil_w;
};

// K of output pixel m (flattened image, row, column): the in-bounds taps of A summed in row-major
// order, divided by kh*kw (sec. 3.2).  Shared by the stand-alone box filter and by the convolution
// kernels when they derive K from A themselves, so both give identical bits.
__device__ __forceinline__ float box_K(const float *__restrict__ A, const ConvGeom &g, uint32_t m)
{
    const uint32_t img = g.div_howo.div(m);
    const uint32_t rem = m - img * (uint32_t)(g.ho * g.wo);
    const uint32_t oy = g.div_wo.div(rem);
    const uint32_t ox = rem - oy * (uint32_t)g.wo;
    const float *Ai = A + (size_t)img * g.h * g.w;
    // Taps are walked in row-major order, four columns at a time with their loads issued
    // together.  An out-of-range tap loads a clamped address and adds +0.0f, which leaves the
    // sum (>= +0) bit for bit as if it were skipped.
    const int iy0 = (int)oy * g.sh - g.ph, ix0 = (int)ox * g.sw - g.pw;
    float s = 0.0f;
    for (int dy = 0; dy < g.kh; ++dy) {
        const int iy = iy0 + dy;
        const bool oky = (uint32_t)iy < (uint32_t)g.h;
        const float *row = Ai + min(max(iy, 0), g.h - 1) * g.w;
        for (int dx0 = 0; dx0 < g.kw; dx0 += 4) {
            float a[4];
            bool ok[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int ix = ix0 + dx0 + u;
                ok[u] = oky && dx0 + u < g.kw && (uint32_t)ix < (uint32_t)g.w;
                a[u] = row[min(max(ix, 0), g.w - 1)];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) s += ok[u] ? a[u] : 0.0f;
        }
    }
    return s / (float)(g.kh * g.kw);
}

inline xnor_status hip_status(hipError_t e) { return e == hipSuccess ? XNOR_OK : XNOR_ERR_HIP; }

// kernels' host launchers (each returns an xnor_status, enqueues on `stream`, never synchronises)
// streamed != 0: the caller states that x is in no cache (read with the non-temporal hint whatever its size)
xnor_status launch_binactiv(const float *x, const float *bn_scale, const float *bn_shift,
                            uint32_t *xbits, float *A, int n, int c, int hw, hipStream_t stream, int streamed = 0);
// the same layer with a max-pool (and optional ReLU) applied to x on load; xbits / A are pooled-size
xnor_status launch_pool_binactiv(const float *x, const float *bn_scale, const float *bn_shift,
                                 uint32_t *xbits, float *A, int n, int c, int h, int w, int ph, int pw,
                                 int sh, int sw, int pad_h, int pad_w, int relu, hipStream_t stream);
xnor_status launch_boxfilter(const float *A, float *K, const ConvGeom &g, hipStream_t stream);
xnor_status launch_pack_weights(const float *w, uint32_t *wbits, float *alpha, void *wmfma,
                                int k_out, int c, int taps, hipStream_t stream, int mode = 0, int aux = 1,
                                float alpha_fill = 1.0f);
// (mode 0: sign(W) and alpha; 1: transposed, rotated filters of the backward convolution; 3: int8 level
// numerators of the aux-bit quantised weights, int8 image only, alpha = alpha_fill)
// k-bit quantisation (kbit.hip): int8 level numerators of q_k(x), [n][hw][Cw][32] (channels innermost)
xnor_status launch_kbit_pack_input(const float *x, int8_t *xq, int k, int n, int c, int hw, hipStream_t stream);
// Binary gradient (bingrad.hip): sign words of gd = g * alpha_k * K over the filters + per-image max |gd|;
// a plane [n][hw] filled with each image's maximum
xnor_status launch_bingrad_binarize(const float *g, const float *K, const float *alpha, uint32_t *gbits,
                                    float *gmax, int n, int k_out, int hw, hipStream_t stream);
xnor_status launch_bingrad_scale_plane(const float *gmax, float *plane, int n, int hw, hipStream_t stream);
// K may be NULL in the convolution launchers: the kernels then compute it from A on the fly.
// wmfma may be NULL (then the canonical wbits order is used, at a lower rate)
xnor_status launch_conv_popcount(const uint32_t *xbits, const uint32_t *wbits, const void *wmfma, const float *K, const float *A,
                                 const float *alpha, float *out, int32_t *dot_out,
                                 const ConvGeom &g, hipStream_t stream);
// Third image of the wmfma buffer (after the int8 and 4-bit images): the packed weight words in
// scalar-path order, [filter block of 32][tap][channel word][32 filters], so that the 32 words a
// wave needs for one (tap, channel word) are one aligned 128-byte scalar load.
__host__ __device__ inline size_t wimg_pop_bytes(int k_out, int c, int taps)
{
    return (size_t)((k_out + 31) / 32) * (size_t)taps * (size_t)((c + 31) / 32) * 128u;
}

// Next block's BatchNorm + BinActiv applied in the convolution's epilogue (block order of sec. 3.2):
// z = fmaf(y, bn_scale[k], bn_shift[k]) (z = y without normalisation), sign bits of z packed over the
// filters into xbits_next[pixel][ceil(k_out/32)], A_next[pixel] = sum_k |z| / k_out.  A workgroup sums
// |z| over its own filters; when the filters span several workgroups the partial sums go to
// `workspace` ([filter tile][pixel]) and a second small kernel adds them in order.
struct FuseArgs {
    const float *bn_scale, *bn_shift;   // per filter, both NULL or both set
    uint32_t *xbits_next;
    float *A_next;
    float *workspace;                   // >= ceil(k_out/32) * m_total floats
};

// fmt 0: int8 operands, fmt 1: 4-bit float operands (both images live in the wmfma buffer).
// fz != NULL selects the fused epilogue above; `out` may then be NULL.
xnor_status launch_conv_mfma(int fmt, const uint32_t *xbits, const void *wmfma, const float *K, const float *A,
                             const float *alpha, float *out, int32_t *dot_out,
                             const ConvGeom &g, hipStream_t stream, const FuseArgs *fz = nullptr);
// the same convolution (4-bit operands) with max-pooling (window ph x pw, stride sh x sw, no padding, optional
// ReLU first) applied in the epilogue: out_pool [n][k_out][hpo][wpo], the unpooled tensor is never written
xnor_status launch_conv_mfma_pool(const uint32_t *xbits, const void *wmfma, const float *K, const float *A,
                                  const float *alpha, float *out_pool, const ConvGeom &g, int ph, int pw, int sh,
                                  int sw, int relu, hipStream_t stream);
void set_mfma_tuning(int tile, int lds_budget);
// Binary-Weight-Network preparation kernels (bwn.hip); the convolution itself is launch_conv_mfma with fmt 2
xnor_status launch_bwn_split(const float *x, void *parts, int n, int c, int hw, hipStream_t stream);
xnor_status launch_bwn_pack(const float *w, float *alpha, void *wimg, int k_out, int c, int taps, hipStream_t stream);
// Sizes of the two matrix-core weight images (int8 first, 4-bit float second), 1 KiB records;
// each image ends with one all-zero record that padded K-steps multiply by.
__host__ __device__ inline size_t wimg_i8_bytes(int k_out, int c, int taps)
{
    return ((size_t)((k_out + 31) / 32) * (size_t)taps * (size_t)((c + 31) / 32) + 1) * 1024u;
}
__host__ __device__ inline size_t wimg_f4_bytes(int k_out, int c, int taps)
{
    return ((size_t)((k_out + 31) / 32) * (((size_t)taps * (size_t)((c + 31) / 32) + 1) / 2) + 1) * 1024u;
}
// Binary-Weight-Network image: one +-1 bfloat16 record per filter block, tap and 16-channel group
// (groups = ceil(c/16)), plus the trailing all-zero record
__host__ __device__ inline size_t wimg_bf16_bytes(int k_out, int groups, int taps)
{
    return ((size_t)((k_out + 31) / 32) * (size_t)taps * (size_t)groups + 1) * 1024u;
}

}  // namespace xnor
