// Internal declarations shared by the translation units of libxnor (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "xnor.h"

namespace xnor {

// Exact unsigned division by a run-time constant: q = floor(x / d) for x*d < 2^32.
struct FastDiv {
    uint32_t magic;  // floor(2^32 / d) + 1, unused when d == 1
    uint32_t d;
    __host__ static FastDiv make(uint32_t d) {
        FastDiv f;
        f.d = d;
        f.magic = (d <= 1) ? 0u : (uint32_t)((0x100000000ull / d) + 1ull);
        return f;
    }
    __device__ __forceinline__ uint32_t div(uint32_t x) const {
        return d == 1 ? x : __umulhi(x, magic);
    }
};

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
};

inline xnor_status hip_status(hipError_t e) { return e == hipSuccess ? XNOR_OK : XNOR_ERR_HIP; }

// kernels' host launchers (each returns an xnor_status, enqueues on `stream`, never synchronises)
xnor_status launch_binactiv(const float *x, const float *bn_scale, const float *bn_shift,
                            uint32_t *xbits, float *A, int n, int c, int hw, hipStream_t stream);
xnor_status launch_boxfilter(const float *A, float *K, const ConvGeom &g, hipStream_t stream);
xnor_status launch_pack_weights(const float *w, uint32_t *wbits, float *alpha, void *wmfma,
                                int k_out, int c, int taps, hipStream_t stream);
xnor_status launch_conv_popcount(const uint32_t *xbits, const uint32_t *wbits, const float *K,
                                 const float *alpha, float *out, int32_t *dot_out,
                                 const ConvGeom &g, hipStream_t stream);
// fmt 0: int8 operands, fmt 1: 4-bit float operands (both images live in the wmfma buffer)
xnor_status launch_conv_mfma(int fmt, const uint32_t *xbits, const void *wmfma, const float *K,
                             const float *alpha, float *out, int32_t *dot_out,
                             const ConvGeom &g, hipStream_t stream);
void set_mfma_tuning(int tile, int lds_budget);

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

}  // namespace xnor
