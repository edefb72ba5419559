// k-bit quantisation (sec. 3.2, paragraph "k-bit Quantization"): q_k(x) = 2*([(2^k - 1)(x + 1)/2]/(2^k - 1) - 1/2)
// in place of sign().  With L = 2^k - 1 and the level index u = [L (x + 1)/2] = sum_p 2^p u_p (bits u_p),
// q_k = (2u - L)/L = sum_p 2^p s_p / L with s_p = 2 u_p - 1 = +-1: a k-bit tensor is k weighted +-1 tensors.
// The convolution of a ka-bit input with kw-bit weights is therefore ka*kw binary convolutions, run as
// ONE launch of the binary kernel over ka*n "images" and kw*k_out "filters" (bit planes stacked along the
// batch and filter axes), followed by the weighted sum of the plane pairs.  Zero padding stays exact
// (every plane contributes 0 there).
#include "xnor_internal.h"
#include <algorithm>

namespace xnor {

__device__ __forceinline__ int qk_level(float x, int L)
{
    // u = floor(((x + 1) * 0.5) * L + 0.5), x clamped to [-1, 1] (NaN -> -1); each operation rounded to
    // float in this order (contraction is disabled for the build): the float value decides the level
    float t = x >= -1.0f ? x : -1.0f;
    t = t <= 1.0f ? t : 1.0f;
    const float v = ((t + 1.0f) * 0.5f) * (float)L + 0.5f;
    return min(max((int)__builtin_floorf(v), 0), L);
}

// x [n][c][hw] float -> planes [k][n][hw][cw] uint32: bit j of word wd of plane p = bit p of the level index
// of channel wd*32 + j.  Work split of the BinActiv kernel: one workgroup = 64 consecutive pixels of one
// image x all channels, lanes along pixels, the 4 waves share the channels in groups of 8 (one byte of a
// packed word per plane), words assembled in LDS ([plane][pixel][word]) and written as k contiguous runs.
template <int KB>
__global__ __launch_bounds__(256) void kbit_pack_kernel(const float *__restrict__ x, uint32_t *__restrict__ planes,
                                                        int n, int c, int hw, int cw, int tiles_per_image)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t wbytes[];      // [KB][64 px][cw words][4 bytes]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned b = blockIdx.x, win = (b >> 6) << 6;
    const int blk = (int)(win + 64u <= gridDim.x ? win + ((b & 7u) << 3) + ((b >> 3) & 7u) : b);
    const int img = blk / tiles_per_image;
    const int p0 = (blk - img * tiles_per_image) * 64;
    const int pc = min(p0 + lane, hw - 1);
    const float *xi = x + (size_t)img * c * hw + pc;
    const int groups = (c + 7) >> 3;
    constexpr int L = (1 << KB) - 1;
    const int plane_bytes = 64 * cw * 4;
#pragma unroll 2
    for (int gidx = wave; gidx < groups; gidx += 4) {
        const int ch0 = gidx * 8;
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = xi[(size_t)min(ch0 + j, c - 1) * hw];
        uint32_t byte[KB];
#pragma unroll
        for (int p = 0; p < KB; ++p) byte[p] = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int u = ch0 + j < c ? qk_level(v[j], L) : 0;
#pragma unroll
            for (int p = 0; p < KB; ++p) byte[p] |= ((uint32_t)(u >> p) & 1u) << j;
        }
#pragma unroll
        for (int p = 0; p < KB; ++p) wbytes[p * plane_bytes + (lane * cw) * 4 + gidx] = (uint8_t)byte[p];
    }
    __syncthreads();
    const int npx = min(64, hw - p0);
    const int nwords = npx * cw;
    const uint32_t tail_mask = 0xFFFFFFFFu >> (8 * (cw * 4 - groups));      // bytes of the last word no group wrote
#pragma unroll
    for (int p = 0; p < KB; ++p) {
        const uint32_t *wsrc = reinterpret_cast<const uint32_t *>(wbytes + p * plane_bytes);
        uint32_t *dst = planes + (((size_t)p * n + img) * hw + p0) * cw;
        for (int i = tid; i < nwords; i += 256) {
            uint32_t word = wsrc[i];
            if (i % cw == cw - 1) word &= tail_mask;
            dst[i] = word;
        }
    }
}

xnor_status launch_kbit_pack_input(const float *x, uint32_t *planes, int k, int n, int c, int hw, hipStream_t stream)
{
    const int cw = (c + 31) / 32;
    const int tiles = (hw + 63) / 64;
    const size_t lds = (size_t)k * 64 * cw * 4;
    if (lds > 64 * 1024 || (long long)n * tiles > 0x7fffffffLL) return XNOR_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)(n * tiles)), block(256);
#define XNOR_KB(B) case B: kbit_pack_kernel<B><<<grid, block, lds, stream>>>(x, planes, n, c, hw, cw, tiles); break
    switch (k) {
        XNOR_KB(1); XNOR_KB(2); XNOR_KB(3); XNOR_KB(4); XNOR_KB(5); XNOR_KB(6); XNOR_KB(7); XNOR_KB(8);
    default: return XNOR_ERR_UNSUPPORTED;
    }
#undef XNOR_KB
    return hip_status(hipGetLastError());
}

// dots [ka*n][kw*k_out][howo]: the +-1 dot products of the plane pairs as floats (exact integers below 2^24).
// num = sum_{p,q} 2^(p+q) dots[p*n + img][q*k_out + f], out = num / (La * Lw) with one rounding.
constexpr int COMBINE_PLANES = 4;
__global__ __launch_bounds__(256) void kbit_combine_kernel(const float *__restrict__ dots, float *__restrict__ out,
                                                           int32_t *__restrict__ num_out, int n, int k_out, int howo,
                                                           int ka, int kw, double scale, int fgroups)
{
    // one workgroup per image and group of 4 filters: no index divisions per element, and the loads of
    // the 4 output planes are independent (small planes would otherwise leave a wave one load deep)
    const int img = blockIdx.x / fgroups, f0 = (blockIdx.x - img * fgroups) * COMBINE_PLANES;
    const size_t kk = (size_t)kw * k_out;
    for (int pix = threadIdx.x; pix < howo; pix += 256) {
        int num[COMBINE_PLANES];                        // fits: the host checked La * Lw * c * taps < 2^31
#pragma unroll
        for (int u = 0; u < COMBINE_PLANES; ++u) num[u] = 0;
        for (int p = 0; p < ka; ++p)
            for (int q = 0; q < kw; ++q) {
                const float *src = dots + (((size_t)p * n + img) * kk + (size_t)q * k_out) * howo + pix;
#pragma unroll
                for (int u = 0; u < COMBINE_PLANES; ++u)
                    num[u] += (int)src[(size_t)min(f0 + u, k_out - 1) * howo] << (p + q);
            }
#pragma unroll
        for (int u = 0; u < COMBINE_PLANES; ++u)
            if (f0 + u < k_out) {
                const size_t o = ((size_t)img * k_out + f0 + u) * howo + pix;
                if (num_out) num_out[o] = num[u];
                out[o] = (float)((double)num[u] / scale);
            }
    }
}

xnor_status launch_kbit_combine(const float *dots, float *out, int32_t *num_out, int n, int k_out, int howo,
                                int ka, int kw, hipStream_t stream)
{
    const int fgroups = (k_out + COMBINE_PLANES - 1) / COMBINE_PLANES;
    if ((long long)n * fgroups > 0x7fffffffLL) return XNOR_ERR_UNSUPPORTED;
    const double scale = (double)((1 << ka) - 1) * (double)((1 << kw) - 1);
    kbit_combine_kernel<<<dim3((unsigned)(n * fgroups)), dim3(256), 0, stream>>>(dots, out, num_out, n, k_out, howo, ka,
                                                                                kw, scale, fgroups);
    return hip_status(hipGetLastError());
}

__global__ __launch_bounds__(256) void fill_ones_kernel(float *__restrict__ p, size_t count)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) p[i] = 1.0f;
}

xnor_status launch_fill_ones(float *p, size_t count, hipStream_t stream)
{
    const unsigned blocks = (unsigned)std::min<size_t>((count + 255) / 256, 4096);
    fill_ones_kernel<<<dim3(blocks), dim3(256), 0, stream>>>(p, count);
    return hip_status(hipGetLastError());
}

}  // namespace xnor
