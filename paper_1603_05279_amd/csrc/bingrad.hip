// Binary gradient (sec. 3.2, paragraph "Binary Gradient"): the gradient that meets the weight filters in
// the backward convolution is binarised like the forward input, with the largest magnitude of the tensor
// as its scaling factor.  The forward layer is out = dot * K * alpha_k, so that gradient is
// gd = (g_out * alpha_k) * K; this file produces its sign words (packed over the filters, the channel
// axis of the backward convolution) and max |gd| per image.  The convolution itself is the forward
// kernel run on the transposed, 180-degree-rotated filters (pack_weights.hip, TRANSPOSED).
#include "xnor_internal.h"
#include <algorithm>

namespace xnor {

// Same work split as the forward BinActiv kernel: one workgroup = 64 consecutive pixels of one image x
// all filters, lanes along the pixels (contiguous in NCHW), the 4 waves share the filters in groups of 8
// (one byte of a packed word), words assembled in LDS and written as one contiguous run.  The maximum
// is reduced over the wave by lane exchanges, over the waves in LDS, and merged into gmax[image] with an
// integer atomic maximum on the float's bit pattern (|gd| >= 0, so the patterns order like the values;
// the result does not depend on the order of arrival; NaN magnitudes are ignored).
template <bool HAS_ALPHA, bool HAS_K>
__global__ __launch_bounds__(256) void bingrad_binarize_kernel(
    const float *__restrict__ g, const float *__restrict__ K, const float *__restrict__ alpha,
    uint32_t *__restrict__ gbits, float *__restrict__ gmax, int c, int hw, int cw, int tiles_per_image)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    float *wmax = reinterpret_cast<float *>(smem);                      // [4]
    uint8_t *wbytes = smem + 16;                                        // [64 px][cw words][4 bytes]
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    // workgroups go to the 8 XCDs round-robin; within every complete window of 64 tiles each XCD takes a
    // run of 8 consecutive ones, so the cache lines that straddle tile boundaries hit in its own L2
    const unsigned b = blockIdx.x, win = (b >> 6) << 6;
    const int blk = (int)(win + 64u <= gridDim.x ? win + ((b & 7u) << 3) + ((b >> 3) & 7u) : b);
    const int img = blk / tiles_per_image;
    const int tile = blk - img * tiles_per_image;
    const int p0 = tile * 64, p = p0 + lane;
    const bool live = p < hw;
    const int pc = live ? p : hw - 1;
    const float *gi = g + (size_t)img * c * hw + pc;
    const float kp = HAS_K ? K[(size_t)img * hw + pc] : 1.0f;
    const int groups = (c + 7) >> 3;
    float m = 0.0f;
#pragma unroll 4
    for (int gidx = wave; gidx < groups; gidx += 4) {
        const int ch0 = gidx * 8;
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = gi[(size_t)min(ch0 + j, c - 1) * hw];
        uint32_t byte = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int ch = min(ch0 + j, c - 1);
            float gd = v[j];
            if (HAS_ALPHA) gd = gd * alpha[ch];
            if (HAS_K) gd = gd * kp;
            const bool ok = ch0 + j < c && live;
            byte |= ((ok && gd >= 0.0f) ? 1u : 0u) << j;
            const float a = __builtin_fabsf(gd);
            m = (ok && a > m) ? a : m;
        }
        wbytes[(lane * cw) * 4 + gidx] = (uint8_t)byte;
    }
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) {
        const float o = __shfl_xor(m, s, 64);
        m = o > m ? o : m;
    }
    if (lane == 0) wmax[wave] = m;
    __syncthreads();
    if (tid == 0) {
        float t = wmax[0];
#pragma unroll
        for (int q = 1; q < 4; ++q) t = wmax[q] > t ? wmax[q] : t;
        atomicMax(reinterpret_cast<unsigned int *>(gmax + img), __float_as_uint(t));
    }
    const int npx = min(64, hw - p0);
    const uint32_t *wsrc = reinterpret_cast<const uint32_t *>(wbytes);
    uint32_t *dst = gbits + ((size_t)img * hw + p0) * cw;
    const int nwords = npx * cw;
    const int tail_bytes = cw * 4 - groups;          // bytes of the last word no group wrote
    const uint32_t tail_mask = 0xFFFFFFFFu >> (8 * tail_bytes);
    for (int i = tid; i < nwords; i += 256) {
        uint32_t word = wsrc[i];
        if (i % cw == cw - 1) word &= tail_mask;
        dst[i] = word;
    }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float *__restrict__ p, int count)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = 0.0f;
}

__global__ __launch_bounds__(256) void bingrad_plane_kernel(const float *__restrict__ gmax,
                                                            float *__restrict__ plane, int hw)
{
    const float m = gmax[blockIdx.y];
    for (int i = blockIdx.x * 256 + threadIdx.x; i < hw; i += gridDim.x * 256)
        plane[(size_t)blockIdx.y * hw + i] = m;
}

xnor_status launch_bingrad_binarize(const float *g, const float *K, const float *alpha, uint32_t *gbits,
                                    float *gmax, int n, int k_out, int hw, hipStream_t stream)
{
    const int cw = (k_out + 31) / 32;
    const int tiles = (hw + 63) / 64;
    const size_t lds = 16 + (size_t)64 * cw * 4;
    if (lds > 64 * 1024 || (long long)n * tiles > 0x7fffffffLL) return XNOR_ERR_UNSUPPORTED;
    // the maxima start at zero: cleared by a kernel, so that the sequence can be captured in a graph
    fill_zero_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(gmax, n);
    const dim3 grid((unsigned)(n * tiles)), block(256);
#define XNOR_BG(HA, HK) bingrad_binarize_kernel<HA, HK><<<grid, block, lds, stream>>>(g, K, alpha, gbits, gmax, k_out, hw, cw, tiles)
    if (alpha) { if (K) XNOR_BG(true, true); else XNOR_BG(true, false); }
    else       { if (K) XNOR_BG(false, true); else XNOR_BG(false, false); }
#undef XNOR_BG
    return hip_status(hipGetLastError());
}

xnor_status launch_bingrad_scale_plane(const float *gmax, float *plane, int n, int hw, hipStream_t stream)
{
    if (n > 65535) return XNOR_ERR_UNSUPPORTED;
    const int bx = std::min((hw + 255) / 256, 64);
    bingrad_plane_kernel<<<dim3((unsigned)bx, (unsigned)n), dim3(256), 0, stream>>>(gmax, plane, hw);
    return hip_status(hipGetLastError());
}

}  // namespace xnor
