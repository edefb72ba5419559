// BinActiv layer (sec. 3.2): sign(I) packed to bits, A = channel mean of |I|, K = box filter of A.
// Optional batch normalisation folded in front (block order BatchNorm -> BinActiv).
#include "xnor_internal.h"

namespace xnor {

// One workgroup = 64 consecutive pixels of one image x all channels.  Lanes run along the pixels
// (contiguous in NCHW, so every channel row is read as 256-byte coalesced segments); the 4 waves
// share the channels in groups of 8 (wave w takes groups w, w+4, ...), so any channel count keeps
// all waves busy with many independent loads in flight.  A group's 8 sign bits are one byte of
// the pixel's packed word: it is assembled in LDS, from where the 64 x Cw words of the tile leave
// as one contiguous, fully coalesced run.  |y| is accumulated per wave in float; the 4 partial
// sums per pixel meet in LDS in a fixed order, so results do not depend on timing.
template <bool WRITE_BITS, bool WRITE_A, bool BN>
__global__ __launch_bounds__(256) void binactiv_kernel(
    const float *__restrict__ x, const float *__restrict__ bn_scale,
    const float *__restrict__ bn_shift, uint32_t *__restrict__ xbits, float *__restrict__ A,
    int c, int hw, int cw, int tiles_per_image, int nblocks)
{
    // Workgroups are dealt to the 8 XCDs round-robin by index.  Neighbouring pixel tiles share the
    // cache lines that straddle their boundary (channel rows are not line aligned), so within
    // every window of 64 tiles each XCD takes a run of 8 consecutive ones: the shared line is then
    // a hit in that XCD's own L2, while all XCDs still stream through the same region of memory.
    // The last, incomplete window keeps the plain order (runs would load the XCDs unevenly there).
    const unsigned b = blockIdx.x, win = (b >> 6) << 6;
    const int blk = (int)(win + 64u <= (unsigned)nblocks ? win + ((b & 7u) << 3) + ((b >> 3) & 7u) : b);
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    float(*part)[64] = reinterpret_cast<float(*)[64]>(smem);            // [4][64]
    uint8_t *wbytes = smem + 4 * 64 * sizeof(float);                    // [64 px][cw words][4 bytes]
    const int tid = threadIdx.x;
    // the wave index as a scalar: channel indices derived from it are then scalar too, and the
    // per-channel scale and shift come through the scalar cache instead of 64-lane loads
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int img = blk / tiles_per_image;
    const int tile = blk - img * tiles_per_image;
    const int p0 = tile * 64;
    const int p = p0 + lane;
    const bool live = p < hw;
    const float *xi = x + (size_t)img * c * hw + (live ? p : hw - 1);
    const int groups = (c + 7) >> 3;
    float asum = 0.0f;
    // Every load is unconditional (indices clamped into the tensor) so that the 8 loads of a group,
    // and those of the next groups, are all in flight together; validity is applied afterwards.
#pragma unroll 4
    for (int gidx = wave; gidx < groups; gidx += 4) {
        const int ch0 = gidx * 8;
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = xi[(size_t)min(ch0 + j, c - 1) * hw];
        uint32_t byte = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int ch = min(ch0 + j, c - 1);
            float y = v[j];
            if (BN) y = __builtin_fmaf(y, bn_scale[ch], bn_shift[ch]);
            const bool ok = ch0 + j < c;
            byte |= ((ok && y >= 0.0f) ? 1u : 0u) << j;
            asum += ok ? __builtin_fabsf(y) : 0.0f;
        }
        if (WRITE_BITS) wbytes[(lane * cw) * 4 + gidx] = (uint8_t)byte;   // byte gidx of the pixel's word run
    }
    if (WRITE_A) part[wave][lane] = asum;
    __syncthreads();
    if (WRITE_A && wave == 0 && live) {
        const float s = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
        A[(size_t)img * hw + p] = s / (float)c;
    }
    if (WRITE_BITS) {
        const int npx = min(64, hw - p0);
        const uint32_t *wsrc = reinterpret_cast<const uint32_t *>(wbytes);
        uint32_t *dst = xbits + ((size_t)img * hw + p0) * cw;
        const int nwords = npx * cw;
        const int tail_bytes = cw * 4 - groups;          // bytes of the last word no group wrote
        const uint32_t tail_mask = 0xFFFFFFFFu >> (8 * tail_bytes);
        int wd = tid % cw;                                // word index within the pixel, advanced by 256 % cw
        const int wstep = 256 % cw;
        for (int i = tid; i < nwords; i += 256) {
            uint32_t word = wsrc[i];
            if (wd == cw - 1) word &= tail_mask;
            dst[i] = word;
            wd += wstep;
            if (wd >= cw) wd -= cw;
        }
    }
}

// hw == 1 (fully connected layers): the channels of one image are contiguous, so lanes run along
// channels and a wave-wide comparison yields 64 sign bits (two packed words) at once.
__global__ __launch_bounds__(256) void binactiv_vec_kernel(
    const float *__restrict__ x, const float *__restrict__ bn_scale,
    const float *__restrict__ bn_shift, uint32_t *__restrict__ xbits, float *__restrict__ A,
    int c, int cw)
{
    __shared__ float part[4];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int img = blockIdx.x;
    const float *xi = x + (size_t)img * c;
    const bool bn = bn_scale != nullptr;
    float asum = 0.0f;
    for (int base = wave * 64; base < c; base += 256) {
        const int ch = base + lane;
        float y = -1.0f;
        if (ch < c) {
            y = xi[ch];
            if (bn) y = __builtin_fmaf(y, bn_scale[ch], bn_shift[ch]);
            asum += __builtin_fabsf(y);
        }
        const unsigned long long mask = __ballot(ch < c && y >= 0.0f);
        if (xbits) {
            const int wd = base >> 5;
            if (lane == 0) xbits[(size_t)img * cw + wd] = (uint32_t)mask;
            if (lane == 1 && wd + 1 < cw) xbits[(size_t)img * cw + wd + 1] = (uint32_t)(mask >> 32);
        }
    }
    if (A) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) asum += __shfl_xor(asum, off, 64);
        if (lane == 0) part[wave] = asum;
        __syncthreads();
        if (tid == 0) A[img] = (((part[0] + part[1]) + part[2]) + part[3]) / (float)c;
    }
}

xnor_status launch_binactiv(const float *x, const float *bn_scale, const float *bn_shift,
                            uint32_t *xbits, float *A, int n, int c, int hw, hipStream_t stream)
{
    const int cw = (c + 31) / 32;
    if (hw == 1) {
        binactiv_vec_kernel<<<dim3((unsigned)n), dim3(256), 0, stream>>>(x, bn_scale, bn_shift, xbits, A, c, cw);
        return hip_status(hipGetLastError());
    }
    const int tiles = (hw + 63) / 64;
    const long long blocks = (long long)n * tiles;
    if (blocks > 0x7ffffff0LL) return XNOR_ERR_SHAPE;
    const size_t lds = 4 * 64 * sizeof(float) + (size_t)64 * cw * 4;
    if (lds > 64 * 1024) return XNOR_ERR_UNSUPPORTED;       // more than ~500k channels per pixel
    dim3 grid((unsigned)blocks), block(256);
#define XNOR_BA(B, AA, N) binactiv_kernel<B, AA, N><<<grid, block, lds, stream>>>(x, bn_scale, bn_shift, xbits, A, c, hw, cw, tiles, (int)blocks)
    const bool bn = bn_scale != nullptr;
    if (xbits && A) { if (bn) XNOR_BA(true, true, true); else XNOR_BA(true, true, false); }
    else if (xbits) { if (bn) XNOR_BA(true, false, true); else XNOR_BA(true, false, false); }
    else            { if (bn) XNOR_BA(false, true, true); else XNOR_BA(false, true, false); }
#undef XNOR_BA
    return hip_status(hipGetLastError());
}

// K[n][oy][ox] = (1/(kh*kw)) * sum over in-bounds taps of A (sec. 3.2).  One thread per output;
// A is 1/c of the input volume and stays in L2, taps are summed in row-major order.
__global__ __launch_bounds__(256) void boxfilter_kernel(const float *__restrict__ A,
                                                        float *__restrict__ K, ConvGeom g)
{
    const uint32_t m = blockIdx.x * 256u + threadIdx.x;
    if (m >= (uint32_t)g.m_total) return;
    K[m] = box_K(A, g, m);
}

xnor_status launch_boxfilter(const float *A, float *K, const ConvGeom &g, hipStream_t stream)
{
    dim3 grid((unsigned)((g.m_total + 255) / 256)), block(256);
    boxfilter_kernel<<<grid, block, 0, stream>>>(A, K, g);
    return hip_status(hipGetLastError());
}

}  // namespace xnor
