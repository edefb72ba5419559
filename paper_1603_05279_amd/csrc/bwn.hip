// Binary-Weight-Network convolution (sec. 3.1): real-valued inputs, weights estimated as alpha * sign(W),
//     I * W  ~  (I (+) B) alpha        (convolution with additions and subtractions only).
// On this chip the +-1 weighted sums run on the bfloat16 matrix cores: a float is the exact sum of
// three bfloat16 numbers, a +-1 weight times a bfloat16 is exact, and the matrix cores accumulate in
// float, so the convolution kernel (conv_mfma.hip, third operand format) returns the float sum of
// exact terms.  This file holds the two preparation kernels: the activation split and the weights.
#include "xnor_internal.h"

namespace xnor {

__device__ __forceinline__ uint32_t bf16_rne(float v)      // round to nearest even (finite inputs)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, v);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float bf16_value(uint32_t h) { return __builtin_bit_cast(float, h << 16); }

// x [n][c][hw] float  ->  parts [n][hw][Cg][3][16] bfloat16, Cg = ceil(c/16): for every pixel and group
// of 16 channels three 32-byte words (hi, mid, lo) with hi + mid + lo == x exactly; channels >= c are 0.
// One workgroup = 64 pixels x 4 channel groups, one group per wave; lanes along pixels (every channel
// row is read as coalesced 256-byte segments, 16 loads in flight per lane).  A lane's 96 bytes go to LDS
// (row stride 4*96 + 16 bytes: 16-byte writes of neighbouring lanes fall on different banks), from where
// the workgroup writes each pixel's 4*96 bytes as one contiguous run, 16 bytes per lane.
constexpr int SPLIT_G = 4, SPLIT_ROW = SPLIT_G * 96 + 16;
__global__ __launch_bounds__(256) void bwn_split_kernel(const float *__restrict__ x, uint8_t *__restrict__ parts,
                                                        int c, int hw, int cg)
{
    __shared__ __attribute__((aligned(16))) uint8_t stage[64 * SPLIT_ROW];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int p0 = blockIdx.x * 64, g0 = blockIdx.y * SPLIT_G, img = blockIdx.z;
    const int grp = g0 + wave;
    const int pc = min(p0 + lane, hw - 1);
    if (grp < cg) {
        const float *xi = x + ((size_t)img * c + (size_t)grp * 16) * hw + pc;
        float v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = xi[(size_t)min(j, c - 1 - grp * 16) * hw];     // clamped, masked below
        uint32_t hi[16], mid[16], lo[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float t = grp * 16 + j < c ? v[j] : 0.0f;
            hi[j] = bf16_rne(t);
            const float r1 = t - bf16_value(hi[j]);          // exact
            mid[j] = bf16_rne(r1);
            const float r2 = r1 - bf16_value(mid[j]);        // exact, at most 8 significant bits left
            lo[j] = bf16_rne(r2);
        }
        uint4 *dst = reinterpret_cast<uint4 *>(stage + lane * SPLIT_ROW + wave * 96);
        auto pack4 = [](const uint32_t *h) { return make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)); };
        dst[0] = pack4(hi);  dst[1] = pack4(hi + 8);
        dst[2] = pack4(mid); dst[3] = pack4(mid + 8);
        dst[4] = pack4(lo);  dst[5] = pack4(lo + 8);
    }
    __syncthreads();
    const int ng = min(SPLIT_G, cg - g0);            // groups of this workgroup
    const int upp = ng * 6;                          // 16-byte units per pixel
    const int npx = min(64, hw - p0);
    uint8_t *out = parts + (((size_t)img * hw + p0) * cg + g0) * 96;
    for (int i = tid; i < npx * upp; i += 256) {
        const int px = i / upp, u = i - px * upp;
        *reinterpret_cast<uint4 *>(out + (size_t)px * cg * 96 + u * 16) =
            *reinterpret_cast<const uint4 *>(stage + px * SPLIT_ROW + u * 16);
    }
}

xnor_status launch_bwn_split(const float *x, void *parts, int n, int c, int hw, hipStream_t stream)
{
    const int cg = (c + 15) / 16;
    const int gblocks = (cg + SPLIT_G - 1) / SPLIT_G;
    if (gblocks > 65535 || n > 65535) return XNOR_ERR_UNSUPPORTED;
    dim3 grid((unsigned)((hw + 63) / 64), (unsigned)gblocks, (unsigned)n);
    bwn_split_kernel<<<grid, dim3(256), 0, stream>>>(x, static_cast<uint8_t *>(parts), c, hw, cg);
    return hip_status(hipGetLastError());
}

// Weight side: alpha_k = ||W_k||_1 / n (sec. 3.1) and the +-1 bfloat16 record image
// [filter block of 32][tap][16-channel group] of 1 KiB records in matrix-operand lane order
// (lane l: filter l & 31, channels 16*group + 8*(l >> 5) .. +7); a record multiplies all three
// parts of its group.  One trailing all-zero record.  One workgroup per filter.
__global__ __launch_bounds__(256) void bwn_pack_kernel(const float *__restrict__ w, float *__restrict__ alpha,
                                                       uint16_t *__restrict__ wimg, int k_out, int c, int taps, int cg)
{
    __shared__ float red[256];
    const int f = blockIdx.x, tid = threadIdx.x;
    const int nw = c * taps;
    const float *wf = w + (size_t)f * nw;
    float s = 0.0f;
    for (int i = tid; i < nw; i += 256) s += __builtin_fabsf(wf[i]);
    red[tid] = s;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {            // fixed-order tree
        if (tid < off) red[tid] += red[tid + off];
        __syncthreads();
    }
    if (tid == 0) alpha[f] = red[0] / (float)nw;
    // records: index (fblk*taps + t)*cg + grp, 512 bfloat16 each; lane slot (f & 31) + 32*half holds 8 values
    const int fblk = f >> 5, row = f & 31;
    for (int i = tid; i < taps * cg * 16; i += 256) {
        const int t = i / (cg * 16), rem = i - t * cg * 16;
        const int grp = rem >> 4, j = rem & 15;           // channel 16*grp + j
        const int ch = grp * 16 + j;
        const uint16_t v = ch < c ? (wf[(size_t)ch * taps + t] >= 0.0f ? 0x3F80 : 0xBF80) : 0;
        const size_t rec = (size_t)(fblk * taps + t) * cg + grp;
        const int slot = (row + 32 * (j >> 3)) * 8 + (j & 7);
        wimg[rec * 512 + slot] = v;
    }
}

__global__ __launch_bounds__(256) void bwn_clear_kernel(uint32_t *__restrict__ p, size_t ndwords)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < ndwords; i += (size_t)gridDim.x * 256) p[i] = 0;
}

xnor_status launch_bwn_pack(const float *w, float *alpha, void *wimg, int k_out, int c, int taps, hipStream_t stream)
{
    const int cg = (c + 15) / 16;
    // rows of the last filter block past k_out and the trailing record must read as zero
    const size_t bytes = wimg_bf16_bytes(k_out, cg, taps);
    bwn_clear_kernel<<<dim3(1024), dim3(256), 0, stream>>>(static_cast<uint32_t *>(wimg), bytes / 4);
    if (xnor_status s = hip_status(hipGetLastError())) return s;
    bwn_pack_kernel<<<dim3((unsigned)k_out), dim3(256), 0, stream>>>(w, alpha, static_cast<uint16_t *>(wimg), k_out, c,
                                                                     taps, cg);
    return hip_status(hipGetLastError());
}

}  // namespace xnor
