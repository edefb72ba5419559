// k-bit quantisation (sec. 3.2, paragraph "k-bit Quantization"): q_k(x) = 2*([(2^k - 1)(x + 1)/2]/(2^k - 1) - 1/2)
// in place of sign().  With L = 2^k - 1 and the level index u = [L (x + 1)/2], q_k = (2u - L)/L: an odd integer
// in [-L, L] over L.  The convolution of ka-bit inputs with kw-bit weights is therefore an integer contraction
// of the numerators divided by La*Lw, and runs as ONE int8 matrix-core convolution (conv_mfma.hip, operand
// format 3: int32 accumulation, exact) on the numerators stored as int8; zero padding stays exact.
// (The same sum could be formed from ka*kw binary convolutions of the bit planes, q_k = sum_p 2^p s_p / L; on
// this chip the int8 contraction is ka*kw times less matrix work at half the 4-bit rate.)
#include "xnor_internal.h"

namespace xnor {

__device__ __forceinline__ int qk_level(float x, int L)
{
    // u = floor(((x + 1) * 0.5) * L + 0.5), x clamped to [-1, 1] (NaN -> -1); each operation rounded to
    // float in this order (contraction is disabled for the build): the float value decides the level
    float t = x >= -1.0f ? x : -1.0f;
    t = t <= 1.0f ? t : 1.0f;
    const float v = ((t + 1.0f) * 0.5f) * (float)L + 0.5f;
    // one bit: the comparison of the sign rule (x + 1 rounds to 1 for -2^-25 < x < 0, which would give +1)
    if (L == 1) return x >= 0.0f ? 1 : 0;
    return min(max((int)__builtin_floorf(v), 0), L);
}

// x [n][c][hw] float -> xq [n][hw][cw][32] int8: byte j of word wd = 2u - L of channel wd*32 + j (0 past the
// last channel).  One workgroup = 64 consecutive pixels of one image x 8 channel words; lanes along pixels
// (every channel row is read as coalesced 256-byte segments), the 4 waves share the 32 groups of 8 channels,
// a group's 8 bytes go to LDS (row stride 8*32 + 16 bytes: neighbouring lanes fall on different banks), from
// where each pixel's words leave as one contiguous run, 16 bytes per lane.
constexpr int KB_WORDS = 8, KB_ROW = KB_WORDS * 32 + 16;
__global__ __launch_bounds__(256) void kbit_levels_kernel(const float *__restrict__ x, int8_t *__restrict__ xq,
                                                          int c, int hw, int cw, int L)
{
    __shared__ __attribute__((aligned(16))) uint8_t stage[64 * KB_ROW];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int p0 = blockIdx.x * 64, w0 = blockIdx.y * KB_WORDS, img = blockIdx.z;
    const int nwords = min(KB_WORDS, cw - w0);
    const int pc = min(p0 + lane, hw - 1);
    const float *xi = x + (size_t)img * c * hw + pc;
#pragma unroll 2
    for (int gidx = wave; gidx < nwords * 4; gidx += 4) {           // groups of 8 channels of this workgroup
        const int ch0 = w0 * 32 + gidx * 8;
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = xi[(size_t)min(ch0 + j, c - 1) * hw];
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int a = ch0 + j < c ? 2 * qk_level(v[j], L) - L : 0;
            if (j < 4) lo |= ((uint32_t)a & 255u) << (8 * j);
            else hi |= ((uint32_t)a & 255u) << (8 * (j - 4));
        }
        *reinterpret_cast<uint2 *>(stage + lane * KB_ROW + gidx * 8) = make_uint2(lo, hi);
    }
    __syncthreads();
    const int upp = nwords * 2;                       // 16-byte units per pixel
    const int npx = min(64, hw - p0);
    int8_t *out = xq + (((size_t)img * hw + p0) * cw + w0) * 32;
    for (int i = tid; i < npx * upp; i += 256) {
        const int px = i / upp, u = i - px * upp;
        *reinterpret_cast<uint4 *>(out + (size_t)px * cw * 32 + u * 16) =
            *reinterpret_cast<const uint4 *>(stage + px * KB_ROW + u * 16);
    }
}

xnor_status launch_kbit_pack_input(const float *x, int8_t *xq, int k, int n, int c, int hw, hipStream_t stream)
{
    const int cw = (c + 31) / 32;
    const int wblocks = (cw + KB_WORDS - 1) / KB_WORDS;
    if (wblocks > 65535 || n > 65535) return XNOR_ERR_UNSUPPORTED;
    dim3 grid((unsigned)((hw + 63) / 64), (unsigned)wblocks, (unsigned)n);
    kbit_levels_kernel<<<grid, dim3(256), 0, stream>>>(x, xq, c, hw, cw, (1 << k) - 1);
    return hip_status(hipGetLastError());
}

}  // namespace xnor
