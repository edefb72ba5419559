// Weight binarisation (sec. 3.1): B = sign(W) packed to bits, alpha = ||W||_1 / n per filter.
// Runs once per layer; at inference only B and alpha are kept.  Also writes the same signs in
// matrix-core operand order, so the convolution can fetch a whole 32-filter operand as one
// contiguous KiB: once as int8 (+1/-1, 0 for channel or filter padding) for the 32x32x32 int8
// instruction and once as 4-bit floats (E2M1 0x2/0xA/0x0) for the 32x32x64 f8f6f4 instruction.
#include "xnor_internal.h"

namespace xnor {

// int8 image: for filter block fb (32 filters), tap t, channel word wd there is a 1 KiB record
// (index (fb*taps + t)*cw + wd); lane l of a wave owns bytes [16*l, 16*l+16): filter
// fb*32 + (l & 31), channels wd*32 + 16*(l >> 5) + 0..15.
// 4-bit image (after the int8 image): the (tap, word) blocks of a filter are numbered
// b = t*cw + wd and taken two per record (record fb*ceil(taps*cw/2) + b/2); lane l owns the 32
// channels of block 2*(b/2) + (l >> 5) as 32 nibbles, channel j in nibble j (low nibble first);
// a block past the end is all zero.
// MODE 1 (transposed): the filters of the data-gradient convolution of the backward pass (sec. 3.2, "Binary
// Gradient"), read straight out of the forward tensor W [c][k_out][taps] (c = forward filters, k_out =
// forward channels in this kernel's naming): filter k, channel ch, tap t is W[ch][k][taps - 1 - t], the
// forward filter rotated by 180 degrees with the two channel axes exchanged.
// MODE 3 (k-bit quantised weights as int8 levels): the int8 image alone is written, its bytes the odd-integer
// numerators 2u - L of q_aux(w) (L = 2^aux - 1) instead of +-1; wbits may be NULL; alpha[k] = `alpha_fill`
// (the caller's 1 / (La * Lw)).
// In mode 1 alpha is written as 1 (the scaling of that convolution is applied elsewhere).
__device__ __forceinline__ int qk_level_index(float x, int L)
{
    // level index u = floor(((x + 1) * 0.5) * L + 0.5) of q_k, x clamped to [-1, 1] (NaN -> -1); every
    // operation rounded to float in this order (the build disables contraction)
    float t = x >= -1.0f ? x : -1.0f;
    t = t <= 1.0f ? t : 1.0f;
    const float v = ((t + 1.0f) * 0.5f) * (float)L + 0.5f;
    if (L == 1) return x >= 0.0f ? 1 : 0;      // one bit: the sign rule's comparison, for every float
    return min(max((int)__builtin_floorf(v), 0), L);
}

template <int MODE>
__global__ __launch_bounds__(256) void pack_weights_kernel(
    const float *__restrict__ w, uint32_t *__restrict__ wbits, float *__restrict__ alpha,
    int8_t *__restrict__ wmfma, int k_out, int c, int taps, int cw, int aux, int stage, float alpha_fill)
{
    constexpr bool TRANSPOSED = MODE == 1;
    __shared__ float red[256];
    const int k = blockIdx.x;              // grid covers the filters padded to a multiple of 32
    const int tid = threadIdx.x;
    const bool real = k < k_out;
    const size_t n = (size_t)c * taps;
    const int kk = real ? k : 0;
    const int kf = kk;
    // element (channel ch, tap t) of this filter, read from the tensor in the mode's order
    struct Source {
        const float *base;
        size_t ch_stride;
        int taps, L;
        __device__ float operator()(int ch, int t) const
        {
            if (MODE == 3) return (float)(2 * qk_level_index(base[(size_t)ch * ch_stride + t], L) - L);
            return TRANSPOSED ? base[(size_t)ch * ch_stride + (taps - 1 - t)] : base[(size_t)ch * ch_stride + t];
        }
    };
    const Source src{TRANSPOSED ? w + (size_t)kf * taps : w + (size_t)kf * n,
                     TRANSPOSED ? (size_t)k_out * taps : (size_t)taps, taps, (1 << aux) - 1};
    // The four images below each walk the whole filter with a 32-channel stride per thread.  When the
    // filter fits the staging buffer it is first copied to LDS in [channel][tap] order (one coalesced pass
    // in mode 0) and every later access reads LDS; larger filters are read from memory each time.
    extern __shared__ float staged[];
    if (stage) {
        for (int i = tid; i < (int)n; i += 256) {
            const int ch = i / taps;
            staged[i] = src(ch, i - ch * taps);
        }
        __syncthreads();
    }
    struct Filter {
        const Source &src;
        const float *lds;
        int taps;
        __device__ float operator()(int ch, int t) const { return lds ? lds[ch * taps + t] : src(ch, t); }
    };
    const Filter wk{src, stage ? staged : nullptr, taps};

    if (real && wbits) {
        for (int item = tid; item < taps * cw; item += 256) {
            const int t = item / cw, wd = item - t * cw;
            const int nch = min(32, c - wd * 32);
            uint32_t word = 0;
            for (int j = 0; j < nch; ++j)
                word |= (wk(wd * 32 + j, t) >= 0.0f ? 1u : 0u) << j;
            wbits[((size_t)k * taps + t) * cw + wd] = word;
        }
    }
    if (real) {
        if (MODE != 0) {
            if (tid == 0) alpha[k] = MODE == 3 ? alpha_fill : 1.0f;
        } else {
            float s = 0.0f;
            for (size_t i = tid; i < n; i += 256) s += __builtin_fabsf(stage ? staged[i] : src.base[i]);
            red[tid] = s;
            __syncthreads();
            for (int step = 128; step > 0; step >>= 1) {
                if (tid < step) red[tid] += red[tid + step];
                __syncthreads();
            }
            if (tid == 0) alpha[k] = red[0] / (float)n;
        }
    }
    if (wmfma) {
        const int fb = k >> 5, row = k & 31;
        for (int item = tid; item < taps * cw * 2; item += 256) {
            const int half = item & 1;
            const int tw = item >> 1;               // t*cw + wd
            const int t = tw / cw, wd = tw - t * cw;
            const int ch0 = wd * 32 + half * 16;
            union { int8_t b[16]; uint4 v; } u;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                int8_t s = 0;
                if (real && ch0 + j < c) s = MODE == 3 ? (int8_t)wk(ch0 + j, t) : (wk(ch0 + j, t) >= 0.0f) ? 1 : -1;
                u.b[j] = s;
            }
            const size_t rec = ((size_t)fb * taps + t) * cw + wd;
            *reinterpret_cast<uint4 *>(wmfma + rec * 1024 + (size_t)(row + 32 * half) * 16) = u.v;
        }
        if (MODE == 3) {        // the int8 image alone: its trailing all-zero record, then done
            if (k == 0 && tid < 64)
                *reinterpret_cast<uint4 *>(wmfma + wimg_i8_bytes(k_out, c, taps) - 1024 + (size_t)tid * 16) = make_uint4(0, 0, 0, 0);
            return;
        }
        int8_t *w4 = wmfma + wimg_i8_bytes(k_out, c, taps);
        const int nblk = taps * cw, nrec = (nblk + 1) / 2;
        for (int item = tid; item < nrec * 2; item += 256) {
            const int half = item & 1, r = item >> 1;
            const int b = 2 * r + half;
            union { uint8_t b[16]; uint4 v; } u;
            u.v = make_uint4(0, 0, 0, 0);
            if (real && b < nblk) {
                const int t = b / cw, wd = b - t * cw;
#pragma unroll
                for (int j = 0; j < 32; ++j) {
                    const int ch = wd * 32 + j;
                    uint32_t code = 0;
                    if (ch < c) code = (wk(ch, t) >= 0.0f) ? 0x2u : 0xAu;
                    u.b[j >> 1] |= (uint8_t)(code << (4 * (j & 1)));
                }
            }
            const size_t rec = (size_t)fb * nrec + r;
            *reinterpret_cast<uint4 *>(w4 + rec * 1024 + (size_t)(row + 32 * half) * 16) = u.v;
        }
        // scalar-path image: this filter's words, 32 filters interleaved per (tap, channel word)
        uint32_t *wp = reinterpret_cast<uint32_t *>(w4 + wimg_f4_bytes(k_out, c, taps));
        for (int item = tid; item < taps * cw; item += 256) {
            const int t = item / cw, wd = item - t * cw;
            uint32_t word = 0;
            if (real) {
                const int nch = min(32, c - wd * 32);
                for (int j = 0; j < nch; ++j)
                    word |= (wk(wd * 32 + j, t) >= 0.0f ? 1u : 0u) << j;
            }
            wp[(((size_t)fb * taps + t) * cw + wd) * 32 + row] = word;
        }
        if (k == 0 && tid < 128) {      // the trailing all-zero record of each image
            int8_t *z = tid < 64 ? w4 - 1024 : w4 + wimg_f4_bytes(k_out, c, taps) - 1024;
            *reinterpret_cast<uint4 *>(z + (size_t)(tid & 63) * 16) = make_uint4(0, 0, 0, 0);
        }
    }
}

xnor_status launch_pack_weights(const float *w, uint32_t *wbits, float *alpha, void *wmfma,
                                int k_out, int c, int taps, hipStream_t stream, int mode, int aux, float alpha_fill)
{
    const int cw = (c + 31) / 32;
    const int kpad = (k_out + 31) / 32 * 32;
    dim3 grid((unsigned)(wmfma ? kpad : k_out)), block(256);
    const size_t fbytes = (size_t)c * taps * sizeof(float);
    const int stage = fbytes <= 60 * 1024 ? 1 : 0;
    const size_t lds = stage ? fbytes : 0;
#define XNOR_PACK(M, AUX) pack_weights_kernel<M><<<grid, block, lds, stream>>>(w, wbits, alpha, (int8_t *)wmfma, k_out, c, taps, cw, AUX, stage, alpha_fill)
    if (mode == 1) XNOR_PACK(1, 1);
    else if (mode == 3) XNOR_PACK(3, aux);
    else XNOR_PACK(0, 1);
#undef XNOR_PACK
    return hip_status(hipGetLastError());
}

}  // namespace xnor
