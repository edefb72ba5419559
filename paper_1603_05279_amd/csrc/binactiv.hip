// BinActiv layer (sec. 3.2): sign(I) packed to bits, A = channel mean of |I|, K = box filter of A.
// Optional batch normalisation folded in front (block order BatchNorm -> BinActiv).
#include "xnor_internal.h"
#include <atomic>
#include <algorithm>

namespace xnor {

// One workgroup = 64 consecutive pixels of one image x all channels.  Lanes run along the pixels
// (contiguous in NCHW, so every channel row is read as 256-byte coalesced segments); the 4 waves
// share the channels in groups of 8 (wave w takes groups w, w+4, ...), so any channel count keeps
// all waves busy with many independent loads in flight.  A group's 8 sign bits are one byte of
// the pixel's packed word: it is assembled in LDS, from where the 64 x Cw words of the tile leave
// as one contiguous, fully coalesced run.  |y| is accumulated per wave in float; the 4 partial
// sums per pixel meet in LDS in a fixed order, so results do not depend on timing.
// Max-pooling in front of the layer (block order BinConv -> Pool -> next block's BatchNorm -> BinActiv,
// sec. 3.2): `hw` then counts pooled pixels and every value is the maximum of its window of the
// h x w input plane.  Out-of-range window positions are skipped; the maximum starts at -inf and skips
// NaN inputs (maxNum), so it is never NaN itself.
struct PoolGeom {
    int h, w, wo;           // input plane, pooled row length
    int ph, pw, sh, sw;     // window, stride
    int pad_h, pad_w;
    int relu;               // max(., 0) before the normalisation (the optional ReLU of sec. 3.2)
    int stage;              // > 0: floats per channel of the per-wave LDS staging buffer (see the kernel)
    int streamed;           // unpooled form: the caller says the input is not in any cache (read with the non-temporal hint)
};

// NW = waves per workgroup.  The pooled form runs 16: a pooled image has few pixels (13 x 13 after
// the 27 x 27 layer), so 64-pixel tiles alone would leave CUs idle and each wave with hundreds of
// dependent window loads; more waves share the channels instead.
// PH x PW > 0: pooling window known at compile time (3 x 3 and 2 x 2 are built): all window loads of
// a channel group are then in flight together; 0: any window, one window position at a time.
// STREAM: the float input is read with the non-temporal hint (see the loads).
template <bool WRITE_BITS, bool WRITE_A, bool BN, bool POOL, int NW, int PH = 0, int PW = 0, bool STREAM = false>
__global__ __launch_bounds__(64 * NW) void binactiv_kernel(
    const float *__restrict__ x, const float *__restrict__ bn_scale,
    const float *__restrict__ bn_shift, uint32_t *__restrict__ xbits, float *__restrict__ A,
    int c, int hw, int cw, int tiles_per_image, int nblocks, PoolGeom pg)
{
    // Workgroups are dealt to the 8 XCDs round-robin by index.  Neighbouring pixel tiles share the
    // cache lines that straddle their boundary (channel rows are not line aligned), so within
    // every window of 64 tiles each XCD takes a run of 8 consecutive ones: the shared line is then
    // a hit in that XCD's own L2, while all XCDs still stream through the same region of memory.
    // The last, incomplete window keeps the plain order (runs would load the XCDs unevenly there).
    const unsigned b = blockIdx.x, win = (b >> 6) << 6;
    const int blk = (int)(win + 64u <= (unsigned)nblocks ? win + ((b & 7u) << 3) + ((b >> 3) & 7u) : b);
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    float(*part)[64] = reinterpret_cast<float(*)[64]>(smem);            // [NW][64]
    uint8_t *wbytes = smem + NW * 64 * sizeof(float);                   // [64 px][cw words][4 bytes]
    float *stage_lds = reinterpret_cast<float *>(wbytes + (size_t)64 * cw * 4);   // [NW][2][pg.stage], pooled form
    const int tid = threadIdx.x;
    // the wave index as a scalar: channel indices derived from it are then scalar too, and the
    // per-channel scale and shift come through the scalar cache instead of 64-lane loads
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int img = blk / tiles_per_image;
    const int tile = blk - img * tiles_per_image;
    const int p0 = tile * 64;
    const int p = p0 + lane;
    const bool live = p < hw;
    const int pc = live ? p : hw - 1;
    const float *xi = x + (size_t)img * c * hw + pc;                       // unpooled: this lane's pixel
    const float *xs = x + (size_t)img * c * pg.h * pg.w;                  // pooled: the image (wave-uniform)
    const int in_hw = POOL ? pg.h * pg.w : hw;
    int iy0 = 0, ix0 = 0;       // window origin of this lane's pooled pixel
    if (POOL) {
        const int oy = pc / pg.wo;
        iy0 = oy * pg.sh - pg.pad_h;
        ix0 = (pc - oy * pg.wo) * pg.sw - pg.pad_w;
    }
    const int groups = (c + 7) >> 3;
    float asum = 0.0f;
    // Every load is unconditional (indices clamped into the tensor) so that the 8 loads of a group,
    // and those of the next groups, are all in flight together; validity is applied afterwards.
#pragma unroll 4
    for (int gidx = wave; gidx < groups; gidx += NW) {
        const int ch0 = gidx * 8;
        float v[8];
        if (!POOL) {
            // An input beyond a quarter of the 256 MB last-level cache cannot be resident anyway and is read once: the
            // non-temporal hint keeps its stream from displacing the previous layers' results, which still wait in that
            // cache to be written back (a whole benchmark step 428 -> 412 us).  Smaller inputs keep the default policy:
            // they are often the previous layer's result, still in cache (with the hint a chain of three 13 x 13 blocks
            // took 93 instead of 86 us).
            if constexpr (STREAM) {
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(xi + (size_t)min(ch0 + j, c - 1) * in_hw);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = xi[(size_t)min(ch0 + j, c - 1) * in_hw];
            }
        } else if constexpr (PH > 0) {
            uint32_t off[PH * PW];       // byte offsets within the channel plane (unsigned: scalar base + 32-bit lane offset)
            bool okw[PH * PW];
#pragma unroll
            for (int dy = 0; dy < PH; ++dy)
#pragma unroll
                for (int dx = 0; dx < PW; ++dx) {
                    const int iy = iy0 + dy, ix = ix0 + dx;
                    okw[dy * PW + dx] = (unsigned)iy < (unsigned)pg.h && (unsigned)ix < (unsigned)pg.w;
                    off[dy * PW + dx] = (uint32_t)(min(max(iy, 0), pg.h - 1) * pg.w + min(max(ix, 0), pg.w - 1)) * 4u;
                }
            // maximum that skips NaN and starts at -inf (never NaN itself); positions outside the
            // image count as -inf
            const bool padded = pg.pad_h != 0 || pg.pad_w != 0;
            auto window_max = [&](const float (&t)[PH * PW]) {
                float m = -__builtin_inff();
                if (padded) {
#pragma unroll
                    for (int q = 0; q < PH * PW; ++q) m = __builtin_fmaxf(m, okw[q] ? t[q] : -__builtin_inff());
                } else {
#pragma unroll
                    for (int q = 0; q < PH * PW; ++q) m = __builtin_fmaxf(m, t[q]);
                }
                return m;
            };
            if (pg.stage > 0) {
                // The windows of neighbouring pooled pixels overlap and sit two floats apart, so loading
                // them lane by lane moves every input element several times through L1 in half-used
                // lines.  Instead the wave copies the input rows its tile touches (one contiguous run
                // per channel) into a private LDS buffer, two channels at a time, fully coalesced and
                // once, and the lanes pick their windows out of LDS.  LDS serves one wave's
                // instructions in order, so the copy needs no barrier beyond the compiler's.
                const int oy_a = p0 / pg.wo, oy_b = min(p0 + 63, hw - 1) / pg.wo;
                const int r0 = max(oy_a * pg.sh - pg.pad_h, 0);
                const int r1 = min(oy_b * pg.sh - pg.pad_h + PH - 1, pg.h - 1);
                const int nfl = (r1 - r0 + 1) * pg.w;             // <= pg.stage by the host's bound
                float *stg = stage_lds + (size_t)wave * 2 * pg.stage;
                uint32_t loff[PH * PW];
#pragma unroll
                for (int q = 0; q < PH * PW; ++q) loff[q] = off[q] / 4u - (uint32_t)(r0 * pg.w);
#pragma unroll
                for (int pr = 0; pr < 4; ++pr) {
                    float r[2][8];              // nfl <= 512 = 8 * 64: all loads of the pair in flight together
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const float *plane = xs + (size_t)min(ch0 + 2 * pr + u, c - 1) * in_hw + r0 * pg.w;
#pragma unroll
                        for (int k = 0; k < 8; ++k) r[u][k] = plane[min(lane + 64 * k, nfl - 1)];
                    }
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int k = 0; k < 8; ++k)
                            if (lane + 64 * k < nfl) stg[u * pg.stage + lane + 64 * k] = r[u][k];
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        float t[PH * PW];
#pragma unroll
                        for (int q = 0; q < PH * PW; ++q) t[q] = stg[u * pg.stage + loff[q]];
                        v[2 * pr + u] = window_max(t);
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            } else {
                float tt[8][PH * PW];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const char *plane = reinterpret_cast<const char *>(xs + (size_t)min(ch0 + j, c - 1) * in_hw);
#pragma unroll
                    for (int q = 0; q < PH * PW; ++q) tt[j][q] = *reinterpret_cast<const float *>(plane + off[q]);
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = window_max(tt[j]);
            }
            if (pg.relu) {
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = v[j] > 0.0f ? v[j] : 0.0f;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = -__builtin_inff();
            for (int dy = 0; dy < pg.ph; ++dy) {
                const int iy = iy0 + dy;
                const bool oky = (unsigned)iy < (unsigned)pg.h;
                const int rowoff = min(max(iy, 0), pg.h - 1) * pg.w;
                for (int dx = 0; dx < pg.pw; ++dx) {
                    const int ix = ix0 + dx;
                    const bool ok = oky && (unsigned)ix < (unsigned)pg.w;
                    const int off = rowoff + min(max(ix, 0), pg.w - 1);
                    float t[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) t[j] = xs[(size_t)min(ch0 + j, c - 1) * in_hw + off];
#pragma unroll
                    for (int j = 0; j < 8; ++j) v[j] = __builtin_fmaxf(v[j], ok ? t[j] : -__builtin_inff());
                }
            }
            if (pg.relu) {
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = v[j] > 0.0f ? v[j] : 0.0f;     // never NaN here
            }
        }
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
        float s = part[0][lane];
#pragma unroll
        for (int q = 1; q < NW; ++q) s += part[q][lane];
        A[(size_t)img * hw + p] = s / (float)c;
    }
    if (WRITE_BITS) {
        const int npx = min(64, hw - p0);
        const uint32_t *wsrc = reinterpret_cast<const uint32_t *>(wbytes);
        uint32_t *dst = xbits + ((size_t)img * hw + p0) * cw;
        const int nwords = npx * cw;
        const int tail_bytes = cw * 4 - groups;          // bytes of the last word no group wrote
        const uint32_t tail_mask = 0xFFFFFFFFu >> (8 * tail_bytes);
        int wd = tid % cw;                                // word index within the pixel, advanced by NT % cw
        const int wstep = (64 * NW) % cw;
        for (int i = tid; i < nwords; i += 64 * NW) {
            uint32_t word = wsrc[i];
            if (wd == cw - 1) word &= tail_mask;
            dst[i] = word;
            wd += wstep;
            if (wd >= cw) wd -= cw;
        }
    }
}

// hw == 1 (fully connected layers): the channels of one image are contiguous, so lanes run along
// channels and a wave-wide comparison yields 64 sign bits (two packed words) at once.  One workgroup of
// NWV waves per image (16 for long rows: a batch is a few hundred workgroups, so the loads in flight per
// CU come from the waves of one workgroup).
template <int NWV>
__global__ __launch_bounds__(64 * NWV) void binactiv_vec_kernel(
    const float *__restrict__ x, const float *__restrict__ bn_scale,
    const float *__restrict__ bn_shift, uint32_t *__restrict__ xbits, float *__restrict__ A,
    int c, int cw)
{
    __shared__ float part[NWV];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int img = blockIdx.x;
    const float *xi = x + (size_t)img * c;
    const bool bn = bn_scale != nullptr;
    float asum = 0.0f;
    // up to twelve 64-channel segments per wave and turn: the loads (clamped; segments past the last channel are skipped,
    // which is uniform per wave) are all in flight together, so a row of 9216 channels costs one trip to memory, not three
    constexpr int SEG = 12;
    for (int base0 = wave * 64; base0 < c; base0 += 64 * SEG * NWV) {
        float v[SEG], sc[SEG], sh[SEG];
#pragma unroll
        for (int u = 0; u < SEG; ++u) {
            v[u] = 0.0f; sc[u] = 1.0f; sh[u] = 0.0f;
            if (base0 + u * 64 * NWV < c) {
                const int chc = min(base0 + u * 64 * NWV + lane, c - 1);
                v[u] = xi[chc];
                if (bn) { sc[u] = bn_scale[chc]; sh[u] = bn_shift[chc]; }
            }
        }
#pragma unroll
        for (int u = 0; u < SEG; ++u) {
            const int base = base0 + u * 64 * NWV, ch = base + lane;
            const float y = bn ? __builtin_fmaf(v[u], sc[u], sh[u]) : v[u];
            const bool ok = ch < c;
            asum += ok ? __builtin_fabsf(y) : 0.0f;
            const unsigned long long mask = __ballot(ok && y >= 0.0f);
            if (xbits && base < c) {
                const int wd = base >> 5;
                if (lane == 0) xbits[(size_t)img * cw + wd] = (uint32_t)mask;
                if (lane == 1 && wd + 1 < cw) xbits[(size_t)img * cw + wd + 1] = (uint32_t)(mask >> 32);
            }
        }
    }
    if (A) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) asum += __shfl_xor(asum, off, 64);
        if (lane == 0) part[wave] = asum;
        __syncthreads();
        if (tid == 0) {
            float s = part[0];
#pragma unroll
            for (int q = 1; q < NWV; ++q) s += part[q];        // fixed order
            A[img] = s / (float)c;
        }
    }
}

template <bool WB, bool WA, bool BN, bool POOL, int NW, int PH, int PW>
static xnor_status launch_binactiv_one(dim3 grid, size_t lds, hipStream_t stream, const float *x,
                                       const float *bn_scale, const float *bn_shift, uint32_t *xbits, float *A, int c,
                                       int hw, int cw, int tiles, int blocks, const PoolGeom &pg)
{
    // (the cache policy is an instruction field: a kernel of its own for streamed inputs)
    const bool stream_in = !POOL && (pg.streamed || (long long)(blocks / tiles) * c * hw * 4 > (64ll << 20));
    auto kern = stream_in ? binactiv_kernel<WB, WA, BN, POOL, NW, PH, PW, !POOL> : binactiv_kernel<WB, WA, BN, POOL, NW, PH, PW, false>;
    if (lds > 48 * 1024) {      // the pooled form's staging buffer can pass the default dynamic LDS limit
        static std::atomic<bool> attr_done;      // false -> true only; a repeated attribute call is harmless
        if (!attr_done.load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    160 * 1024) != hipSuccess)
                return XNOR_ERR_HIP;
            attr_done.store(true, std::memory_order_release);
        }
    }
    kern<<<grid, dim3(64 * NW), lds, stream>>>(x, bn_scale, bn_shift, xbits, A, c, hw, cw, tiles, blocks, pg);
    return hip_status(hipGetLastError());
}

template <bool POOL, int PH, int PW, int NW>
static xnor_status launch_binactiv_nw(const float *x, const float *bn_scale, const float *bn_shift,
                                      uint32_t *xbits, float *A, int n, int c, int hw, const PoolGeom &pg,
                                      hipStream_t stream);

template <bool POOL, int PH = 0, int PW = 0>
static xnor_status launch_binactiv_impl(const float *x, const float *bn_scale, const float *bn_shift,
                                        uint32_t *xbits, float *A, int n, int c, int hw, const PoolGeom &pg,
                                        hipStream_t stream)
{
    const int cw = (c + 31) / 32;
    const int tiles = (hw + 63) / 64;
    const long long blocks = (long long)n * tiles;
    if (blocks > 0x7ffffff0LL) return XNOR_ERR_SHAPE;
    // 16 waves per workgroup for the pooled form and wherever 4-wave workgroups would leave the CUs with fewer
    // than 8 waves each (small planes: a 7 x 7 image is one 64-pixel tile): more loads in flight per CU
    if (!POOL && blocks * 4 < 256 * 8 && c >= 128)
        return launch_binactiv_nw<POOL, PH, PW, 16>(x, bn_scale, bn_shift, xbits, A, n, c, hw, pg, stream);
    return launch_binactiv_nw<POOL, PH, PW, POOL ? 16 : 4>(x, bn_scale, bn_shift, xbits, A, n, c, hw, pg, stream);
}

template <bool POOL, int PH, int PW, int NW>
static xnor_status launch_binactiv_nw(const float *x, const float *bn_scale, const float *bn_shift,
                                      uint32_t *xbits, float *A, int n, int c, int hw, const PoolGeom &pg,
                                      hipStream_t stream)
{
    const int cw = (c + 31) / 32;
    const int tiles = (hw + 63) / 64;
    const long long blocks = (long long)n * tiles;
    size_t lds = NW * 64 * sizeof(float) + (size_t)64 * cw * 4;
    if (lds > 64 * 1024) return XNOR_ERR_UNSUPPORTED;       // more than ~500k channels per pixel
    lds += (size_t)NW * 2 * pg.stage * sizeof(float);
    dim3 grid((unsigned)blocks);
#define XNOR_BA(B, AA, N) \
    return launch_binactiv_one<B, AA, N, POOL, NW, PH, PW>(grid, lds, stream, x, bn_scale, bn_shift, xbits, A, c, hw, cw, \
                                                           tiles, (int)blocks, pg)
    const bool bn = bn_scale != nullptr;
    if (xbits && A) { if (bn) XNOR_BA(true, true, true); else XNOR_BA(true, true, false); }
    else if (xbits) { if (bn) XNOR_BA(true, false, true); else XNOR_BA(true, false, false); }
    else            { if (bn) XNOR_BA(false, true, true); else XNOR_BA(false, true, false); }
#undef XNOR_BA
}

xnor_status launch_binactiv(const float *x, const float *bn_scale, const float *bn_shift,
                            uint32_t *xbits, float *A, int n, int c, int hw, hipStream_t stream, int streamed)
{
    if (hw == 1) {
        const int cw = (c + 31) / 32;
        if (c >= 4096)
            binactiv_vec_kernel<16><<<dim3((unsigned)n), dim3(1024), 0, stream>>>(x, bn_scale, bn_shift, xbits, A, c, cw);
        else
            binactiv_vec_kernel<4><<<dim3((unsigned)n), dim3(256), 0, stream>>>(x, bn_scale, bn_shift, xbits, A, c, cw);
        return hip_status(hipGetLastError());
    }
    PoolGeom pg{};
    pg.streamed = streamed;
    return launch_binactiv_impl<false>(x, bn_scale, bn_shift, xbits, A, n, c, hw, pg, stream);
}

xnor_status launch_pool_binactiv(const float *x, const float *bn_scale, const float *bn_shift,
                                 uint32_t *xbits, float *A, int n, int c, int h, int w, int ph, int pw,
                                 int sh, int sw, int pad_h, int pad_w, int relu, hipStream_t stream)
{
    PoolGeom pg;
    pg.h = h; pg.w = w; pg.ph = ph; pg.pw = pw; pg.sh = sh; pg.sw = sw; pg.pad_h = pad_h; pg.pad_w = pad_w;
    pg.relu = relu;
    const int ho = (h + 2 * pad_h - ph) / sh + 1, wo = (w + 2 * pad_w - pw) / sw + 1;
    pg.wo = wo;
    // LDS staging of the input rows a 64-pixel tile touches (compile-time windows only): at most
    // ceil-ish (64 + wo - 2)/wo + 1 pooled rows, hence (rows - 1)*sh + ph input rows of w floats
    pg.stage = 0;
    if ((ph == 3 && pw == 3) || (ph == 2 && pw == 2)) {
        const long long prows = std::min<long long>(ho, (64 + wo - 2) / wo + 1);
        const long long nfl = std::min<long long>(h, (prows - 1) * sh + ph) * w;
        if (nfl <= 512) pg.stage = (int)nfl;      // 16 waves x 2 channels x 512 floats = 64 KB
    }
    if (ph == 3 && pw == 3) return launch_binactiv_impl<true, 3, 3>(x, bn_scale, bn_shift, xbits, A, n, c, ho * wo, pg, stream);
    if (ph == 2 && pw == 2) return launch_binactiv_impl<true, 2, 2>(x, bn_scale, bn_shift, xbits, A, n, c, ho * wo, pg, stream);
    return launch_binactiv_impl<true>(x, bn_scale, bn_shift, xbits, A, n, c, ho * wo, pg, stream);
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
