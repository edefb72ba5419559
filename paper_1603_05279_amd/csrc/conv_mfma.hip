// Binary convolution on the int8 matrix cores (sec. 3.2).  The +-1 product-sum that XNOR +
// bitcount evaluates is the same integer as an int8 dot product of the sign tensors, with 0 for
// padded positions, so the convolution is run as an implicit GEMM
//     D[filter][pixel] = sum_{tap, channel} sW[filter][tap][channel] * sI[pixel + tap][channel]
// on v_mfma_i32_32x32x32_i8, followed by the fused scaling by K and alpha.
//
// Work split: a workgroup owns FT = 32*FW*WF filters x PT = 32*PW*WP consecutive output pixels
// (pixels flattened over image, row, column so small images still fill the tile).  Per channel
// chunk it widens the packed activation bits of the input rows its pixels touch (halo included,
// halo = 0) to int8 in LDS once; every tap then reads the same LDS image at a shifted offset.
// Weights come from the pre-widened image written by the weight packer, one contiguous KiB per
// 32-filter operand.  Filters are the M operand and pixels the N operand, so each lane of the
// result holds one pixel column: stores along a filter plane are contiguous across lanes.
#include "xnor_internal.h"

namespace xnor {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct MfmaPlan {
    int cc_words;     // channel words widened per chunk (divides cw)
    int ps;           // bytes per pixel in LDS: cc_words*32 + 16 (odd multiple of 16: no bank conflicts)
    int max_rows;     // padded input rows a pixel tile can touch
    int region_bytes; // max_rows * wp * ps
    FastDiv div_wp, div_hp, div_ccw;
};

// 4 sign bits -> 4 int8 lanes of a dword: bit 1 -> +1 (0x01), bit 0 -> -1 (0xFF).
__device__ __forceinline__ uint32_t widen4(uint32_t nibble)
{
    const uint32_t t = __umul24(nibble, 0x00204081u) & 0x01010101u;   // bit i -> byte i
    return __builtin_amdgcn_perm(0x000001FFu, 0x000001FFu, t);         // byte = table[t], table = {0xFF, 0x01}
}

template <int FW, int PW, int WF, int WP>
__global__ __launch_bounds__(64 * WF * WP) void conv_mfma_i8_kernel(
    const uint32_t *__restrict__ xbits, const v4i *__restrict__ wmfma,
    const float *__restrict__ K, const float *__restrict__ alpha, float *__restrict__ out,
    int32_t *__restrict__ dot_out, ConvGeom g, MfmaPlan pl)
{
    constexpr int NT = 64 * WF * WP;
    constexpr int FT = 32 * FW * WF;
    constexpr int PT = 32 * PW * WP;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    int *rowinfo = reinterpret_cast<int *>(lds + pl.region_bytes);

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, half = lane >> 5;
    const int wf = wave % WF, wp = wave / WF;
    const uint32_t m0 = blockIdx.x * (uint32_t)PT;
    const int f0 = blockIdx.y * FT;
    const uint32_t howo = (uint32_t)(g.ho * g.wo);

    // padded input rows this tile touches: R = image*hp + padded row
    const uint32_t m_last = min(m0 + (uint32_t)PT, (uint32_t)g.m_total) - 1u;
    const uint32_t img_a = g.div_howo.div(m0), img_b = g.div_howo.div(m_last);
    const uint32_t oy_a = g.div_wo.div(m0 - img_a * howo), oy_b = g.div_wo.div(m_last - img_b * howo);
    const int r_lo = (int)(img_a * g.hp + oy_a * g.sh);
    const int r_hi = (int)(img_b * g.hp + oy_b * g.sh) + g.kh - 1;
    const int nrows = r_hi - r_lo + 1;

    for (int rr = tid; rr < nrows; rr += NT) {
        const uint32_t R = (uint32_t)(r_lo + rr);
        const uint32_t img = pl.div_hp.div(R);
        const int y = (int)(R - img * g.hp) - g.ph;
        rowinfo[rr] = (y >= 0 && y < g.h) ? (int)(((img * g.h + y) * g.w) * g.cw) : -1;
    }

    // LDS byte offset of each of this lane's pixel columns (window origin in the padded frame)
    int pbase[PW];
#pragma unroll
    for (int j = 0; j < PW; ++j) {
        const uint32_t m = min(m0 + (uint32_t)((wp * PW + j) * 32 + l32), (uint32_t)g.m_total - 1u);
        const uint32_t img = g.div_howo.div(m);
        const uint32_t pix = m - img * howo;
        const uint32_t oy = g.div_wo.div(pix), ox = pix - oy * g.wo;
        pbase[j] = (((int)(img * g.hp + oy * g.sh) - r_lo) * g.wp + (int)ox * g.sw) * pl.ps + 16 * half;
    }
    int fblk[FW];
#pragma unroll
    for (int i = 0; i < FW; ++i) fblk[i] = min(f0 / 32 + wf * FW + i, g.fblocks - 1);

    v16i acc[FW][PW];
#pragma unroll
    for (int i = 0; i < FW; ++i)
#pragma unroll
        for (int j = 0; j < PW; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    const int ccw = pl.cc_words;
    for (int wbase = 0; wbase < g.cw; wbase += ccw) {
        __syncthreads();   // rowinfo visible / previous chunk fully consumed
        const int items = nrows * g.wp * ccw;
        for (int it = tid; it < items; it += NT) {
            const uint32_t px = pl.div_ccw.div((uint32_t)it);
            const int wl = it - (int)px * ccw;
            const uint32_t rr = pl.div_wp.div(px);
            const int col = (int)(px - rr * g.wp);
            const int xcol = col - g.pw;
            const int rowbase = rowinfo[rr];
            const bool ok = rowbase >= 0 && xcol >= 0 && xcol < g.w;
            uint4 lo = make_uint4(0, 0, 0, 0), hi = make_uint4(0, 0, 0, 0);
            if (ok) {
                const uint32_t bits = xbits[(size_t)rowbase + (size_t)xcol * g.cw + wbase + wl];
                lo.x = widen4(bits & 15u);         lo.y = widen4((bits >> 4) & 15u);
                lo.z = widen4((bits >> 8) & 15u);  lo.w = widen4((bits >> 12) & 15u);
                hi.x = widen4((bits >> 16) & 15u); hi.y = widen4((bits >> 20) & 15u);
                hi.z = widen4((bits >> 24) & 15u); hi.w = widen4(bits >> 28);
                const int nch = g.c - (wbase + wl) * 32;   // channels present in this word
                if (nch < 32) {                              // zero the channel padding
                    uint32_t *d = reinterpret_cast<uint32_t *>(&lo);
                    uint32_t *e = reinterpret_cast<uint32_t *>(&hi);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int r0 = nch - 4 * q, r1 = nch - 16 - 4 * q;
                        d[q] &= r0 >= 4 ? 0xFFFFFFFFu : (r0 <= 0 ? 0u : (1u << (8 * r0)) - 1u);
                        e[q] &= r1 >= 4 ? 0xFFFFFFFFu : (r1 <= 0 ? 0u : (1u << (8 * r1)) - 1u);
                    }
                }
            }
            uint8_t *dst = lds + (size_t)px * pl.ps + wl * 32;
            *reinterpret_cast<uint4 *>(dst) = lo;
            *reinterpret_cast<uint4 *>(dst + 16) = hi;
        }
        __syncthreads();

        for (int dy = 0; dy < g.kh; ++dy)
            for (int dx = 0; dx < g.kw; ++dx) {
                const int tapoff = (dy * g.wp + dx) * pl.ps;
                const int t = dy * g.kw + dx;
                for (int ks = 0; ks < ccw; ++ks) {
                    v4i wfr[FW], xfr[PW];
#pragma unroll
                    for (int i = 0; i < FW; ++i)
                        wfr[i] = wmfma[(((size_t)fblk[i] * g.taps + t) * g.cw + wbase + ks) * 64 + lane];
#pragma unroll
                    for (int j = 0; j < PW; ++j)
                        xfr[j] = *reinterpret_cast<const v4i *>(lds + pbase[j] + tapoff + ks * 32);
#pragma unroll
                    for (int i = 0; i < FW; ++i)
#pragma unroll
                        for (int j = 0; j < PW; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wfr[i], xfr[j], acc[i][j], 0, 0, 0);
                }
            }
    }

    // epilogue: out = float(dot) * K * alpha; result register v of a lane is filter row
    // 8*(v/4) + 4*half + v%4 of the 32-filter block, pixel column l32.
#pragma unroll
    for (int j = 0; j < PW; ++j) {
        const uint32_t m = m0 + (uint32_t)((wp * PW + j) * 32 + l32);
        if (m >= (uint32_t)g.m_total) continue;
        const uint32_t img = g.div_howo.div(m);
        const uint32_t pix = m - img * howo;
        const float Km = K[m];
#pragma unroll
        for (int i = 0; i < FW; ++i) {
            const int kb = f0 + (wf * FW + i) * 32 + 4 * half;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = kb + 8 * (v >> 2) + (v & 3);
                if (k < g.k_out) {
                    const int dot = acc[i][j][v];
                    const size_t o = ((size_t)img * g.k_out + k) * howo + pix;
                    out[o] = (float)dot * Km * alpha[k];
                    if (dot_out) dot_out[o] = dot;
                }
            }
        }
    }
}

// Padded input rows touched by the worst pixel tile of PT consecutive output pixels.
static int worst_rows(const ConvGeom &g, int PT)
{
    int worst = 0;
    const int howo = g.ho * g.wo;
    for (long long m0 = 0; m0 < g.m_total; m0 += PT) {
        const long long m1 = (m0 + PT < g.m_total ? m0 + PT : g.m_total) - 1;
        const int ia = (int)(m0 / howo), ib = (int)(m1 / howo);
        const int oa = (int)(m0 % howo) / g.wo, ob = (int)(m1 % howo) / g.wo;
        const int rows = (ib * g.hp + ob * g.sh + g.kh - 1) - (ia * g.hp + oa * g.sh) + 1;
        if (rows > worst) worst = rows;
    }
    return worst;
}

static const int LDS_LIMIT = 160 * 1024;

static bool make_plan(const ConvGeom &g, int PT, int lds_budget, MfmaPlan *pl)
{
    const int rows = worst_rows(g, PT);
    for (int ccw = g.cw; ccw >= 1; --ccw) {
        if (g.cw % ccw) continue;
        const long long ps = (long long)ccw * 32 + 16;
        const long long region = (long long)rows * g.wp * ps;
        const long long total = region + (long long)rows * 4 + 16;
        if (total > lds_budget && ccw > 1) continue;
        if (total > LDS_LIMIT) return false;
        if (region * 1 >= (1ll << 30)) return false;
        pl->cc_words = ccw;
        pl->ps = (int)ps;
        pl->max_rows = rows;
        pl->region_bytes = (int)region;
        pl->div_wp = FastDiv::make((uint32_t)g.wp);
        pl->div_hp = FastDiv::make((uint32_t)g.hp);
        pl->div_ccw = FastDiv::make((uint32_t)ccw);
        return true;
    }
    return false;
}

template <int FW, int PW, int WF, int WP>
static xnor_status launch_cfg(const uint32_t *xbits, const void *wmfma, const float *K,
                              const float *alpha, float *out, int32_t *dot_out, const ConvGeom &g,
                              hipStream_t stream)
{
    constexpr int FT = 32 * FW * WF, PT = 32 * PW * WP;
    MfmaPlan pl;
    if (!make_plan(g, PT, 64 * 1024, &pl)) return XNOR_ERR_UNSUPPORTED;
    const size_t lds = (size_t)pl.region_bytes + (size_t)pl.max_rows * 4 + 16;
    auto kern = conv_mfma_i8_kernel<FW, PW, WF, WP>;
    static bool attr_done = false;   // per instantiation
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_LIMIT) != hipSuccess)
            return XNOR_ERR_HIP;
        attr_done = true;
    }
    dim3 grid((unsigned)((g.m_total + PT - 1) / PT), (unsigned)((g.k_out + FT - 1) / FT)), block(64 * WF * WP);
    if (grid.y > 65535u) return XNOR_ERR_UNSUPPORTED;
    kern<<<grid, block, lds, stream>>>(xbits, reinterpret_cast<const v4i *>(wmfma), K, alpha, out, dot_out, g, pl);
    return hip_status(hipGetLastError());
}

xnor_status launch_conv_mfma_i8(const uint32_t *xbits, const void *wmfma, const float *K,
                                const float *alpha, float *out, int32_t *dot_out,
                                const ConvGeom &g, hipStream_t stream)
{
    if (g.k_out <= 64)
        return launch_cfg<2, 2, 1, 4>(xbits, wmfma, K, alpha, out, dot_out, g, stream);
    return launch_cfg<2, 2, 2, 2>(xbits, wmfma, K, alpha, out, dot_out, g, stream);
}

}  // namespace xnor
