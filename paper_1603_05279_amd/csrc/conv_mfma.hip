// Binary convolution on the matrix cores (sec. 3.2).  The +-1 product-sum that XNOR + bitcount
// evaluates is the same integer as a dot product of the sign tensors with 0 at padded positions,
// so the convolution is run as an implicit GEMM
//     D[filter][pixel] = sum_{tap, channel} sW[filter][tap][channel] * sI[pixel + tap][channel]
// followed by the fused scaling by K and alpha.  Two operand encodings, same kernel:
//   I8: signs widened to int8 (+1, -1, 0), v_mfma_i32_32x32x32_i8, int32 accumulation;
//   F4: signs widened to 4-bit floats (E2M1 codes 0x2 = +1, 0xA = -1, 0x0 = 0),
//       v_mfma_scale_f32_32x32x64_f8f6f4 with unit scales.  Products are +-1 or 0 and the sums
//       stay far below 2^24, so the float accumulation is exact.
//
// Work split: a workgroup owns FT = 32*FW*WF filters x PT = 32*PW*WP consecutive output pixels
// (pixels flattened over image, row, column so small images still fill the tile).  Per channel
// chunk it widens the packed activation bits of the input rows its pixels touch (halo included,
// halo = 0) into LDS once; every tap then reads the same LDS image at a shifted offset.
// Weights come from the pre-widened image written by the weight packer, one contiguous KiB per
// 32-filter operand, prefetched several K-steps ahead in registers.  Filters are the M operand
// and pixels the N operand, so each lane of the result holds one pixel column: stores along a
// filter plane are contiguous across lanes.
#include "mfma_common.h"
#include <algorithm>
#include <atomic>
#include <type_traits>

namespace xnor {

// Sum of a KH x KW window of the staged matrix A (row pitch `pitch` floats), taps added in row-major order
// starting from +0: every read is issued before the first addition.
template <int KH, int KW> __device__ __forceinline__ float box_sum_lds(const float *ap, int pitch)
{
    float a[KH * KW];
#pragma unroll
    for (int dy = 0; dy < KH; ++dy)
#pragma unroll
        for (int dx = 0; dx < KW; ++dx) a[dy * KW + dx] = ap[dy * pitch + dx];
    float s = 0.0f;
#pragma unroll
    for (int t = 0; t < KH * KW; ++t) s += a[t];
    return s;
}

// Accumulator tiles of up to 8 result blocks leave room for two waves per SIMD (256 registers each).
// KS > 1: KS groups of WF x WP waves share the K loop of the same tile (group k takes the k-th run of steps) and add
// their accumulators through LDS at the end: more weight loads in flight and more waves for the staging where a
// problem offers few output tiles and a long K (fully connected layers).  Consecutive-record streams only.
template <int FMT, int FW, int PW, int WF, int WP, bool FUSE, bool LINEAR, bool POOL = false, int KS = 1>
__global__ __launch_bounds__(64 * WF * WP * KS, (FW * PW <= (FMT == 2 ? 6 : 8) ? 2 : 1)) void conv_mfma_kernel(
    const uint32_t *__restrict__ xbits, const v4i *__restrict__ wimg, uint32_t wimg_bytes,
    const float *__restrict__ K, const float *__restrict__ A, const float *__restrict__ alpha,
    float *__restrict__ out, int32_t *__restrict__ dot_out, ConvGeom g, MfmaPlan pl, FuseArgs fz)
{
    typedef Enc<FMT> E;
    // operands staged as they are (no sign bits to widen, no K): bfloat16 parts and int8 levels
    constexpr bool RAW = FMT == 2 || FMT == 3;
    typedef typename E::acc_t acc_t;
    static_assert(KS == 1 || (LINEAR && !FUSE && !POOL), "waves along K: plain epilogue, consecutive records");
    constexpr int NT = 64 * WF * WP * KS;
    constexpr int FT = 32 * FW * WF;
    constexpr int PT = 32 * PW * WP;
    // Weight prefetch depth.  Five steps pay off on long K loops; the 64-filter tiles serve layers
    // with short K loops and many workgroups, and the fused epilogue needs registers of its own:
    // there three steps keep more waves resident.
    // A wave tile of a single result block (fully connected layers: few output tiles, long K) issues one matrix
    // instruction per KiB of weights: only a deep ring keeps enough bytes in flight to cover the L2 latency.
    // The division-free staging loop costs four more registers at the kernel's peak (the end of the K loop).  The
    // 64 x 256 and 128 x 64 tilings sit exactly at a count where one more wave per SIMD fits (127 and 96): they keep
    // the general loop (measured: ResNet 64x56 41 -> 44 us with the fast loop).
    constexpr bool FAST_STAGING = !(FW == 2 && PW == 2 && WF == 1 && WP == 4) && !(FW == 1 && PW == 2 && WF == 4 && WP == 1);
    constexpr int DW = (FW * PW == 1 && FMT < 2 && !FUSE) ? 7 : (FUSE || FT <= 64 || FMT == 2) ? 3 : 5;      // (bfloat16 parts: a step is three times as long)
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    int *rowinfo = reinterpret_cast<int *>(lds + pl.region_bytes);
    int *xoff_tab = rowinfo + pl.max_rows;     // [(nsteps + KLOOP_TABLE_PAD) * BPS]
    float *a_lds = reinterpret_cast<float *>(xoff_tab + (pl.nsteps + KLOOP_TABLE_PAD) * E::BPS);   // [max_rows * wp], halo = 0
    float *ktile = a_lds + pl.max_rows * g.wp;                                   // [PT]
    float *asum_lds = ktile + PT;                                                // [WF][PT], fused epilogue only
    uint32_t *wtile_lds = reinterpret_cast<uint32_t *>(asum_lds + WF * PT);      // [PT][FT/32], fused epilogue only
    // sign byte -> operand bytes table, after everything else (16-byte aligned by the plan)
    const uint8_t *lut = lds + pl.lut_offset;

    // Workgroups go to the 8 XCDs round-robin by (linear) index, and every XCD has its own L2.
    //  - Usual case (activations outweigh weights): within every window of 64 pixel tiles each XCD
    //    takes a run of 8 consecutive ones, so that the output lines two neighbouring tiles both
    //    write in part (and the input rows they share) meet in one XCD's L2.  The last, incomplete
    //    window keeps the plain order: runs would load the XCDs unevenly there.
    //  - Weight-heavy problems (fully connected layers): all pixel tiles of one filter tile go to
    //    one XCD, so that each XCD fetches only its own filter tiles' weights from HBM instead of
    //    all eight fetching everything.  1-D grid: XCD = index % 8, filter tile = 8 * (slot /
    //    ptiles) + XCD, pixel tile = slot % ptiles, slot = index / 8.
    uint32_t ptile, ftile;
    if (pl.wmajor) {
        const uint32_t xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;
        ftile = (slot / (uint32_t)pl.ptiles) * 8u + xcd;
        ptile = slot % (uint32_t)pl.ptiles;
        if (ftile >= (uint32_t)pl.ftiles) return;
    } else {
        const uint32_t bx = blockIdx.x;
        const uint32_t win = (bx >> 6) << 6;
        ptile = win + 64u <= (uint32_t)pl.ptiles ? win + ((bx & 7u) << 3) + ((bx >> 3) & 7u) : bx;
        ftile = blockIdx.y;
        if (ptile >= (uint32_t)pl.ptiles) return;
    }
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, half = lane >> 5;
    const int wk = wave / (WF * WP);                  // the wave's run of K-steps (0 without waves along K)
    const int wf = (wave % (WF * WP)) % WF, wp = (wave % (WF * WP)) / WF;
    const int f0 = (int)ftile * FT;
    const uint32_t howo = (uint32_t)(g.ho * g.wo);
    // the tile's run of flattened output pixels [m0, m_end): PT consecutive ones, or (pooled epilogue) the
    // convolution rows under a group of pooled rows of one image
    uint32_t m0, m_end;
    uint32_t pool_img = 0;
    int pool_py0 = 0, pool_rows = 0;               // first pooled row and pooled rows of this tile
    if constexpr (POOL) {
        pool_img = pl.pool.div_groups.div(ptile);
        const int gi = (int)(ptile - pool_img * (uint32_t)pl.pool.groups);
        pool_py0 = gi * pl.pool.pr;
        pool_rows = min(pl.pool.pr, pl.pool.hpo - pool_py0);
        m0 = pool_img * howo + (uint32_t)(pool_py0 * pl.pool.sh * g.wo);
        m_end = m0 + (uint32_t)(((pool_rows - 1) * pl.pool.sh + pl.pool.ph) * g.wo);
    } else {
        m0 = ptile * (uint32_t)PT;
        m_end = min(m0 + (uint32_t)PT, (uint32_t)g.m_total);
    }
    const int ccw = pl.cc_words;
    const int nsteps = pl.nsteps;

    // padded input rows this tile touches: R = image*hp + padded row
    const uint32_t m_last = m_end - 1u;
    const uint32_t img_a = g.div_howo.div(m0), img_b = g.div_howo.div(m_last);
    const uint32_t oy_a = g.div_wo.div(m0 - img_a * howo), oy_b = g.div_wo.div(m_last - img_b * howo);
    const int r_lo = (int)(img_a * g.hp + oy_a * g.sh);
    const int r_hi = (int)(img_b * g.hp + oy_b * g.sh) + g.kh - 1;
    const int nrows = r_hi - r_lo + 1;

    E::build_lut(lds + pl.lut_offset, tid, NT);
    // alpha (fused epilogue: also scale and shift) of this workgroup's filters, staged once behind the
    // widening table ([FT] each); filters past the last one repeat it and are masked later
    float *par_lds = reinterpret_cast<float *>(lds + pl.lut_offset + E::LUT_BYTES);
    for (int t = tid; t < FT; t += NT) {
        const int kc = min(f0 + t, g.k_out - 1);
        par_lds[t] = alpha[kc];
        if constexpr (FUSE) {
            par_lds[FT + t] = fz.bn_scale ? fz.bn_scale[kc] : 1.0f;
            par_lds[2 * FT + t] = fz.bn_scale ? fz.bn_shift[kc] : 0.0f;
        }
    }
    for (int rr = tid; rr < nrows; rr += NT) {
        const uint32_t R = (uint32_t)(r_lo + rr);
        const uint32_t img = pl.div_hp.div(R);
        const int y = (int)(R - img * g.hp) - g.ph;
        // first pixel of the (real) input row, -1 for padding rows and the zero rows of a dilated input
        const uint32_t ry = g.div_dil_h.div_small((uint32_t)max(y, 0));
        const bool rv = y >= 0 && y < g.h && (int)ry * g.dil_h == y && (int)ry < g.real_h;
        rowinfo[rr] = rv ? (int)((img * g.real_h + ry) * g.real_w) : -1;
    }
    // LDS offset of every channel block of a chunk relative to a pixel's window origin:
    // block b = tap * ccw + word  ->  (dy*wp + dx)*ps + word*BPB
    {
        const int nblk = g.taps * ccw;
        for (int b = tid; b < (nsteps + KLOOP_TABLE_PAD) * E::BPS; b += NT) {     // padding repeats the last block
            const uint32_t bb = (uint32_t)min(b, nblk - 1);
            const uint32_t t = pl.div_ccw.div_small(bb);
            const uint32_t wl = bb - t * ccw;
            const uint32_t dy = g.div_kw.div_small(t);
            const uint32_t dx = t - dy * g.kw;
            xoff_tab[b] = (int)(dy * pl.row_pitch + dx * pl.ps + wl * E::BPB);
        }
    }
    // LDS byte offset of each of this lane's pixel columns (window origin in the padded frame)
    int pbase[PW];
#pragma unroll
    for (int j = 0; j < PW; ++j) {
        const uint32_t m = min(m0 + (uint32_t)((wp * PW + j) * 32 + l32), m_end - 1u);
        const uint32_t img = g.div_howo.div(m);
        const uint32_t pix = m - img * howo;
        const uint32_t oy = g.div_wo.div(pix), ox = pix - oy * g.wo;
        pbase[j] = ((int)(img * g.hp + oy * g.sh) - r_lo) * pl.row_pitch + (int)ox * g.sw * pl.ps +
                   (E::HALF_SPLIT ? 16 * half : 0);
    }
    // weight records of this wave's filter blocks: record index = fblk * recs_per_fblock + step record
    const int recs_per_fb = (g.taps * g.cw + E::BPS - 1) / E::BPS;
    // Weight records are fetched with buffer loads: scalar record offset + the lane's 16-byte slot,
    // so the K loop spends no vector registers or ALU work on weight addresses.
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<v4i *>(wimg), 0, (int)wimg_bytes, 0x00020000);
    const int wlane = lane * 16;
    const int zero_rec = (int)(wimg_bytes >> 10) - 1;      // the image ends with an all-zero record
    int wrec0[FW];
#pragma unroll
    for (int i = 0; i < FW; ++i) {
        const int fb = min(f0 / 32 + wf * FW + i, g.fblocks - 1);
        wrec0[i] = __builtin_amdgcn_readfirstlane(fb * recs_per_fb);
    }
    const int tab_lane = (E::HALF_SPLIT ? 0 : half);

    acc_t acc[FW][PW];
#pragma unroll
    for (int i = 0; i < FW; ++i)
#pragma unroll
        for (int j = 0; j < PW; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    const int steps_per_tap = pl.tap_jump ? ccw / E::BPS : 0x7fffffff;
    for (int wbase = 0; wbase < g.cw; wbase += ccw) {
        __syncthreads();   // tables visible / previous chunk fully consumed
        // the first words of the matrix A are requested before the activation words, so that the two round trips
        // to memory overlap
        constexpr int FA = FW * PW > 4 ? 2 : 0;       // (small tiles: the registers are worth more as a fourth wave per SIMD)
        float a_reg[FA + 1];
        const bool stageA = !RAW && wbase == 0 && !K;
        auto a_load = [&](int it) -> float {
            const uint32_t rr = pl.div_wp.div_small((uint32_t)it);
            const int xcol = it - (int)rr * g.wp - g.pw;
            const int rowbase = rowinfo[rr];
            const bool ok = rowbase >= 0 && xcol >= 0 && xcol < g.w;
            return ok ? A[(size_t)rowbase + xcol] : 0.0f;
        };
#pragma unroll
        for (int u = 0; u < FA; ++u) a_reg[u] = (stageA && tid + u * NT < nrows * g.wp) ? a_load(tid + u * NT) : 0.0f;
        if (!RAW && pl.dense == 1) {
          if constexpr (!RAW) {
            // 1x1 filter without padding: the tile's pixels are consecutive pixels of the input and their packed
            // words one contiguous, 16-byte aligned run of memory: four words per load, up to twelve loads in flight
            // (a fully connected layer's 36 words per thread in one round trip)
            constexpr int FD = FW * PW == 1 ? 12 : 4;     // (the one-block wave tiles of fully connected layers have the registers)
            const int nwords = (int)(m_end - m0) * ccw;
            const uint4 *src = reinterpret_cast<const uint4 *>(xbits + (size_t)m0 * g.cw);
            for (int i0 = tid * 4; i0 < nwords; i0 += NT * 4 * FD) {
                uint4 v[FD];
#pragma unroll
                for (int u = 0; u < FD; ++u) {
                    const int i = i0 + u * NT * 4;
                    v[u] = src[min(i, nwords - 4) >> 2];
                }
#pragma unroll
                for (int u = 0; u < FD; ++u) {
                    const int i = i0 + u * NT * 4;
                    if (i < nwords) {
                        const uint32_t px = pl.div_ccw.div_small((uint32_t)i);
                        const int wl = i - (int)px * ccw;
                        const uint32_t m = m0 + px;
                        const uint32_t R = g.div_wo.div(m);                 // image row of the pixel (h_out = h, w_out = w)
                        uint8_t *dst = lds + ((int)R - r_lo) * pl.row_pitch + (int)(m - R * g.wo) * pl.ps + wl * E::BPB;
                        const uint32_t wv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            E::widen_word_lut(dst + q * E::BPB, lut, wv[q], true, g.c - (wl + q) * 32);
                    }
                }
            }
          }
        } else if (!RAW && FAST_STAGING && pl.dense == 2) {
          if constexpr (!RAW && FAST_STAGING) {
            // (row, column, word) of the thread's current item, advanced by the stride's increments with carries
            const int items = nrows * g.wp * ccw;
            const uint32_t q0 = pl.div_ccw.div_small((uint32_t)tid);
            int wl = tid - (int)q0 * ccw;
            int rr = (int)pl.div_wp.div_small(q0);
            int xc = (int)q0 - rr * g.wp;
            int it = tid;
            // what one workgroup-wide stride of NT items adds to (word, column, row): wave-uniform
            const uint32_t dq = pl.div_ccw.div_small((uint32_t)NT);
            const int st_dwl = NT - (int)dq * ccw;
            const int st_drr = (int)pl.div_wp.div_small(dq);
            const int st_dx = (int)dq - st_drr * g.wp;
            const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<uint32_t *>(xbits), 0, (int)((uint32_t)(g.n * g.h * g.w) * (uint32_t)g.cw * 4u), 0x00020000);
            constexpr int FB = 8;
            for (; it < items;) {
                uint32_t bits[FB];
                int dst[FB];
                bool ok[FB];
#pragma unroll
                for (int u = 0; u < FB; ++u) {
                    const int rowbase = rowinfo[min(rr, nrows - 1)];
                    const int xv = xc - g.pw;
                    ok[u] = rowbase >= 0 && (uint32_t)xv < (uint32_t)g.w && it < items;
                    // word index (rowbase + xv) * cw + wbase + wl, in bytes; outside the image: beyond the buffer
                    const int woff = (int)__umul24((uint32_t)(rowbase + xv), (uint32_t)g.cw) + wbase + wl;
                    bits[u] = __builtin_amdgcn_raw_buffer_load_b32(xrsrc, ok[u] ? woff * 4 : (int)0x80000000u, 0, 0);
                    dst[u] = it < items ? (int)(__umul24((uint32_t)rr, (uint32_t)pl.row_pitch) +
                                                __umul24((uint32_t)xc, (uint32_t)pl.ps)) + wl * E::BPB
                                        : -1;
                    it += NT;
                    wl += st_dwl;
                    const int c1 = wl >= ccw ? 1 : 0;
                    wl -= c1 ? ccw : 0;
                    xc += st_dx + c1;
                    const int c2 = xc >= g.wp ? 1 : 0;
                    xc -= c2 ? g.wp : 0;
                    rr += st_drr + c2;
                }
#pragma unroll
                for (int u = 0; u < FB; ++u)
                    if (dst[u] >= 0) E::widen_word_lut(lds + dst[u], lut, bits[u], ok[u], 32);
            }
          }
        } else {
        const int items = nrows * g.wp * ccw;
        constexpr int FB = RAW ? 4 : 8;        // items in flight per thread: loads first, then widening (every batch costs one round trip to L2 or HBM)
        for (int it0 = tid; it0 < items; it0 += NT * FB) {
            uint32_t bits[FB];
            uint4 raw[FB][2];              // FMT 2: the 32-byte word itself
            int dst[FB], nch[FB];
            bool ok[FB];
#pragma unroll
            for (int u = 0; u < FB; ++u) {
                const int it = it0 + u * NT;
                const uint32_t itc = (uint32_t)min(it, items - 1);
                const uint32_t px = pl.div_ccw.div_small(itc);
                const int wl = (int)(itc - px * ccw);
                const uint32_t rr = pl.div_wp.div_small(px);
                const int xv = (int)(px - rr * g.wp) - g.pw;                 // column of the (virtual) input
                const int xcol = (int)g.div_dil_w.div_small((uint32_t)max(xv, 0));  // column of the real tensor
                const int rowbase = rowinfo[rr];
                ok[u] = rowbase >= 0 && xv >= 0 && xv < g.w && xcol * g.dil_w == xv && xcol < g.real_w;
                dst[u] = it < items ? (int)(rr * pl.row_pitch + (px - rr * g.wp) * pl.ps + wl * E::BPB) : -1;
                nch[u] = g.c - (wbase + wl) * 32;
                bits[u] = 0;
                if constexpr (RAW) {
                    raw[u][0] = raw[u][1] = make_uint4(0, 0, 0, 0);
                    if (ok[u]) {
                        const uint4 *src = reinterpret_cast<const uint4 *>(xbits) +
                                           (((size_t)rowbase + xcol) * g.cw + wbase + wl) * 2;
                        raw[u][0] = src[0];
                        raw[u][1] = src[1];
                    }
                } else {
                    if (ok[u]) bits[u] = xbits[((size_t)rowbase + xcol) * g.cw + wbase + wl];
                }
            }
#pragma unroll
            for (int u = 0; u < FB; ++u)
                if (dst[u] >= 0) {
                    if constexpr (RAW) {
                        *reinterpret_cast<uint4 *>(lds + dst[u]) = raw[u][0];
                        *reinterpret_cast<uint4 *>(lds + dst[u] + 16) = raw[u][1];
                    } else {
                        E::widen_word_lut(lds + dst[u], lut, bits[u], ok[u], nch[u]);
                    }
                }
        }
        }
        if (stageA) {
            // the matrix A of the same input rows (0 in the halo), for the K of this tile
#pragma unroll
            for (int u = 0; u < FA; ++u)
                if (tid + u * NT < nrows * g.wp) a_lds[tid + u * NT] = a_reg[u];
            for (int it = tid + FA * NT; it < nrows * g.wp; it += NT) a_lds[it] = a_load(it);
        }
        __syncthreads();
        // K of the tile's output pixels, an equal share per wave: the kh x kw taps of A in row-major order over the
        // staged rows (halo entries add +0.0f, the same bits as skipping them), divided by kh*kw
        constexpr int KPW = (PT + WF * WP * KS - 1) / (WF * WP * KS);
        if (!RAW && wbase == 0 && !K) for (int kt = wave * KPW + lane; kt < min((wave + 1) * KPW, PT); kt += 64) {
            const uint32_t m = min(m0 + (uint32_t)kt, m_end - 1u);
            const uint32_t img = g.div_howo.div(m);
            const uint32_t pix = m - img * howo;
            const uint32_t oy = g.div_wo.div(pix), ox = pix - oy * g.wo;
            const float *ap = a_lds + ((int)(img * g.hp + oy * g.sh) - r_lo) * g.wp + (int)ox * g.sw;
            // the common filters with every tap's read in flight at once (one LDS latency instead of one per group
            // of four taps); the additions keep the row-major order either way
            float s;
            if (g.kh == 3 && g.kw == 3) s = box_sum_lds<3, 3>(ap, g.wp);
            else if (g.kh == 5 && g.kw == 5) s = box_sum_lds<5, 5>(ap, g.wp);
            else if (g.kh == 1 && g.kw == 1) s = 0.0f + ap[0];
            else {
                s = 0.0f;
                for (int dy = 0; dy < g.kh; ++dy, ap += g.wp)
                    for (int dx0 = 0; dx0 < g.kw; dx0 += 4) {
                        float a[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) a[u] = ap[min(dx0 + u, g.kw - 1)];
#pragma unroll
                        for (int u = 0; u < 4; ++u) s += dx0 + u < g.kw ? a[u] : 0.0f;
                    }
            }
            ktile[kt] = s / (float)(g.kh * g.kw);
        }

        // ---- software-pipelined K loop over this chunk's steps --------------------------------
        // record of step s: rec0 + s + (s / steps_per_tap) * tap_jump
        if constexpr (LINEAR && KS > 1) {
            const int per = (nsteps + KS - 1) / KS;
            const int s0 = __builtin_amdgcn_readfirstlane(wk * per);
            const int ns = max(0, min(per, nsteps - s0));
            // (problems that take this form are all weights: an image read once per call, which passes every XCD's L2 on its
            // way and should not settle in the last-level cache: fully connected layer inside a step 27.3 -> 24.3 us)
            WStreamLinear<FW, 2> ws(wimg, wrec0, wbase / E::BPS + s0, ns, wlane);
            mfma_kloop<E, FW, PW, DW, 1>(acc, lds, pbase, xoff_tab + s0 * E::BPS, tab_lane, ws, ns);
        } else if constexpr (LINEAR) {      // the chunk holds every channel word: consecutive records
            WStreamLinear<FW> ws(wimg, wrec0, wbase / E::BPS, nsteps, wlane);
            mfma_kloop<E, FW, PW, DW, 1>(acc, lds, pbase, xoff_tab, tab_lane, ws, nsteps);
        } else {
            WStreamChunked<FW> ws(wrsrc, wrec0, zero_rec, wbase / E::BPS, nsteps, steps_per_tap, pl.tap_jump, wlane);
            mfma_kloop<E, FW, PW, DW, 1>(acc, lds, pbase, xoff_tab, tab_lane, ws, nsteps);
        }
    }
    // epilogue: out = float(dot) * K * alpha; result register v of a lane is filter row
    // 8*(v/4) + 4*half + v%4 of the 32-filter block, pixel column l32.  alpha of the lane's
    // filter rows is fetched once (clamped index, no branch), stores are predicated.
    if (!RAW && !K) __syncthreads();      // the K tile is complete
    if constexpr (KS > 1) {
        // the wave groups' partial sums (exact integers) meet in LDS, laid over the finished activation region
        // ([group - 1][wave][block][register][lane]: consecutive lanes, consecutive words); group 0 adds them in order
        __syncthreads();                  // every wave is done reading activations
        typedef typename std::remove_reference<decltype(acc[0][0][0])>::type elem_t;
        elem_t *redw = reinterpret_cast<elem_t *>(lds);
        const int slot = ((wk - 1) * WF * WP + (wave % (WF * WP))) * FW * PW;
        if (wk > 0) {
#pragma unroll
            for (int i = 0; i < FW; ++i)
#pragma unroll
                for (int j = 0; j < PW; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) redw[((slot + i * PW + j) * 16 + v) * 64 + lane] = acc[i][j][v];
        }
        __syncthreads();
        if (wk > 0) return;               // (no barrier follows in the plain epilogue)
#pragma unroll
        for (int k = 1; k < KS; ++k)
#pragma unroll
            for (int i = 0; i < FW; ++i)
#pragma unroll
                for (int j = 0; j < PW; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        acc[i][j][v] += redw[(((k - 1) * WF * WP + wave) * FW * PW + i * PW + j) * 16 * 64 + v * 64 + lane];
    }
    uint32_t pimg[PW], ppix[PW];
    float Km[PW];
    bool plive[PW];
#pragma unroll
    for (int j = 0; j < PW; ++j) {
        const int pl_idx = (wp * PW + j) * 32 + l32;
        const uint32_t m = m0 + (uint32_t)pl_idx;
        plive[j] = m < m_end;
        const uint32_t mc = plive[j] ? m : m_end - 1u;
        pimg[j] = g.div_howo.div(mc);
        ppix[j] = mc - pimg[j] * howo;
        Km[j] = RAW ? 1.0f : (K ? K[mc] : ktile[pl_idx]);      // real and k-bit activations carry no K
    }
    // Float (and optional integer) results leave through buffer stores: the resource starts at the
    // tile's first image, a lane's vector offset names its pixel (plus its half-wave's four rows),
    // the filter row is a scalar offset, so a store needs no per-lane address arithmetic.  Dead
    // pixel columns and rows past the last filter get an offset beyond the resource, which the
    // buffer bounds check discards.  (The host refuses shapes whose tile span exceeds 2 GiB.)
    const size_t img_elems = (size_t)g.k_out * howo;
    const uint32_t span = (uint32_t)min((size_t)(g.n - (int)img_a) * img_elems * 4, (size_t)0x7ffffff0);
    const uint32_t OOB = 0x80000000u;
    uint32_t voff[PW];
#pragma unroll
    for (int j = 0; j < PW; ++j)
        voff[j] = plive[j] ? (uint32_t)(((pimg[j] - img_a) * (uint32_t)img_elems + ppix[j] + 4u * half * howo) * 4u) : OOB;
    const int wf_s = __builtin_amdgcn_readfirstlane(wf);
    auto store_rows = [&](auto *dst, int i, int j, auto value_of) {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(dst + (size_t)img_a * img_elems, 0, (int)span, 0x00020000);
        const int row0 = f0 + (wf_s * FW + i) * 32;                 // wave-uniform
        if (row0 + 32 <= g.k_out && howo == 1u && (g.k_out & 3) == 0) {
            // planes of one pixel (fully connected layers): a lane's four consecutive filter rows are 16
            // contiguous, aligned bytes
#pragma unroll
            for (int q = 0; q < 4; ++q)
                __builtin_amdgcn_raw_buffer_store_b128(v4u{value_of(4 * q), value_of(4 * q + 1), value_of(4 * q + 2),
                                                           value_of(4 * q + 3)},
                                                       rs, (int)voff[j], (row0 + 8 * q) * 4, 0);
            return;
        }
        // Results larger than a quarter of the 256 MB last-level cache leave with the non-temporal hint (measured: a
        // 205 MB result 59 -> 44 us, 103 MB 42 -> 32 us, while 51 MB and smaller results are 10 us slower with it).
        // The cache policy is part of the instruction: one run of stores per policy, chosen by a uniform branch.
        auto rows = [&](auto aux) {
            constexpr int AUX = decltype(aux)::value;
            if (row0 + 32 <= g.k_out) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    __builtin_amdgcn_raw_buffer_store_b32(value_of(v), rs, (int)voff[j],
                                                          (row0 + 8 * (v >> 2) + (v & 3)) * (int)howo * 4, AUX);
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row0 + 8 * (v >> 2) + (v & 3);
                    const bool fin = row + 4 * half < g.k_out;
                    __builtin_amdgcn_raw_buffer_store_b32(value_of(v), rs, (int)(fin ? voff[j] : OOB),
                                                          min(row, g.k_out - 1) * (int)howo * 4, AUX);
                }
            }
        };
        if (pl.stream_out) rows(std::integral_constant<int, 2>{});
        else rows(std::integral_constant<int, 0>{});
    };
    if constexpr (POOL) {
    // Pooled epilogue: y = float(dot) * K * alpha (optionally max(y, 0)) of one filter block goes to a
    // per-wave LDS tile [32 filters][PT + 1 pixels] laid over the (finished) activation region; lanes
    // then take the maximum over the pooling windows and store the pooled rows of this tile.  LDS serves
    // one wave's instructions in order, so a wave's own writes are visible to its reads without a
    // workgroup barrier.  The maximum starts at -inf and skips NaN (maxNum).
    constexpr int YP = PT + 1;
    float al[FW][16];
#pragma unroll
    for (int i = 0; i < FW; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 a4 = *reinterpret_cast<const float4 *>(par_lds + (wf * FW + i) * 32 + 8 * q + 4 * half);
            al[i][4 * q] = a4.x; al[i][4 * q + 1] = a4.y; al[i][4 * q + 2] = a4.z; al[i][4 * q + 3] = a4.w;
        }
    __syncthreads();                              // every wave is done reading activations (and alpha is in registers)
    // 16 filter rows at a time (register groups v = 0..7, then 8..15): [16][PT + 1] floats per wave
    float *ystage = reinterpret_cast<float *>(lds) + (size_t)wave * 16 * YP;
    const PoolPlan &pp = pl.pool;
    const int npool = pool_rows * pp.wpo;         // pooled pixels of this tile
    // lanes -> (filter offset, pooled pixel): as many filters side by side as fit into the wave; a lane
    // keeps its pooled pixel and walks the filters in steps of nf, eight filters' window loads in flight
    const int nf = npool >= 64 ? 1 : min(64 / npool, 16);
    const int fo = npool >= 64 ? 0 : lane / npool;
    const int pq = lane - fo * npool;
    const int pstep = npool >= 64 ? 64 : npool;
    const bool lane_on = fo < nf;
    float *pooled = reinterpret_cast<float *>(out);
    const size_t plane = (size_t)pp.hpo * pp.wpo;
    // maxima of 8 filters (rows fb + u*nf + fo of the staged 16) over one pooled pixel's window
    auto window_max = [&](auto PHc, auto PWc, const float *win, const int (&roff)[8], float (&mx)[8]) {
        constexpr int CH = decltype(PHc)::value, CW = decltype(PWc)::value;       // 0: run-time window
        if constexpr (CH > 0) {
            float t[CH * CW][8];
#pragma unroll
            for (int dy = 0; dy < CH; ++dy)
#pragma unroll
                for (int dx = 0; dx < CW; ++dx)
#pragma unroll
                    for (int u = 0; u < 8; ++u) t[dy * CW + dx][u] = win[roff[u] + dy * g.wo + dx];
#pragma unroll
            for (int w9 = 0; w9 < CH * CW; ++w9)
#pragma unroll
                for (int u = 0; u < 8; ++u) mx[u] = __builtin_fmaxf(mx[u], t[w9][u]);
        } else {
            for (int dy = 0; dy < pp.ph; ++dy)
                for (int dx = 0; dx < pp.pw; ++dx) {
                    float t[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) t[u] = win[roff[u] + dy * g.wo + dx];
#pragma unroll
                    for (int u = 0; u < 8; ++u) mx[u] = __builtin_fmaxf(mx[u], t[u]);
                }
        }
    };
    const int wkind = (pp.ph == 3 && pp.pw == 3) ? 3 : (pp.ph == 2 && pp.pw == 2) ? 2 : 0;
#pragma unroll
    for (int i = 0; i < FW; ++i) {
#pragma unroll
        for (int hq = 0; hq < 2; ++hq) {          // filter rows 16*hq .. 16*hq + 15 of the block
#pragma unroll
            for (int j = 0; j < PW; ++j)
#pragma unroll
                for (int v8 = 0; v8 < 8; ++v8) {
                    const int v = 8 * hq + v8;
                    float y = E::to_float(acc[i][j], v) * Km[j] * al[i][v];
                    if (pp.relu) y = y > 0.0f ? y : 0.0f;
                    ystage[(8 * (v8 >> 2) + 4 * half + (v8 & 3)) * YP + (wp * PW + j) * 32 + l32] = y;
                }
            __builtin_amdgcn_wave_barrier();
            const int row0 = f0 + (wf * FW + i) * 32 + 16 * hq;
            const int nrow = min(16, g.k_out - row0);       // staged filters that exist (wave-uniform, may be <= 0)
            for (int q = pq; q < npool; q += pstep) {
                const uint32_t py = pp.div_wpo.div_small((uint32_t)q);
                const int px = q - (int)py * pp.wpo;
                const float *win = ystage + (int)py * pp.sh * g.wo + px * pp.sw;
                float *dst = pooled + ((size_t)pool_img * g.k_out + row0 + fo) * plane + (size_t)pool_py0 * pp.wpo + q;
                for (int fb = 0; fb < nrow; fb += 8 * nf) {       // wave-uniform trip count
                    int roff[8];
                    float mx[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        roff[u] = min(fb + u * nf + fo, 15) * YP;      // clamped: always inside the wave's tile
                        mx[u] = -__builtin_inff();
                    }
                    if (wkind == 3) window_max(std::integral_constant<int, 3>{}, std::integral_constant<int, 3>{}, win, roff, mx);
                    else if (wkind == 2) window_max(std::integral_constant<int, 2>{}, std::integral_constant<int, 2>{}, win, roff, mx);
                    else window_max(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, win, roff, mx);
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (lane_on && fb + u * nf + fo < nrow) dst[(size_t)(fb + u * nf) * plane] = mx[u];
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
    } else if constexpr (!FUSE) {
#pragma unroll
    for (int i = 0; i < FW; ++i) {
        float al[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {           // rows 8q + 4*half .. +3 of the block: one 16-byte read
            const float4 a4 = *reinterpret_cast<const float4 *>(par_lds + (wf * FW + i) * 32 + 8 * q + 4 * half);
            al[4 * q] = a4.x; al[4 * q + 1] = a4.y; al[4 * q + 2] = a4.z; al[4 * q + 3] = a4.w;
        }
#pragma unroll
        for (int j = 0; j < PW; ++j) {
            store_rows(out, i, j, [&](int v) {
                return __builtin_bit_cast(uint32_t, E::to_float(acc[i][j], v) * Km[j] * al[v]);
            });
            if (dot_out) store_rows(dot_out, i, j, [&](int v) { return (uint32_t)E::to_int(acc[i][j], v); });
        }
    }
    } else {
    // Fused epilogue: the next block's BatchNorm and BinActiv on y = float(dot) * K * alpha while it
    // is still in registers.  A lane holds 16 of the 32 filter rows of a block for one pixel; the
    // other 16 sit in the lane 32 further on, so one cross-half exchange completes the sign word
    // and the |z| sum of the block.  Exchanges run for every lane (dead pixel columns carry
    // clamped data); only the stores are predicated.
    const int cwn = g.fblocks;                    // words per pixel of the next layer's input
    constexpr int WT = FT / 32;                   // words per pixel this workgroup produces
    float asum[PW];
#pragma unroll
    for (int j = 0; j < PW; ++j) asum[j] = 0.0f;
#pragma unroll
    for (int i = 0; i < FW; ++i) {
        const int fblk = f0 / 32 + wf * FW + i;
        const int kb = fblk * 32 + 4 * half;
        float al[16], bs[16], bb[16];
        const bool whole = kb + 28 < g.k_out;     // all 16 rows of this lane exist (uniform per half-wave pair)
#pragma unroll
        for (int q = 0; q < 4; ++q) {           // rows 8q + 4*half .. +3 of the block: one 16-byte read each
            const int t = (wf * FW + i) * 32 + 8 * q + 4 * half;
            const float4 a4 = *reinterpret_cast<const float4 *>(par_lds + t);
            const float4 s4 = *reinterpret_cast<const float4 *>(par_lds + FT + t);
            const float4 b4 = *reinterpret_cast<const float4 *>(par_lds + 2 * FT + t);
            al[4 * q] = a4.x; al[4 * q + 1] = a4.y; al[4 * q + 2] = a4.z; al[4 * q + 3] = a4.w;
            bs[4 * q] = s4.x; bs[4 * q + 1] = s4.y; bs[4 * q + 2] = s4.z; bs[4 * q + 3] = s4.w;
            bb[4 * q] = b4.x; bb[4 * q + 1] = b4.y; bb[4 * q + 2] = b4.z; bb[4 * q + 3] = b4.w;
        }
#pragma unroll
        for (int j = 0; j < PW; ++j) {
            // sign word built at the rows' positions for half 0 (compile-time masks), moved to this
            // half's rows by one shift at the end
            uint32_t word = 0;
            float sabs = 0.0f;
            if (whole) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float y = E::to_float(acc[i][j], v) * Km[j] * al[v];
                    const float z = fmaf(y, bs[v], bb[v]);          // scale 1, shift 0 without normalisation: z == y
                    word |= z >= 0.0f ? 1u << (8 * (v >> 2) + (v & 3)) : 0u;
                    sabs += fabsf(z);
                }
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int kr = 8 * (v >> 2) + (v & 3);
                    const bool fin = kb + kr < g.k_out;             // rows past the last filter: bit 0, no |z|
                    const float y = E::to_float(acc[i][j], v) * Km[j] * al[v];
                    const float z = fmaf(y, bs[v], bb[v]);          // scale 1, shift 0 without normalisation: z == y
                    word |= (fin && z >= 0.0f) ? 1u << kr : 0u;
                    sabs += fin ? fabsf(z) : 0.0f;
                }
            }
            word <<= 4 * half;
            if (out)                              // callers that also want the real tensor
                store_rows(out, i, j, [&](int v) {
                    return __builtin_bit_cast(uint32_t, E::to_float(acc[i][j], v) * Km[j] * al[v]);
                });
            word |= (uint32_t)__shfl_xor((int)word, 32);
            asum[j] += sabs + __shfl_xor(sabs, 32);
            if (half == 0) wtile_lds[((wp * PW + j) * 32 + l32) * WT + wf * FW + i] = word;
        }
        __builtin_amdgcn_sched_barrier(0);        // one block's alpha / scale / shift live at a time
    }
    // |z| summed over this workgroup's filters: waves along the filter axis combine through LDS in
    // a fixed order.  Sign words leave through LDS too, so that consecutive threads write
    // consecutive words of a pixel (the whole tile is one contiguous run when the workgroup holds
    // every filter).
    if (half == 0) {
#pragma unroll
        for (int j = 0; j < PW; ++j) asum_lds[wf * PT + (wp * PW + j) * 32 + l32] = asum[j];
    }
    __syncthreads();
    for (int t = tid; t < PT * WT; t += NT) {
        const uint32_t m = m0 + (uint32_t)(t / WT);
        const int fblk = f0 / 32 + t % WT;
        if (m < (uint32_t)g.m_total && fblk < cwn) fz.xbits_next[(size_t)m * cwn + fblk] = wtile_lds[t];
    }
    for (int t = tid; t < PT; t += NT) {
        const uint32_t m = m0 + (uint32_t)t;
        if (m >= (uint32_t)g.m_total) continue;
        float sum = 0.0f;
#pragma unroll
        for (int q = 0; q < WF; ++q) sum += asum_lds[q * PT + t];
        if (pl.ftiles == 1) fz.A_next[m] = sum / (float)g.k_out;
        else fz.workspace[(size_t)ftile * g.m_total + m] = sum;
    }
    }
}

static const int LDS_LIMIT = 160 * 1024;

// fuse_rows: rows of PT words for the fused epilogue's |z| sums and sign words (0 without it)
// par_bytes: alpha (fused epilogue: also scale and shift) of the workgroup's filters
// channel words per K-step and bytes of the widening table of an operand format (Enc<fmt>::BPS, LUT_BYTES)
static constexpr int fmt_bps(int fmt) { return fmt == 1 ? 2 : fmt == 2 ? 3 : 1; }
static constexpr int fmt_lut_bytes(int fmt) { return fmt == 0 ? 512 * 8 : 0; }     // int8 operands only
static size_t plan_lds_bytes(const MfmaPlan &pl, int fmt, int wp, int PT, int fuse_rows, int par_bytes)
{
    const size_t rest = (size_t)pl.region_bytes + (size_t)pl.max_rows * 4 +
                        (size_t)((pl.nsteps + KLOOP_TABLE_PAD) * fmt_bps(fmt)) * 4 + (size_t)pl.max_rows * wp * 4 +
                        (size_t)PT * 4 * (1 + fuse_rows) + 16;
    return (rest + 15) / 16 * 16 + fmt_lut_bytes(fmt) + par_bytes;       // + the widening table
}
static int plan_lut_offset(const MfmaPlan &pl, int fmt, int wp, int PT, int fuse_rows, int par_bytes)
{
    return (int)(plan_lds_bytes(pl, fmt, wp, PT, fuse_rows, par_bytes) - fmt_lut_bytes(fmt) - par_bytes);
}

static bool make_plan(const ConvGeom &g, int PT, int fmt, int lds_budget, int fuse_rows, int par_bytes, MfmaPlan *pl,
                      int rows_override = 0, bool lone = false)
{
    const int bps = fmt_bps(fmt), bpb = fmt == 1 ? 16 : 32;
    const int rows = rows_override ? rows_override : worst_region_rows(g, PT, PT);
    for (int ccw = g.cw; ccw >= 1; --ccw) {
        if (g.cw % ccw) continue;
        // 4-bit operands take two channel words per step, bfloat16 parts three: chunks must keep the
        // words of a step together
        if (ccw != g.cw && (ccw % bps)) continue;
        const long long row_bytes = (long long)ccw * bpb;
        const long long ps = row_bytes + ((row_bytes / 16) % 2 == 0 ? 16 : 0);
        // LDS row pitch: at least wp pixels, padded so that stepping from the last output pixel of a row
        // to the first of the next continues the bank pattern of the steps within a row
        // (sh * pitch = wo * sw * ps modulo the 256-byte bank period): operand reads of a wave that
        // spans a row boundary then stay conflict-free
        long long pitch = (long long)g.wp * ps;
        for (int add = 0; add < 256; add += 16)
            if (((long long)g.sh * (pitch + add) - (long long)g.wo * g.sw * ps) % 256 == 0) { pitch += add; break; }
        const long long region = (long long)rows * pitch;
        pl->row_pitch = (int)pitch;
        pl->cc_words = ccw;
        pl->ps = (int)ps;
        pl->max_rows = rows;
        pl->nsteps = (g.taps * ccw + bps - 1) / bps;
        pl->tap_jump = (ccw == g.cw) ? 0 : (g.cw - ccw) / bps;
        if (region >= (1ll << 30)) continue;
        pl->region_bytes = (int)region;
        const long long total = (long long)plan_lds_bytes(*pl, fmt, g.wp, PT, fuse_rows, par_bytes);
        const bool last = ccw <= bps;
        // one chunk with all channel words keeps the weight records consecutive (the K loop without
        // bookkeeping) and saves the refills: worth up to half the CU's LDS (two workgroups per CU)
        // (`lone`: the launch has at most one workgroup per CU, which may then take nearly all of the CU's LDS)
        const long long whole = lone ? 156 * 1024 : 80 * 1024;
        const long long budget = ccw == g.cw ? (lds_budget > whole ? lds_budget : whole) : lds_budget;
        if (total > budget && !last) continue;
        if (total > LDS_LIMIT) return false;
        pl->div_wp = FastDiv::make((uint32_t)g.wp);
        pl->div_hp = FastDiv::make((uint32_t)g.hp);
        pl->div_ccw = FastDiv::make((uint32_t)ccw);
        pl->div_cw = FastDiv::make((uint32_t)g.cw);
        return true;
    }
    return false;
}

static std::atomic<int> g_tile_override{0};
static std::atomic<int> g_lds_budget{64 * 1024};
void set_mfma_tuning(int tile, int lds_budget)
{
    g_tile_override.store(tile, std::memory_order_relaxed);
    if (lds_budget > 0) g_lds_budget.store(lds_budget, std::memory_order_relaxed);
}

// Raises a kernel's dynamic LDS limit once per instantiation (the library drives one GPU per process).  Concurrent first calls may both
// set the attribute (the call is idempotent); the flag only ever goes from false to true.
template <class Kern> static xnor_status allow_full_lds(Kern kern, std::atomic<bool> &done)
{
    if (done.load(std::memory_order_acquire)) return XNOR_OK;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            LDS_LIMIT) != hipSuccess)
        return XNOR_ERR_HIP;
    done.store(true, std::memory_order_release);
    return XNOR_OK;
}

// second kernel of the fused epilogue when the filters span several workgroups:
// A_next[m] = (part[0][m] + part[1][m] + ...) / k_out, planes added in order
__global__ __launch_bounds__(256) void sum_planes_kernel(const float *__restrict__ part, float *__restrict__ A_next,
                                                        int m_total, int planes, float k_out)
{
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m >= m_total) return;
    float s = 0.0f;
    for (int p = 0; p < planes; ++p) s += part[(size_t)p * m_total + m];
    A_next[m] = s / k_out;
}

template <int FMT, int FW, int PW, int WF, int WP, bool FUSE, int KS = 1>
static xnor_status launch_cfg(const uint32_t *xbits, const void *wimg, const float *K, const float *A,
                              const float *alpha, float *out, int32_t *dot_out, const ConvGeom &g,
                              hipStream_t stream, const FuseArgs *fz)
{
    constexpr int FT = 32 * FW * WF, PT = 32 * PW * WP;
    // results are stored through a buffer resource with 32-bit offsets from the tile's first image
    const long long howo = (long long)g.ho * g.wo;
    if ((PT / howo + 2) * g.k_out * howo * 4 >= 0x7ffffff0LL) return XNOR_ERR_UNSUPPORTED;
    MfmaPlan pl;
    constexpr int FROWS = FUSE ? WF + FT / 32 : 0, PARB = (FUSE ? 3 : 1) * FT * 4;
    const long long wg_count = (long long)((g.m_total + PT - 1) / PT) * ((g.k_out + FT - 1) / FT);
    if (!make_plan(g, PT, FMT, g_lds_budget.load(std::memory_order_relaxed), FROWS, PARB, &pl, 0, wg_count <= 256))
        return XNOR_ERR_UNSUPPORTED;
    const size_t lds = plan_lds_bytes(pl, FMT, g.wp, PT, FROWS, PARB);
    pl.lut_offset = plan_lut_offset(pl, FMT, g.wp, PT, FROWS, PARB);
    // two builds of every tiling: weight records consecutive (one chunk holds all channel words) or not
    // (a chunk of a 1x1 filter is a run of consecutive records too)
    const bool linear = pl.tap_jump == 0 || g.taps == 1;
    // waves along K: consecutive weight records only, and the partial sums need the activation region's room
    if (KS > 1 && (!linear || (size_t)pl.region_bytes < (size_t)(KS - 1) * WF * WP * FW * PW * 16 * 64 * 4))
        return XNOR_ERR_UNSUPPORTED;
    auto kern = linear ? conv_mfma_kernel<FMT, FW, PW, WF, WP, FUSE, true, false, KS>
                       : conv_mfma_kernel<FMT, FW, PW, WF, WP, FUSE, KS != 1, false, KS>;
    static std::atomic<bool> attr_done[2];       // per instantiation (zero-initialised: false)
    if (xnor_status s = allow_full_lds(kern, attr_done[linear])) return s;
    pl.ptiles = (g.m_total + PT - 1) / PT;
    pl.ftiles = (g.k_out + FT - 1) / FT;
    pl.dense = FMT < 2 && g.taps == 1 && g.ph == 0 && g.pw == 0 && g.sh == 1 && g.sw == 1 && g.dil_h == 1 &&
               g.dil_w == 1 && pl.cc_words == g.cw && g.cw % 4 == 0;
    set_fast_staging(&pl, g, FMT);
    // (measured on whole benchmark steps: 64 MiB 382 us, 40 MiB 403 us, 120 MiB 408 us, never 428 us)
    pl.stream_out = (long long)g.m_total * g.k_out * 4 > (64ll << 20);
    // weight-heavy: the weight image outweighs the packed activations and there are filter tiles to spread
    pl.wmajor = pl.ftiles >= 8 && (long long)g.k_out * g.taps * g.c > 4LL * g.n * g.h * g.w * g.c;
    dim3 grid((unsigned)pl.ptiles, (unsigned)pl.ftiles), block(64 * WF * WP * KS);
    if (pl.wmajor) {
        const long long wg = (long long)((pl.ftiles + 7) / 8) * pl.ptiles * 8;
        if (wg > 0x7fffffffLL) return XNOR_ERR_UNSUPPORTED;
        grid = dim3((unsigned)wg, 1u);
    }
    if (grid.y > 65535u) return XNOR_ERR_UNSUPPORTED;
    const size_t img_bytes = FMT == 1 ? wimg_f4_bytes(g.k_out, g.c, g.taps)
                             : FMT == 2 ? wimg_bf16_bytes(g.k_out, g.cw / 3, g.taps)
                                        : wimg_i8_bytes(g.k_out, g.c, g.taps);
    if (img_bytes > 0x7fffffffull) return XNOR_ERR_UNSUPPORTED;
    kern<<<grid, block, lds, stream>>>(xbits, reinterpret_cast<const v4i *>(wimg), (uint32_t)img_bytes, K, A, alpha,
                                       out, dot_out, g, pl, FUSE ? *fz : FuseArgs{});
    if (xnor_status s = hip_status(hipGetLastError())) return s;
    if (FUSE && pl.ftiles > 1) {
        sum_planes_kernel<<<dim3((unsigned)((g.m_total + 255) / 256)), dim3(256), 0, stream>>>(
            fz->workspace, fz->A_next, g.m_total, pl.ftiles, (float)g.k_out);
        return hip_status(hipGetLastError());
    }
    return XNOR_OK;
}

// Pooled-epilogue launch of one tiling (4-bit operands): a pixel tile is a group of pooled rows of one image.
template <int FW, int PW, int WF, int WP>
static xnor_status launch_cfg_pool(const uint32_t *xbits, const void *wimg, const float *K, const float *A,
                                   const float *alpha, float *out_pool, const ConvGeom &g, const PoolPlan &pool,
                                   hipStream_t stream)
{
    constexpr int FT = 32 * FW * WF, PT = 32 * PW * WP, WAVES = WF * WP;
    MfmaPlan pl;
    const int conv_rows = (pool.pr - 1) * pool.sh + pool.ph;          // convolution rows under a tile
    if (conv_rows * g.wo > PT) return XNOR_ERR_UNSUPPORTED;
    if (!make_plan(g, PT, 1, g_lds_budget.load(std::memory_order_relaxed), 0, FT * 4, &pl, (conv_rows - 1) * g.sh + g.kh)) return XNOR_ERR_UNSUPPORTED;
    size_t lds = plan_lds_bytes(pl, 1, g.wp, PT, 0, FT * 4);
    pl.lut_offset = plan_lut_offset(pl, 1, g.wp, PT, 0, FT * 4);
    lds = std::max(lds, (size_t)WAVES * 16 * (PT + 1) * sizeof(float));       // the epilogue's per-wave y tiles
    if (lds > (size_t)LDS_LIMIT) return XNOR_ERR_UNSUPPORTED;
    const bool linear = pl.tap_jump == 0 || g.taps == 1;
    auto kern = linear ? conv_mfma_kernel<1, FW, PW, WF, WP, false, true, true>
                       : conv_mfma_kernel<1, FW, PW, WF, WP, false, false, true>;
    static std::atomic<bool> attr_done[2];
    if (xnor_status s = allow_full_lds(kern, attr_done[linear])) return s;
    const long long ptiles = (long long)g.n * pool.groups;
    if (ptiles > 0x7fffffffLL) return XNOR_ERR_UNSUPPORTED;
    pl.ptiles = (int)ptiles;
    pl.ftiles = (g.k_out + FT - 1) / FT;
    pl.wmajor = 0;
    pl.dense = 0;
    set_fast_staging(&pl, g, 1);
    pl.stream_out = 0;
    pl.pool = pool;
    if (pl.ftiles > 65535) return XNOR_ERR_UNSUPPORTED;
    const size_t img_bytes = wimg_f4_bytes(g.k_out, g.c, g.taps);
    if (img_bytes > 0x7fffffffull) return XNOR_ERR_UNSUPPORTED;
    // the XCD-aware tile order works on whole windows of 64 pixel tiles; the grid is not padded beyond ptiles
    kern<<<dim3((unsigned)pl.ptiles, (unsigned)pl.ftiles), dim3(64 * WAVES), lds, stream>>>(
        xbits, reinterpret_cast<const v4i *>(wimg), (uint32_t)img_bytes, K, A, alpha, out_pool, nullptr, g, pl, FuseArgs{});
    return hip_status(hipGetLastError());
}

xnor_status launch_conv_mfma_pool(const uint32_t *xbits, const void *wmfma, const float *K, const float *A,
                                  const float *alpha, float *out_pool, const ConvGeom &g, int ph, int pw, int sh,
                                  int sw, int relu, hipStream_t stream)
{
    if ((long long)g.c * g.taps >= (1ll << 24)) return XNOR_ERR_UNSUPPORTED;       // exact float accumulation
    PoolPlan pool;
    pool.ph = ph; pool.pw = pw; pool.sh = sh; pool.sw = sw; pool.relu = relu;
    pool.hpo = (g.ho - ph) / sh + 1;
    pool.wpo = (g.wo - pw) / sw + 1;
    pool.div_wpo = FastDiv::make((uint32_t)pool.wpo);
    // Tile: 256 filters x 96, 160 or 192 pixels.  Each holds as many pooled rows as its pixels allow; the
    // choice minimises (rounds of workgroups over the CUs' workgroup slots) x (pixels per tile), the smaller
    // tile on a tie.
    const int pts[3] = {96, 160, 192};
    int best = -1, best_pr = 0;
    long long best_cost = 0;
    const int ftiles = (g.k_out + 255) / 256;
    for (int t = 0; t < 3; ++t) {
        const int rows_fit = pts[t] / g.wo;                     // convolution rows a tile can hold
        if (rows_fit < ph) continue;
        const int pr = std::min((rows_fit - ph) / sh + 1, pool.hpo);
        const long long groups = (pool.hpo + pr - 1) / pr;
        const long long wgs = (long long)g.n * groups * ftiles;
        const long long slots = t == 0 ? 512 : 256;            // two workgroups of the 96-pixel tile share a CU
        const long long cost = (wgs + slots - 1) / slots * pts[t];
        if (best < 0 || cost < best_cost) { best = t; best_cost = cost; best_pr = pr; }
    }
    if (best < 0) return XNOR_ERR_UNSUPPORTED;                  // a pooling window's rows do not fit any tile
    pool.pr = best_pr;
    pool.groups = (pool.hpo + best_pr - 1) / best_pr;
    pool.div_groups = FastDiv::make((uint32_t)pool.groups);
    const uint8_t *img = static_cast<const uint8_t *>(wmfma) + wimg_i8_bytes(g.k_out, g.c, g.taps);
    switch (best) {
    case 0: return launch_cfg_pool<2, 3, 4, 1>(xbits, img, K, A, alpha, out_pool, g, pool, stream);
    case 1: return launch_cfg_pool<2, 5, 4, 1>(xbits, img, K, A, alpha, out_pool, g, pool, stream);
    default: return launch_cfg_pool<2, 6, 4, 1>(xbits, img, K, A, alpha, out_pool, g, pool, stream);
    }
}

template <int FMT>
static xnor_status launch_fmt(const uint32_t *xbits, const void *wimg, const float *K, const float *A,
                              const float *alpha, float *out, int32_t *dot_out, const ConvGeom &g,
                              hipStream_t stream, const FuseArgs *fz)
{
    int tile = g_tile_override.load(std::memory_order_relaxed);
    if (tile == 0) {
        // Measured rules (fp4, all benchmark layers).  Up to 64 filters: 64 x 256 when that still gives every
        // CU two workgroups, else 64 x 128; up to 128 filters: 128 x 64, else 64 x 128 (fused epilogue:
        // 64 x 256 or 128 x 128, so that one workgroup holds every filter).  129..256 filters: a tile that
        // holds every filter (weights stream through L1 once per pixel tile, the fused epilogue needs no
        // partial sums), 256 x 96 or 256 x 128, whichever leaves fewer CUs idle in its last round of
        // workgroups.  More filters: 256 x 128 when the filter count is a multiple of 256, else 128 x 128.
        // Problems with few output tiles (fully connected layers: few "pixels", long K) take the largest
        // smaller tile that still gives every CU a workgroup.
        auto wgs = [&](int ft, int pt) {
            return (long long)((g.m_total + pt - 1) / pt) * ((g.k_out + ft - 1) / ft);
        };
        const int cus = 256;
        auto waste = [&](long long w) { return (double)((w + cus - 1) / cus * cus) / (double)w; };
        if (FMT == 2) {
            // real activations (bfloat16 parts): the K loop is 24 times longer per channel, so the
            // tiles with the larger register blocks win wherever the filter count fills them
            // (measured): up to 64 filters 64 x 256, up to 128 filters 128 x 128; beyond that the tile
            // among 256 x 96 (when one tile holds every filter), 128 x 128 and 128 x 64 that leaves the
            // fewest CUs idle in the last round, the larger one on a tie
            if (g.k_out <= 64) tile = 2;
            else if (g.k_out <= 128) tile = 1;
            else {
                const double w4 = g.k_out <= 256 ? waste(wgs(256, 96)) : 1e30;
                const double w1 = waste(wgs(128, 128)), w13 = waste(wgs(128, 64));
                tile = w4 <= 1.03 * w1 && w4 <= 1.03 * w13 ? 4 : w1 <= 1.03 * w13 ? 1 : 13;
            }
        } else if (g.k_out <= 64) tile = (fz || wgs(64, 256) >= 2 * cus) ? 2 : 11;
        else if (g.k_out <= 128) tile = fz ? 1 : wgs(128, 64) >= 2 * cus ? 13 : 11;
        else if (g.k_out <= 256) tile = waste(wgs(256, 96)) <= waste(wgs(256, 128)) ? 4 : 5;
        else tile = g.k_out % 256 == 0 ? 5 : fz ? 13 : 1;      // (fused epilogue: 128 x 64 ahead of 128 x 128)
        const long long w0 = tile == 11 ? wgs(64, 128) : tile == 2 ? wgs(64, 256) : tile == 4 ? wgs(256, 96)
                             : tile == 5 ? wgs(256, 128) : tile == 13 ? wgs(128, 64) : wgs(128, 128);
        if (w0 < (FMT == 2 ? 128 : 160)) {
            if (wgs(64, 128) >= cus) tile = 11;
            else if (wgs(128, 64) >= cus) tile = 13;
            else tile = (FMT < 2 && !fz && g.taps == 1) ? 15 : 14;       // 128 x 32 (measured ahead of 64 x 64 at equal workgroup count), with eight waves where the records are consecutive
        }
    }
    // every tiling is built with and without the fused epilogue (bfloat16 parts and k-bit levels: without only)
#define XNOR_TILE_F(ID, FW, PW, WF, WP)                                                                   \
    case ID:                                                                                              \
        if constexpr (FMT < 2) {                                                                          \
            if (fz) return launch_cfg<FMT, FW, PW, WF, WP, true>(xbits, wimg, K, A, alpha, out, dot_out, g, stream, fz); \
        }                                                                                                 \
        return launch_cfg<FMT, FW, PW, WF, WP, false>(xbits, wimg, K, A, alpha, out, dot_out, g, stream, nullptr);
    switch (tile) {
        XNOR_TILE_F(1, 2, 2, 2, 2);   // 128 filters x 128 pixels
        XNOR_TILE_F(2, 2, 2, 1, 4);   //  64 x 256
        XNOR_TILE_F(4, 2, 3, 4, 1);   // 256 x  96
        XNOR_TILE_F(5, 2, 4, 4, 1);   // 256 x 128
        XNOR_TILE_F(11, 1, 2, 2, 2);  //  64 x 128
        XNOR_TILE_F(13, 1, 2, 4, 1);  // 128 x  64
        XNOR_TILE_F(14, 1, 1, 4, 1);  // 128 x  32
    case 15:                          // 128 x  32, two groups of four waves along K (no fused epilogue, packed-bit operands)
        if constexpr (FMT < 2) {
            if (!fz) {
                const xnor_status s = launch_cfg<FMT, 1, 1, 4, 1, false, 2>(xbits, wimg, K, A, alpha, out, dot_out, g, stream, nullptr);
                // (the library's own choice falls back to the four-wave form where this one does not apply)
                if (s != XNOR_ERR_UNSUPPORTED || g_tile_override.load(std::memory_order_relaxed) == 15) return s;
                return launch_cfg<FMT, 1, 1, 4, 1, false>(xbits, wimg, K, A, alpha, out, dot_out, g, stream, nullptr);
            }
        }
        return XNOR_ERR_UNSUPPORTED;
    default: return XNOR_ERR_UNSUPPORTED;
    }
#undef XNOR_TILE_F
}

xnor_status launch_conv_mfma(int fmt, const uint32_t *xbits, const void *wmfma, const float *K, const float *A,
                             const float *alpha, float *out, int32_t *dot_out,
                             const ConvGeom &g, hipStream_t stream, const FuseArgs *fz)
{
    const uint8_t *img = static_cast<const uint8_t *>(wmfma);
    // fmt 2: real activations in bfloat16 parts (xbits = 32-byte words, g.c = 32 x words per pixel,
    // wmfma = the +-1 bfloat16 record image alone); no K, no fused epilogue
    if (fmt == 2) return fz ? XNOR_ERR_UNSUPPORTED : launch_fmt<2>(xbits, img, nullptr, nullptr, alpha, out, nullptr, g, stream, nullptr);
    // fmt 3: int8 level numerators (xbits = 32-byte words of 32 channels, wmfma = an int8 record image); no K
    if (fmt == 3) return fz ? XNOR_ERR_UNSUPPORTED : launch_fmt<3>(xbits, img, nullptr, nullptr, alpha, out, dot_out, g, stream, nullptr);
    // float accumulation of the 4-bit path is exact while every sum stays below 2^24
    if (fmt != 0 && (long long)g.c * g.taps >= (1ll << 24)) return XNOR_ERR_UNSUPPORTED;
    if (fmt == 0) return launch_fmt<0>(xbits, img, K, A, alpha, out, dot_out, g, stream, fz);
    img += wimg_i8_bytes(g.k_out, g.c, g.taps);
    return launch_fmt<1>(xbits, img, K, A, alpha, out, dot_out, g, stream, fz);
}

}  // namespace xnor
