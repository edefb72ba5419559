// Pipelined, persistent form of the matrix-core binary convolution (sec. 3.2).
//
// Same arithmetic as conv_mfma.hip (implicit GEMM over sign operands widened on chip, fused
// K*alpha scaling); what changes is the schedule.  At the benchmark sizes one layer is only a few
// microseconds of matrix work per CU, about as long as writing its float output to HBM, so a
// workgroup that widens, multiplies and stores one after the other leaves the matrix cores idle
// for most of its life.  Here one workgroup per CU stays resident and splits into two roles:
//   waves 0-3 ("matrix" waves, one per SIMD) only run K loops;
//   waves 4-7 ("service" waves) widen the activation rows of the NEXT stage into the other half
//     of a double-buffered LDS image, and turn the results of the PREVIOUS output tile, handed
//     over through LDS as int16 (|dot| <= c*kh*kw < 32768), into scaled float stores.
// A stage is (pixel sub-tile, filter group, channel chunk); one workgroup barrier per stage.
// Output pixels are split evenly over the workgroups in units of 32, so every CU gets the same
// amount of matrix work whatever the image size.
#include "mfma_common.h"

namespace xnor {

#ifdef XNOR_TIMELINE
__device__ long long *g_timeline_pipe = nullptr;
#define XNOR_TLP(slot, who)                                                                   \
    do {                                                                                      \
        if (threadIdx.x == (who) && g_timeline_pipe)                                          \
            g_timeline_pipe[(size_t)blockIdx.x * 16 + (slot)] = wall_clock64();                \
    } while (0)
#else
#define XNOR_TLP(slot, who) do { } while (0)
#endif

struct PipePlan {
    int cc_words, ps, max_rows, region_bytes, nsteps, tap_jump;
    int nchunks;        // channel chunks per output tile
    int fgroups;        // filter groups of FG filters
    int total_frags;    // ceil(m_total / 32)
    int res_stride;     // bytes per filter row of a result buffer
    int off_x[2], off_res[2], off_alds[2], off_ktile[2], off_obase[2], off_xoff, off_alpha;   // LDS byte offsets
    FastDiv div_wp, div_hp, div_ccw;
};

template <int FMT, int FW, int PW, int WF, bool LINEAR>
__global__ __launch_bounds__(512, 2) void conv_mfma_pipe_kernel(
    const uint32_t *__restrict__ xbits, const v4i *__restrict__ wimg, uint32_t wimg_bytes,
    const float *__restrict__ K, const float *__restrict__ A, const float *__restrict__ alpha,
    float *__restrict__ out, int32_t *__restrict__ dot_out, ConvGeom g, PipePlan pl)
{
    typedef Enc<FMT> E;
    typedef typename E::acc_t acc_t;
    constexpr int WP = 4 / WF;                 // matrix waves along pixels
    constexpr int PT = 32 * PW * WP;           // pixels per sub-tile
    constexpr int FG = 32 * FW * WF;           // filters per group
    constexpr int NS_THREADS = 256;            // service threads
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    int *xoff_tab = reinterpret_cast<int *>(lds + pl.off_xoff);

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, half = lane >> 5;
    const bool matrix_role = wave < 4;
    const uint32_t howo = (uint32_t)(g.ho * g.wo);
    const int ccw = pl.cc_words;

    // this workgroup's share of the output pixels, in 32-pixel blocks
    const int fa = (int)(((long long)pl.total_frags * blockIdx.x) / gridDim.x);
    const int fb = (int)(((long long)pl.total_frags * (blockIdx.x + 1)) / gridDim.x);
    const int ntiles = (fb - fa + PW * WP - 1) / (PW * WP);
    if (ntiles == 0) return;
    const int nstages = ntiles * pl.fgroups * pl.nchunks;

    auto tile_m0 = [&](int T) -> uint32_t { return (uint32_t)(fa + T * PW * WP) * 32u; };
    auto tile_m1 = [&](int T) -> uint32_t {        // one past the last pixel of sub-tile T
        const uint32_t e = (uint32_t)min(fa + (T + 1) * PW * WP, fb) * 32u;
        return min(e, (uint32_t)g.m_total);
    };
    auto tile_rlo = [&](int T) -> int {            // first padded input row of sub-tile T
        const uint32_t m0 = tile_m0(T);
        const uint32_t img = g.div_howo.div(m0);
        const uint32_t oy = g.div_wo.div(m0 - img * howo);
        return (int)(img * g.hp + oy * g.sh);
    };
    auto tile_rows = [&](int T) -> int {
        const uint32_t ml = tile_m1(T) - 1u;
        const uint32_t img = g.div_howo.div(ml);
        const uint32_t oy = g.div_wo.div(ml - img * howo);
        return (int)(img * g.hp + oy * g.sh) + g.kh - 1 - tile_rlo(T) + 1;
    };

    // ---------------------------------------------------------------- service-wave routines
    XNOR_TLP(0, 0);
    // The service waves issue few instructions but sit on the same SIMDs as the matrix waves, whose
    // queued MFMAs would otherwise win the vector issue slot every time: give them priority.
    if (!matrix_role) __builtin_amdgcn_s_setprio(3);
    const int htid = tid - 256;
    // widen the packed bits of sub-tile T, channel chunk ch, into x buffer xb
    auto fill_x = [&](int T, int ch, int xb) {
        uint8_t *dstbase = lds + pl.off_x[xb];
        const int r_lo = tile_rlo(T), nrows = tile_rows(T);
        const int wbase = ch * ccw;
        const int items = nrows * g.wp * ccw;
        constexpr int FB = 4;
        for (int it0 = htid; it0 < items; it0 += NS_THREADS * FB) {
            uint32_t bits[FB];
            int dst[FB], nch[FB];
            bool ok[FB];
#pragma unroll
            for (int u = 0; u < FB; ++u) {
                const int it = it0 + u * NS_THREADS;
                const uint32_t itc = (uint32_t)min(it, items - 1);
                const uint32_t px = pl.div_ccw.div(itc);
                const int wl = (int)(itc - px * ccw);
                const uint32_t rr = pl.div_wp.div(px);
                const int xcol = (int)(px - rr * g.wp) - g.pw;
                const uint32_t R = (uint32_t)r_lo + rr;
                const uint32_t img = pl.div_hp.div(R);
                const int y = (int)(R - img * g.hp) - g.ph;
                ok[u] = y >= 0 && y < g.h && xcol >= 0 && xcol < g.w;
                dst[u] = it < items ? (int)(px * pl.ps + wl * E::BPB) : -1;
                nch[u] = g.c - (wbase + wl) * 32;
                bits[u] = 0;
                if (ok[u]) bits[u] = xbits[((size_t)(img * g.h + y) * g.w + xcol) * g.cw + wbase + wl];
            }
#pragma unroll
            for (int u = 0; u < FB; ++u)
                if (dst[u] >= 0) E::widen_word(dstbase + dst[u], bits[u], ok[u], nch[u]);
        }
    };
    // the matrix A over the same input rows (0 in the halo), for the K of sub-tile T
    auto stage_a = [&](int T) {
        if (K) return;
        float *a_lds = reinterpret_cast<float *>(lds + pl.off_alds[T & 1]);
        const int r_lo = tile_rlo(T), nrows = tile_rows(T);
        for (int it = htid; it < nrows * g.wp; it += NS_THREADS) {
            const uint32_t rr = pl.div_wp.div((uint32_t)it);
            const int xcol = it - (int)rr * g.wp - g.pw;
            const uint32_t R = (uint32_t)r_lo + rr;
            const uint32_t img = pl.div_hp.div(R);
            const int y = (int)(R - img * g.hp) - g.ph;
            const bool ok = y >= 0 && y < g.h && xcol >= 0 && xcol < g.w;
            a_lds[it] = ok ? A[(size_t)(img * g.h + y) * g.w + xcol] : 0.0f;
        }
    };
    // K and the output offset of every pixel of sub-tile T
    auto make_pixel_tables = [&](int T) {
        const float *a_lds = reinterpret_cast<const float *>(lds + pl.off_alds[T & 1]);
        float *ktile = reinterpret_cast<float *>(lds + pl.off_ktile[T & 1]);
        unsigned long long *obase = reinterpret_cast<unsigned long long *>(lds + pl.off_obase[T & 1]);
        const uint32_t m0 = tile_m0(T);
        const int r_lo = tile_rlo(T);
        for (int kt = htid; kt < PT; kt += NS_THREADS) {
            const uint32_t m = min(m0 + (uint32_t)kt, (uint32_t)g.m_total - 1u);
            const uint32_t img = g.div_howo.div(m);
            const uint32_t pix = m - img * howo;
            obase[kt] = (unsigned long long)img * g.k_out * howo + pix;
            if (K) {
                ktile[kt] = K[m];
            } else {
                // kh x kw taps of A in row-major order over the staged rows (halo adds +0.0f, the
                // same bits as skipping it), divided by kh*kw: identical to the box-filter kernel
                const uint32_t oy = g.div_wo.div(pix), ox = pix - oy * g.wo;
                const float *ap = a_lds + ((int)(img * g.hp + oy * g.sh) - r_lo) * g.wp + (int)ox * g.sw;
                float s = 0.0f;
                for (int dy = 0; dy < g.kh; ++dy, ap += g.wp)
                    for (int dx0 = 0; dx0 < g.kw; dx0 += 4) {
                        float a[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) a[u] = ap[min(dx0 + u, g.kw - 1)];
#pragma unroll
                        for (int u = 0; u < 4; ++u) s += dx0 + u < g.kw ? a[u] : 0.0f;
                    }
                ktile[kt] = s / (float)(g.kh * g.kw);
            }
        }
    };
    // out = float(dot) * K * alpha for output tile (T, fg), results read from result buffer rb.
    // A lane takes four consecutive pixels of one filter row and writes them with one 16-byte
    // store when they are four consecutive floats of the output (same image, inside the tile);
    // a whole output tile is then a dozen store instructions per wave, all in flight at once.
    // Everything a lane needs comes from LDS: a vector load in here would wait for the stores
    // before it (loads and stores share one completion counter on this chip).
    auto drain = [&](int T, int fg, int rb) {
        typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
        typedef int i4u __attribute__((ext_vector_type(4), aligned(4)));
        constexpr int PQ = PT / 4;                 // pixel quads per filter row
        const uint8_t *res = lds + pl.off_res[rb];
        const float *ktile = reinterpret_cast<const float *>(lds + pl.off_ktile[T & 1]);
        const unsigned long long *obase = reinterpret_cast<const unsigned long long *>(lds + pl.off_obase[T & 1]);
        const float *alpha_lds = reinterpret_cast<const float *>(lds + pl.off_alpha);
        const int npx = (int)(tile_m1(T) - tile_m0(T));
        const int f0 = fg * FG;
        const int nf = min(FG, g.k_out - f0);
        const int items = nf * PQ;
        for (int it = htid; it < items; it += NS_THREADS) {
            const int row = it / PQ, px0 = (it - row * PQ) * 4;
            if (px0 >= npx) continue;
            const int2 d2 = *reinterpret_cast<const int2 *>(res + (size_t)row * pl.res_stride + px0 * 2);
            const float4 k4 = *reinterpret_cast<const float4 *>(ktile + px0);
            const float al = alpha_lds[f0 + row];
            const int last = min(px0 + 3, npx - 1);
            const unsigned long long ob0 = obase[px0], ob3 = obase[last];
            const int dot[4] = {(int)(short)(d2.x & 0xffff), d2.x >> 16, (int)(short)(d2.y & 0xffff), d2.y >> 16};
            const float kk[4] = {k4.x, k4.y, k4.z, k4.w};
            float y[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) y[u] = (float)dot[u] * kk[u] * al;
            const size_t frow = (size_t)(f0 + row) * howo;
            if (px0 + 3 < npx && ob3 - ob0 == 3ull) {
                *reinterpret_cast<f4u *>(out + ob0 + frow) = f4u{y[0], y[1], y[2], y[3]};
                if (dot_out) *reinterpret_cast<i4u *>(dot_out + ob0 + frow) = i4u{dot[0], dot[1], dot[2], dot[3]};
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (px0 + u < npx) {
                        const size_t o = (size_t)obase[px0 + u] + frow;
                        out[o] = y[u];
                        if (dot_out) dot_out[o] = dot[u];
                    }
            }
        }
    };

    // ---------------------------------------------------------------- prologue
    {   // LDS offset of every channel block of a chunk relative to a pixel's window origin
        const int nblk = g.taps * ccw;
        for (int b = tid; b < (pl.nsteps + KLOOP_TABLE_PAD) * E::BPS; b += 512) {
            const uint32_t bb = (uint32_t)min(b, nblk - 1);
            const uint32_t t = pl.div_ccw.div(bb);
            const uint32_t wl = bb - t * ccw;
            const uint32_t dy = g.div_kw.div(t);
            const uint32_t dx = t - dy * g.kw;
            xoff_tab[b] = (int)((dy * g.wp + dx) * pl.ps + wl * E::BPB);
        }
    }
    {   // every filter's alpha, for the drains
        float *alpha_lds = reinterpret_cast<float *>(lds + pl.off_alpha);
        for (int f = tid; f < g.k_out; f += 512) alpha_lds[f] = alpha[f];
    }
    if (!matrix_role) {
        fill_x(0, 0, 0);
        stage_a(0);
    }
    __syncthreads();
    XNOR_TLP(1, 0);

    // ---------------------------------------------------------------- matrix-wave state
    const int mw = wave & 3;
    const int wf = mw % WF, wp = mw / WF;
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<v4i *>(wimg), 0, (int)wimg_bytes, 0x00020000);
    const int wlane = lane * 16;
    const int zero_rec = (int)(wimg_bytes >> 10) - 1;
    const int recs_per_fb = E::BPS == 1 ? g.taps * g.cw : (g.taps * g.cw + 1) / 2;
    const int tab_lane = (E::BPS == 2 ? half : 0);
    const int steps_per_tap = pl.tap_jump ? ccw / E::BPS : 0x7fffffff;
    int pbase[PW];
    acc_t acc[FW][PW];

    // ---------------------------------------------------------------- stage loop
    int T = 0, fg = 0, ch = 0;      // current stage
    int xcur = 0;                   // x buffer the current stage reads
    int rt = 0;                     // output tiles completed so far (selects the result buffer)
    int pend_T = -1, pend_fg = 0, pend_rb = 0;   // output tile waiting to be drained
    for (int st = 0; st < nstages; ++st) {
        // next stage
        int Tn = T, fgn = fg, chn = ch + 1;
        if (chn == pl.nchunks) { chn = 0; ++fgn; }
        if (fgn == pl.fgroups) { fgn = 0; ++Tn; }
        const bool has_next = st + 1 < nstages;
        const bool refill = has_next && (pl.nchunks > 1 || Tn != T);
        const bool completes = ch == pl.nchunks - 1;

        if (matrix_role) {
            if (fg == 0 && ch == 0) {
                const uint32_t m0 = tile_m0(T);
                const int r_lo = tile_rlo(T);
#pragma unroll
                for (int j = 0; j < PW; ++j) {
                    const uint32_t m = min(m0 + (uint32_t)((wp * PW + j) * 32 + l32), (uint32_t)g.m_total - 1u);
                    const uint32_t img = g.div_howo.div(m);
                    const uint32_t pix = m - img * howo;
                    const uint32_t oy = g.div_wo.div(pix), ox = pix - oy * g.wo;
                    pbase[j] = (((int)(img * g.hp + oy * g.sh) - r_lo) * g.wp + (int)ox * g.sw) * pl.ps +
                               (E::BPS == 1 ? 16 * half : 0);
                }
            }
            if (ch == 0) {
#pragma unroll
                for (int i = 0; i < FW; ++i)
#pragma unroll
                    for (int j = 0; j < PW; ++j)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
            }
            int wrec0[FW];
#pragma unroll
            for (int i = 0; i < FW; ++i) {
                const int fblk = min(fg * (FG / 32) + wf * FW + i, g.fblocks - 1);
                wrec0[i] = __builtin_amdgcn_readfirstlane(fblk * recs_per_fb);
            }
            if (st == 0) XNOR_TLP(8, 0);
            if (st == 1) XNOR_TLP(10, 0);
            if constexpr (LINEAR) {
                WStreamLinear<FW> ws(wimg, wrec0, 0, pl.nsteps, wlane);
                mfma_kloop<E, FW, PW, 5, 2>(acc, lds + pl.off_x[xcur], pbase, xoff_tab, tab_lane, ws, pl.nsteps);
            } else {
                WStreamChunked<FW> ws(wrsrc, wrec0, zero_rec, (ch * ccw) / E::BPS, pl.nsteps, steps_per_tap,
                                      pl.tap_jump, wlane);
                mfma_kloop<E, FW, PW, 5, 2>(acc, lds + pl.off_x[xcur], pbase, xoff_tab, tab_lane, ws, pl.nsteps);
            }
            if (st == 0) XNOR_TLP(9, 0);
            if (st == 1) XNOR_TLP(11, 0);
            if (completes) {
                // hand the integers to the service waves: res[filter row][pixel] as int16
                uint8_t *res = lds + pl.off_res[rt & 1];
#pragma unroll
                for (int i = 0; i < FW; ++i)
#pragma unroll
                    for (int j = 0; j < PW; ++j) {
                        const int px = (wp * PW + j) * 32 + l32;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int frow = (wf * FW + i) * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                            *reinterpret_cast<int16_t *>(res + (size_t)frow * pl.res_stride + px * 2) =
                                (int16_t)E::to_int(acc[i][j], v);
                        }
                    }
            }
        } else {
            // stores first: they complete on their own while the next stage is prepared
            if (pend_T >= 0) drain(pend_T, pend_fg, pend_rb);
            if (st == 1) XNOR_TLP(12, 256);
            if (refill) fill_x(Tn, chn, xcur ^ 1);
            if (st == 0) XNOR_TLP(13, 256);
            if (has_next && Tn != T) stage_a(Tn);
            if (st == 0) XNOR_TLP(14, 256);
            if (fg == 0 && ch == 0) make_pixel_tables(T);
        }
        if (st == 0) { XNOR_TLP(2, 0); XNOR_TLP(3, 256); }
        if (st == 1) { XNOR_TLP(4, 0); XNOR_TLP(5, 256); }
        // bookkeeping common to both roles (uniform)
        pend_T = -1;
        if (completes) { pend_T = T; pend_fg = fg; pend_rb = rt & 1; ++rt; }
        if (refill) xcur ^= 1;
        T = Tn; fg = fgn; ch = chn;
        __syncthreads();
    }
    XNOR_TLP(6, 0);
    if (!matrix_role && pend_T >= 0) drain(pend_T, pend_fg, pend_rb);
    XNOR_TLP(7, 256);
}

#ifdef XNOR_TIMELINE
extern "C" int xnor_debug_timeline_pipe(long long *buf)
{
    return hipMemcpyToSymbol(HIP_SYMBOL(g_timeline_pipe), &buf, sizeof(buf)) == hipSuccess ? 0 : -5;
}
#endif

static const int PIPE_LDS_LIMIT = 160 * 1024;

static bool make_pipe_plan(const ConvGeom &g, int fmt, int PT, int FG, PipePlan *pl, size_t *lds_bytes)
{
    const int bps = fmt == 0 ? 1 : 2, bpb = fmt == 0 ? 32 : 16;
    if ((long long)g.c * g.taps >= 32768) return false;       // results travel as int16
    const int rows = worst_region_rows(g, PT, 32);
    // result rows: PT int16 plus padding so the two half-waves (rows f and f+4) hit different banks
    int res_stride = PT * 2;
    while ((res_stride / 4) % 8 != 4) res_stride += 4;
    const long long res_bytes = (long long)FG * res_stride;
    for (int ccw = g.cw; ccw >= 1; --ccw) {
        if (g.cw % ccw) continue;
        if (bps == 2 && ccw != g.cw && (ccw % 2)) continue;
        const long long row_bytes = (long long)ccw * bpb;
        const long long ps = row_bytes + ((row_bytes / 16) % 2 == 0 ? 16 : 0);
        const long long region = ((long long)rows * g.wp * ps + 15) / 16 * 16;
        const int nsteps = (g.taps * ccw + bps - 1) / bps;
        const long long alds = ((long long)rows * g.wp * 4 + 15) / 16 * 16;
        long long off = 0;
        pl->off_x[0] = (int)off; off += region;
        pl->off_x[1] = (int)off; off += region;
        pl->off_res[0] = (int)off; off += res_bytes;
        pl->off_res[1] = (int)off; off += res_bytes;
        pl->off_alds[0] = (int)off; off += alds;
        pl->off_alds[1] = (int)off; off += alds;
        pl->off_ktile[0] = (int)off; off += PT * 4;
        pl->off_ktile[1] = (int)off; off += PT * 4;
        pl->off_obase[0] = (int)off; off += PT * 8;
        pl->off_obase[1] = (int)off; off += PT * 8;
        pl->off_xoff = (int)off; off += ((long long)(nsteps + KLOOP_TABLE_PAD) * bps * 4 + 31) / 16 * 16;
        pl->off_alpha = (int)off; off += ((long long)g.k_out * 4 + 15) / 16 * 16;
        if (off > PIPE_LDS_LIMIT) continue;
        pl->cc_words = ccw;
        pl->ps = (int)ps;
        pl->max_rows = rows;
        pl->region_bytes = (int)region;
        pl->nsteps = nsteps;
        pl->tap_jump = (ccw == g.cw) ? 0 : (g.cw - ccw) / bps;
        pl->nchunks = g.cw / ccw;
        pl->fgroups = (g.k_out + FG - 1) / FG;
        pl->total_frags = (g.m_total + 31) / 32;
        pl->res_stride = res_stride;
        pl->div_wp = FastDiv::make((uint32_t)g.wp);
        pl->div_hp = FastDiv::make((uint32_t)g.hp);
        pl->div_ccw = FastDiv::make((uint32_t)ccw);
        *lds_bytes = (size_t)off;
        return true;
    }
    return false;
}

static int cu_count()
{
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
    }
    return n;
}

template <int FMT, int FW, int PW, int WF>
static xnor_status launch_pipe_cfg(const uint32_t *xbits, const void *wimg, size_t img_bytes, const float *K,
                                   const float *A, const float *alpha, float *out, int32_t *dot_out,
                                   const ConvGeom &g, hipStream_t stream)
{
    constexpr int PT = 32 * PW * (4 / WF), FG = 32 * FW * WF;
    PipePlan pl;
    size_t lds = 0;
    if (!make_pipe_plan(g, FMT, PT, FG, &pl, &lds)) return XNOR_ERR_UNSUPPORTED;
    const bool linear = pl.tap_jump == 0;
    auto kern = linear ? conv_mfma_pipe_kernel<FMT, FW, PW, WF, true> : conv_mfma_pipe_kernel<FMT, FW, PW, WF, false>;
    static bool attr_done[2] = {false, false};
    if (!attr_done[linear]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, PIPE_LDS_LIMIT) != hipSuccess)
            return XNOR_ERR_HIP;
        attr_done[linear] = true;
    }
    const int wgs = min(cu_count(), pl.total_frags);
    kern<<<dim3((unsigned)wgs), dim3(512), lds, stream>>>(xbits, reinterpret_cast<const v4i *>(wimg),
                                                         (uint32_t)img_bytes, K, A, alpha, out, dot_out, g, pl);
    return hip_status(hipGetLastError());
}

xnor_status launch_conv_mfma_pipe(int fmt, const uint32_t *xbits, const void *wmfma, const float *K,
                                  const float *A, const float *alpha, float *out, int32_t *dot_out,
                                  const ConvGeom &g, hipStream_t stream)
{
    const uint8_t *img = static_cast<const uint8_t *>(wmfma);
    const size_t i8 = wimg_i8_bytes(g.k_out, g.c, g.taps), f4 = wimg_f4_bytes(g.k_out, g.c, g.taps);
    const size_t img_bytes = fmt == 0 ? i8 : f4;
    if (img_bytes > 0x7fffffffull) return XNOR_ERR_UNSUPPORTED;
    if (fmt != 0) img += i8;
    // matrix waves along filters (4, 2 or 1; the rest go along pixels): the split that pads the
    // filter count least, larger splits first on ties
    int WFv = 4;
    long long best = -1;
    for (int cand : {4, 2, 1}) {
        const int fgc = 64 * cand;
        const long long padded = (long long)((g.k_out + fgc - 1) / fgc) * fgc;
        if (best < 0 || padded < best) { best = padded; WFv = cand; }
    }
#define XNOR_PIPE(F, WFC) \
    return launch_pipe_cfg<F, 2, 3, WFC>(xbits, img, img_bytes, K, A, alpha, out, dot_out, g, stream)
    if (fmt == 0) {
        if (WFv == 1) XNOR_PIPE(0, 1);
        if (WFv == 2) XNOR_PIPE(0, 2);
        XNOR_PIPE(0, 4);
    } else {
        if (WFv == 1) XNOR_PIPE(1, 1);
        if (WFv == 2) XNOR_PIPE(1, 2);
        XNOR_PIPE(1, 4);
    }
#undef XNOR_PIPE
}

}  // namespace xnor
