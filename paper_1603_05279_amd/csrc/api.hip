// C ABI of libxnor: argument validation and dispatch.  Declarations and contracts: include/xnor.h.
#include "xnor_internal.h"
#include <mutex>

using namespace xnor;

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Validates a descriptor and derives the kernel geometry.
xnor_status make_geom(const xnor_conv_desc *d, ConvGeom *g)
{
    if (!d) return XNOR_ERR_NULL;
    if (d->n <= 0 || d->c <= 0 || d->h_in <= 0 || d->w_in <= 0 || d->k_out <= 0 || d->kh <= 0 ||
        d->kw <= 0 || d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0)
        return XNOR_ERR_SHAPE;
    const long long hp = (long long)d->h_in + 2LL * d->pad_h, wp = (long long)d->w_in + 2LL * d->pad_w;
    if (d->kh > hp || d->kw > wp) return XNOR_ERR_SHAPE;
    if (d->pad_h >= d->kh || d->pad_w >= d->kw) return XNOR_ERR_UNSUPPORTED;  // windows made of padding only
    const long long ho = (hp - d->kh) / d->stride_h + 1, wo = (wp - d->kw) / d->stride_w + 1;
    const long long cw = ((long long)d->c + 31) / 32;
    const long long lim = 0x7fffffffLL;
    const long long m = (long long)d->n * ho * wo;
    if (m > lim || m * d->k_out > (lim << 4) || (long long)d->n * d->h_in * d->w_in * cw > lim ||
        (long long)d->n * hp > lim || (long long)d->k_out * d->kh * d->kw * cw > lim ||
        hp > 65535 || wp > 65535 || (long long)d->kh * d->kw > 4096)
        return XNOR_ERR_SHAPE;
    g->n = d->n; g->c = d->c; g->h = d->h_in; g->w = d->w_in;
    g->k_out = d->k_out; g->kh = d->kh; g->kw = d->kw;
    g->sh = d->stride_h; g->sw = d->stride_w; g->ph = d->pad_h; g->pw = d->pad_w;
    g->ho = (int)ho; g->wo = (int)wo; g->cw = (int)cw; g->taps = d->kh * d->kw;
    g->hp = (int)hp; g->wp = (int)wp; g->m_total = (int)m;
    g->fblocks = (d->k_out + 31) / 32;
    g->div_wo = FastDiv::make((uint32_t)wo);
    g->div_howo = FastDiv::make((uint32_t)(ho * wo));
    g->div_kw = FastDiv::make((uint32_t)d->kw);
    g->dil_h = g->dil_w = 1;
    g->real_h = g->h; g->real_w = g->w;
    g->div_dil_h = g->div_dil_w = FastDiv::make(1u);
    return XNOR_OK;
}

xnor_status check_bn(const float *bn_scale, const float *bn_shift)
{
    if ((bn_scale == nullptr) != (bn_shift == nullptr)) return XNOR_ERR_NULL;
    if (!aligned16(bn_scale) || !aligned16(bn_shift)) return XNOR_ERR_ALIGN;
    return XNOR_OK;
}

}  // namespace

extern "C" {

int xnor_words_per_pixel(int c) { return c > 0 ? (c + 31) / 32 : 0; }

int xnor_output_hw(const xnor_conv_desc *d, int *h_out, int *w_out)
{
    ConvGeom g;
    const xnor_status s = make_geom(d, &g);
    if (s != XNOR_OK) return s;
    if (h_out) *h_out = g.ho;
    if (w_out) *w_out = g.wo;
    return XNOR_OK;
}

const char *xnor_status_string(int status)
{
    switch (status) {
    case XNOR_OK: return "ok";
    case XNOR_ERR_NULL: return "a required pointer is NULL";
    case XNOR_ERR_SHAPE: return "invalid shape";
    case XNOR_ERR_UNSUPPORTED: return "unsupported configuration";
    case XNOR_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case XNOR_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

size_t xnor_wmfma_bytes(int k_out, int c, int kh, int kw)
{
    if (k_out <= 0 || c <= 0 || kh <= 0 || kw <= 0) return 0;
    if ((long long)kh * kw > 4096) return 0;
    return wimg_i8_bytes(k_out, c, kh * kw) + wimg_f4_bytes(k_out, c, kh * kw) + wimg_pop_bytes(k_out, c, kh * kw);
}

int xnor_set_tuning(int mfma_tile, int lds_budget_bytes)
{
    if (mfma_tile < 0 || mfma_tile > 15 || lds_budget_bytes < 0 || lds_budget_bytes > 160 * 1024)
        return XNOR_ERR_UNSUPPORTED;
    set_mfma_tuning(mfma_tile, lds_budget_bytes);
    return XNOR_OK;
}

int xnor_binarize_pack(const float *x, const float *bn_scale, const float *bn_shift,
                       uint32_t *xbits, int n, int c, int h, int w, void *hip_stream)
{
    if (!x || !xbits) return XNOR_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return XNOR_ERR_SHAPE;
    if ((long long)h * w > 0x7fffffffLL || (long long)n * h * w * ((c + 31) / 32) > 0x7fffffffLL)
        return XNOR_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(xbits)) return XNOR_ERR_ALIGN;
    if (xnor_status s = check_bn(bn_scale, bn_shift)) return s;
    return launch_binactiv(x, bn_scale, bn_shift, xbits, nullptr, n, c, h * w, (hipStream_t)hip_stream);
}

int xnor_compute_K(const float *x, const float *bn_scale, const float *bn_shift,
                   float *A, float *K, const xnor_conv_desc *d, void *hip_stream)
{
    if (!x || !A || !K) return XNOR_ERR_NULL;
    ConvGeom g;
    if (xnor_status s = make_geom(d, &g)) return s;
    if (!aligned16(x) || !aligned16(A) || !aligned16(K)) return XNOR_ERR_ALIGN;
    if (xnor_status s = check_bn(bn_scale, bn_shift)) return s;
    hipStream_t st = (hipStream_t)hip_stream;
    if (xnor_status s = launch_binactiv(x, bn_scale, bn_shift, nullptr, A, g.n, g.c, g.h * g.w, st)) return s;
    return launch_boxfilter(A, K, g, st);
}

static int binactiv_entry(const float *x, const float *bn_scale, const float *bn_shift, uint32_t *xbits, float *A,
                          float *K, const xnor_conv_desc *d, void *hip_stream, int streamed)
{
    if (!x || !xbits || !A) return XNOR_ERR_NULL;
    ConvGeom g;
    if (xnor_status s = make_geom(d, &g)) return s;
    if (!aligned16(x) || !aligned16(xbits) || !aligned16(A) || !aligned16(K)) return XNOR_ERR_ALIGN;
    if (xnor_status s = check_bn(bn_scale, bn_shift)) return s;
    hipStream_t st = (hipStream_t)hip_stream;
    if (xnor_status s = launch_binactiv(x, bn_scale, bn_shift, xbits, A, g.n, g.c, g.h * g.w, st, streamed)) return s;
    return K ? launch_boxfilter(A, K, g, st) : XNOR_OK;
}

int xnor_binactiv(const float *x, const float *bn_scale, const float *bn_shift,
                  uint32_t *xbits, float *A, float *K, const xnor_conv_desc *d, void *hip_stream)
{
    return binactiv_entry(x, bn_scale, bn_shift, xbits, A, K, d, hip_stream, 0);
}

int xnor_binactiv_streamed(const float *x, const float *bn_scale, const float *bn_shift,
                           uint32_t *xbits, float *A, float *K, const xnor_conv_desc *d, void *hip_stream)
{
    return binactiv_entry(x, bn_scale, bn_shift, xbits, A, K, d, hip_stream, 1);
}

int xnor_pool_binactiv(const float *x, const float *bn_scale, const float *bn_shift,
                       uint32_t *xbits, float *A, int n, int c, int h_in, int w_in,
                       int pool_h, int pool_w, int stride_h, int stride_w, int pad_h, int pad_w, int relu,
                       void *hip_stream)
{
    if (!x || !xbits || !A) return XNOR_ERR_NULL;
    if (n <= 0 || c <= 0 || h_in <= 0 || w_in <= 0 || pool_h <= 0 || pool_w <= 0 || stride_h <= 0 ||
        stride_w <= 0 || pad_h < 0 || pad_w < 0)
        return XNOR_ERR_SHAPE;
    if (2 * pad_h > pool_h || 2 * pad_w > pool_w) return XNOR_ERR_SHAPE;     // every window holds an input value
    const long long hp = (long long)h_in + 2LL * pad_h, wp = (long long)w_in + 2LL * pad_w;
    if (pool_h > hp || pool_w > wp) return XNOR_ERR_SHAPE;
    const long long ho = (hp - pool_h) / stride_h + 1, wo = (wp - pool_w) / stride_w + 1;
    if ((long long)h_in * w_in > 0x7fffffffLL || ho * wo > 0x7fffffffLL ||
        (long long)n * ho * wo * ((c + 31) / 32) > 0x7fffffffLL || (long long)n * c > 0x7fffffffLL)
        return XNOR_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(xbits) || !aligned16(A)) return XNOR_ERR_ALIGN;
    if (xnor_status s = check_bn(bn_scale, bn_shift)) return s;
    return launch_pool_binactiv(x, bn_scale, bn_shift, xbits, A, n, c, h_in, w_in, pool_h, pool_w, stride_h,
                                stride_w, pad_h, pad_w, relu ? 1 : 0, (hipStream_t)hip_stream);
}

int xnor_pack_weights(const float *w, uint32_t *wbits, float *alpha, void *wmfma,
                      int k_out, int c, int kh, int kw, void *hip_stream)
{
    if (!w || !wbits || !alpha) return XNOR_ERR_NULL;
    if (k_out <= 0 || c <= 0 || kh <= 0 || kw <= 0) return XNOR_ERR_SHAPE;
    if ((long long)kh * kw > 4096 || (long long)k_out * kh * kw * ((c + 31) / 32) > 0x7fffffffLL ||
        (long long)c * kh * kw > 0x7fffffffLL)
        return XNOR_ERR_SHAPE;
    if (!aligned16(w) || !aligned16(wbits) || !aligned16(alpha) || !aligned16(wmfma)) return XNOR_ERR_ALIGN;
    return launch_pack_weights(w, wbits, alpha, wmfma, k_out, c, kh * kw, (hipStream_t)hip_stream);
}

namespace {
// Inner-loop choice for a validated geometry.  A dilated input (transposed convolution of a strided layer) is
// staged by the matrix-core kernels only, and needs K given (A of the virtual image does not exist).
xnor_status conv_dispatch(const ConvGeom &g, const uint32_t *xbits, const uint32_t *wbits, const void *wmfma,
                          const float *K, const float *A, const float *alpha, float *out, int32_t *dot_out,
                          int algo, hipStream_t st)
{
    const bool dilated = g.dil_h > 1 || g.dil_w > 1;
    if (dilated && !K) return XNOR_ERR_UNSUPPORTED;
    switch (algo) {
    case XNOR_ALGO_POPCOUNT:
        if (dilated) return XNOR_ERR_UNSUPPORTED;
        return launch_conv_popcount(xbits, wbits, wmfma, K, A, alpha, out, dot_out, g, st);
    case XNOR_ALGO_MFMA_I8:
    case XNOR_ALGO_MFMA_F4:
        if (!wmfma) return XNOR_ERR_NULL;
        return launch_conv_mfma(algo == XNOR_ALGO_MFMA_F4 ? 1 : 0, xbits, wmfma, K, A, alpha, out, dot_out, g, st);
    case XNOR_ALGO_AUTO: {
        if (wmfma) {        // 4-bit operands, then int8 (sums of 2^24 and more terms), then the vector ALU
            xnor_status s = launch_conv_mfma(1, xbits, wmfma, K, A, alpha, out, dot_out, g, st);
            if (s != XNOR_ERR_UNSUPPORTED) return s;
            s = launch_conv_mfma(0, xbits, wmfma, K, A, alpha, out, dot_out, g, st);
            if (s != XNOR_ERR_UNSUPPORTED) return s;
        }
        if (dilated) return XNOR_ERR_UNSUPPORTED;
        return launch_conv_popcount(xbits, wbits, wmfma, K, A, alpha, out, dot_out, g, st);
    }
    default:
        return XNOR_ERR_UNSUPPORTED;
    }
}
}  // namespace

int xnor_conv2d(const uint32_t *xbits, const uint32_t *wbits, const void *wmfma,
                const float *K, const float *A, const float *alpha, float *out, int32_t *dot_out,
                const xnor_conv_desc *d, int algo, void *hip_stream)
{
    if (!xbits || !wbits || (!K && !A) || !alpha || !out) return XNOR_ERR_NULL;
    ConvGeom g;
    if (xnor_status s = make_geom(d, &g)) return s;
    if (!aligned16(xbits) || !aligned16(wbits) || !aligned16(wmfma) || !aligned16(K) || !aligned16(A) ||
        !aligned16(alpha) || !aligned16(out) || !aligned16(dot_out))
        return XNOR_ERR_ALIGN;
    return conv_dispatch(g, xbits, wbits, wmfma, K, A, alpha, out, dot_out, algo, (hipStream_t)hip_stream);
}

int xnor_conv2d_pool(const uint32_t *xbits, const void *wmfma, const float *K, const float *A,
                     const float *alpha, float *out_pool, const xnor_conv_desc *d,
                     int pool_h, int pool_w, int pstride_h, int pstride_w, int relu, void *hip_stream)
{
    if (!xbits || !wmfma || (!K && !A) || !alpha || !out_pool) return XNOR_ERR_NULL;
    ConvGeom g;
    if (xnor_status s = make_geom(d, &g)) return s;
    if (pool_h <= 0 || pool_w <= 0 || pstride_h <= 0 || pstride_w <= 0 || pool_h > g.ho || pool_w > g.wo)
        return XNOR_ERR_SHAPE;
    if (!aligned16(xbits) || !aligned16(wmfma) || !aligned16(K) || !aligned16(A) || !aligned16(alpha) ||
        !aligned16(out_pool))
        return XNOR_ERR_ALIGN;
    return launch_conv_mfma_pool(xbits, wmfma, K, A, alpha, out_pool, g, pool_h, pool_w, pstride_h, pstride_w,
                                 relu ? 1 : 0, (hipStream_t)hip_stream);
}

int xnor_pool_fusion_choice(const xnor_conv_desc *d, int pool_h, int pool_w, int pstride_h, int pstride_w)
{
    ConvGeom g;
    if (xnor_status s = make_geom(d, &g)) return s;
    if (pool_h <= 0 || pool_w <= 0 || pstride_h <= 0 || pstride_w <= 0 || pool_h > g.ho || pool_w > g.wo)
        return XNOR_ERR_SHAPE;
    // the pooled epilogue needs the convolution rows under one pooled row inside its largest pixel tile
    if ((long long)pool_h * g.wo > 192 || (long long)g.c * g.taps >= (1ll << 24)) return XNOR_POOL_ON_LOAD;
    return g.wo <= 16 ? XNOR_POOL_IN_EPILOGUE : XNOR_POOL_ON_LOAD;
}

size_t xnor_conv2d_binactiv_workspace_bytes(const xnor_conv_desc *d)
{
    ConvGeom g;
    if (make_geom(d, &g) != XNOR_OK) return 0;
    // up to 64 filters every workgroup tiling covers all of them: no partial sums
    return g.k_out <= 64 ? 0 : (size_t)g.fblocks * (size_t)g.m_total * sizeof(float);
}

int xnor_conv2d_binactiv(const uint32_t *xbits, const uint32_t *wbits, const void *wmfma,
                         const float *K, const float *A, const float *alpha,
                         const float *bn_scale_next, const float *bn_shift_next,
                         uint32_t *xbits_next, float *A_next, float *out, void *workspace,
                         const xnor_conv_desc *d, int algo, void *hip_stream)
{
    if (!xbits || !wbits || (!K && !A) || !alpha || !xbits_next || !A_next) return XNOR_ERR_NULL;
    ConvGeom g;
    if (xnor_status s = make_geom(d, &g)) return s;
    if (!workspace && g.k_out > 64) return XNOR_ERR_NULL;
    if ((long long)g.m_total * g.fblocks > 0x7fffffffLL) return XNOR_ERR_SHAPE;
    if (!aligned16(xbits) || !aligned16(wbits) || !aligned16(wmfma) || !aligned16(K) || !aligned16(A) ||
        !aligned16(alpha) || !aligned16(xbits_next) || !aligned16(A_next) || !aligned16(out) ||
        !aligned16(workspace))
        return XNOR_ERR_ALIGN;
    if (xnor_status s = check_bn(bn_scale_next, bn_shift_next)) return s;
    if (algo != XNOR_ALGO_AUTO && algo != XNOR_ALGO_MFMA_I8 && algo != XNOR_ALGO_MFMA_F4)
        return XNOR_ERR_UNSUPPORTED;      // the fused epilogue lives in the matrix-core kernels only
    if (!wmfma) return XNOR_ERR_NULL;
    FuseArgs fz;
    fz.bn_scale = bn_scale_next; fz.bn_shift = bn_shift_next;
    fz.xbits_next = xbits_next; fz.A_next = A_next; fz.workspace = static_cast<float *>(workspace);
    hipStream_t st = (hipStream_t)hip_stream;
    if (algo != XNOR_ALGO_MFMA_I8) {
        const xnor_status s = launch_conv_mfma(1, xbits, wmfma, K, A, alpha, out, nullptr, g, st, &fz);
        if (s != XNOR_ERR_UNSUPPORTED || algo == XNOR_ALGO_MFMA_F4) return s;
    }
    return launch_conv_mfma(0, xbits, wmfma, K, A, alpha, out, nullptr, g, st, &fz);
}

/* ---- xnor_conv2d_binactiv for callers that cannot allocate ------------------------------------------ */

}  // extern "C" (file-scope device memory and its host-side bookkeeping follow)

// Library-owned scratch for the partial |z| sums of xnor_conv2d_binactiv_noalloc.  Every GPU the library
// runs on holds its own copy at its own address until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress: kernels are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[XNOR_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES];          // device address of `scratch` per device ordinal, NULL = not asked yet

// Address of the current device's copy of `scratch` (asked once per device, with that device current).
xnor_status scratch_address(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return XNOR_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return XNOR_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return XNOR_OK;
}
}  // namespace

extern "C" {

int xnor_conv2d_binactiv_noalloc(const uint32_t *xbits, const uint32_t *wbits, const void *wmfma,
                                 const float *K, const float *A, const float *alpha,
                                 const float *bn_scale_next, const float *bn_shift_next,
                                 uint32_t *xbits_next, float *A_next, float *out,
                                 const xnor_conv_desc *d, int algo, void *hip_stream)
{
    const size_t need = xnor_conv2d_binactiv_workspace_bytes(d);     // 0 also for an invalid descriptor: caught below
    if (need > (size_t)XNOR_NOALLOC_SCRATCH_BYTES) return XNOR_ERR_UNSUPPORTED;
    void *ws = nullptr;
    if (xnor_status s = scratch_address(&ws)) return s;
    // Nothing in the scratch has to start at zero: the second kernel reads only the partial sums the first
    // one wrote in this call.
    return xnor_conv2d_binactiv(xbits, wbits, wmfma, K, A, alpha, bn_scale_next, bn_shift_next, xbits_next, A_next,
                                out, ws, d, algo, hip_stream);
}

/* ---- Binary-Weight-Network convolution: real activations, +-1 weights (sec. 3.1) ------------------ */

size_t xnor_bwn_parts_bytes(int n, int c, int h, int w)
{
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return 0;
    return (size_t)n * h * w * ((c + 15) / 16) * 96u;
}

size_t xnor_bwn_wimg_bytes(int k_out, int c, int kh, int kw)
{
    if (k_out <= 0 || c <= 0 || kh <= 0 || kw <= 0 || (long long)kh * kw > 4096) return 0;
    return wimg_bf16_bytes(k_out, (c + 15) / 16, kh * kw);
}

int xnor_bwn_split(const float *x, void *parts, int n, int c, int h, int w, void *hip_stream)
{
    if (!x || !parts) return XNOR_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return XNOR_ERR_SHAPE;
    if ((long long)h * w > 0x7fffffffLL || (long long)n * h * w * ((c + 15) / 16) * 3 > 0x7fffffffLL)
        return XNOR_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(parts)) return XNOR_ERR_ALIGN;
    return launch_bwn_split(x, parts, n, c, h * w, (hipStream_t)hip_stream);
}

int xnor_bwn_pack_weights(const float *w, float *alpha, void *wimg, int k_out, int c, int kh, int kw,
                          void *hip_stream)
{
    if (!w || !alpha || !wimg) return XNOR_ERR_NULL;
    if (k_out <= 0 || c <= 0 || kh <= 0 || kw <= 0) return XNOR_ERR_SHAPE;
    if ((long long)kh * kw > 4096 || (long long)c * kh * kw > 0x7fffffffLL ||
        (long long)k_out * kh * kw * ((c + 15) / 16) * 3 > 0x7fffffffLL / 32)
        return XNOR_ERR_SHAPE;
    if (!aligned16(w) || !aligned16(alpha) || !aligned16(wimg)) return XNOR_ERR_ALIGN;
    return launch_bwn_pack(w, alpha, wimg, k_out, c, kh * kw, (hipStream_t)hip_stream);
}

int xnor_bwn_conv2d(const void *parts, const void *wimg, const float *alpha, float *out,
                    const xnor_conv_desc *d, void *hip_stream)
{
    if (!parts || !wimg || !alpha || !out) return XNOR_ERR_NULL;
    if (!d) return XNOR_ERR_NULL;
    // the matrix-core kernel sees 3*ceil(c/16) operand words of 32 bytes per pixel
    xnor_conv_desc dd = *d;
    if (d->c <= 0 || d->c > 0x7fffffff / 96) return XNOR_ERR_SHAPE;
    dd.c = 96 * ((d->c + 15) / 16);
    ConvGeom g;
    if (xnor_status s = make_geom(&dd, &g)) return s;
    if (!aligned16(parts) || !aligned16(wimg) || !aligned16(alpha) || !aligned16(out)) return XNOR_ERR_ALIGN;
    return launch_conv_mfma(2, static_cast<const uint32_t *>(parts), wimg, nullptr, nullptr, alpha, out, nullptr, g,
                            (hipStream_t)hip_stream);
}

int xnor_bingrad_pack_weights(const float *w, uint32_t *wtbits, float *ones, void *wtmfma,
                              int k_out, int c, int kh, int kw, void *hip_stream)
{
    if (!w || !wtbits || !ones) return XNOR_ERR_NULL;
    if (k_out <= 0 || c <= 0 || kh <= 0 || kw <= 0) return XNOR_ERR_SHAPE;
    if ((long long)kh * kw > 4096 || (long long)c * kh * kw * ((k_out + 31) / 32) > 0x7fffffffLL ||
        (long long)k_out * kh * kw > 0x7fffffffLL || (long long)k_out * c * kh * kw > 0x7fffffffLL)
        return XNOR_ERR_SHAPE;
    if (!aligned16(w) || !aligned16(wtbits) || !aligned16(ones) || !aligned16(wtmfma)) return XNOR_ERR_ALIGN;
    // the backward convolution has c filters over k_out channels
    return launch_pack_weights(w, wtbits, ones, wtmfma, c, k_out, kh * kw, (hipStream_t)hip_stream, 1);
}

int xnor_bingrad_binarize(const float *g_out, const float *K, const float *alpha, uint32_t *gbits,
                          float *gmax, const xnor_conv_desc *d, void *hip_stream)
{
    if (!g_out || !gbits || !gmax) return XNOR_ERR_NULL;
    ConvGeom g;
    if (xnor_status s = make_geom(d, &g)) return s;
    if ((long long)g.m_total * ((g.k_out + 31) / 32) > 0x7fffffffLL) return XNOR_ERR_SHAPE;
    if (!aligned16(g_out) || !aligned16(K) || !aligned16(alpha) || !aligned16(gbits) || !aligned16(gmax))
        return XNOR_ERR_ALIGN;
    return launch_bingrad_binarize(g_out, K, alpha, gbits, gmax, g.n, g.k_out, g.ho * g.wo, (hipStream_t)hip_stream);
}

int xnor_bingrad_conv2d(const uint32_t *gbits, const uint32_t *wtbits, const void *wtmfma,
                        const float *gmax, const float *ones, float *scale_plane, float *g_in,
                        int32_t *dot_out, const xnor_conv_desc *d, int algo, void *hip_stream)
{
    if (!gbits || !wtbits || !gmax || !ones || !scale_plane || !g_in) return XNOR_ERR_NULL;
    ConvGeom fwd;
    if (xnor_status s = make_geom(d, &fwd)) return s;
    // Transpose of the forward correlation: a stride-1 correlation of the gradient, dilated by the forward
    // stride (zeros between its pixels) and extended by the input rows and columns the last forward window
    // left uncovered, with the c rotated filters and padding kh-1-pad; it gives back h_in x w_in.
    xnor_conv_desc t;
    t.n = fwd.n; t.c = fwd.k_out;
    t.h_in = fwd.h + 2 * fwd.ph - fwd.kh + 1;            // = (h_out-1)*stride_h + 1 + uncovered rows
    t.w_in = fwd.w + 2 * fwd.pw - fwd.kw + 1;
    t.k_out = fwd.c; t.kh = fwd.kh; t.kw = fwd.kw;
    t.stride_h = 1; t.stride_w = 1;
    t.pad_h = fwd.kh - 1 - fwd.ph; t.pad_w = fwd.kw - 1 - fwd.pw;
    if (!aligned16(gbits) || !aligned16(wtbits) || !aligned16(wtmfma) || !aligned16(gmax) || !aligned16(ones) ||
        !aligned16(scale_plane) || !aligned16(g_in) || !aligned16(dot_out))
        return XNOR_ERR_ALIGN;
    ConvGeom g;
    if (xnor_status s = make_geom(&t, &g)) return s;
    if (g.ho != fwd.h || g.wo != fwd.w) return XNOR_ERR_SHAPE;
    g.dil_h = fwd.sh; g.dil_w = fwd.sw;
    g.real_h = fwd.ho; g.real_w = fwd.wo;
    g.div_dil_h = FastDiv::make((uint32_t)fwd.sh);
    g.div_dil_w = FastDiv::make((uint32_t)fwd.sw);
    // what conv_dispatch would refuse for this algo, before the first launch touches scale_plane
    const bool dilated = g.dil_h > 1 || g.dil_w > 1;
    if (algo != XNOR_ALGO_AUTO && algo != XNOR_ALGO_POPCOUNT && algo != XNOR_ALGO_MFMA_I8 && algo != XNOR_ALGO_MFMA_F4)
        return XNOR_ERR_UNSUPPORTED;
    if (algo == XNOR_ALGO_POPCOUNT && dilated) return XNOR_ERR_UNSUPPORTED;
    if ((algo == XNOR_ALGO_MFMA_I8 || algo == XNOR_ALGO_MFMA_F4) && !wtmfma) return XNOR_ERR_NULL;
    if (algo == XNOR_ALGO_AUTO && dilated && !wtmfma) return XNOR_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)hip_stream;
    if (xnor_status s = launch_bingrad_scale_plane(gmax, scale_plane, fwd.n, fwd.h * fwd.w, st)) return s;
    return conv_dispatch(g, gbits, wtbits, wtmfma, scale_plane, nullptr, ones, g_in, dot_out, algo, st);
}

size_t xnor_kbit_input_bytes(int n, int c, int h, int w)
{
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return 0;
    return (size_t)n * h * w * (size_t)((c + 31) / 32) * 32u;
}

size_t xnor_kbit_wimg_bytes(int k_out, int c, int kh, int kw)
{
    if (k_out <= 0 || c <= 0 || kh <= 0 || kw <= 0 || (long long)kh * kw > 4096) return 0;
    return wimg_i8_bytes(k_out, c, kh * kw);
}

int xnor_kbit_pack_input(const float *x, void *xq, int ka, int n, int c, int h, int w, void *hip_stream)
{
    if (!x || !xq) return XNOR_ERR_NULL;
    if (ka < 1 || ka > 7 || n <= 0 || c <= 0 || h <= 0 || w <= 0) return XNOR_ERR_SHAPE;
    if ((long long)h * w > 0x7fffffffLL || (long long)n * h * w * ((c + 31) / 32) > 0x7fffffffLL / 8 ||
        (long long)n * c > 0x7fffffffLL)
        return XNOR_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(xq)) return XNOR_ERR_ALIGN;
    return launch_kbit_pack_input(x, static_cast<int8_t *>(xq), ka, n, c, h * w, (hipStream_t)hip_stream);
}

int xnor_kbit_pack_weights(const float *w, float *scale, void *wq, int ka, int kw_bits,
                           int k_out, int c, int kh, int kw, void *hip_stream)
{
    if (!w || !scale || !wq) return XNOR_ERR_NULL;
    if (ka < 1 || ka > 7 || kw_bits < 1 || kw_bits > 7 || k_out <= 0 || c <= 0 || kh <= 0 || kw <= 0) return XNOR_ERR_SHAPE;
    if ((long long)kh * kw > 4096 || (long long)k_out * kh * kw * ((c + 31) / 32) > 0x7fffffffLL ||
        (long long)c * kh * kw > 0x7fffffffLL)
        return XNOR_ERR_SHAPE;
    if (!aligned16(w) || !aligned16(scale) || !aligned16(wq)) return XNOR_ERR_ALIGN;
    const double s = (double)((1 << ka) - 1) * (double)((1 << kw_bits) - 1);
    return launch_pack_weights(w, nullptr, scale, wq, k_out, c, kh * kw, (hipStream_t)hip_stream, 3, kw_bits,
                               (float)(1.0 / s));
}

int xnor_kbit_conv2d(const void *xq, const void *wq, const float *scale, float *out, int32_t *num_out,
                     const xnor_conv_desc *d, int ka, int kw_bits, void *hip_stream)
{
    if (!xq || !wq || !scale || !out) return XNOR_ERR_NULL;
    if (ka < 1 || ka > 7 || kw_bits < 1 || kw_bits > 7) return XNOR_ERR_SHAPE;
    ConvGeom g;
    if (xnor_status s = make_geom(d, &g)) return s;
    const long long lw = (long long)((1 << ka) - 1) * ((1 << kw_bits) - 1);
    if (lw * g.c * g.taps > 0x7fffffffLL) return XNOR_ERR_UNSUPPORTED;       // the int32 accumulator holds every sum
    if (!aligned16(xq) || !aligned16(wq) || !aligned16(scale) || !aligned16(out) || !aligned16(num_out))
        return XNOR_ERR_ALIGN;
    return launch_conv_mfma(3, static_cast<const uint32_t *>(xq), wq, nullptr, nullptr, scale, out, num_out, g,
                            (hipStream_t)hip_stream);
}

int xnor_linear(const uint32_t *xbits, const uint32_t *wbits, const void *wmfma,
                const float *Krow, const float *alpha, float *out, int32_t *dot_out,
                int batch, int in_features, int out_features, int algo, void *hip_stream)
{
    // A fully connected layer is the convolution whose 1x1 "image" has in_features channels.
    xnor_conv_desc d;
    d.n = batch; d.c = in_features; d.h_in = 1; d.w_in = 1;
    d.k_out = out_features; d.kh = 1; d.kw = 1;
    d.stride_h = 1; d.stride_w = 1; d.pad_h = 0; d.pad_w = 0;
    return xnor_conv2d(xbits, wbits, wmfma, Krow, nullptr, alpha, out, dot_out, &d, algo, hip_stream);
}

}  // extern "C"
