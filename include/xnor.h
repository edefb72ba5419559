/*
 * libxnor — forward binary convolution of XNOR-Net on AMD MI355X (gfx950).
 *
 *     I * W  ~  (sign(I) (*) sign(W)) . K alpha            (sec. 3.2, binary-convolution equation)
 *
 * with  alpha = ||W||_1 / n  per filter, n = c*kh*kw        (sec. 3.1, optimal scaling factor),
 *       A     = (1/c) sum_c |I[c]|                          (sec. 3.2, matrix A),
 *       K     = A filtered by the constant kh x kw box 1/(kh*kw)   (sec. 3.2, matrix K),
 * and (*) the convolution of +-1 tensors evaluated with XNOR + bitcount (sec. 3.2).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every pointer is a DEVICE pointer to memory the CALLER owns, except descriptors
 *    (`const xnor_conv_desc*`), which are HOST pointers read during the call.
 *    The library allocates nothing, frees nothing and keeps no pointer after returning.
 *  - `hip_stream` is a hipStream_t (NULL = the default stream).  All work is enqueued on it
 *    asynchronously; no entry point synchronises.
 *  - Return value: XNOR_OK (0) or a negative xnor_status.  Arguments are validated before anything is
 *    launched.  The entry points that enqueue two kernels (xnor_compute_K, xnor_binactiv and xnor_binactiv_streamed with K,
 *    xnor_bingrad_binarize, xnor_bingrad_conv2d, xnor_conv2d_binactiv) may have enqueued the first one
 *    when the second reports XNOR_ERR_UNSUPPORTED (no kernel fits the shape) or XNOR_ERR_HIP; the first
 *    kernel writes only that call's own outputs or scratch.
 *  - Real tensors are float32, NCHW, densely packed, row-major:
 *        x   [n][c][h_in][w_in]      w [k_out][c][kh][kw]      out [n][k_out][h_out][w_out]
 *    h_out = (h_in + 2*pad_h - kh)/stride_h + 1 (floor), same for w_out.
 *  - Packed tensors put channels innermost, 32 channels per uint32 word, Cw = ceil(c/32):
 *        xbits [n][h_in][w_in][Cw]         wbits [k_out][kh][kw][Cw]
 *    bit j of word i <-> channel 32*i + j; bit 1 <-> value >= 0 (+1), bit 0 <-> value < 0 (-1)
 *    (sign rule of sec. 3.1, decided by a comparison: -0.0 -> +1, NaN -> -1).
 *    Bits of channels >= c are 0 in both operands.
 *  - Padding: a padded position contributes 0 to the dot product and 0 to A; the divisor of
 *    K is always kh*kw.  The operation is a correlation (no filter flip).  No bias, groups = 1,
 *    dilation = 1 (the paper's filters have no bias; sec. 3).
 *  - All device pointers must be 16-byte aligned (XNOR_ERR_ALIGN otherwise).
 */
#ifndef XNOR_H
#define XNOR_H

#include <stddef.h>
#include <stdint.h>

/* Only the functions declared with XNOR_API are exported by the shared library. */
#define XNOR_API __attribute__((visibility("default")))

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    XNOR_OK = 0,
    XNOR_ERR_NULL = -1,        /* a required pointer is NULL                                  */
    XNOR_ERR_SHAPE = -2,       /* non-positive size, filter larger than padded input, overflow */
    XNOR_ERR_UNSUPPORTED = -3, /* a combination this build has no kernel for                  */
    XNOR_ERR_ALIGN = -4,       /* a device pointer is not 16-byte aligned                     */
    XNOR_ERR_HIP = -5          /* the HIP runtime reported an error at launch                 */
} xnor_status;

/* Which inner loop xnor_conv2d / xnor_linear run.  Both produce the same integers. */
typedef enum {
    XNOR_ALGO_AUTO = 0,     /* the library's choice for the shape                                  */
    XNOR_ALGO_POPCOUNT = 1, /* XOR + bitcount on the vector ALU over the packed words              */
    XNOR_ALGO_MFMA_I8 = 2,  /* +-1 (0 for padding) widened to int8 on chip, int8 matrix cores      */
    XNOR_ALGO_MFMA_F4 = 3   /* same, widened to 4-bit floats (E2M1), f8f6f4 matrix cores; exact:   */
                            /* products are +-1 or 0 and the float sums stay below 2^24             */
} xnor_algo;

/* Problem statement of sec. 3: input c x w_in x h_in, filters c x w x h, plus stride and pad. */
typedef struct {
    int n, c, h_in, w_in;   /* input  [n][c][h_in][w_in]                 */
    int k_out, kh, kw;      /* filters [k_out][c][kh][kw]                */
    int stride_h, stride_w; /* >= 1                                      */
    int pad_h, pad_w;       /* >= 0, zero padding on both sides          */
} xnor_conv_desc;

/* Cw = ceil(c/32): uint32 words per pixel of a packed tensor. */
XNOR_API int xnor_words_per_pixel(int c);

/* Output extent of the convolution; returns XNOR_ERR_SHAPE if the descriptor is invalid. */
XNOR_API int xnor_output_hw(const xnor_conv_desc *d, int *h_out, int *w_out);

/* Static string for a status code. */
XNOR_API const char *xnor_status_string(int status);

/* Bytes of the matrix-core weight image written by xnor_pack_weights (0 if the shape is invalid). */
XNOR_API size_t xnor_wmfma_bytes(int k_out, int c, int kh, int kw);

/*
 * sign(I) packed to bits (BinActiv layer, sec. 3.2; sign rule of sec. 3.1).
 * Optional batch normalisation first (block order BatchNorm -> BinActiv, sec. 3.2):
 * y = fmaf(x, bn_scale[ch], bn_shift[ch]) in float32; bn_scale == bn_shift == NULL means y = x.
 *   x      in   float32 [n][c][h][w]
 *   xbits  out  uint32  [n][h][w][Cw]
 */
XNOR_API int xnor_binarize_pack(const float *x, const float *bn_scale, const float *bn_shift,
                       uint32_t *xbits, int n, int c, int h, int w, void *hip_stream);

/*
 * A = channel mean of |y| and K = A box-filtered by 1/(kh*kw) at the output positions (sec. 3.2).
 *   x  in   float32 [n][c][h_in][w_in]   (y as in xnor_binarize_pack)
 *   A  out  float32 [n][h_in][w_in]      (required: K is computed from it)
 *   K  out  float32 [n][h_out][w_out]
 */
XNOR_API int xnor_compute_K(const float *x, const float *bn_scale, const float *bn_shift,
                   float *A, float *K, const xnor_conv_desc *d, void *hip_stream);

/*
 * The whole BinActiv layer in one pass over x: xbits, A and K as the two calls above produce them
 * (bit-identical), reading the float input once.  K may be NULL when the following xnor_conv2d is
 * given A instead: it then derives K itself and the separate box-filter launch is saved.
 */
XNOR_API int xnor_binactiv(const float *x, const float *bn_scale, const float *bn_shift,
                  uint32_t *xbits, float *A, float *K, const xnor_conv_desc *d, void *hip_stream);

/*
 * xnor_binactiv for an input that is in no cache (a network's input, a tensor nobody has touched since it went to
 * memory): the same results bit for bit, with x read under the non-temporal hint, so that its stream does not push
 * other kernels' results, which still wait in the last-level cache to be written back, out in front of it.
 * xnor_binactiv itself does that only for inputs beyond a quarter of that cache (64 MiB); for smaller ones it cannot
 * know where x is, and the hint is the slower choice when x was just written by the previous layer.
 */
XNOR_API int xnor_binactiv_streamed(const float *x, const float *bn_scale, const float *bn_shift,
                           uint32_t *xbits, float *A, float *K, const xnor_conv_desc *d, void *hip_stream);

/*
 * Max-pooling (and the optional ReLU) between one block's BinConv and the next block's BatchNorm and
 * BinActiv (block order BatchNorm -> BinActiv -> BinConv -> Pool of sec. 3.2, "Training XNOR-Networks"),
 * applied to the float tensor on load: the pooled tensor is never written.
 *     p[n][ch][oy][ox] = max over the pool_h x pool_w window at (oy*stride_h - pad_h, ox*stride_w - pad_w)
 *                        of x, window positions outside the image skipped (output extent as for a
 *                        convolution: floor((h_in + 2*pad_h - pool_h)/stride_h) + 1); 2*pad <= pool.
 *                        The running maximum starts at -inf and a value replaces it only when it
 *                        compares greater (NaN inputs are skipped).
 *     relu != 0:         p = max(p, 0)
 *     then exactly xnor_binactiv on p with K = NULL:  y = fmaf(p, bn_scale, bn_shift), xbits, A.
 *   x      in   float32 [n][c][h_in][w_in]
 *   xbits  out  uint32  [n][h_out][w_out][Cw]
 *   A      out  float32 [n][h_out][w_out]
 */
XNOR_API int xnor_pool_binactiv(const float *x, const float *bn_scale, const float *bn_shift,
                       uint32_t *xbits, float *A, int n, int c, int h_in, int w_in,
                       int pool_h, int pool_w, int stride_h, int stride_w, int pad_h, int pad_w, int relu,
                       void *hip_stream);

/*
 * B = sign(W) packed to bits and alpha = ||W||_1/n per filter (sec. 3.1; first loop of the
 * training algorithm).  Run once per layer: at inference only B and alpha are kept.
 *   w      in   float32 [k_out][c][kh][kw]
 *   wbits  out  uint32  [k_out][kh][kw][Cw]
 *   alpha  out  float32 [k_out]
 *   wmfma  out  (nullable) xnor_wmfma_bytes(...) bytes: the same signs laid out for the matrix
 *               cores; required by the XNOR_ALGO_MFMA_* loops, opaque to the caller.
 */
XNOR_API int xnor_pack_weights(const float *w, uint32_t *wbits, float *alpha, void *wmfma,
                      int k_out, int c, int kh, int kw, void *hip_stream);

/*
 * BinConv layer: out = float(dot) * K * alpha with
 * dot[n][k][oy][ox] = sum over in-bounds taps and channels of sign(I)*sign(W)
 *                   = n_valid - 2*bitcount(xbits XOR wbits)        (sec. 3.2).
 *   xbits, wbits, alpha  in   as produced above
 *   K        in   (nullable) float32 [n][h_out][w_out]
 *   A        in   (nullable) float32 [n][h_in][w_in]; used only when K is NULL: the kernel then
 *                 evaluates K = box filter of A per output pixel (same bits as xnor_compute_K).
 *                 K and A must not both be NULL.
 *   wmfma    in   (nullable) from xnor_pack_weights; NULL forces XNOR_ALGO_POPCOUNT under AUTO and
 *                 is an XNOR_ERR_NULL under XNOR_ALGO_MFMA_*
 *   out      out  float32 [n][k_out][h_out][w_out]
 *   dot_out  out  (nullable) int32 same shape: the exact integer map, for verification
 *   algo          an xnor_algo
 */
XNOR_API int xnor_conv2d(const uint32_t *xbits, const uint32_t *wbits, const void *wmfma,
                const float *K, const float *A, const float *alpha, float *out, int32_t *dot_out,
                const xnor_conv_desc *d, int algo, void *hip_stream);

/*
 * BinConv of one block followed by the BatchNorm and BinActiv of the NEXT block (block order
 * BatchNorm -> BinActiv -> BinConv of sec. 3.2, "Training XNOR-Networks": what consumes a BinConv output is
 * the next block's normalisation and sign), without the float tensor travelling through memory:
 *     y = float(dot) * K * alpha                          as xnor_conv2d
 *     z = fmaf(y, bn_scale_next[k], bn_shift_next[k])     float32; z = y when both are NULL
 *     xbits_next [n][h_out][w_out][ceil(k_out/32)]        bit k%32 of word k/32 = (z >= 0), tail bits 0
 *     A_next     [n][h_out][w_out] = (1/k_out) sum_k |z|  (sec. 3.2, matrix A of the next block's input)
 * xbits_next and A_next are what xnor_binactiv(out, bn_scale_next, bn_shift_next, ...) would produce from
 * the output of xnor_conv2d: the bits are identical, A_next agrees to float rounding (the |z| are added in
 * a different order).  The next layer then runs xnor_conv2d(xbits_next, ..., K = NULL, A = A_next, ...).
 *   xbits, wbits, wmfma, K, A, alpha   in   as for xnor_conv2d (wmfma is required)
 *   bn_scale_next, bn_shift_next       in   (nullable, both or neither) float32 [k_out]
 *   out        out  (nullable) float32 [n][k_out][h_out][w_out]: y, for callers that also need the real output
 *   workspace       device scratch of xnor_conv2d_binactiv_workspace_bytes(d) bytes (partial |z| sums of the
 *                   filter tiles), contents undefined afterwards; may be NULL when that size is 0
 *   algo            XNOR_ALGO_AUTO, XNOR_ALGO_MFMA_I8 or XNOR_ALGO_MFMA_F4 (XNOR_ERR_UNSUPPORTED otherwise)
 */
XNOR_API size_t xnor_conv2d_binactiv_workspace_bytes(const xnor_conv_desc *d);
XNOR_API int xnor_conv2d_binactiv(const uint32_t *xbits, const uint32_t *wbits, const void *wmfma,
                         const float *K, const float *A, const float *alpha,
                         const float *bn_scale_next, const float *bn_shift_next,
                         uint32_t *xbits_next, float *A_next, float *out, void *workspace,
                         const xnor_conv_desc *d, int algo, void *hip_stream);

/*
 * xnor_conv2d_binactiv for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * launches as xnor_conv2d_binactiv, minus `workspace`: the partial |z| sums go to a buffer of
 * XNOR_NOALLOC_SCRATCH_BYTES that lives in the library's device image (every GPU the process uses holds one
 * until the process ends).  The call allocates and frees nothing.
 *   - XNOR_ERR_UNSUPPORTED when xnor_conv2d_binactiv_workspace_bytes(d) exceeds XNOR_NOALLOC_SCRATCH_BYTES
 *     (4 MiB: every layer of the AlexNet / ResNet-18 shapes at batch 256 needs at most 3.2 MiB).
 *   - All calls on one GPU share that buffer: calls that may overlap on one GPU (different streams, or
 *     graphs replayed concurrently) race on it and must be serialised by the caller.  Nothing in it needs
 *     clearing between calls.
 *   - XNOR_ERR_HIP when the buffer's device address cannot be obtained (asked once per device, at the first
 *     call with that device current).
 */
#define XNOR_NOALLOC_SCRATCH_BYTES (4u << 20)
XNOR_API int xnor_conv2d_binactiv_noalloc(const uint32_t *xbits, const uint32_t *wbits, const void *wmfma,
                                          const float *K, const float *A, const float *alpha,
                                          const float *bn_scale_next, const float *bn_shift_next,
                                          uint32_t *xbits_next, float *A_next, float *out,
                                          const xnor_conv_desc *d, int algo, void *hip_stream);

/*
 * Binary convolution with the block's pooling layer applied in the epilogue (block order BinConv -> Pool,
 * with the optional ReLU after BinConv; sec. 3.2):
 *   out_pool[n][k][py][px] = max over the pool_h x pool_w window at (py*pstride_h, px*pstride_w) of
 *                            y = float(dot) * K * alpha   (y = max(y, 0) first when relu != 0),
 * h_pool = floor((h_out - pool_h)/pstride_h) + 1, w_pool likewise (no pooling padding; the window must fit the
 * convolution output).  The unpooled tensor is never written.  The maximum skips NaN and is never NaN.
 * Arguments as xnor_conv2d (K or A, alpha, wmfma required: matrix-core path with 4-bit operands only);
 * out_pool float32 [n][k_out][h_pool][w_pool].  XNOR_ERR_UNSUPPORTED when the convolution rows under one
 * pooled row (pool_h rows of w_out pixels) exceed the largest pixel tile (192 pixels), or c*kh*kw >= 2^24.
 */
/*
 * Which of the two pooling fusions is the faster chain for a layer (block order BinConv -> Pool -> next block's
 * BatchNorm -> BinActiv, sec. 3.2):
 *   XNOR_POOL_IN_EPILOGUE (1): xnor_conv2d_pool, then xnor_binactiv on the pooled tensor
 *   XNOR_POOL_ON_LOAD     (0): xnor_conv2d, then xnor_pool_binactiv on the unpooled tensor
 * Pooling in the epilogue recomputes the convolution rows that neighbouring groups of pooled rows share and
 * sends every result through LDS once more; measured on the AlexNet / ResNet-18 layer shapes it wins where
 * output rows are short (w_out <= 16: 13- and 14-pixel rows, 1.1 to 1.25 times the matrix work) and loses on
 * 27- and 28-pixel rows.  Also XNOR_POOL_ON_LOAD when xnor_conv2d_pool has no kernel for the geometry.
 * Returns a negative xnor_status for an invalid descriptor or window.  Host-only, launches nothing.
 */
#define XNOR_POOL_ON_LOAD 0
#define XNOR_POOL_IN_EPILOGUE 1
XNOR_API int xnor_pool_fusion_choice(const xnor_conv_desc *d, int pool_h, int pool_w, int pstride_h, int pstride_w);

XNOR_API int xnor_conv2d_pool(const uint32_t *xbits, const void *wmfma, const float *K, const float *A,
                     const float *alpha, float *out_pool, const xnor_conv_desc *d,
                     int pool_h, int pool_w, int pstride_h, int pstride_w, int relu, void *hip_stream);

/*
 * Binary-Weight-Network convolution (sec. 3.1, "Binary-Weight-Networks"): real-valued input, weights
 * estimated by alpha * sign(W):
 *     out[n][k][oy][ox] = alpha_k * sum over in-bounds taps and channels of  I * sign(W)
 * (additions and subtractions of the inputs only; zero padding, correlation, no bias, as above).
 * The sums run on the bfloat16 matrix cores and are float sums of exact terms: xnor_bwn_split writes
 * every input as three bfloat16 numbers whose sum is the float exactly (finite inputs), the weights
 * are +-1.  Three calls:
 *   xnor_bwn_split         x float32 [n][c][h][w]  ->  parts, xnor_bwn_parts_bytes(n, c, h, w) bytes (opaque)
 *   xnor_bwn_pack_weights  w float32 [k_out][c][kh][kw]  ->  alpha float32 [k_out] (as xnor_pack_weights),
 *                          wimg, xnor_bwn_wimg_bytes(k_out, c, kh, kw) bytes (opaque); once per layer
 *   xnor_bwn_conv2d        parts, wimg, alpha  ->  out float32 [n][k_out][h_out][w_out]; d describes the
 *                          convolution with the real channel count c
 * Differences between this result and one accumulated in double stay within float rounding of the
 * running sums (about 1e-7 * sqrt(c*kh*kw) of the magnitude of the terms).
 */
XNOR_API size_t xnor_bwn_parts_bytes(int n, int c, int h, int w);
XNOR_API size_t xnor_bwn_wimg_bytes(int k_out, int c, int kh, int kw);
XNOR_API int xnor_bwn_split(const float *x, void *parts, int n, int c, int h, int w, void *hip_stream);
XNOR_API int xnor_bwn_pack_weights(const float *w, float *alpha, void *wimg, int k_out, int c, int kh, int kw,
                          void *hip_stream);
XNOR_API int xnor_bwn_conv2d(const void *parts, const void *wimg, const float *alpha, float *out,
                    const xnor_conv_desc *d, void *hip_stream);

/*
 * Binary gradient (sec. 3.2, paragraph "Binary Gradient"): the backward convolution between the weight
 * filters and the incoming gradient, with that gradient binarised and scaled by its largest magnitude
 * (not by its mean).  d is always the FORWARD layer's descriptor (input n x c x h_in x w_in, k_out filters),
 * any stride.  All pointers are device pointers, 16-byte
 * aligned, caller-owned; work is enqueued on hip_stream without synchronising.
 *
 *   xnor_bingrad_pack_weights  w float32 [k_out][c][kh][kw] (the forward tensor)  ->  the filters of the
 *       backward convolution, sign(W) rotated by 180 degrees with the channel axes exchanged:
 *       wtbits uint32 [c][kh*kw][ceil(k_out/32)], wtmfma = xnor_wmfma_bytes(c, k_out, kh, kw) bytes (may be
 *       NULL: vector-ALU path only), ones float32 [c] (written with 1.0, the per-filter factor of that
 *       convolution).  Once per layer.
 *   xnor_bingrad_binarize      g_out float32 [n][k_out][h_out][w_out], K float32 [n][h_out][w_out] or NULL,
 *       alpha float32 [k_out] or NULL  ->  gbits uint32 [n][h_out][w_out][ceil(k_out/32)]: bit = (gd >= 0) with
 *       gd = (g_out * alpha_k) * K in float32, the gradient that reaches the binary dot product of the forward
 *       layer out = dot * K * alpha (absent factors count as 1); gmax float32 [n] = max |gd| over the image
 *       (0 for an all-zero image, NaN magnitudes ignored).  Two launches (gmax is cleared first).
 *   xnor_bingrad_conv2d        gbits, wtbits, wtmfma, gmax, ones  ->  g_in float32 [n][c][h_in][w_in] =
 *       gmax[n] * sum over filters and taps of sign(gd) * sign(W) (positions that were padding in the forward
 *       pass receive and contribute nothing); dot_out int32 [n][c][h_in][w_in] (may be NULL) = the integer sum.
 *       scale_plane float32 [n][h_in][w_in] is scratch the caller provides (overwritten).  algo as xnor_conv2d;
 *       for a forward stride above 1 the gradient is staged with zeros between its pixels, which the matrix-core
 *       paths do (wtmfma required; XNOR_ALGO_POPCOUNT gives XNOR_ERR_UNSUPPORTED).
 * The straight-through factor of sign() on the forward input and the gradient through K are not part of
 * these calls.
 */
XNOR_API int xnor_bingrad_pack_weights(const float *w, uint32_t *wtbits, float *ones, void *wtmfma,
                              int k_out, int c, int kh, int kw, void *hip_stream);
XNOR_API int xnor_bingrad_binarize(const float *g_out, const float *K, const float *alpha, uint32_t *gbits,
                          float *gmax, const xnor_conv_desc *d, void *hip_stream);
XNOR_API int xnor_bingrad_conv2d(const uint32_t *gbits, const uint32_t *wtbits, const void *wtmfma,
                        const float *gmax, const float *ones, float *scale_plane, float *g_in,
                        int32_t *dot_out, const xnor_conv_desc *d, int algo, void *hip_stream);

/*
 * k-bit quantisation (sec. 3.2, paragraph "k-bit Quantization"): q_k(x) = 2*([(2^k-1)(x+1)/2]/(2^k-1) - 1/2) in
 * place of sign(), x in [-1, 1] (values outside are clamped, NaN counts as -1; halves round up, so q_1 = sign
 * with sign(0) = +1; the level is decided in float32 as u = floor(((x + 1) * 0.5) * (2^k - 1) + 0.5), except
 * k = 1, which is decided by the comparison x >= 0 so that q_1 is the sign rule for every float, also for
 * -2^-25 < x < 0 where x + 1 rounds to 1).
 * q_k = (2u - L)/L with L = 2^k - 1, so the convolution of ka-bit inputs with kw-bit weights is an exact integer
 * sum of numerator products divided by La * Lw; it runs on the int8 matrix cores:
 *   out[n][k_out][h_out][w_out] = sum q_ka(x) * q_kw(w) over the in-bounds window, no K, no alpha.
 * ka, kw in 1..7 (the numerators of 7-bit levels, -127..127, are the widest that fit int8).  Device pointers,
 * 16-byte aligned, caller-owned; enqueued on hip_stream.
 *   xnor_kbit_pack_input    x float32 [n][c][h][w] -> xq, xnor_kbit_input_bytes(n, c, h, w) bytes: the numerators
 *                           2u - La as int8, [n][h][w][ceil(c/32)][32], 0 past the last channel
 *   xnor_kbit_pack_weights  w float32 [k_out][c][kh][kw] -> wq, xnor_kbit_wimg_bytes(k_out, c, kh, kw) bytes
 *                           (opaque), scale float32 [k_out] (written with 1 / (La * Lw)); once per layer
 *   xnor_kbit_conv2d        num_out int32 [n][k_out][h_out][w_out] (may be NULL) = the integer numerator
 *                           sum (2u_x - La)(2u_w - Lw), out = float(num) * scale (two float roundings: within
 *                           2e-7 relative of num / (La * Lw)).  XNOR_ERR_UNSUPPORTED when La * Lw * c * kh * kw
 *                           does not fit 31 bits.
 */
XNOR_API size_t xnor_kbit_input_bytes(int n, int c, int h, int w);
XNOR_API size_t xnor_kbit_wimg_bytes(int k_out, int c, int kh, int kw);
XNOR_API int xnor_kbit_pack_input(const float *x, void *xq, int ka, int n, int c, int h, int w, void *hip_stream);
XNOR_API int xnor_kbit_pack_weights(const float *w, float *scale, void *wq, int ka, int kw_bits,
                           int k_out, int c, int kh, int kw, void *hip_stream);
XNOR_API int xnor_kbit_conv2d(const void *xq, const void *wq, const float *scale, float *out, int32_t *num_out,
                     const xnor_conv_desc *d, int ka, int kw_bits, void *hip_stream);

/*
 * Fully connected layer = convolution whose filter covers the whole input (footnote of sec. 1).
 *   xbits [batch][Fw], wbits [out_features][Fw], Fw = ceil(in_features/32)
 *   Krow  [batch]  = mean_j |x[b][j]|  (xnor_compute_K / xnor_binactiv with c = in_features, 1x1)
 *   alpha [out_features], out / dot_out [batch][out_features]
 *   wmfma as in xnor_conv2d, packed with (k_out = out_features, c = in_features, 1, 1).
 */
XNOR_API int xnor_linear(const uint32_t *xbits, const uint32_t *wbits, const void *wmfma,
                const float *Krow, const float *alpha, float *out, int32_t *dot_out,
                int batch, int in_features, int out_features, int algo, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* XNOR_H */
