// Operand encodings and the LDS plan shared by the matrix-core convolution kernels.
#pragma once
#include "xnor_internal.h"

namespace xnor {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

// Max-pooling applied in the convolution's epilogue (block order BinConv -> Pool, sec. 3.2).  A pixel tile is
// then a group of `pr` pooled rows of one image: the (pr-1)*sh + ph convolution rows under them, all
// columns, as one run of consecutive flattened output pixels (neighbouring groups overlap by ph - sh rows,
// which are computed twice).
struct PoolPlan {
    int ph, pw, sh, sw;   // window, stride (no padding)
    int hpo, wpo;         // pooled extent
    int pr;               // pooled rows per tile
    int groups;           // tiles per image = ceil(hpo / pr)
    int relu;             // max(., 0) before pooling (the optional ReLU after BinConv)
    FastDiv div_groups, div_wpo;
};

struct MfmaPlan {
    int cc_words;     // channel words widened per chunk (divides cw)
    int ps;           // bytes per pixel in LDS (an odd multiple of 16: conflict-free 16-byte reads)
    int max_rows;     // padded input rows a pixel tile can touch
    int region_bytes; // max_rows * row_pitch
    int row_pitch;    // LDS bytes per padded input row (>= wp * ps)
    int nsteps;       // K-steps per chunk
    int tap_jump;     // weight records skipped when a chunk moves to the next tap
    int ptiles;       // pixel tiles of the launch (the grid is padded beyond it)
    int lut_offset;   // LDS byte offset of the sign-byte widening table
    int ftiles;       // filter tiles of the launch
    int wmajor;       // 1: 1-D grid that keeps the pixel tiles of a filter tile on one XCD
    int dense;        // 1: 1x1 filter, no padding, stride 1, one chunk, words per pixel a multiple of 4: the tile's
                      //    packed words are one contiguous run of memory, staged 16 bytes per load
                      // 2: staging without per-item divisions or 64-bit addresses (see set_fast_staging)
    int stream_out;   // 1: float results are stored with the non-temporal hint (they exceed a quarter of the last-level cache)
    FastDiv div_wp, div_hp, div_ccw, div_cw;
    PoolPlan pool;    // used by the pooled-epilogue instantiations only
};

// The staging loop walks the items (padded row, padded column, channel word), word fastest, a workgroup-wide stride
// of `threads` items at a time.  When the input is not dilated, every channel word is full (c a multiple of 32) and
// pixel and byte counts fit 24 and 31 bits, a thread keeps its (row, column, word) in registers and advances them by
// the stride's constant increments with carries, addresses LDS and memory with 24-bit multiply-adds, and reads the
// packed words through a bounds-checked buffer (positions outside the image get an offset beyond it): no division,
// no 64-bit arithmetic and no branch per item.
inline void set_fast_staging(MfmaPlan *pl, const ConvGeom &g, int fmt)
{
    const long long px = (long long)g.n * g.h * g.w;
    if (fmt < 2 && !pl->dense && g.dil_h == 1 && g.dil_w == 1 && g.c % 32 == 0 && px < (1 << 24) &&
        g.cw < (1 << 16) && px * g.cw * 4 < 0x7fffffffLL && pl->row_pitch < (1 << 23))
        pl->dense = 2;
}

// Most padded input rows touched by any run of `run` consecutive (flattened) output pixels that
// starts at a multiple of `step`.  The row span only depends on the start modulo the pixels of one
// image, so one period of starts is enough (the host pays a few dozen iterations per launch).
inline int worst_region_rows(const ConvGeom &g, int run, int step)
{
    const long long howo = (long long)g.ho * g.wo;
    long long a = step, b = howo;
    while (b) { const long long t = a % b; a = b; b = t; }      // gcd(step, howo)
    const long long period = howo / a;
    const long long starts = (g.m_total + step - 1) / step;
    const long long n = starts < period ? starts : period;
    int worst = 0;
    for (long long i = 0; i < n; ++i) {
        const long long m0 = i * step;
        const long long m1 = (m0 + run < g.m_total ? m0 + run : g.m_total) - 1;
        const int ia = (int)(m0 / howo), ib = (int)(m1 / howo);
        const int oa = (int)((m0 % howo) / g.wo), ob = (int)((m1 % howo) / g.wo);
        const int rows = (ib * g.hp + ob * g.sh + g.kh - 1) - (ia * g.hp + oa * g.sh) + 1;
        if (rows > worst) worst = rows;
    }
    return worst;
}

template <int FMT> struct Enc;

template <> struct Enc<0> {                    // int8
    static constexpr int BPS = 1;              // channel words per K-step (= per weight record)
    static constexpr int NX = 1;               // matrix instructions per K-step and result block
    static constexpr bool HALF_SPLIT = true;   // a lane's half-wave picks 16 of a word's 32 bytes
    static constexpr int BPB = 32;             // LDS bytes per pixel per channel word
    typedef v16i acc_t;
    static __device__ __forceinline__ acc_t mfma(v4i w, v4i x, acc_t c) {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(w, x, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int to_int(acc_t a, int v) { return a[v]; }
    static __device__ __forceinline__ float to_float(acc_t a, int v) { return (float)a[v]; }
    // 4 sign bits -> 4 int8: bit 1 -> 0x01, bit 0 -> 0xFF
    static __device__ __forceinline__ uint32_t widen4(uint32_t nibble) {
        const uint32_t t = __umul24(nibble, 0x00204081u) & 0x01010101u;     // bit i -> byte i
        return __builtin_amdgcn_perm(0x000001FFu, 0x000001FFu, t);           // byte = {0xFF, 0x01}[t]
    }
    // one channel word -> 32 bytes at dst; channels >= nch are 0
    static __device__ __forceinline__ void widen_word(uint8_t *dst, uint32_t bits, bool ok, int nch) {
        uint4 lo = make_uint4(0, 0, 0, 0), hi = make_uint4(0, 0, 0, 0);
        if (ok) {
            lo.x = widen4(bits & 15u);         lo.y = widen4((bits >> 4) & 15u);
            lo.z = widen4((bits >> 8) & 15u);  lo.w = widen4((bits >> 12) & 15u);
            hi.x = widen4((bits >> 16) & 15u); hi.y = widen4((bits >> 20) & 15u);
            hi.z = widen4((bits >> 24) & 15u); hi.w = widen4(bits >> 28);
            if (nch < 32) {
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
        *reinterpret_cast<uint4 *>(dst) = lo;
        *reinterpret_cast<uint4 *>(dst + 16) = hi;
    }
    // The same through a table in LDS: entry b (8 bytes) = the 8 operand bytes of sign byte b,
    // entries 256..511 are zero (selected for positions outside the image).  Three instructions
    // per sign byte instead of a dozen: the widening is instruction-issue bound.
    static constexpr int LUT_BYTES = 512 * 8;
    static __device__ __forceinline__ void build_lut(uint8_t *lut, int tid, int nthreads) {
        uint2 *t = reinterpret_cast<uint2 *>(lut);
        for (int b = tid; b < 512; b += nthreads)
            t[b] = b < 256 ? make_uint2(widen4(b & 15u), widen4((uint32_t)b >> 4)) : make_uint2(0, 0);
    }
    static __device__ __forceinline__ void widen_word_lut(uint8_t *dst, const uint8_t *lut, uint32_t bits, bool ok,
                                                          int nch) {
        const uint8_t *base = lut + (ok ? 0 : 256 * 8);
        const uint2 a = *reinterpret_cast<const uint2 *>(base + (bits & 255u) * 8);
        const uint2 b = *reinterpret_cast<const uint2 *>(base + ((bits >> 8) & 255u) * 8);
        const uint2 c = *reinterpret_cast<const uint2 *>(base + ((bits >> 16) & 255u) * 8);
        const uint2 d = *reinterpret_cast<const uint2 *>(base + (bits >> 24) * 8);
        uint4 lo = make_uint4(a.x, a.y, b.x, b.y), hi = make_uint4(c.x, c.y, d.x, d.y);
        if (nch < 32) {
            uint32_t *p = reinterpret_cast<uint32_t *>(&lo);
            uint32_t *q = reinterpret_cast<uint32_t *>(&hi);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const int r0 = nch - 4 * w, r1 = nch - 16 - 4 * w;
                p[w] &= r0 >= 4 ? 0xFFFFFFFFu : (r0 <= 0 ? 0u : (1u << (8 * r0)) - 1u);
                q[w] &= r1 >= 4 ? 0xFFFFFFFFu : (r1 <= 0 ? 0u : (1u << (8 * r1)) - 1u);
            }
        }
        *reinterpret_cast<uint4 *>(dst) = lo;
        *reinterpret_cast<uint4 *>(dst + 16) = hi;
    }
};

template <> struct Enc<1> {                    // 4-bit float E2M1
    static constexpr int BPS = 2;
    static constexpr int NX = 1;
    static constexpr bool HALF_SPLIT = false;  // a lane's half-wave picks one word of the step's pair
    static constexpr int BPB = 16;
    typedef v16f acc_t;
    static __device__ __forceinline__ acc_t mfma(v4i w, v4i x, acc_t c) {
        // 4-bit operands occupy the low four dwords; the rest is left undefined (never read)
        const v8i w8 = __builtin_shufflevector(w, w, 0, 1, 2, 3, -1, -1, -1, -1);
        const v8i x8 = __builtin_shufflevector(x, x, 0, 1, 2, 3, -1, -1, -1, -1);
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(w8, x8, c, 4, 4, 0, 127, 0, 127);
    }
    static __device__ __forceinline__ int to_int(acc_t a, int v) { return (int)a[v]; }
    static __device__ __forceinline__ float to_float(acc_t a, int v) { return a[v]; }   // an exact integer already
    // 8 sign bits -> 8 nibbles: bit 1 -> 0x2 (+1.0), bit 0 -> 0xA (-1.0)
    static __device__ __forceinline__ uint32_t widen8(uint32_t byte) {
        uint32_t x = byte;                                   // bit i -> bit 4i by three shift-or steps
        x = (x | (x << 12)) & 0x000F000Fu;
        x = (x | (x << 6)) & 0x03030303u;
        x = (x | (x << 3)) & 0x11111111u;
        return 0xAAAAAAAAu ^ (x << 3);
    }
    static __device__ __forceinline__ void widen_word(uint8_t *dst, uint32_t bits, bool ok, int nch) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (ok) {
            v.x = widen8(bits & 255u);         v.y = widen8((bits >> 8) & 255u);
            v.z = widen8((bits >> 16) & 255u); v.w = widen8(bits >> 24);
            if (nch < 32) {
                uint32_t *d = reinterpret_cast<uint32_t *>(&v);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int r0 = nch - 8 * q;
                    d[q] &= r0 >= 8 ? 0xFFFFFFFFu : (r0 <= 0 ? 0u : (1u << (4 * r0)) - 1u);
                }
            }
        }
        *reinterpret_cast<uint4 *>(dst) = v;
    }
    // 8 sign bits -> 8 nibbles with one byte permute: an output byte holds two channels, i.e. one of four values
    // (0xAA, 0xA2, 0x2A, 0x22 for the bit pairs 00, 01, 10, 11), and v_perm_b32 picks four bytes out of a 32-bit
    // table by four selector bytes.  The selectors are the byte's four bit pairs spread to byte positions by two
    // shift-ors and a mask: four vector instructions per output dword, no table in LDS (whose reads would hit
    // random banks).  `byte` must be clean above bit 7.
    static __device__ __forceinline__ uint32_t widen8_perm(uint32_t byte, uint32_t tbl = 0x222AA2AAu) {
        uint32_t t = (byte << 6) | byte;
        t = (t << 12) | t;
        return __builtin_amdgcn_perm(0u, tbl, t & 0x03030303u);
    }
    static constexpr int LUT_BYTES = 0;
    static __device__ __forceinline__ void build_lut(uint8_t *, int, int) {}
    static __device__ __forceinline__ uint4 widen_word_regs(uint32_t bits, bool ok, int nch) {
        // positions outside the image pick from an all-zero table (code 0x0 = 0.0)
        const uint32_t tbl = ok ? 0x222AA2AAu : 0u;
        uint4 v;
        v.x = widen8_perm(bits & 255u, tbl);
        v.y = widen8_perm((bits >> 8) & 255u, tbl);
        v.z = widen8_perm((bits >> 16) & 255u, tbl);
        v.w = widen8_perm(bits >> 24, tbl);
        if (nch < 32) {
            uint32_t *d = reinterpret_cast<uint32_t *>(&v);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int r0 = nch - 8 * q;
                d[q] &= r0 >= 8 ? 0xFFFFFFFFu : (r0 <= 0 ? 0u : (1u << (4 * r0)) - 1u);
            }
        }
        return v;
    }
    static __device__ __forceinline__ void widen_word_lut(uint8_t *dst, const uint8_t *, uint32_t bits, bool ok,
                                                          int nch) {
        *reinterpret_cast<uint4 *>(dst) = widen_word_regs(bits, ok, nch);
    }
};


constexpr int ring_lcm(int a, int b)
{
    int m = a;
    while (m % b) m += a;
    return m;
}

// Binary-Weight-Network operands (sec. 3.1: real inputs, +-1 weights).  The real activations arrive
// pre-split into three bfloat16 parts (hi + mid + lo == the float exactly), 16 channels x one part
// = one 32-byte "word" per pixel; the weights are +-1.0 (0 past the last channel or filter) in
// bfloat16, one record per 16-channel group that multiplies all three parts (the record is fetched
// once per K-step and feeds three matrix instructions per result block).  Products are exact,
// accumulation is float: the result is the float sum of exact terms.  Layout-wise a word is like the
// int8 encoding's (32 bytes per pixel and word, the half-wave picks its 16 bytes), with nothing to widen.
template <> struct Enc<2> {
    static constexpr int BPS = 3;       // a K-step = one 16-channel group = the three parts' words, one weight record
    static constexpr int NX = 3;        // matrix instructions per step and result block (one per part)
    static constexpr bool HALF_SPLIT = true;
    static constexpr int BPB = 32;
    typedef v16f acc_t;
    typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ acc_t mfma(v4i w, v4i x, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, w), __builtin_bit_cast(v8bf, x), c, 0, 0,
                                                       0);
    }
    static __device__ __forceinline__ int to_int(acc_t a, int v) { return (int)a[v]; }
    static __device__ __forceinline__ float to_float(acc_t a, int v) { return a[v]; }
    static constexpr int LUT_BYTES = 0;
    static __device__ __forceinline__ void build_lut(uint8_t *, int, int) {}
};

// k-bit quantised operands (sec. 3.2, "k-bit Quantization"): activations and weights arrive as the odd-integer
// numerators 2u - L of their levels in int8 (32 channels = one 32-byte word per pixel, 0 past the last
// channel), so the int8 matrix instruction accumulates the exact integer sum of products; nothing to widen.
template <> struct Enc<3> : Enc<0> {
    static constexpr int LUT_BYTES = 0;
    static __device__ __forceinline__ void build_lut(uint8_t *, int, int) {}
};

// Steps the offset table is padded by beyond the last K-step (copies of the last entry): operand
// prefetches run ahead of the loop's end by at most one turn plus the activation depth.
constexpr int KLOOP_TABLE_PAD = 20;

// Weight record stream of a chunk that holds every channel word: the records of a filter block are
// consecutive, so each block gets its own buffer resource covering exactly nsteps records and the
// lane's offset advances by 1 KiB per step.  Prefetches past the end (never multiplied) fall outside
// the resource and are answered with zeros by the buffer bounds check instead of touching memory;
// the check covers the vector offset only, which is why the step lives there and not in the scalar
// offset.  No other bookkeeping in the loop.
// AUX: cache policy of the loads (2 = non-temporal hint).
template <int FW, int AUX = 0> struct WStreamLinear {
    __amdgpu_buffer_rsrc_t rsrc[FW];
    int voff;
    __device__ __forceinline__ WStreamLinear(const v4i *wimg, const int (&wrec0)[FW], int rec_start, int nsteps,
                                             int wlane)
        : voff(wlane)
    {
#pragma unroll
        for (int i = 0; i < FW; ++i)
            rsrc[i] = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<v4i *>(wimg + (size_t)(wrec0[i] + rec_start) * 64), 0, nsteps * 1024, 0x00020000);
    }
    __device__ __forceinline__ void load(v4i (&dst)[FW])
    {
#pragma unroll
        for (int i = 0; i < FW; ++i) {
            const v4u r = __builtin_amdgcn_raw_buffer_load_b128(rsrc[i], voff, 0, AUX);
            dst[i] = v4i{(int)r[0], (int)r[1], (int)r[2], (int)r[3]};
        }
        voff += 1024;
    }
};

// Weight record stream of a chunk that holds part of the channel words: +1 record per step and
// +tap_jump more when the chunk moves to the next tap; steps past the end read the all-zero record.
// Branch-free scalar bookkeeping, so the loop body stays one basic block.
template <int FW> struct WStreamChunked {
    __amdgpu_buffer_rsrc_t rsrc;
    int wrec0[FW];
    int wlane, zero_rec, w_rec, w_cnt, w_left, steps_per_tap, tap_jump;
    __device__ __forceinline__ WStreamChunked(__amdgpu_buffer_rsrc_t rsrc_, const int (&wrec0_)[FW], int zero_rec_,
                                              int rec_start, int nsteps, int steps_per_tap_, int tap_jump_,
                                              int wlane_)
        : rsrc(rsrc_), wlane(wlane_), zero_rec(zero_rec_), w_rec(rec_start), w_cnt(0), w_left(nsteps),
          steps_per_tap(steps_per_tap_), tap_jump(tap_jump_)
    {
#pragma unroll
        for (int i = 0; i < FW; ++i) wrec0[i] = wrec0_[i];
    }
    __device__ __forceinline__ void load(v4i (&dst)[FW])
    {
        const int live = w_left > 0 ? 1 : 0;
#pragma unroll
        for (int i = 0; i < FW; ++i) {
            const int rec = live ? wrec0[i] + w_rec : zero_rec;
            const v4u r = __builtin_amdgcn_raw_buffer_load_b128(rsrc, wlane, rec * 1024, 0);
            dst[i] = v4i{(int)r[0], (int)r[1], (int)r[2], (int)r[3]};
        }
        w_left -= live;
        w_cnt += live;
        const int wrap = w_cnt == steps_per_tap ? 1 : 0;
        w_cnt = wrap ? 0 : w_cnt;
        w_rec += live + (wrap ? tap_jump : 0);
    }
};

// One chunk's K loop of a wave: acc[i][j] += W(filter block i, step s) x X(pixel block j, step s)
// for s = 0 .. nsteps-1, weights from the stream `ws` (one of the two above), activations from LDS
// through the per-step offset table (padded by KLOOP_TABLE_PAD steps).  Operands are requested DW
// steps (weights: buffer loads with a scalar offset, L2 latency) and DX steps (activations) ahead
// of their use and live in register rings of DW+1 and DX+1 slots; the body is unrolled until both
// rings are back at slot 0.  A wave issues one instruction every four cycles, so everything that is
// not a matrix instruction competes with them for issue slots: the loop carries no address or
// bounds arithmetic beyond PW + 1 vector adds per step.
// The scheduling barriers pin the order written here (next operands requested, then the current
// step's matrix instructions interleaved with those requests), which the compiler otherwise
// regroups into one burst of loads followed by one burst of MFMAs with the latencies exposed.
template <class E, int FW, int PW, int DW, int DX, class WS>
__device__ __forceinline__ void mfma_kloop(typename E::acc_t (&acc)[FW][PW], const uint8_t *lds_x,
                                           const int (&pbase)[PW], const int *xoff_tab, int tab_lane, WS &ws,
                                           int nsteps)
{
    constexpr int RW = DW + 1, RX = DX + 1;
    constexpr int TURN = ring_lcm(RW, RX);     // sub-steps after which both rings are back at slot 0
    static_assert(RX <= RW && TURN <= 16 && TURN % 2 == 0, "unrolled turn: even, at most 16 sub-steps");
    static_assert(TURN + DX + 2 <= KLOOP_TABLE_PAD, "offset table padding");
    auto load_w = [&](v4i (&dst)[FW]) { ws.load(dst); };
    const int *tab = xoff_tab + tab_lane;
    auto load_t = [&](int s) -> int { return tab[s * E::BPS]; };
    constexpr int NX = E::NX;                  // words of a step that share its weight record
    auto load_x = [&](v4i (&dst)[PW][NX], int toff) {
#pragma unroll
        for (int j = 0; j < PW; ++j)
#pragma unroll
            for (int q = 0; q < NX; ++q)
                dst[j][q] = *reinterpret_cast<const v4i *>(lds_x + pbase[j] + toff + q * E::BPB);
    };
    auto fma_all = [&](const v4i (&w)[FW], const v4i (&x)[PW][NX]) {
#pragma unroll
        for (int q = 0; q < NX; ++q)
#pragma unroll
            for (int j = 0; j < PW; ++j)
#pragma unroll
                for (int i = 0; i < FW; ++i) acc[i][j] = E::mfma(w[i], x[j][q], acc[i][j]);
    };

    v4i w[RW][FW], x[RX][PW][NX];
    int tq[2];
#pragma unroll
    for (int u = 0; u < DW; ++u) load_w(w[u]);
#pragma unroll
    for (int u = 0; u < DX; ++u) load_x(x[u], load_t(u));
    tq[0] = load_t(DX);
    auto substep = [&](int s, int u) {
        load_w(w[(u + DW) % RW]);                       // step s+u+DW
        tq[(u + 1) & 1] = load_t(s + u + DX + 1);
        load_x(x[(u + DX) % RX], tq[u & 1]);            // step s+u+DX, offset read one sub-step ago
        fma_all(w[u % RW], x[u % RX]);
        // one LDS read behind each of the first PW*NX+1 MFMAs, then the FW weight loads
#pragma unroll
        for (int q = 0; q < PW * NX + 1; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
#pragma unroll
        for (int q = 0; q < FW; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, FW * PW * NX - PW * NX - 1 - FW, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    int s = 0;
    for (; s + TURN <= nsteps; s += TURN) {             // whole turns: one basic block, no exits
#pragma unroll
        for (int u = 0; u < TURN; ++u) substep(s, u);
    }
    // the last, partial turn.  The accumulators are pinned before every exit test: otherwise the
    // matrix instructions sink below the branches and run in one burst behind all the loads.
#pragma unroll
    for (int u = 0; u < TURN - 1; ++u) {
        if (s + u >= nsteps) break;
        substep(s, u);
#pragma unroll
        for (int i = 0; i < FW; ++i)
#pragma unroll
            for (int j = 0; j < PW; ++j) asm volatile("" : "+v"(acc[i][j]));
    }
}

}  // namespace xnor
