// Exact unsigned division by a run-time constant, usable from host and device code (no HIP headers
// needed, so that a plain host compiler can check it).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define XNOR_HD __host__ __device__
#else
#define XNOR_HD
#endif

namespace xnor {

// q = floor(x / d) for every 32-bit x and every divisor 1 <= d <= 2^31.
// magic = floor(2^32 / d) + 1 = (2^32 + e) / d with 1 <= e <= d, so
//     x * magic / 2^32 = x / d + x * e / (d * 2^32),   0 <= x * e / (d * 2^32) < 1:
// the high product word is floor(x / d) or one more, and one multiply-compare takes the excess back.
// d == 1 has no 32-bit magic: magic = 0 and `pass` = ~0 hand x through.
struct FastDiv {
    uint32_t magic;
    uint32_t pass;
    uint32_t d;
    static FastDiv make(uint32_t d)
    {
        FastDiv f;
        f.magic = (d <= 1) ? 0u : (uint32_t)((0x100000000ull / d) + 1ull);
        f.pass = (d <= 1) ? 0xFFFFFFFFu : 0u;
        f.d = d ? d : 1u;
        return f;
    }
    static XNOR_HD inline uint32_t mulhi(uint32_t a, uint32_t b)
    {
#if defined(__HIP_DEVICE_COMPILE__)
        return __umulhi(a, b);
#else
        return (uint32_t)(((uint64_t)a * b) >> 32);
#endif
    }
    XNOR_HD inline uint32_t div(uint32_t x) const
    {
        const uint32_t q = mulhi(x, magic) + (x & pass);
        // remainder in wrapping arithmetic: below d when q is right, at least 2^32 - d >= d when q is one too
        // many (divisors are at most 2^31)
        const uint32_t r = x - q * d;
        return q - (r >= d ? 1u : 0u);
    }
    // Without the correction: exact while x * d < 2^32.  For the inner loops whose operands the host
    // bounds (indices into an LDS image of at most 160 KiB, filter taps).
    XNOR_HD inline uint32_t div_small(uint32_t x) const { return mulhi(x, magic) + (x & pass); }
};

}  // namespace xnor
