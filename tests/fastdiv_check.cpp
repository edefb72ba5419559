// Host-side check of csrc/fastdiv.h: FastDiv::div against x / d over divisors the kernels use
// (output planes, padded rows, channel chunks) and the whole 32-bit range of x; prints the number of
// mismatches of the exact form and exits non-zero when there is one.  Compiled and run by tests/test_fastdiv.py.
#include "fastdiv.h"
#include <cstdio>
#include <initializer_list>

int main()
{
    using xnor::FastDiv;
    unsigned long long bad = 0;
    const uint32_t ds[] = {1, 2, 3, 5, 7, 13, 49, 169, 196, 729, 784, 3136, 4096, 12544, 16384, 50176,
                           65535, 65536, 1000003, 0x7fffffffu, 0x80000000u};
    for (uint32_t d : ds) {
        const FastDiv f = FastDiv::make(d);
        // dense near both ends, strided in between
        for (uint64_t x = 0; x < 0x100000000ull; x += (x < 200000 || x > 0xfffd0000ull) ? 1 : 9973)
            bad += f.div((uint32_t)x) != (uint32_t)x / d;
        // both sides of every multiple of d (sampled when there are many)
        const uint64_t nq = 0x100000000ull / d, step = nq > 2000000 ? nq / 1000000 : 1;
        for (uint64_t q = 1; q * d < 0x100000000ull; q += step) {
            const uint64_t x = q * d;
            bad += f.div((uint32_t)x) != q;
            bad += f.div((uint32_t)(x - 1)) != q - 1;
        }
    }
    // last output pixel of batches whose pixel index times the plane size passes 2^32
    // (plane, batch): 224x224 x 2, 64x64 x 257, 112x112 x 33, 56x56 x 1259
    const uint32_t cases[][2] = {{224 * 224, 2}, {64 * 64, 257}, {112 * 112, 33}, {56 * 56, 1259}};
    for (const auto &c : cases) {
        const FastDiv f = FastDiv::make(c[0]);
        const uint32_t x = c[0] * c[1] - 1;
        bad += f.div(x) != c[1] - 1;
        std::printf("plane %u batch %u: last pixel -> image %u (uncorrected form: %u)\n", c[0], c[1], f.div(x),
                    f.div_small(x));
    }
    std::printf("mismatches %llu\n", bad);
    return bad != 0;
}
