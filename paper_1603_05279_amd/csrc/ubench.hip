// Machine microbenchmarks behind the measured peaks bench.py prints next to the published ones
// (include/xnor_ubench.h): register-only matrix-instruction and XOR + bitcount loops, streaming fill / read / copy.
#include "xnor_internal.h"
#include "xnor_ubench.h"

namespace xnor {

typedef int ub_v4i __attribute__((ext_vector_type(4)));
typedef int ub_v8i __attribute__((ext_vector_type(8)));
typedef int ub_v16i __attribute__((ext_vector_type(16)));
typedef float ub_v16f __attribute__((ext_vector_type(16)));

constexpr int UB_ACC = 8;

__global__ __launch_bounds__(256) void ubench_mfma_f4_kernel(float *out, int iters)
{
    ub_v8i a = {(int)threadIdx.x, 0x22222222, 0x2a2a2a2a, 0x22aa22aa, 0, 0, 0, 0};
    ub_v8i b = {0x2222aaaa, 0x22222222, (int)threadIdx.x, 0x2a2a2a2a, 0, 0, 0, 0};
    ub_v16f acc[UB_ACC];
    for (int i = 0; i < UB_ACC; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < UB_ACC; ++i)
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], 4, 4, 0, 127, 0, 127);
    }
    float s = 0.0f;
    for (int i = 0; i < UB_ACC; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    if (s == 1.2345e30f) out[0] = s;            // keeps the loop alive; never true
}

// The same loop on operands that change with every instruction (four A and four B register sets of pseudo-random +-1
// codes): real operands toggle the multiplier inputs, and the chip lowers its clock under that load.  Thread 0 of
// workgroup 0 reports the loop's core-clock count and its 100 MHz wall-clock ticks.
__global__ __launch_bounds__(256) void ubench_mfma_f4_data_kernel(unsigned long long *out, int iters)
{
    ub_v8i a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t h = (threadIdx.x * 8u + j) * 2654435761u + i * 0x9e3779b9u;
            h ^= h >> 15; h *= 0x85ebca6bu; h ^= h >> 13;
            const uint32_t g = h * 0xc2b2ae35u ^ (h >> 16);
            a[i][j] = j < 4 ? (int)(0x22222222u | (h & 0x88888888u)) : 0;      // each nibble 0x2 (+1) or 0xA (-1)
            b[i][j] = j < 4 ? (int)(0x22222222u | (g & 0x88888888u)) : 0;
        }
    }
    ub_v16f acc[UB_ACC];
#pragma unroll
    for (int i = 0; i < UB_ACC; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    const unsigned long long c0 = __builtin_readcyclecounter(), r0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < UB_ACC; ++i)
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i & 3], b[(i >> 1) & 3], acc[i], 4, 4, 0, 127, 0, 127);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < UB_ACC; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    const unsigned long long c1 = __builtin_readcyclecounter(), r1 = wall_clock64();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = c1 - c0 + (s == 1.2345e30f ? 1u : 0u);      // (the sums have to be used)
        out[1] = r1 - r0;
    }
}

__global__ __launch_bounds__(256) void ubench_mfma_i8_kernel(int *out, int iters)
{
    ub_v4i a = {(int)threadIdx.x, 0x01ff01ff, 0x0101ffff, 0x01010101}, b = {0x01ff01ff, (int)threadIdx.x, 0x01010101, 0x0101ffff};
    ub_v16i acc[UB_ACC];
    for (int i = 0; i < UB_ACC; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < UB_ACC; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
    }
    int s = 0;
    for (int i = 0; i < UB_ACC; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    if (s == 0x7fffffff) out[0] = s;
}

__global__ __launch_bounds__(256) void ubench_popcount_kernel(uint32_t *out, int iters, uint32_t seed)
{
    uint32_t acc[16], a[8];
    for (int i = 0; i < 16; ++i) acc[i] = 0;
    for (int j = 0; j < 8; ++j) a[j] = threadIdx.x * 2654435761u + j * seed;
    uint32_t w = seed;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[i] += __builtin_popcount(a[j] ^ (w + i));       // v_xor, v_bcnt with accumulate
        w = w * 1664525u + 1013904223u;
    }
    uint32_t s = 0;
    for (int i = 0; i < 16; ++i) s += acc[i];
    if (s == 0xffffffffu) out[0] = s;
}

__global__ __launch_bounds__(256) void ubench_fill_kernel(uint4 *dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = make_uint4(1, 2, 3, 4);
}

// the same stores with the non-temporal hint (what the convolution uses for results beyond a quarter of the last-level cache)
__global__ __launch_bounds__(256) void ubench_fill_nt_kernel(ub_v4i *dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(ub_v4i{1, 2, 3, 4}, dst + i);
}

__global__ __launch_bounds__(256) void ubench_read_kernel(const uint4 *src, uint32_t *out, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    uint32_t s = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        const uint4 v = src[i];
        s += v.x ^ v.y ^ v.z ^ v.w;
    }
    if (s == 0x9e3779b9u) out[0] = s;           // practically never: the sum only has to be used
}

// Every workgroup streams `passes` times over its own 64 KiB window of a small buffer that stays in L2 (window =
// workgroup index modulo the number of windows): twice the vector L1, so nearly every line comes from L2, the way the
// convolution's weight records do.
__global__ __launch_bounds__(256) void ubench_l2_read_kernel(const uint4 *src, uint32_t *out, int windows, int passes)
{
    const uint4 *w = src + (size_t)(blockIdx.x % (unsigned)windows) * 4096 + threadIdx.x;
    uint32_t s = 0;
    for (int p = 0; p < passes; ++p) {
        uint4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = w[u * 256];
#pragma unroll
        for (int u = 0; u < 16; ++u) s += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
        asm volatile("" : "+v"(s));          // keeps every pass's loads
    }
    if (s == 0x9e3779b9u) out[0] = s;
}

__global__ __launch_bounds__(256) void ubench_copy_kernel(const uint4 *src, uint4 *dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace xnor

using namespace xnor;

extern "C" int xnor_ubench(int kind, int workgroups, int iters, void *buf, size_t bytes, void *hip_stream)
{
    if (!buf) return XNOR_ERR_NULL;
    if (workgroups <= 0 || workgroups > (1 << 20) || iters < 0 || bytes < 4) return XNOR_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(buf) & 15u) return XNOR_ERR_ALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    const dim3 grid((unsigned)workgroups), block(256);
    switch (kind) {
    case XNOR_UBENCH_MFMA_F4: ubench_mfma_f4_kernel<<<grid, block, 0, st>>>(static_cast<float *>(buf), iters); break;
    case XNOR_UBENCH_MFMA_I8: ubench_mfma_i8_kernel<<<grid, block, 0, st>>>(static_cast<int *>(buf), iters); break;
    case XNOR_UBENCH_POPCOUNT: ubench_popcount_kernel<<<grid, block, 0, st>>>(static_cast<uint32_t *>(buf), iters, 0x9e3779b9u); break;
    case XNOR_UBENCH_FILL:
        if (bytes % 32) return XNOR_ERR_SHAPE;
        ubench_fill_kernel<<<grid, block, 0, st>>>(static_cast<uint4 *>(buf), bytes / 16);
        break;
    case XNOR_UBENCH_FILL_NT:
        if (bytes % 32) return XNOR_ERR_SHAPE;
        ubench_fill_nt_kernel<<<grid, block, 0, st>>>(static_cast<ub_v4i *>(buf), bytes / 16);
        break;
    case XNOR_UBENCH_READ:
        if (bytes % 32) return XNOR_ERR_SHAPE;
        ubench_read_kernel<<<grid, block, 0, st>>>(static_cast<const uint4 *>(buf), static_cast<uint32_t *>(buf), bytes / 16);
        break;
    case XNOR_UBENCH_COPY:
        if (bytes % 32) return XNOR_ERR_SHAPE;
        ubench_copy_kernel<<<grid, block, 0, st>>>(static_cast<const uint4 *>(buf), static_cast<uint4 *>(buf) + bytes / 32, bytes / 32);
        break;
    case XNOR_UBENCH_MFMA_F4_DATA:
        if (bytes < 16) return XNOR_ERR_SHAPE;
        ubench_mfma_f4_data_kernel<<<grid, block, 0, st>>>(static_cast<unsigned long long *>(buf), iters);
        break;
    case XNOR_UBENCH_L2_READ:
        if (bytes % 65536 || bytes == 0 || bytes / 65536 > 0x7fffffffu) return XNOR_ERR_SHAPE;
        ubench_l2_read_kernel<<<grid, block, 0, st>>>(static_cast<const uint4 *>(buf), static_cast<uint32_t *>(buf),
                                                      (int)(bytes / 65536), iters);
        break;
    default: return XNOR_ERR_UNSUPPORTED;
    }
    return hip_status(hipGetLastError());
}
