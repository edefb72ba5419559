/*
 * libxnor - machine microbenchmarks behind the roofline figures of bench.py: what this GPU delivers on the
 * three inner loops the binary convolution of sec. 3.2 can run on (4-bit-float and int8 matrix
 * instructions, XOR + bitcount on the vector ALU) and on plain streaming of device memory.  Not part of the
 * method; kept beside it so that measured peaks come from committed code.
 */
#ifndef XNOR_UBENCH_H
#define XNOR_UBENCH_H

#include "xnor.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    XNOR_UBENCH_MFMA_F4 = 0,  /* register-only v_mfma_scale_f32_32x32x64_f8f6f4 (4-bit operands), 8 accumulators */
    XNOR_UBENCH_MFMA_I8 = 1,  /* register-only v_mfma_i32_32x32x32_i8, 8 accumulators per wave            */
    XNOR_UBENCH_POPCOUNT = 2, /* register-only v_xor + v_bcnt (accumulating), 128 pairs per iteration      */
    XNOR_UBENCH_FILL = 3,     /* 16-byte stores over `bytes` of buf                                         */
    XNOR_UBENCH_READ = 4,     /* 16-byte loads over `bytes` of buf                                          */
    XNOR_UBENCH_COPY = 5      /* 16-byte loads from the first half of buf, stores to the second half       */
} xnor_ubench_kind;

/*
 * Enqueues one microbenchmark kernel on hip_stream (no synchronisation; the caller times it with events).
 *   kind       an xnor_ubench_kind
 *   workgroups grid size (256 threads each); the compute loops want a multiple of the 256 compute units
 *   iters      compute kinds: loop iterations per wave (8 matrix instructions, or 128 XOR + bitcount pairs,
 *              per iteration); ignored by the memory kinds
 *   buf, bytes device buffer the memory kinds stream over (bytes a multiple of 32, 16-byte aligned; COPY moves
 *              bytes/2); the compute kinds write one word per thread to it only when a result has an impossible
 *              value (so it needs at least 4 bytes)
 * Work per launch: MFMA_F4 workgroups*4*iters*8 instructions of 2*32*32*64 flop; MFMA_I8 the same count of
 * 2*32*32*32 op; POPCOUNT workgroups*256*iters*128 lane-operations of 32 binary multiply-accumulates.
 * Returns an xnor_status.
 */
XNOR_API int xnor_ubench(int kind, int workgroups, int iters, void *buf, size_t bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* XNOR_UBENCH_H */
