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
    XNOR_UBENCH_COPY = 5,     /* 16-byte loads from the first half of buf, stores to the second half       */
    XNOR_UBENCH_MFMA_F4_DATA = 6, /* MFMA_F4 on operands that change with every instruction (pseudo-random +-1 codes);
                                     writes two 64-bit counts to buf: core clocks and 100 MHz ticks of workgroup 0's loop */
    XNOR_UBENCH_L2_READ = 7,  /* every workgroup reads its 64 KiB window of buf `iters` times with 16-byte loads:
                                 a stream out of L2, like the convolution's weight records                 */
    XNOR_UBENCH_FILL_NT = 8   /* FILL with the non-temporal hint on every store                             */
} xnor_ubench_kind;

/*
 * Enqueues one microbenchmark kernel on hip_stream (no synchronisation; the caller times it with events).
 *   kind       an xnor_ubench_kind
 *   workgroups grid size (256 threads each); the compute loops want a multiple of the 256 compute units
 *   iters      compute kinds: loop iterations per wave (8 matrix instructions, or 128 XOR + bitcount pairs,
 *              per iteration); L2_READ: passes over the window; ignored by FILL, FILL_NT, READ and COPY
 *   buf, bytes device buffer the memory kinds stream over (bytes a multiple of 32, 16-byte aligned; COPY moves
 *              bytes/2; L2_READ: a multiple of 64 KiB, workgroup i reads window i modulo bytes/64 KiB); the compute
 *              kinds write one word per thread to it only when a result has an impossible value (so it needs at
 *              least 4 bytes; MFMA_F4_DATA: 16 bytes, which receive the two counts)
 * Work per launch: MFMA_F4 workgroups*4*iters*8 instructions of 2*32*32*64 flop; MFMA_I8 the same count of
 * 2*32*32*32 op; POPCOUNT workgroups*256*iters*128 lane-operations of 32 binary multiply-accumulates; MFMA_F4_DATA as
 * MFMA_F4; L2_READ workgroups*iters*65536 bytes.
 * Returns an xnor_status.
 */
XNOR_API int xnor_ubench(int kind, int workgroups, int iters, void *buf, size_t bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* XNOR_UBENCH_H */
