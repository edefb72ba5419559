/*
 * libxnor - development hook for tests and benchmarks, kept out of xnor.h on purpose: production callers
 * never need it, results never depend on it.
 */
#ifndef XNOR_TUNING_H
#define XNOR_TUNING_H

#include "xnor.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Forces one workgroup tiling of the matrix-core convolution kernels (sec. 3.2, binary convolution) for every
 * later call of the process, so that tests can run each tiling on small shapes and benchmarks can compare them:
 * mfma_tile = one of the ids listed in csrc/conv_mfma.hip (1, 2, 4, 5, 11, 13, 14, 15), 0 restores the library's per-shape choice;
 * lds_budget_bytes > 0 caps the LDS image of a workgroup (0 keeps the current cap).  Process-global host state
 * (two relaxed atomics): calls racing with it see either setting.  XNOR_ERR_UNSUPPORTED for an unknown id or a
 * budget above 160 KiB.
 */
XNOR_API int xnor_set_tuning(int mfma_tile, int lds_budget_bytes);

#ifdef __cplusplus
}
#endif
#endif /* XNOR_TUNING_H */
