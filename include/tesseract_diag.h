/*
 * tesseract_diag.h -- measurement and diagnostic aids of the Tesseract linear library.
 * Not part of the product interface (tesseract.h): nothing here is needed to compute a
 * layer.  Benchmarks and tests use it to calibrate against the matrix cores' own rate, to
 * check the workgroup -> tile map on the host and to force launch shapes in sweeps.
 */
#ifndef TESSERACT_DIAG_H_
#define TESSERACT_DIAG_H_

#include "tesseract.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Enqueues a register-resident loop of bf16 32x32x16 MFMAs (no memory traffic) on
 * `workgroups` workgroups of 256 threads, `iters` x 16 MFMAs per wavefront (a 4 x 4 grid of
 * accumulator tiles, as in the GEMM kernel), and writes one float per thread to `sink`
 * (device, workgroups*256 floats) so that the loop is not optimised away.  Timing it gives
 * the matrix-core rate this device sustains: workgroups * 4 * iters * 16 * 32768 flop.
 *   data = 0: operands of small integers, the same for every MFMA (little switching);
 *   data = 1: operands drawn like the workloads' (N(0,1) x N(0,0.02), bf16), four A and
 *             four B fragments per lane: the rate the board's power limit leaves to
 *             matrix-core work on realistic operands, with no data movement at all.      */
tess_status tess_probe_mfma_rate(void* sink, int32_t workgroups, int32_t iters, int32_t data,
                                 void* hip_stream);

/* The output tile (tile row *tm, tile column *tn) that workgroup `block` of a launch over
 * a tiles_m x tiles_n tile grid computes.  The same function the kernels use; a bijection
 * from [0, tiles_m*tiles_n) onto the grid.  Pure host arithmetic. */
tess_status tess_tile_of_block(int32_t block, int32_t tiles_m, int32_t tiles_n, int32_t* tm,
                               int32_t* tn);

/* Forces the macro tile (128 or 256; 0 = cost model) and the number of equal K parts (>= 1;
 * 0 = cost model) of every later call of this process, where the shape allows them.
 * tess_linear_plan, tess_linear_workspace_bytes and the launches all see the same
 * override.  Process-wide and not synchronised with running calls: for sweeps and tests. */
tess_status tess_diag_set_plan_override(int32_t tile, int32_t k_splits);

#ifdef __cplusplus
}
#endif
#endif /* TESSERACT_DIAG_H_ */
