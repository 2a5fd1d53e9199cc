/*
 * Test and measurement hook of libdpc.so.  NOT part of the public C ABI
 * (include/dpc.h): the symbol is exported so that the parity tests and the
 * benchmark can run one problem through every stage-2 kernel shape, whatever
 * its size, and compare the results, which are bit-identical for every shape.
 */
#ifndef DPC_HOOKS_H
#define DPC_HOOKS_H

#include "dpc.h"

#ifdef __cplusplus
extern "C" {
#endif

/* `shape` of dpc_stage2_knapsack_shape:
 *   0                      the choice dpc_stage2_knapsack makes from B, L, P
 *   DPC_SHAPE_ROWS         one launch per row, M read from global memory
 *   DPC_SHAPE_WAVE_BASE+k  persistent kernel with wave-private windows, task
 *                          shape k (rows per group x waves per task of 256
 *                          columns each): 1 8x4, 2 8x8, 3 8x2, 4 8x1, 5 16x4,
 *                          6 16x8, 8 16x16
 * (tables narrower than 16 budgets always take the row family) */
#define DPC_SHAPE_ROWS      1
#define DPC_SHAPE_WAVE_BASE 30

/* dpc_stage2_knapsack with the kernel shape as a per-call argument; every
 * other argument, the outputs and the return codes are those of
 * dpc_stage2_knapsack, plus DPC_ERR_SHAPE for an unknown shape. */
int dpc_stage2_knapsack_shape(int32_t B, int32_t L, int32_t P, const int32_t *Topt,
                              const float *I, float *M, uint8_t *K, void *workspace,
                              size_t workspace_bytes, int32_t shape, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DPC_HOOKS_H */
