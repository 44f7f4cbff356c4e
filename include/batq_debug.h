/*
 * libbatq - introspection hooks for tests of the library itself.  Not part of the interface a model uses; the
 * functions are exported by libbatq.so but may change with its internals.
 */
#ifndef BATQ_DEBUG_H
#define BATQ_DEBUG_H

#include "batq.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------------------------
 * Introspection (HOST only, no GPU needed): the work split of the tiled GEMM kernels for an M x K x N problem
 * (M > 64; 0 tiles below) on a device with `compute_units` compute units, as the kernels would walk it (shapes
 * with at most one 128 x 64 tile per compute unit go to another kernel, one tile per workgroup).  Writes 7 ints per
 * tile to tiles[capacity * 7] (HOST): workgroup, first row, first column, width in 64-column strips, K part,
 * first K group (256 elements) and number of K groups; returns the number of tiles (also when capacity is
 * smaller; -1 for invalid arguments).  glu: the gated-output mode of batq_gemm_glu (N % 64 == 0);
 * allow_ksplit: K parts as chosen with a workspace of batq_gemm_workspace() bytes.  For tests of the schedule. */
int batq_debug_tile_schedule(int M, int N, int K, int compute_units, int glu, int allow_ksplit,
                             int* tiles, int capacity);

#ifdef __cplusplus
}
#endif
#endif /* BATQ_DEBUG_H */
