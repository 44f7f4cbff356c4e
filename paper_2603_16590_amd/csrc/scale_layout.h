// Internal layout of E8M0 scale bytes used between the library's own kernels.
//
// The GEMM consumes, per 32-row operand fragment and per 256-wide K stage, one dword per lane
// holding the scales of the four MX blocks that lane feeds to four consecutive matrix
// instructions: lanes 0-31 own the even blocks of the stage, lanes 32-63 the odd ones.
// Scales are therefore stored grouped by 8 K-blocks, group-major, with the even blocks of a
// group first:
//   byte index(row, k) = ((k / 8) * rows + row) * 8 + (k % 8) / 2 + 4 * (k % 2)
// so that a wave reads 32 consecutive rows x 8 bytes = 256 contiguous bytes per fragment.
// Groups are padded to 8 blocks with the neutral scale 127 (2^0); the matching codes are zero.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace batq {

__host__ __device__ inline int scale_groups(int nb) { return (nb + 7) >> 3; }

__host__ __device__ inline size_t scale_bytes_internal(int rows, int nb) {
    return (size_t)scale_groups(nb) * (size_t)rows * 8;
}

__host__ __device__ inline size_t scale_index_internal(int row, int k, int rows) {
    return ((size_t)(k >> 3) * (size_t)rows + (size_t)row) * 8 + (size_t)(((k & 7) >> 1) | ((k & 1) << 2));
}

}  // namespace batq
