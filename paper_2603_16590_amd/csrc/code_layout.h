// Layout of packed E2M1 codes shared by the quantiser, the weight preparation and the GEMM.
//
// The GEMM streams operands global -> LDS in pieces of 1 KiB = 16 rows x 128 K elements
// (64 code bytes per row, one 16-byte chunk per MX block), one piece per wave-level
// LDS-direct load.  Codes are stored so that such a piece is contiguous in memory and is
// already the LDS image the matrix-instruction fragment reads expect:
//   piece(rg, ks)   rg = row / 16, ks = k / 128 (k = K element index), at byte
//                   (rg * stages + ks) * 1024, stages = Kp / 128, Kp = K rounded up to 256
//   inside a piece  row r = row % 16 at byte 64 r; MX block c = (k / 32) % 4 in 16-byte
//                   slot c ^ ((r / 4) % 4) (bank swizzle); element j = k % 32 in byte j / 2,
//                   even j in the low nibble.
// Rows are padded to a multiple of 32 (pad rows are never read into results) and K to a
// multiple of 256 with zero codes (and neutral scales), which contribute nothing.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace batq {

__host__ __device__ inline int code_stages(int nb) { return ((nb + 7) >> 3) << 1; }      // Kp / 128

// Rows are padded to a multiple of 32 so that a 32-row tile of the quantiser always stores two
// whole pieces.
__host__ __device__ inline size_t code_bytes_blocked(int rows, int nb) {
    return (size_t)(((rows + 31) >> 5) << 1) * (size_t)code_stages(nb) * 1024;
}

// Byte offset of the 16-byte chunk holding MX block k of `row`.
__host__ __device__ inline size_t code_chunk_offset(int row, int k, int nb) {
    const int r = row & 15;
    return ((size_t)(row >> 4) * (size_t)code_stages(nb) + (size_t)(k >> 2)) * 1024 + (size_t)r * 64 +
           (size_t)(((k & 3) ^ ((r >> 2) & 3)) << 4);
}

// ---- MXFP8 activation codes (1 byte per element): the same 1 KiB pieces of 16 rows x 64 bytes, a piece
// now covering 64 K elements = 2 MX blocks; the 32 bytes of a block are two 16-byte slots
// (elements 0-15 and 16-31), slot q = 2 (k % 2) + h of row r stored at q ^ ((r / 4) % 4).
__host__ __device__ inline int code8_stages(int nb) { return ((nb + 7) >> 3) << 2; }     // Kp / 64

__host__ __device__ inline size_t code8_bytes_blocked(int rows, int nb) {
    return (size_t)(((rows + 31) >> 5) << 1) * (size_t)code8_stages(nb) * 1024;
}

__host__ __device__ inline size_t code8_slot_offset(int row, int k, int h, int nb) {
    const int r = row & 15;
    return ((size_t)(row >> 4) * (size_t)code8_stages(nb) + (size_t)(k >> 1)) * 1024 + (size_t)r * 64 +
           (size_t)((((k & 1) << 1 | h) ^ ((r >> 2) & 3)) << 4);
}

}  // namespace batq
