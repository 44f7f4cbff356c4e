// MXFP4 x MXFP4 GEMM (the low-bit product of Sec. 3.1: Q(XP) Q(P^-1 W)) on gfx950's
// block-scaled FP4 matrix instruction, fp32 accumulation.
//
// v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in FP4: lane l supplies, for matrix
// row (l % 32), the 32 consecutive K elements of MX block (l / 32) as 16 packed bytes, plus
// that block's E8M0 scale; so one 16-byte chunk of the code layout (code_layout.h) is exactly
// one operand fragment.  Accumulator register r of lane l is element
// (8*(r/4) + 4*(l/32) + r%4, l % 32) of the 32x32 tile.
//
// Kernels:
//   gemm_skinny - M <= 64: 32 output columns per workgroup, K split over its 8 waves.
//   gemm_tiled  - persistent workgroups of 4 or 8 waves, output tiles of 256 rows x 64..256 columns;
//                 codes and scales stream global -> LDS with LDS-direct loads through a 4-stage ring
//                 (XOR-swizzled 16-byte slots); every workgroup takes an equal share of the output,
//                 and the shares of one XCD form a compact block for its L2.  8 waves (two per SIMD)
//                 where the tiles are three or four strips wide.
//   gemm_mid    - few rows and strips: one 128 x 64 tile (and K part) per workgroup, at most one
//                 workgroup per compute unit; X fragments straight from the L2 to registers.
//   gemm_direct - one wave per 32x32 tile with operands straight from global memory; only for
//                 operand arrays of 2 GiB or more (the other kernels use 32-bit load offsets).
#include <algorithm>
#include <type_traits>

#include "batq_internal.h"
#include "code_layout.h"
#include "mxfp4_device.h"
#include "scale_layout.h"
#include "tile_plan.h"

namespace batq {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// element type of the K-split kernels' partial-sum array (selects the partial-sum epilogue)
struct partial_f32 { float v; };
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

template <typename YT>
__device__ __forceinline__ void store_y(YT* p, float v);
template <>
__device__ __forceinline__ void store_y<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_y<uint16_t>(uint16_t* p, float v) { *p = (uint16_t)float_to_bf16_bits(v); }

__device__ __forceinline__ uint4 as_uint4(const batq_u32x4 v) { return uint4{v.x, v.y, v.z, v.w}; }
__device__ __forceinline__ v8i frag(const uint4 v) {
    return v8i{(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};
}

// FP8 (E4M3) operand of one lane (verified on the device with one-hot operands): registers 0-3 hold
// elements 16 kg .. 16 kg + 15 of the instruction's first MX block, registers 4-7 the same elements of
// its second block (kg = lane / 32); the lane's scale byte is still that of block kg.
__device__ __forceinline__ v8i frag8(const uint4 lo, const uint4 hi) {
    return v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
}

// One block-scaled matrix instruction; A8 = the A operand is MXFP8 (cbsz 0) instead of MXFP4 (cbsz 4);
// the B operand (weights) is always MXFP4.
template <bool A8, int OPSEL>
__device__ __forceinline__ v16f mx_mfma(const v8i a, const v8i b, const v16f c, int sa, int sb) {
    if constexpr (A8) return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 4, OPSEL, sa, OPSEL, sb);
    else return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 4, 4, OPSEL, sa, OPSEL, sb);
}

// ------------------------------------------------------------------------------------------
// canonical [rows][nb]  <->  internal group-major scale layout
__global__ void __launch_bounds__(256)
scales_to_internal(const uint8_t* __restrict__ canon, uint8_t* __restrict__ internal, int rows, int nb) {
    const int nbp = scale_groups(nb) * 8;
    const size_t total = (size_t)rows * nbp;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int row = (int)(i / nbp), k = (int)(i % nbp);
        internal[scale_index_internal(row, k, rows)] = k < nb ? canon[(size_t)row * nb + k] : (uint8_t)127;
    }
}

__global__ void __launch_bounds__(256)
scales_to_canonical(const uint8_t* __restrict__ internal, uint8_t* __restrict__ canon, int rows, int nb) {
    const size_t total = (size_t)rows * nb;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int row = (int)(i / nb), k = (int)(i % nb);
        canon[i] = internal[scale_index_internal(row, k, rows)];
    }
}

// row-major [rows][nb*16]  <->  blocked code layout (one thread per 16-byte chunk)
__global__ void __launch_bounds__(256)
codes_to_blocked(const uint8_t* __restrict__ rowmajor, uint8_t* __restrict__ blocked, int rows, int nb) {
    const int nbp = scale_groups(nb) * 8;
    const size_t total = (size_t)rows * nbp;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int row = (int)(i / nbp), k = (int)(i % nbp);
        uint4 v = {0, 0, 0, 0};
        if (k < nb) v = *reinterpret_cast<const uint4*>(rowmajor + ((size_t)row * nb + k) * 16);
        *reinterpret_cast<uint4*>(blocked + code_chunk_offset(row, k, nb)) = v;
    }
}

__global__ void __launch_bounds__(256)
codes_to_rowmajor(const uint8_t* __restrict__ blocked, uint8_t* __restrict__ rowmajor, int rows, int nb) {
    const size_t total = (size_t)rows * nb;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int row = (int)(i / nb), k = (int)(i % nb);
        *reinterpret_cast<uint4*>(rowmajor + i * 16) =
            *reinterpret_cast<const uint4*>(blocked + code_chunk_offset(row, k, nb));
    }
}

// 8-bit codes: row-major [rows][nb*32]  <->  blocked 8-bit layout (one thread per 16-byte slot)
__global__ void __launch_bounds__(256)
codes8_to_blocked(const uint8_t* __restrict__ rowmajor, uint8_t* __restrict__ blocked, int rows, int nb) {
    const int nbp = scale_groups(nb) * 8;
    const size_t total = (size_t)rows * nbp * 2;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int row = (int)(i / (2 * nbp)), kh = (int)(i % (2 * nbp)), k = kh >> 1, h = kh & 1;
        uint4 v = {0, 0, 0, 0};
        if (k < nb) v = *reinterpret_cast<const uint4*>(rowmajor + ((size_t)row * nb + k) * 32 + h * 16);
        *reinterpret_cast<uint4*>(blocked + code8_slot_offset(row, k, h, nb)) = v;
    }
}

__global__ void __launch_bounds__(256)
codes8_to_rowmajor(const uint8_t* __restrict__ blocked, uint8_t* __restrict__ rowmajor, int rows, int nb) {
    const size_t total = (size_t)rows * nb * 2;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int row = (int)(i / (2 * nb)), kh = (int)(i % (2 * nb));
        *reinterpret_cast<uint4*>(rowmajor + i * 16) =
            *reinterpret_cast<const uint4*>(blocked + code8_slot_offset(row, kh >> 1, kh & 1, nb));
    }
}

// ------------------------------------------------------------------------------------------
template <typename YT, bool A8>
__global__ void __launch_bounds__(256)
gemm_direct(const uint8_t* __restrict__ xc, const uint8_t* __restrict__ xs, const uint8_t* __restrict__ wc,
            const uint8_t* __restrict__ ws, int M, int N, int nb, YT* __restrict__ Y, int64_t ldy) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m0 = blockIdx.y * 64 + (wave >> 1) * 32;
    const int n0 = blockIdx.x * 64 + (wave & 1) * 32;
    if (m0 >= M || n0 >= N) return;                       // wave-uniform
    const int i = lane & 31, kg = lane >> 5;
    const int am = min(m0 + i, M - 1), bn = min(n0 + i, N - 1);   // rows past the edge are computed, not stored
    v16f acc = {};
    const int steps = nb >> 1;
    auto load_a = [&](int k) -> v8i {
        if constexpr (A8)   // half kg of both blocks of the step (K is zero-padded to whole groups)
            return frag8(*reinterpret_cast<const uint4*>(xc + code8_slot_offset(am, k & ~1, kg, nb)),
                         *reinterpret_cast<const uint4*>(xc + code8_slot_offset(am, k | 1, kg, nb)));
        else
            return frag(*reinterpret_cast<const uint4*>(xc + code_chunk_offset(am, k, nb)));
    };
    for (int s = 0; s < steps; ++s) {
        const v8i a = load_a(2 * s + kg);
        const uint4 b = *reinterpret_cast<const uint4*>(wc + code_chunk_offset(bn, 2 * s + kg, nb));
        const int sa = xs[scale_index_internal(am, 2 * s + kg, M)];
        const int sb = ws[scale_index_internal(bn, 2 * s + kg, N)];
        acc = mx_mfma<A8, 0>(a, frag(b), acc, sa, sb);
    }
    if (nb & 1) {
        // odd block count: the upper half-wave contributes an all-zero operand
        const int s = steps;
        v8i a = {0, 0, 0, 0, 0, 0, 0, 0};
        uint4 b = {0, 0, 0, 0};
        int sa = 127, sb = 127;
        if (A8 || kg == 0) a = load_a(2 * s);              // 8-bit: every lane holds half of the last block
        if (kg == 0) {
            b = *reinterpret_cast<const uint4*>(wc + code_chunk_offset(bn, 2 * s, nb));
            sa = xs[scale_index_internal(am, 2 * s, M)];
            sb = ws[scale_index_internal(bn, 2 * s, N)];
        }
        acc = mx_mfma<A8, 0>(a, frag(b), acc, sa, sb);
    }
    const int col = n0 + i;
    if (col < N) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = m0 + 8 * (r >> 2) + 4 * kg + (r & 3);
            if (row < M) store_y<YT>(Y + (size_t)row * ldy + col, acc[r]);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Small M (decode shapes): the time goes into streaming the weight codes once, so the work is
// split along K as well.  A workgroup of 8 waves owns 32 output columns (all rows); wave w takes an
// equal share of the K groups (256 elements = 4 matrix instructions, whose 8 scale bytes per row
// are two dwords), issues all loads of a group before its matrix instructions, and the 8 partial
// tiles are summed through LDS in a fixed order.  K is zero-padded to whole groups in both
// operands, so there is no K tail.
constexpr int kSkinnyWaves = 8;

// RT = 32-row tiles of X handled together (1 or 2), sharing the weight loads; A8 = MXFP8 activations;
// GLU = gated output: a workgroup owns 32 output columns = the 32 gate and the 32 up columns of one
// 64-column group of the interleaved weight (sharing the loads of X), and stores silu(gate) * up to M x N/2.
// WIDE (not with GLU): a workgroup owns 64 output columns instead of 32, which halves how often the X codes
// are read; used when N is large enough that 64-column workgroups still fill the chip.
// NARROW (not with GLU or WIDE): a workgroup owns 16 output columns, for N so small that 32-column workgroups would
// leave half the compute units without one: lanes 16-31 of each half wave load what lanes 0-15 load (the same cache
// lines) and their columns of the matrix instructions' results are dropped.
template <typename YT, int RT, bool A8, bool GLU, bool WIDE, bool NARROW = false>
__global__ void __launch_bounds__(kSkinnyWaves * 64)
gemm_skinny(const uint8_t* __restrict__ xc, const uint8_t* __restrict__ xs, const uint8_t* __restrict__ wc,
            const uint8_t* __restrict__ ws, int M, int N, int nb, YT* __restrict__ Y, int64_t ldy,
            float* __restrict__ partial) {
    static_assert(!(GLU && WIDE), "the gated kernel already takes two column groups");
    static_assert(!(NARROW && (GLU || WIDE)), "16 columns only for the plain kernel");
    constexpr int NG = (GLU || WIDE) ? 2 : 1;               // 32-column groups of the weight per workgroup
    __shared__ float part[kSkinnyWaves][16][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n0 = blockIdx.x * (NARROW ? 16 : 32 * NG);    // first weight column
    const int i = lane & 31, kg = lane >> 5;
    const int groups = scale_groups(nb);
    // gridDim.y > 1: the K groups are first cut into gridDim.y parts, one per workgroup row, whose sums go
    // to partial[part][M][N] (fp32) for splitk_reduce_rows
    const int p_begin = groups * blockIdx.y / gridDim.y, p_groups = groups * (blockIdx.y + 1) / gridDim.y - p_begin;
    const int g_begin = p_begin + p_groups * wave / kSkinnyWaves, g_end = p_begin + p_groups * (wave + 1) / kSkinnyWaves;
    // block k = 8 g + 2 j + kg (j = 0..3): chunk (k / 4, k % 4) = (2 g + j / 2, 2 (j % 2) + kg)
    int bn[NG], swb[NG];
    const uint8_t* pb[NG];
#pragma unroll
    for (int c = 0; c < NG; ++c) {
        bn[c] = min(n0 + 32 * c + (NARROW ? (i & 15) : i), N - 1);   // rows and columns past the edge are computed, not stored
        const int rb = bn[c] & 15;
        pb[c] = wc + (size_t)(bn[c] >> 4) * code_stages(nb) * 1024 + rb * 64;
        swb[c] = (rb >> 2) & 3;
    }
    int am[RT], swa[RT];
    const uint8_t* pa[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        am[t] = min(32 * t + i, M - 1);
        const int ra = am[t] & 15;
        pa[t] = xc + (size_t)(am[t] >> 4) * (A8 ? code8_stages(nb) : code_stages(nb)) * 1024 + ra * 64;
        swa[t] = (ra >> 2) & 3;
    }
    constexpr int AR = A8 ? 2 : 1;                          // 16-byte slots of A per lane and matrix instruction
    v16f acc[RT][NG];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int c = 0; c < NG; ++c) acc[t][c] = v16f{};
    // operands of group g are fetched while group g-1 is multiplied
    uint4 a[RT][4][AR], b[NG][4], an[RT][4][AR], bn4[NG][4];
    int sa[RT], sb[NG], san[RT], sbn[NG];
    auto load_group = [&](int g, uint4 (&ga)[RT][4][AR], uint4 (&gb)[NG][4], int (&gsa)[RT], int (&gsb)[NG]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int piece = 2 * g + (j >> 1), slot = 2 * (j & 1) + kg;
#pragma unroll
            for (int c = 0; c < NG; ++c)
                gb[c][j] = *reinterpret_cast<const uint4*>(pb[c] + (size_t)piece * 1024 + ((slot ^ swb[c]) << 4));
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                if constexpr (A8) {
                    // 8-bit pieces hold the 2 blocks of one matrix instruction: piece 4 g + j, and the lane takes
                    // elements 16 kg .. 16 kg + 15 of both (slots kg and 2 + kg)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        ga[t][j][h] = *reinterpret_cast<const uint4*>(pa[t] + (size_t)(4 * g + j) * 1024 +
                                                                     (((2 * h + kg) ^ swa[t]) << 4));
                } else {
                    ga[t][j][0] = *reinterpret_cast<const uint4*>(pa[t] + (size_t)piece * 1024 + ((slot ^ swa[t]) << 4));
                }
            }
        }
        // byte j of the dword at 4 kg of the row's scale word is the scale of block 8 g + 2 j + kg
#pragma unroll
        for (int c = 0; c < NG; ++c) gsb[c] = *reinterpret_cast<const int*>(ws + ((size_t)g * N + bn[c]) * 8 + 4 * kg);
#pragma unroll
        for (int t = 0; t < RT; ++t) gsa[t] = *reinterpret_cast<const int*>(xs + ((size_t)g * M + am[t]) * 8 + 4 * kg);
    };
    if (g_begin < g_end) load_group(g_begin, a, b, sa, sb);
    for (int g = g_begin; g < g_end; ++g) {
        if (g + 1 < g_end) load_group(g + 1, an, bn4, san, sbn);
        auto afrag = [&](int t, int j) -> v8i {
            if constexpr (A8) return frag8(a[t][j][0], a[t][j][1]);
            else return frag(a[t][j][0]);
        };
#pragma unroll
        for (int t = 0; t < RT; ++t)
#pragma unroll
            for (int c = 0; c < NG; ++c) {
                acc[t][c] = mx_mfma<A8, 0>(afrag(t, 0), frag(b[c][0]), acc[t][c], sa[t], sb[c]);
                acc[t][c] = mx_mfma<A8, 1>(afrag(t, 1), frag(b[c][1]), acc[t][c], sa[t], sb[c]);
                acc[t][c] = mx_mfma<A8, 2>(afrag(t, 2), frag(b[c][2]), acc[t][c], sa[t], sb[c]);
                acc[t][c] = mx_mfma<A8, 3>(afrag(t, 3), frag(b[c][3]), acc[t][c], sa[t], sb[c]);
            }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int c = 0; c < NG; ++c) b[c][j] = bn4[c][j];
#pragma unroll
            for (int t = 0; t < RT; ++t)
#pragma unroll
                for (int h = 0; h < AR; ++h) a[t][j][h] = an[t][j][h];
        }
#pragma unroll
        for (int c = 0; c < NG; ++c) sb[c] = sbn[c];
#pragma unroll
        for (int t = 0; t < RT; ++t) sa[t] = san[t];
    }
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        // 1024 outputs per 32 x 32 tile, two per thread; element (r, l) of the tile is
        // (8 (r / 4) + 4 (l / 32) + r % 4, l % 32)
        float v[NG][2];
#pragma unroll
        for (int c = 0; c < NG; ++c) {
            if (t > 0 || c > 0) __syncthreads();            // the previous tile's partial sums have been read
#pragma unroll
            for (int r = 0; r < 16; ++r) part[wave][r][lane] = acc[t][c][r];
            __syncthreads();
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int e = threadIdx.x + h * kSkinnyWaves * 64;
                const int r = e >> 6, l = e & 63;
                float sum = part[0][r][l];
#pragma unroll
                for (int w = 1; w < kSkinnyWaves; ++w) sum += part[w][r][l];
                v[c][h] = sum;
            }
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int e = threadIdx.x + h * kSkinnyWaves * 64;
            const int r = e >> 6, l = e & 63;
            const int row = 32 * t + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
            if constexpr (GLU) {
                const int col = blockIdx.x * 32 + (l & 31);
                if (row < M && col < N / 2) store_y<YT>(Y + (size_t)row * ldy + col, swiglu_f32(v[0][h], v[1][h]));
            } else {
#pragma unroll
                for (int c = 0; c < NG; ++c) {
                    const int col = n0 + 32 * c + (l & 31);
                    if (row < M && col < N && (!NARROW || (l & 31) < 16)) {
                        if (gridDim.y > 1) partial[((size_t)blockIdx.y * M + row) * N + col] = v[c][h];
                        else store_y<YT>(Y + (size_t)row * ldy + col, v[c][h]);
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Tiled kernel.  Persistent workgroups, one per compute unit.  An output tile is 256 rows by 64 NJ
// columns (NJ = 1..4 "strips" of 64 columns); the waves sit (8 / RT) x 2 on it, each holding RT x NJ
// matrix tiles (32 RT x 32 NJ outputs) in up to 64 RT accumulator registers.  RT = 4: 4 waves, one per
// SIMD (the 8-bit kernel); RT = 2: 8 waves, two per SIMD, 128 accumulator and 128 other registers each:
// while one wave of a SIMD converts and stores its outputs or waits for LDS, the other one issues.
// K advances in stages of 128 elements (64 code bytes per row).  Codes and scales go
// global -> LDS with LDS-direct loads (no VGPR staging, no ds_write): a ring of 4 stage
// buffers keeps three stages in flight.  Scales of a whole 256-element K group (two stages)
// are fetched once per group into a 2-deep ring.
//
// Work split: the strips of all row panels are put in one linear order (column bands, inside
// a band row panel by row panel) and every workgroup takes an equal contiguous share of it,
// which it cuts into tiles of at most 4 strips.  Workgroups go to the 8 XCDs round-robin, so
// workgroup b works on share (b % 8) * (workgroups / 8) + b / 8: the shares of one XCD are
// contiguous and its L2 sees a compact block of the output.
constexpr int kStageBytes = 64;            // code bytes per row per stage (128 elements, 4 MX blocks)
constexpr int kOperandStage = kTile * kStageBytes;        // 16 KiB per operand per stage
constexpr int kStageLds = 2 * kOperandStage;               // A then B
constexpr int kRing = 4;                   // stage buffers
constexpr int kScaleGroupLds = 2 * kTile * 8;              // A then B scale bytes of one K group (4 KiB)
constexpr int kEpilogueWaveLds = 16 * 256;                 // per wave of 4: 16 output rows x 256 bytes
constexpr int kEpilogueLds0 = kRing * kStageLds + 2 * kScaleGroupLds;
constexpr int kTiledLds = kEpilogueLds0 + 4 * kEpilogueWaveLds;     // 152 KiB
// rows of a wave's staged output block and the bytes of its staging area: 16 KiB per workgroup either way
template <int RT> constexpr int kEpilogueBlockRows = RT == 4 ? 16 : 8;
template <int RT> constexpr int kEpilogueWaveBytes = kEpilogueBlockRows<RT> * 256;

// 16-byte slot swizzle inside a 64-byte LDS row: the 32 rows a fragment read touches, and the
// 16 rows x 4 slots an LDS-direct load writes, both spread over all banks.
__device__ __forceinline__ int slot_swizzle(int row) { return (row >> 2) & 3; }

// LDS-direct loads: lane i of the wave writes its 16 (4) bytes at LDS address m0 + 16 i (4 i).
// `gbase` and `lds_addr` are wave-uniform.  Completion is tracked by vmcnt, in issue order.
__device__ __forceinline__ void dma16(const void* gbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(gbase), "s"(lds_addr) : "memory");
}
__device__ __forceinline__ void dma4(const void* gbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :: "v"(voff), "s"(gbase), "s"(lds_addr) : "memory");
}
// Loads to registers whose completion the caller awaits itself (wait_vmcnt, in issue order with the LDS-direct
// loads): the compiler sees no memory access, so it neither adds waits of its own nor knows that the result is
// late - every use must follow the wait and a ready() on the register.
__device__ __forceinline__ void load16_async(batq_u32x4& dst, const void* gbase, uint32_t voff) {
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(gbase) : "memory");
}
__device__ __forceinline__ void load4_async(int& dst, const void* gbase, uint32_t voff) {
    asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(voff), "s"(gbase) : "memory");
}
template <typename V>
__device__ __forceinline__ void ready(V& v) { asm volatile("; landed: %0" : "+v"(v)); }
// s_waitcnt vmcnt(N) only (expcnt and lgkmcnt left at their maxima), gfx9 encoding.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// s_waitcnt lgkmcnt(0) only: the wave's LDS reads have delivered.
__device__ __forceinline__ void wait_lds() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// One matrix instruction of the grid of 32x32 tiles a wave owns; ZERO starts the accumulation.
template <int KK, bool ZERO>
__device__ __forceinline__ void mfma_one(v16f& acc, const uint4& a, const uint4& b, int sa, int sb) {
    if constexpr (ZERO)
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag(a), frag(b), v16f{}, 4, 4, KK, sa, KK, sb);
    else
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag(a), frag(b), acc, 4, 4, KK, sa, KK, sb);
}

template <int RT>
struct TiledCtx {
    static_assert(RT == 4 || RT == 2, "4 or 8 waves");
    static constexpr int kWaves = 16 / RT;          // 2 columns of 8 / RT waves
    static constexpr int kPA = RT;                  // 1 KiB pieces of A per wave and stage (16 in all)
    static constexpr int kPBMax = RT;               // most pieces of B per wave and stage
    static constexpr int kSc = RT / 2;              // scale loads per wave, operand and K group (64 dwords each)
    // pieces of B per wave and stage for a tile nj strips wide (4 nj in all; with 8 waves the last ones may
    // fall beyond the tile: they are loaded like the others, into the unused rest of the stage buffer)
    static constexpr __device__ __host__ int pb(int nj) { return (4 * nj + kWaves - 1) / kWaves; }
    // global -> LDS
    const uint8_t* xc; const uint8_t* wc; const uint8_t* xs; const uint8_t* ws;
    uint32_t aoff[kPA], boff[kPBMax], sao[kSc], sbo[kSc];
    uint32_t lds0, lds_sc, row_group_bytes;   // bytes of one 16-row group of a code array (all of K)
    int M, N, wave, lane;
    int T, s0;        // stages of the aimed tile and the first of them (stage = 128 K elements; K parts start on K groups)
    // LDS -> registers
    const uint8_t* smem;
    int a_rd, b_rd, sc_a_rd, sc_b_rd, kg, fsw;

    // Per-lane load offsets of a tile.  Wave w, load j copies the 1 KiB piece of row group
    // (tile row / 16 + kPA w + j) of A, and (tile column / 16 + pb w + j) of B, into LDS rows
    // 16 (kPA w + j) .. + 15 (16 (pb w + j) ..) of a stage buffer; the blocked code layout already is
    // the swizzled LDS image, so lane i just moves bytes 16 i .. 16 i + 15.  Row groups past the
    // edge are clamped to the last one (their results are never stored).
    __device__ __forceinline__ void aim(const Tile& t) {
        const int rgA = (M + 15) >> 4, rgB = (N + 15) >> 4;
        int lane = this->lane;
        asm volatile("" : "+v"(lane));      // recompute the lane terms per tile instead of keeping them in registers
        T = 2 * t.ng;
        s0 = 2 * t.g0;
        const int npb = pb(t.nj);
#pragma unroll
        for (int j = 0; j < kPA; ++j)
            aoff[j] = (uint32_t)min((t.m0 >> 4) + kPA * wave + j, rgA - 1) * row_group_bytes + lane * 16;
#pragma unroll
        for (int j = 0; j < kPBMax; ++j)
            boff[j] = (uint32_t)min((t.n0 >> 4) + npb * wave + j, rgB - 1) * row_group_bytes + lane * 16;
        // scales: per K group, A and B each 256 rows x 2 dwords; wave w loads dwords 64 kSc w .. + 64 kSc - 1
        // of each (pieces of 64).  B rows beyond the tile's 64 nj are fetched and not used.
#pragma unroll
        for (int j = 0; j < kSc; ++j) {
            const int d = 64 * kSc * wave + 64 * j + lane;
            sao[j] = ((uint32_t)min(t.m0 + (d >> 1), M - 1) * 2 + (d & 1)) * 4;
            sbo[j] = ((uint32_t)min(t.n0 + (d >> 1), N - 1) * 2 + (d & 1)) * 4;
        }
    }
    // The loads of one stage, in a fixed order: parts 0..kPA-1 = this wave's A pieces, parts kPA..kPA+pb-1
    // its B pieces, part kPA+pb = the scales of the K group an even stage opens (2 kSc dword loads).
    // Completion is counted per thread in this order.
    __device__ __forceinline__ void issue_scales(int s) const {
        const int g = s >> 1;
        const uint32_t sbuf = lds_sc + (uint32_t)(g & 1) * kScaleGroupLds + (uint32_t)wave * (256 * kSc);
        const uint8_t* sag = xs + (size_t)(g + (s0 >> 1)) * M * 8;
        const uint8_t* sbg = ws + (size_t)(g + (s0 >> 1)) * N * 8;
#pragma unroll
        for (int j = 0; j < kSc; ++j) dma4(sag, sao[j], sbuf + j * 256);
#pragma unroll
        for (int j = 0; j < kSc; ++j) dma4(sbg, sbo[j], sbuf + kTile * 8 + j * 256);
    }
    template <int PART>
    __device__ __forceinline__ void issue_part(int s, int nj, bool even) const {
        const uint32_t buf = lds0 + (uint32_t)(s & (kRing - 1)) * kStageLds;
        if constexpr (PART < kPA) {
            dma16(xc + (size_t)(s + s0) * 1024, aoff[PART], buf + (uint32_t)(kPA * wave + PART) * 1024);
        } else {
            const int npb = pb(nj);
            if (PART < kPA + npb)
                dma16(wc + (size_t)(s + s0) * 1024, boff[(PART - kPA) & (kPBMax - 1)],
                      buf + kOperandStage + (uint32_t)(npb * wave + PART - kPA) * 1024);
            else if (PART == kPA + npb && even)
                issue_scales(s);
        }
    }
    // First stages of a tile (all ring slots must be free): kPA + pb loads each, 2 kSc more on even stages.
    __device__ __forceinline__ void issue_prologue(int nj) const {
        const int n = T < kRing ? T : kRing;
        const int npb = pb(nj);
        for (int s = 0; s < n; ++s) {
            issue_part<0>(s, nj, false);
            issue_part<1>(s, nj, false);
            if constexpr (kPA == 4) {
                issue_part<2>(s, nj, false);
                issue_part<3>(s, nj, false);
            }
            issue_part<kPA>(s, nj, false);
            if (npb > 1) issue_part<kPA + 1>(s, nj, false);
            if constexpr (kPBMax == 4) {
                if (npb > 2) issue_part<kPA + 2>(s, nj, false);
                if (npb > 3) issue_part<kPA + 3>(s, nj, false);
            }
            if ((s & 1) == 0) issue_scales(s);
        }
    }
    // Where this lane reads its fragments and scales from: row (wave row base + 32 i + l32),
    // slot ((2 half + kg) ^ f(row)).
    __device__ __forceinline__ void aim_reads(int nj, int wm, int wn, int l32) {
        a_rd = (wm * 32 * RT + l32) * kStageBytes;
        b_rd = kOperandStage + (wn * 32 * nj + l32) * kStageBytes;
        sc_a_rd = ((wm * 32 * RT + l32) * 2 + kg) * 4;
        sc_b_rd = kTile * 8 + ((wn * 32 * nj + l32) * 2 + kg) * 4;
    }
    // in the order the matrix instructions consume them: a0, b0.., a1..
    template <int NJ>
    __device__ __forceinline__ void read_frags(int s, int half, uint4 (&fa)[RT], uint4 (&fb)[NJ]) const {
        const uint8_t* base = smem + (s & (kRing - 1)) * kStageLds + (((2 * half + kg) ^ fsw) << 4);
        fa[0] = *reinterpret_cast<const uint4*>(base + a_rd);
#pragma unroll
        for (int j = 0; j < NJ; ++j) fb[j] = *reinterpret_cast<const uint4*>(base + b_rd + j * 32 * kStageBytes);
#pragma unroll
        for (int i = 1; i < RT; ++i) fa[i] = *reinterpret_cast<const uint4*>(base + a_rd + i * 32 * kStageBytes);
    }
    // fragment IDX of that order alone
    template <int NJ, int IDX>
    __device__ __forceinline__ void read_frag_one(int s, int half, uint4 (&fa)[RT], uint4 (&fb)[NJ]) const {
        const uint8_t* base = smem + (s & (kRing - 1)) * kStageLds + (((2 * half + kg) ^ fsw) << 4);
        if constexpr (IDX == 0) fa[0] = *reinterpret_cast<const uint4*>(base + a_rd);
        else if constexpr (IDX <= NJ) fb[IDX - 1] = *reinterpret_cast<const uint4*>(base + b_rd + (IDX - 1) * 32 * kStageBytes);
        else fa[IDX - NJ] = *reinterpret_cast<const uint4*>(base + a_rd + (IDX - NJ) * 32 * kStageBytes);
    }
    template <int NJ>
    __device__ __forceinline__ void read_scales(int g, int (&sa)[RT], int (&sb)[NJ]) const {
        const uint8_t* sp = smem + kRing * kStageLds + (g & 1) * kScaleGroupLds;
#pragma unroll
        for (int i = 0; i < RT; ++i) sa[i] = *reinterpret_cast<const int*>(sp + sc_a_rd + i * 256);
#pragma unroll
        for (int j = 0; j < NJ; ++j) sb[j] = *reinterpret_cast<const int*>(sp + sc_b_rd + j * 256);
    }
};

// Loads [P0, P1) of stage s, in the fixed order (NJ static).
template <int RT, int NJ, bool EVEN, int P0, int P1>
__device__ __forceinline__ void issue_range(const TiledCtx<RT>& c, int s) {
    if constexpr (P0 < P1) {
        if constexpr (P0 < TiledCtx<RT>::kPA + TiledCtx<RT>::pb(NJ)) c.template issue_part<P0>(s, NJ, false);
        else if constexpr (EVEN) c.issue_scales(s);
        issue_range<RT, NJ, EVEN, P0 + 1, P1>(c, s);
    }
}
// Fragments [R0, R1) of the consumption order.
template <int RT, int NJ, int R0, int R1>
__device__ __forceinline__ void read_frag_range(const TiledCtx<RT>& c, int s, int half, uint4 (&fa)[RT], uint4 (&fb)[NJ]) {
    if constexpr (R0 < R1) {
        c.template read_frag_one<NJ, R0>(s, half, fa, fb);
        read_frag_range<RT, NJ, R0 + 1, R1>(c, s, half, fa, fb);
    }
}

// One K step of a stage: its RT x NJ matrix instructions in row-major tile order, and after each of them one LDS
// fragment read (two where a K step has fewer instructions than fragments) and its share of a set of load parts, so that neither the
// LDS pipe nor the vector-memory address path sees a burst (a wave that blocks on either cannot issue its next
// matrix instruction: measured on cfg3, bunched reads and loads cost 360 of 1490 cycles per stage).
//   KK      scale byte of the K step (op_sel); ZERO: the K step starts the accumulators
//   RD      read the fragments of (rd_stage, rd_half) into ra / rb, one per matrix instruction, in the order the
//           next K step consumes them (a0, b0.., a1..)
//   TE      the stage `st` whose load parts [P0, P1) are issued here is even (its last part = the scales of a K group)
template <int RT, int NJ, int KK, bool ZERO, bool RD, bool TE, int P0, int P1, int M>
__device__ __forceinline__ void wide_k_step(const TiledCtx<RT>& c, v16f (&acc)[RT][NJ], const uint4 (&a)[RT],
                                            const uint4 (&b)[NJ], const int (&sa)[RT], const int (&sb)[NJ], int rd_stage,
                                            int rd_half, uint4 (&ra)[RT], uint4 (&rb)[NJ], int st) {
    constexpr int NM = RT * NJ, NR = RT + NJ, kPer = (NR + NM - 1) / NM;
    if constexpr (M < NM) {
        constexpr int i = M / NJ, j = M % NJ;
        mfma_one<KK, ZERO>(acc[i][j], a[i], b[j], sa[i], sb[j]);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (RD)
            read_frag_range<RT, NJ, (M * kPer < NR ? M * kPer : NR), ((M + 1) * kPer < NR ? (M + 1) * kPer : NR)>(
                c, rd_stage, rd_half, ra, rb);
        constexpr int np = P1 - P0;
        issue_range<RT, NJ, TE, P0 + M * np / NM, P0 + (M + 1) * np / NM>(c, st);
        __builtin_amdgcn_sched_barrier(0);
        wide_k_step<RT, NJ, KK, ZERO, RD, TE, P0, P1, M + 1>(c, acc, a, b, sa, sb, rd_stage, rd_half, ra, rb, st);
    }
}

// One K stage (two matrix-instruction K steps) of the software pipeline (with 4 waves: tiles three or four strips
// wide).
//   NJ       32-column matrix tiles per wave
//   PAR      parity of the stage inside its K group (selects the scale bytes: op_sel 2 PAR, 2 PAR + 1)
//   WAIT     loads that may stay in flight once stage s+1 has landed (-1: there is no stage s+1)
//   ISSUE_A  start the loads of stage s+4 (the first half of its parts) after the barrier, into the ring slot this
//            stage frees there
//   ISSUE_B  finish the loads of stage s+3 (the second half of its parts; the slot was freed by the barrier of
//            stage s-1) during the first K step
//   FIRST    first stage of a tile: its first K step starts the accumulators from zero
// On entry a0/b0 hold the fragments of (s, first half); on exit those of (s+1, first half).  The barrier sits
// between the two K steps: by then every wave has stage s completely in registers (the second half's fragments are
// read under the first K step), and once all have also seen stage s+1 land, its fragments are read under the second
// K step.  The loads of a stage are thus issued one by one over a whole stage length, from the middle of stage s-4
// to the middle of stage s-3, and have two to three stages to land.  When stage s+1 is awaited, stages s+2 and s+3
// have been issued completely and stage s+4 not at all.
template <int RT, int NJ, int PAR, int WAIT, bool ISSUE_A, bool ISSUE_B, bool FIRST>
__device__ __forceinline__ void tiled_stage(const TiledCtx<RT>& c, int s, v16f (&acc)[RT][NJ], uint4 (&a0)[RT],
                                            uint4 (&b0)[NJ], int (&sa)[RT], int (&sb)[NJ]) {
    constexpr int kParts = TiledCtx<RT>::kPA + TiledCtx<RT>::pb(NJ) + 1, kA = (kParts + 1) / 2;
    uint4 a1[RT], b1[NJ];
    // first K step: the second half's fragments, and the rest of stage s+3's loads (stage s+3 has the other parity)
    wide_k_step<RT, NJ, 2 * PAR, FIRST, true, PAR == 1, (ISSUE_B ? kA : 0), (ISSUE_B ? kParts : 0), 0>(
        c, acc, a0, b0, sa, sb, s, 1, a1, b1, s + 3);
    int sna[RT], snb[NJ];
    if constexpr (WAIT >= 0) {
        wait_vmcnt<WAIT>();
        wait_lds();                                         // this wave's fragments of stage s are in registers
        __syncthreads();
        if constexpr (PAR == 1) c.template read_scales<NJ>((s + 1) >> 1, sna, snb);
    }
    __builtin_amdgcn_sched_barrier(0);
    // second K step: the next stage's first fragments, and the first loads of stage s+4 (same parity as s)
    wide_k_step<RT, NJ, 2 * PAR + 1, false, (WAIT >= 0), PAR == 0, 0, ((WAIT >= 0 && ISSUE_A) ? kA : 0), 0>(
        c, acc, a1, b1, sa, sb, s + 1, 0, a0, b0, s + 4);
    if constexpr (WAIT >= 0 && PAR == 1) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < RT; ++i) sa[i] = sna[i];
#pragma unroll
        for (int j = 0; j < NJ; ++j) sb[j] = snb[j];
    }
}

// The same stage for tiles one or two strips wide, 4 waves.  Their 8 or 16 matrix instructions per stage are too few to
// hide a barrier followed by the LDS reads of the next fragments in the last quarter of the stage, so here the
// fragments run a whole stage ahead: on entry a/b hold both K steps of stage s, the barrier at the top makes
// stage s+1 visible (and the slot of stage s, read a stage ago, free), and the reads of stage s+1 and the loads
// of stage s+4 are spread under the stage's own matrix instructions.  Same WAIT / ISSUE / FIRST meaning and the
// same load accounting as tiled_stage: no load of stage s+4 has been issued when stage s+1 is awaited.
template <int NJ, int PAR, int WAIT, bool ISSUE, bool FIRST>
__device__ __forceinline__ void narrow_stage(const TiledCtx<4>& c, int s, v16f (&acc)[4][NJ], uint4 (&a)[2][4],
                                             uint4 (&b)[2][NJ], int (&sa)[4], int (&sb)[NJ]) {
    static_assert(NJ <= 2, "narrow tiles only");
    uint4 na[2][4], nb[2][NJ];
    int sna[4], snb[NJ];
    constexpr bool kNext = WAIT >= 0, kIssue = WAIT >= 0 && ISSUE;
    if constexpr (kNext) {
        wait_vmcnt<WAIT>();
        wait_lds();                                         // this wave's fragments of stage s are in registers
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) mfma_one<2 * PAR, FIRST>(acc[i][j], a[0][i], b[0][j], sa[i], sb[j]);
        __builtin_amdgcn_sched_barrier(0);
        if (i == 0) {
            if constexpr (kNext) c.read_frags<NJ>(s + 1, 0, na[0], nb[0]);
        } else if (i == 1) {
            if constexpr (kIssue) issue_range<4, NJ, PAR == 0, 0, 2>(c, s + 4);
        } else if (i == 2) {
            if constexpr (kNext) c.read_frags<NJ>(s + 1, 1, na[1], nb[1]);
        } else {
            if constexpr (kIssue) issue_range<4, NJ, PAR == 0, 2, 4>(c, s + 4);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) mfma_one<2 * PAR + 1, false>(acc[i][j], a[1][i], b[1][j], sa[i], sb[j]);
        __builtin_amdgcn_sched_barrier(0);
        if (i == 0) {
            if constexpr (kNext && PAR == 1) c.read_scales<NJ>((s + 1) >> 1, sna, snb);
        } else if (i == 1) {
            if constexpr (kIssue) issue_range<4, NJ, PAR == 0, 4, 5 + NJ>(c, s + 4);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (kNext) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int i = 0; i < 4; ++i) a[h][i] = na[h][i];
#pragma unroll
            for (int j = 0; j < NJ; ++j) b[h][j] = nb[h][j];
        }
        if constexpr (PAR == 1) {
#pragma unroll
            for (int i = 0; i < 4; ++i) sa[i] = sna[i];
#pragma unroll
            for (int j = 0; j < NJ; ++j) sb[j] = snb[j];
        }
    }
}

// Stage of a tile NJ strips wide: with 4 waves, narrow tiles keep both K steps' fragments in `a`, `b`; all others
// the first K step's.
// ISSUE: stage s+4 exists and is loaded into the slot this stage frees; PREV: the same was true of stage s-1 (wide
// tiles issue a stage's loads in two halves, the second half during the following stage).
template <int RT, int NJ> constexpr bool kNarrowStages = RT == 4 && NJ <= 2;
template <int RT, int NJ, int PAR, int WAIT, bool ISSUE, bool FIRST, bool PREV = true>
__device__ __forceinline__ void any_stage(const TiledCtx<RT>& c, int s, v16f (&acc)[RT][NJ], uint4 (&a)[2][RT],
                                          uint4 (&b)[2][NJ], int (&sa)[RT], int (&sb)[NJ]) {
    if constexpr (kNarrowStages<RT, NJ>) narrow_stage<NJ, PAR, WAIT, ISSUE, FIRST>(c, s, acc, a, b, sa, sb);
    else tiled_stage<RT, NJ, PAR, WAIT, ISSUE, (PREV && !FIRST), FIRST>(c, s, acc, a[0], b[0], sa, sb);
}

// Epilogue of a tile: RT x NJ output tiles of 32 x 32 of this wave (rows m0 + wm*32*RT.., columns n0 + wn*32*NJ..)
// -> Y; value(i, j, e) = element e (accumulator register order) of output tile (i, j).
// `ep_lds` is the wave's private LDS staging area (kEpilogueWaveBytes<RT>).
template <int NJ, typename YT, int RT, typename F>
__device__ __forceinline__ void store_tile_impl(F value, uint8_t* ep_lds, int lane, int wm, int wn, int m0, int n0,
                                                int M, int N, YT* __restrict__ Y, int64_t ldy) {
    // ---- epilogue: accumulators -> Y
    // (lane-derived addresses are recomputed per tile rather than kept in registers across the main loop)
    int lane_e = lane;
    asm volatile("" : "+v"(lane_e));
    if constexpr (sizeof(YT) == 2) {
        // bf16: transpose through a wave-private LDS buffer so that every lane stores 16 contiguous
        // bytes.  Needs the wave's whole width inside N and 16-byte aligned rows (wave-uniform).
        const bool fast = n0 + (wn + 1) * 32 * NJ <= N && (ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(Y) & 15) == 0;
        if (fast) {
            const bool big = (size_t)M * (size_t)N * sizeof(YT) > (size_t(128) << 20);     // kernel-uniform
            constexpr int BR = kEpilogueBlockRows<RT>;      // rows staged at a time
            uint8_t* ep = ep_lds;   // [BR rows][256 bytes]
            const int odd = lane_e & 1, l32 = lane_e & 31, kg = lane_e >> 5;
            // Lanes pair up: from its two packed values (rows r, r+1 of its column) and the neighbour's,
            // the even lane assembles row r and the odd lane row r+1 of the column pair.
            const uint32_t sel = odd ? 0x03020706u : 0x05040100u;
            // Value pair (j, u) of a block (16 rows = accumulator registers 8 h .. 8 h + 7, or 8 rows = registers
            // 4 h .. 4 h + 3) goes to block row 8 (u / 2) + 2 (u % 2) + (4 kg + odd) and
            // 16-byte chunk (4 j + l32 / 8) ^ swizzle(row); the swizzle only depends on the lane
            // (row & 1 = odd, (row >> 2) & 1 = kg), so it folds into per-lane base pointers, one per j.
            uint8_t* pj[NJ];
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                pj[j] = ep + (4 * kg + odd) * 256 + ((4 * (j ^ (odd | (kg << 1))) + (l32 >> 3)) << 4) + ((l32 >> 1) & 3) * 4;
            // read-back: one instruction covers kRows rows of 4 NJ 16-byte units (NJ = 3 leaves lanes
            // 48..63 idle); row pointers advance by additions only
            constexpr int kUnits = 4 * NJ, kRows = NJ == 3 ? 4 : (64 / kUnits < BR ? 64 / kUnits : BR);
            const int rl = lane_e / kUnits, unit = lane_e % kUnits;
            const bool lane_on = kRows * kUnits == 64 || lane_e < kRows * kUnits;
            int row = m0 + wm * 32 * RT + rl;
            YT* yrow = Y + (size_t)row * ldy + n0 + wn * 32 * NJ + unit * 8;
            const int64_t ystep = (int64_t)kRows * ldy;
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int h = 0; h < 32 / BR; ++h) {
                    __builtin_amdgcn_sched_barrier(0);      // one block at a time: keeps register use flat
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
#pragma unroll
                        for (int u = 0; u < BR / 4; ++u) {
                            f32x2 pr;
                            pr.x = value(i, j, (BR / 2) * h + 2 * u);
                            pr.y = value(i, j, (BR / 2) * h + 2 * u + 1);
                            const int mine = __builtin_bit_cast(int, __builtin_convertvector(pr, bf16x2));
                            const int theirs = __builtin_amdgcn_mov_dpp(mine, 0xB1, 0xF, 0xF, true);
                            *reinterpret_cast<uint32_t*>(pj[j] + (8 * (u >> 1) + 2 * (u & 1)) * 256) =
                                __builtin_amdgcn_perm((uint32_t)theirs, (uint32_t)mine, sel);
                        }
                    // wave-private buffer: the wave's own LDS operations complete in order
#pragma unroll
                    for (int it = 0; it < BR / kRows; ++it) {
                        const int R = it * kRows + rl;
                        const int chunk = unit ^ (((R & 1) << 2) | (((R >> 2) & 1) << 3));
                        const uint4 v = *reinterpret_cast<const uint4*>(ep + R * 256 + chunk * 16);
                        // written through the L2 (device scope): nothing in this kernel reads Y, and lines left
                        // dirty in the eight L2s would be written back at the end of the kernel (cfg2 back to
                        // back: plain stores 69.5 us, non-temporal 67.9, write-through 65.7)
                        // (an output beyond 128 MB also non-temporally: 8192 x 18944 bf16, 310 MB, 274.8 -> 262.0 us;
                        // 2048 x 14336, 59 MB, no difference either way)
                        if (lane_on && row < M) {
                            if (big) store16_through_nt(yrow, batq_u32x4{v.x, v.y, v.z, v.w});
                            else store16_through(yrow, batq_u32x4{v.x, v.y, v.z, v.w});
                        }
                        row += kRows;
                        yrow += ystep;
                    }
                }
            return;
        }
    }
    // general path: element-wise stores with edge checks; rows visited in increasing order per lane
    const int col0 = n0 + wn * 32 * NJ + (lane_e & 31);
    int row = m0 + wm * 32 * RT + 4 * (lane_e >> 5);
    YT* yp = Y + (size_t)row * ldy + col0;
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (row < M) {
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        if (col0 + 32 * j < N) {
                            if constexpr (sizeof(YT) == 4) {
                                // 32 lanes fill a 128-byte line: written through the L2 like the bf16 rows above
                                const float fv = value(i, j, 4 * q + r);
                                asm volatile("global_store_dword %0, %1, off sc1" :: "v"(yp + 32 * j), "v"(fv) : "memory");
                            } else {
                                store_y<YT>(yp + 32 * j, value(i, j, 4 * q + r));
                            }
                        }
                }
                ++row;
                yp += ldy;
            }
            row += 4;
            yp += 4 * ldy;
        }
}

// GLU: the weight columns interleave gate and up in groups of 32 (columns 64 p .. 64 p + 31 = gate columns
// 32 p .., 64 p + 32 .. 64 p + 63 = the matching up columns), so matrix tiles 2 j and 2 j + 1 of a wave hold
// gate and up of the same outputs in the same lanes and registers; what is stored is silu(gate) * up, to the
// M x N/2 array Y (N here = its column count).  NJ must be even.
template <int NJ, typename YT, bool GLU, int RT = 4>
__device__ __forceinline__ void store_tile(v16f (&acc_in)[RT][NJ], uint8_t* ep_lds, int lane, int wm, int wn,
                                           const Tile& t, int M, int N, YT* __restrict__ Y, int64_t ldy) {
    static_assert(!GLU || NJ % 2 == 0, "gated output needs gate/up tile pairs");
    auto value = [&](int i, int j, int e) -> float {
        if constexpr (GLU) return swiglu_f32(acc_in[i][2 * j][e], acc_in[i][2 * j + 1][e]);
        else return acc_in[i][j][e];
    };
    store_tile_impl<(GLU ? NJ / 2 : NJ), YT, RT>(value, ep_lds, lane, wm, wn, t.m0, GLU ? t.n0 / 2 : t.n0, M, N, Y, ldy);
}

// Partial sums of a K part, in the order the accumulators hold them: 32x32 blocks, block (rb, cb) of the
// padded output as 4 pieces of 64 lanes x 4 floats; piece q of lane (l32, kg) = rows 32 rb + 8 q + 4 kg .. + 3
// of column 32 cb + l32.  Every store instruction writes 1 KiB of consecutive memory.
constexpr int kPartialBlockFloats = 32 * 32;
template <int NJ, int RT = 4>
__device__ __forceinline__ void store_partial(v16f (&acc)[RT][NJ], float* __restrict__ P, int lane, int wm, int wn,
                                              const Tile& t, int col_blocks) {
    int lane_e = lane;
    asm volatile("" : "+v"(lane_e));
    const int rb0 = (t.m0 >> 5) + RT * wm, cb0 = (t.n0 >> 5) + NJ * wn;
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (cb0 + j >= col_blocks) continue;            // (a workgroup of two strips whose second does not exist)
            float* blk = P + ((size_t)(rb0 + i) * col_blocks + cb0 + j) * kPartialBlockFloats + lane_e * 4;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                *reinterpret_cast<f32x4*>(blk + q * 256) = v;
            }
        }
}

// One output tile: on entry the loads of its first stages are in flight (issue_prologue); before
// the epilogue the loads of the next tile's first stages are started, so they run underneath it.
// YT = partial_f32 (K parts): Y is the partial-sum array in accumulator order (store_partial), `ldy` its number
// of 32-column blocks and `part_stride` the floats of one part; for every other YT part_stride is unused.
template <int RT, int NJ, typename YT, bool GLU>
__device__ __forceinline__ void run_tile(TiledCtx<RT>& c, const Tile& t, bool has_next, const Tile& next,
                                         YT* __restrict__ Y, int64_t ldy, int64_t part_stride) {
    const int lane = c.lane, wave = c.wave;
    const int wm = wave >> 1, wn = wave & 1;
    const int T = c.T, G = T >> 1;
    c.aim_reads(NJ, wm, wn, lane & 31);
    // tile-variant as far as the compiler can tell: addresses derived from them for all four tile widths would
    // otherwise be kept in registers across the whole kernel
    asm volatile("" : "+v"(c.a_rd), "+v"(c.b_rd), "+v"(c.sc_a_rd), "+v"(c.sc_b_rd));

    v16f acc[RT][NJ];
    uint4 fa[2][RT], fb[2][NJ];
    int sa[RT], sb[NJ];

    // Loads per thread: kPA + pb per stage (4 + NJ with 4 waves), plus 2 kSc for the scales of a K group
    // issued with the group's even stage; they complete in issue order.  In steady state stages s+2 and s+3
    // stay in flight while stage s+1 is awaited.  Stores of the previous tile that are still pending only make
    // a wait longer than needed.
    constexpr int kOdd = TiledCtx<RT>::kPA + TiledCtx<RT>::pb(NJ), kSteady = 2 * kOdd + 2 * TiledCtx<RT>::kSc;
    if (T >= 4) wait_vmcnt<kSteady + kOdd>();
    else wait_vmcnt<kOdd>();
    __syncthreads();
    c.template read_scales<NJ>(0, sa, sb);
    c.template read_frags<NJ>(0, 0, fa[0], fb[0]);
    if constexpr (kNarrowStages<RT, NJ>) c.template read_frags<NJ>(0, 1, fa[1], fb[1]);

    // the first stage of a tile starts the accumulators from zero
    if (G >= 3) {
        any_stage<RT, NJ, 0, kSteady, true, true>(c, 0, acc, fa, fb, sa, sb);
        any_stage<RT, NJ, 1, kSteady, true, false>(c, 1, acc, fa, fb, sa, sb);
        for (int g = 1; g + 2 < G; ++g) {
            any_stage<RT, NJ, 0, kSteady, true, false>(c, 2 * g, acc, fa, fb, sa, sb);
            any_stage<RT, NJ, 1, kSteady, true, false>(c, 2 * g + 1, acc, fa, fb, sa, sb);
        }
        any_stage<RT, NJ, 0, kSteady, false, false>(c, T - 4, acc, fa, fb, sa, sb);            // finishes the loads of stage T-1
        any_stage<RT, NJ, 1, kOdd, false, false, false>(c, T - 3, acc, fa, fb, sa, sb);
        any_stage<RT, NJ, 0, 0, false, false, false>(c, T - 2, acc, fa, fb, sa, sb);
    } else if (G == 2) {
        any_stage<RT, NJ, 0, kSteady, false, true>(c, 0, acc, fa, fb, sa, sb);
        any_stage<RT, NJ, 1, kOdd, false, false, false>(c, 1, acc, fa, fb, sa, sb);
        any_stage<RT, NJ, 0, 0, false, false, false>(c, 2, acc, fa, fb, sa, sb);
    } else {
        any_stage<RT, NJ, 0, 0, false, true>(c, 0, acc, fa, fb, sa, sb);
    }
    any_stage<RT, NJ, 1, -1, false, false, false>(c, T - 1, acc, fa, fb, sa, sb);

    __syncthreads();                                      // every wave is done with the stage ring
    if (has_next) {
        c.aim(next);
        c.issue_prologue(next.nj);
    }

    // ---- epilogue: accumulators -> Y
    if constexpr (std::is_same_v<YT, partial_f32>) {
        store_partial<NJ, RT>(acc, reinterpret_cast<float*>(Y) + t.part * part_stride, lane, wm, wn, t, (int)ldy);
    } else {
        store_tile<NJ, YT, GLU, RT>(acc, const_cast<uint8_t*>(c.smem) + kEpilogueLds0 + wave * kEpilogueWaveBytes<RT>,
                                    lane, wm, wn, t, c.M, GLU ? c.N / 2 : c.N, Y, ldy);
    }
}

// Requires operand code arrays below 2 GiB (32-bit load offsets) and gridDim.x == pl.workers.
// pl.ksplit > 1: tiles cover one K part each and store their partial sums to Y + part * part_stride
// (fp32, summed by splitk_reduce); used when there are fewer strips than workgroups.
// GLU: gated output (see store_tile); the plan then hands out tiles 2 or 4 strips wide, and Y is M x N/2.
template <typename YT, bool GLU, int RT>
__global__ void __launch_bounds__(1024 / RT, 1)
gemm_tiled(const uint8_t* __restrict__ xc, const uint8_t* __restrict__ xs, const uint8_t* __restrict__ wc,
           const uint8_t* __restrict__ ws, int M, int N, int nb, TilePlan pl, YT* __restrict__ Y, int64_t ldy,
           int64_t part_stride) {
    extern __shared__ __align__(16) uint8_t smem[];
    typedef __attribute__((address_space(3))) uint8_t lds_byte;

    // this workgroup's share of the linear strip order
    int cur, end;
    worker_share(pl, blockIdx.x, cur, end);
    TileWalk walk;
    walk_begin(pl, blockIdx.x, cur, end, walk);

    Tile t, next;
    if (!next_tile(pl, walk, t)) return;                  // workgroup-uniform

    const int lane = threadIdx.x & 63;
    TiledCtx<RT> c;
    c.xc = xc; c.wc = wc; c.xs = xs; c.ws = ws;
    c.M = M; c.N = N; c.smem = smem;
    c.row_group_bytes = (uint32_t)(2 * ((nb + 7) >> 3)) * 1024u;   // stages of 128 K elements (K zero-padded to 256)
    c.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    c.lane = lane;
    c.lds0 = (uint32_t)(uintptr_t)(lds_byte*)smem;            // LDS byte address of the stage ring
    c.lds_sc = c.lds0 + kRing * kStageLds;                    // scale ring
    c.kg = lane >> 5;
    c.fsw = slot_swizzle(lane & 31);

    c.aim(t);
    c.issue_prologue(t.nj);
    for (;;) {
        const bool has_next = next_tile(pl, walk, next);
        if constexpr (GLU) {
            if (t.nj == 4) run_tile<RT, 4, YT, true>(c, t, has_next, next, Y, ldy, part_stride);
            else run_tile<RT, 2, YT, true>(c, t, has_next, next, Y, ldy, part_stride);
        } else {
            switch (t.nj) {
                case 4: run_tile<RT, 4, YT, false>(c, t, has_next, next, Y, ldy, part_stride); break;
                case 3: run_tile<RT, 3, YT, false>(c, t, has_next, next, Y, ldy, part_stride); break;
                case 2: run_tile<RT, 2, YT, false>(c, t, has_next, next, Y, ldy, part_stride); break;
                default: run_tile<RT, 1, YT, false>(c, t, has_next, next, Y, ldy, part_stride); break;
            }
        }
        if (!has_next) break;
        t = next;
    }
}

// ------------------------------------------------------------------------------------------
// Kernel for shapes with so few rows and strips that 128-row panels x strips (x K parts) give at most one
// workgroup per compute unit, where the tiled kernel's 256-row tiles leave compute units idle or half empty.
// A workgroup of 4 waves computes 128 RT rows x 64 NS columns (RT = 1 is what the launch code uses; NS = 1 strip,
// or 2 where only pairs of strips give at most one workgroup per compute unit), wave w the rows
// 32 RT w .. + 32 RT - 1 of all its columns: the rows of X a wave multiplies belong to it alone, so their
// fragments go from global memory (the L2) straight to registers, D - 2 stages ahead, and only the weight strips
// (4 KiB per strip and stage, read by all four waves) go through LDS, each wave fetching one of a strip's four
// 1 KiB pieces: with one strip, per stage 12 KiB enter the compute unit and 8 KiB of fragments are read from LDS,
// against 20 KiB and 40 KiB for a 256 x 64 tile of the tiled kernel.
//
// Loads of a wave complete in the order it issued them.  Stage q's are: NS strip pieces, 2 RT fragments of X
// and, for even q, RT + 2 NS scale dwords (those of the K group q opens); stages are issued in order.  At the top
// of stage s a wave waits until only loads of the stages after s + 1 can be outstanding, then meets the others at
// the barrier: the whole strip stage s + 1 is in LDS and is read to registers under the matrix instructions of
// stage s, and every wave is done with stage s - 1, whose LDS slot and registers the loads of stage s + D - 1
// then overwrite (issued after the stage's own matrix instructions, which still read the scale registers of the
// K group they complete).
constexpr int kMidStripLds = 64 * kStageBytes;      // 4 KiB: one stage of one 64-column strip.  A workgroup keeps D
                                                    // stages of its NS strips in LDS (a wave works D - 2 stages
                                                    // ahead); the epilogue's staging reuses them

template <int RT, int D, int NS>
struct MidCtx {
    static_assert(D % 2 == 0 && D >= 4, "stages come in K groups of two");
    static constexpr int NJ = 2 * NS;           // 32-column matrix tiles of a wave
    uint32_t aoff[RT][2], boff[NS], sao[RT], sbo[NJ], lds0;
    int wave, T;
    // the next stage to load: its index, where its codes and the scales of its K group start
    int q;
    const uint8_t* xq; const uint8_t* wq; const uint8_t* sag; const uint8_t* sbg;
    size_t sa_step, sb_step;                    // bytes of one K group of scales (rows x 8)

    // The loads of the next stage, in the counted order, into LDS slot `slot` and the given registers.  Every
    // stage index gets the same number of loads, so that the waits are the same everywhere and no load is
    // conditional (a register an asynchronous load writes must not meet another value at a control-flow join:
    // the compiler would copy it while it is still in flight).  Past the K part's T stages all lanes fetch the
    // first 16 bytes of the last stage instead: one cache line per instruction, into a free LDS slot and dead
    // registers.
    // LIVE: the caller knows that the stage exists (q < T) and that it is not the last one either, so the masks
    // and the clamped pointer steps (a dozen scalar and vector instructions per stage, in a loop whose pace is set by
    // the instructions a wave issues) are left out.
    template <bool EVEN, bool LIVE = false>
    __device__ __forceinline__ void issue(int slot, batq_u32x4 (&a)[RT][2], int (&sa)[RT], int (&sb)[NJ]) {
        if constexpr (LIVE) {
#pragma unroll
            for (int n = 0; n < NS; ++n)
                dma16(wq, boff[n], lds0 + (uint32_t)(slot * NS + n) * kMidStripLds + (uint32_t)wave * 1024);
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int h = 0; h < 2; ++h) load16_async(a[i][h], xq, aoff[i][h]);
            if constexpr (EVEN) {
#pragma unroll
                for (int i = 0; i < RT; ++i) load4_async(sa[i], sag, sao[i]);
#pragma unroll
                for (int j = 0; j < NJ; ++j) load4_async(sb[j], sbg, sbo[j]);
            }
            ++q;
            xq += 1024;
            wq += 1024;
            if constexpr (!EVEN) {
                sag += sa_step;
                sbg += sb_step;
            }
            return;
        }
        const uint32_t m = q < T ? ~0u : 0u;
#pragma unroll
        for (int n = 0; n < NS; ++n)
            dma16(wq, boff[n] & m, lds0 + (uint32_t)(slot * NS + n) * kMidStripLds + (uint32_t)wave * 1024);
#pragma unroll
        for (int i = 0; i < RT; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h) load16_async(a[i][h], xq, aoff[i][h] & m);
        if constexpr (EVEN) {
#pragma unroll
            for (int i = 0; i < RT; ++i) load4_async(sa[i], sag, sao[i] & m);
#pragma unroll
            for (int j = 0; j < NJ; ++j) load4_async(sb[j], sbg, sbo[j] & m);
        }
        ++q;
        const bool more = q < T;                      // uniform; the pointers stay on the last stage otherwise
        xq += more ? 1024 : 0;
        wq += more ? 1024 : 0;
        if constexpr (!EVEN) {
            sag += more ? sa_step : 0;
            sbg += more ? sb_step : 0;
        }
    }
    // loads a wave issues for a stage of parity p
    static constexpr __device__ int count(int p) { return NS + 2 * RT + ((p & 1) == 0 ? RT + NJ : 0); }
};

// Loads of stage indices Q .. D - 2, before the first stage is multiplied.
template <int RT, int D, int NS, int Q>
__device__ __forceinline__ void mid_prologue(MidCtx<RT, D, NS>& c, batq_u32x4 (&a)[D][RT][2], int (&sa)[D / 2][RT],
                                             int (&sb)[D / 2][2 * NS]) {
    if constexpr (Q < D - 1) {
        c.template issue<(Q & 1) == 0>(Q, a[Q], sa[Q >> 1], sb[Q >> 1]);
        mid_prologue<RT, D, NS, Q + 1>(c, a, sa, sb);
    }
}

// This lane's fragments of the strips' stage in LDS slot `slot`: matrix tile j = 32 columns, K steps 0 and 1.
template <int D, int NS>
__device__ __forceinline__ void mid_read_strips(const uint8_t* smem, int slot, int b_rd0, int b_rd1, uint4 (&b)[2 * NS][2]) {
    const uint8_t* bs = smem + slot * NS * kMidStripLds;
#pragma unroll
    for (int j = 0; j < 2 * NS; ++j) {
        b[j][0] = *reinterpret_cast<const uint4*>(bs + b_rd0 + j * 32 * kStageBytes);
        b[j][1] = *reinterpret_cast<const uint4*>(bs + b_rd1 + j * 32 * kStageBytes);
    }
}

// Stages base + U .. base + D - 1 of a K part (base a multiple of D, so stage base + U lives in LDS
// slot and register slot U and has parity U % 2).  ALL: all of them exist.  On entry b[U % 2] holds the strip
// fragments of stage base + U; those of the next stage are read under its matrix instructions.
// LIVE: the stages base + D - 1 .. base + 2 D - 2 whose loads are issued here exist and are not the last one.
template <int RT, int D, int NS, int U, bool ALL, bool LIVE = false>
__device__ __forceinline__ void mid_steps(MidCtx<RT, D, NS>& c, int base, const uint8_t* smem, int b_rd0, int b_rd1,
                                          v16f (&acc)[RT][2 * NS], batq_u32x4 (&a)[D][RT][2],
                                          int (&sa)[D / 2][RT], int (&sb)[D / 2][2 * NS], uint4 (&b)[2][2 * NS][2]) {
    using Ctx = MidCtx<RT, D, NS>;
    constexpr int NJ = 2 * NS;
    if constexpr (U < D) {
        const int s = base + U;
        // stage s + 1 has landed (this wave's loads; the barrier adds the other waves' strip pieces): only the
        // loads of stage indices s + 2 .. s + D - 2 can be outstanding
        wait_vmcnt<(D - 4) / 2 * (Ctx::count(0) + Ctx::count(1)) + Ctx::count(U)>();
        wait_lds();                                                // the fragments of stage s are in registers
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        constexpr int u1 = (U + 1) % D;
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            ready(a[u1][i][0]);
            ready(a[u1][i][1]);
            if constexpr ((u1 & 1) == 0) ready(sa[u1 >> 1][i]);
        }
        if constexpr ((u1 & 1) == 0) {
#pragma unroll
            for (int j = 0; j < NJ; ++j) ready(sb[u1 >> 1][j]);
        }
        mid_read_strips<D, NS>(smem, u1, b_rd0, b_rd1, b[u1 & 1]);
        // the reads go out first and are not waited for here: this stage's matrix instructions take the fragments
        // read a stage ago (left alone, the compiler moves matrix instructions across the stage boundary and then
        // waits for a read it has just issued)
        __builtin_amdgcn_sched_barrier(0);
        if (ALL || s < c.T) {                                      // workgroup-uniform
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    mfma_one<2 * (U & 1), false>(acc[i][j], as_uint4(a[U][i][0]), b[U & 1][j][0], sa[U >> 1][i], sb[U >> 1][j]);
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    mfma_one<2 * (U & 1) + 1, false>(acc[i][j], as_uint4(a[U][i][1]), b[U & 1][j][1], sa[U >> 1][i], sb[U >> 1][j]);
        }
        // Every wave has read the fragments of stage s - 1 and finished its matrix instructions on them: the LDS
        // slot and registers of stage s - 1 take stage s + D - 1.  (After this stage's matrix instructions: for odd
        // s they still read the scale registers that the K group of stage s + D - 1 takes over.)
        constexpr int un = (U + D - 1) % D;
        c.template issue<(un & 1) == 0, LIVE>(un, a[un], sa[un >> 1], sb[un >> 1]);
        __builtin_amdgcn_sched_barrier(0);
        mid_steps<RT, D, NS, U + 1, ALL, LIVE>(c, base, smem, b_rd0, b_rd1, acc, a, sa, sb, b);
    }
}

// Requires operand code arrays below 2 GiB (32-bit load offsets).  Grid: (groups of NS strips, row panels of 128 RT,
// K parts); YT = partial_f32: partial sums of K part blockIdx.z in store_partial order (ldy = 32-column blocks of the
// padded output, part_stride = floats of a part).
template <typename YT, int RT, int D, int NS>
__global__ void __launch_bounds__(256, 2)
gemm_mid(const uint8_t* __restrict__ xc, const uint8_t* __restrict__ xs, const uint8_t* __restrict__ wc,
         const uint8_t* __restrict__ ws, int M, int N, int nb, int ksplit, YT* __restrict__ Y, int64_t ldy,
         int64_t part_stride) {
    constexpr int NJ = 2 * NS;
    __shared__ __align__(16) uint8_t smem[D * NS * kMidStripLds];
    typedef __attribute__((address_space(3))) uint8_t lds_byte;
    const int lane = threadIdx.x & 63, l32 = lane & 31, kg = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int groups = (nb + 7) >> 3;
    Tile t;
    t.n0 = blockIdx.x * (kStrip * NS);
    t.m0 = blockIdx.y * (128 * RT);
    t.nj = NS;
    t.part = blockIdx.z;
    t.g0 = 0;
    t.ng = groups;
    if (ksplit > 1) {                                           // (divisions only where there are K parts)
        t.g0 = groups * t.part / ksplit;
        t.ng = groups * (t.part + 1) / ksplit - t.g0;
    }
    const int T = 2 * t.ng;                                     // stages of 128 K elements

    MidCtx<RT, D, NS> c;
    c.wave = wave;
    c.T = T;
    c.q = 0;
    c.xq = xc + (size_t)(2 * t.g0) * 1024;
    c.wq = wc + (size_t)(2 * t.g0) * 1024;
    c.sa_step = (size_t)M * 8;
    c.sb_step = (size_t)N * 8;
    c.sag = xs + t.g0 * c.sa_step;
    c.sbg = ws + t.g0 * c.sb_step;
    c.lds0 = (uint32_t)(uintptr_t)(lds_byte*)smem;
    const uint32_t row_group_bytes = (uint32_t)(2 * groups) * 1024u;
    const int rgA = (M + 15) >> 4, rgB = (N + 15) >> 4;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        // row groups past the edge are clamped to the last one (their results are never stored)
        const int R = t.m0 + 32 * RT * wave + 32 * i + l32, r = R & 15;
#pragma unroll
        for (int h = 0; h < 2; ++h)
            c.aoff[i][h] = (uint32_t)min(R >> 4, rgA - 1) * row_group_bytes + r * 64 + (((2 * h + kg) ^ slot_swizzle(r)) << 4);
        c.sao[i] = (uint32_t)(min(R, M - 1) * 2 + kg) * 4;
    }
    // wave w fetches the 16-column piece w of each of the workgroup's strips
#pragma unroll
    for (int n = 0; n < NS; ++n)
        c.boff[n] = (uint32_t)min((t.n0 >> 4) + 4 * n + wave, rgB - 1) * row_group_bytes + lane * 16;
#pragma unroll
    for (int j = 0; j < NJ; ++j) c.sbo[j] = (uint32_t)(min(t.n0 + 32 * j + l32, N - 1) * 2 + kg) * 4;
    // this lane's fragment of strip row (32 j + l32), K step h: slot (2 h + kg) ^ swizzle(row)
    const int b_rd0 = l32 * kStageBytes + ((kg ^ slot_swizzle(l32)) << 4);
    const int b_rd1 = l32 * kStageBytes + (((2 + kg) ^ slot_swizzle(l32)) << 4);

    v16f acc[RT][NJ];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = v16f{};
    batq_u32x4 a[D][RT][2];
    int sa[D / 2][RT], sb[D / 2][NJ];

    uint4 b[2][NJ][2];
    mid_prologue<RT, D, NS, 0>(c, a, sa, sb);
    // stage 0 has landed: stage indices 1 .. D - 2 may be outstanding
    wait_vmcnt<(D - 2) / 2 * (MidCtx<RT, D, NS>::count(1) + MidCtx<RT, D, NS>::count(0))>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        ready(a[0][i][0]);
        ready(a[0][i][1]);
        ready(sa[0][i]);
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) ready(sb[0][j]);
    mid_read_strips<D, NS>(smem, 0, b_rd0, b_rd1, b[0]);

    int base = 0;
    for (; base + 2 * D <= T; base += D) mid_steps<RT, D, NS, 0, true, true>(c, base, smem, b_rd0, b_rd1, acc, a, sa, sb, b);
    for (; base + D <= T; base += D) mid_steps<RT, D, NS, 0, true>(c, base, smem, b_rd0, b_rd1, acc, a, sa, sb, b);
    if (base < T) mid_steps<RT, D, NS, 0, false>(c, base, smem, b_rd0, b_rd1, acc, a, sa, sb, b);
    wait_vmcnt<0>();                                            // the loads past the last stage have landed, too
    // their destinations count as in use until here: a register the compiler took for something else would be
    // overwritten when the load lands
#pragma unroll
    for (int d = 0; d < D; ++d) {
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            ready(a[d][i][0]);
            ready(a[d][i][1]);
            ready(sa[d >> 1][i]);
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) ready(sb[d >> 1][j]);
    }
    wait_lds();
    __builtin_amdgcn_s_barrier();                               // every wave is done with the strip ring
    asm volatile("" ::: "memory");
    if constexpr (std::is_same_v<YT, partial_f32>) {
        store_partial<NJ, RT>(acc, reinterpret_cast<float*>(Y) + t.part * part_stride, lane, wave, 0, t, (int)ldy);
    } else {
        store_tile<NJ, YT, false, RT>(acc, smem + wave * kEpilogueWaveBytes<RT>, lane, wave, 0, t, M, N, Y, ldy);
    }
}

// ------------------------------------------------------------------------------------------
// Tiled kernel for MXFP8 activations (W4A8).  Same persistent work split, tile shapes, LDS-direct
// loads and epilogue as gemm_tiled; what differs follows from the 8-bit A operand: a matrix
// instruction takes twice as long (the pipe runs at the FP8 rate), so a stage is one K step of 64
// elements: 256 rows x 64 bytes of A (whole 1 KiB pieces of the 8-bit code layout) and 256 rows x 32
// bytes of B (half of each row of a 4-bit piece, gathered by the load's per-lane addresses).  Ring
// of 4 stages x 24 KiB.  Always 256 rows of B are loaded, whatever the tile width, so that every
// wave issues the same number of loads per stage (6, plus 4 for the scales of a K group with its
// first stage).
constexpr int kA8StageA = kTile * 64;                       // 16 KiB
constexpr int kA8StageB = kTile * 32;                       // 8 KiB
constexpr int kA8Stage = kA8StageA + kA8StageB;
constexpr int kA8ScaleLds0 = kRing * kA8Stage;              // 96 KiB
constexpr int kA8EpilogueLds0 = kA8ScaleLds0 + 2 * kScaleGroupLds;
constexpr int kA8Lds = kA8EpilogueLds0 + 4 * kEpilogueWaveLds;      // 120 KiB

struct A8Ctx {
    const uint8_t* xc; const uint8_t* wc; const uint8_t* xs; const uint8_t* ws;
    uint32_t aoff[4], boff[2], sao[2], sbo[2];
    uint32_t lds0, lds_sc, row_group_bytes;   // bytes of one 16-row group of the 8-bit code array (all of K)
    int M, N, wave, lane;
    int T, s0;        // stages of the aimed tile and the first of them (stage = 64 K elements; K parts start on K groups)
    const uint8_t* smem;
    int a_rd, b_rd, sc_a_rd, sc_b_rd, kg;

    __device__ __forceinline__ void aim(const Tile& t) {
        const int rgA = (M + 15) >> 4, rgB = (N + 15) >> 4;
        int lane = this->lane;
        asm volatile("" : "+v"(lane));      // recompute the lane terms per tile instead of keeping them in registers
        T = 4 * t.ng;
        s0 = 4 * t.g0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            aoff[j] = (uint32_t)min((t.m0 >> 4) + 4 * wave + j, rgA - 1) * row_group_bytes + lane * 16;
        // B: load q of wave w fills LDS rows 32 (2 w + q) .. + 31 (32 bytes each); lane i -> row i / 2, 16-byte
        // position i % 2, which holds block (i % 2) ^ ((row / 8) % 2) of the K step (8 rows of 32 bytes span
        // all LDS banks once); in the 4-bit piece
        // (16 rows x 64 bytes, 2 K steps) that block sits in slot (2 (s % 2) + block) ^ ((row % 16) / 4);
        // the offset below is for an even stage, an odd stage flips bit 5.
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int rho = lane >> 1, p = lane & 1;
            const int r16 = rho & 15;
            const int blk = p ^ ((rho >> 3) & 1);
            const int rg = min((t.n0 >> 4) + 2 * (2 * wave + q) + (rho >> 4), rgB - 1);
            boff[q] = (uint32_t)rg * (row_group_bytes >> 1) + r16 * 64 + ((blk ^ ((r16 >> 2) & 3)) << 4);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int d = 128 * wave + 64 * j + lane;
            sao[j] = ((uint32_t)min(t.m0 + (d >> 1), M - 1) * 2 + (d & 1)) * 4;
            sbo[j] = ((uint32_t)min(t.n0 + (d >> 1), N - 1) * 2 + (d & 1)) * 4;
        }
    }
    // loads of stage s in their fixed order: parts 0..3 A pieces, 4..5 B, 6 = scales (first stage of a K group)
    template <int PART, int PAR>
    __device__ __forceinline__ void issue_part(int s) const {
        const uint32_t buf = lds0 + (uint32_t)(s & (kRing - 1)) * kA8Stage;
        if constexpr (PART < 4) {
            dma16(xc + (size_t)(s + s0) * 1024, aoff[PART], buf + (uint32_t)(4 * wave + PART) * 1024);
        } else if constexpr (PART < 6) {
            dma16(wc + (size_t)((s + s0) >> 1) * 1024, boff[PART - 4] ^ ((PAR & 1) << 5),
                  buf + kA8StageA + (uint32_t)(2 * wave + PART - 4) * 1024);
        } else if constexpr (PAR == 0) {
            const int g = s >> 2;
            const uint32_t sbuf = lds_sc + (uint32_t)(g & 1) * kScaleGroupLds + (uint32_t)wave * 512;
            const uint8_t* sag = xs + (size_t)(g + (s0 >> 2)) * M * 8;
            const uint8_t* sbg = ws + (size_t)(g + (s0 >> 2)) * N * 8;
#pragma unroll
            for (int j = 0; j < 2; ++j) dma4(sag, sao[j], sbuf + j * 256);
#pragma unroll
            for (int j = 0; j < 2; ++j) dma4(sbg, sbo[j], sbuf + kTile * 8 + j * 256);
        }
    }
    template <int PAR>
    __device__ __forceinline__ void issue_stage(int s) const {
        issue_part<0, PAR>(s); issue_part<1, PAR>(s); issue_part<2, PAR>(s); issue_part<3, PAR>(s);
        issue_part<4, PAR>(s); issue_part<5, PAR>(s); issue_part<6, PAR>(s);
    }
    __device__ __forceinline__ void aim_reads(int nj, int wm, int wn, int l32) {
        const int sw = (l32 >> 2) & 3;
        // A: this lane's halves (kg) of the two blocks of the step: slots kg and 2 + kg of its 64-byte row
        a_rd = (wm * 128 + l32) * 64 + ((kg ^ sw) << 4);
        // B: block kg of the step, 32-byte rows
        b_rd = kA8StageA + (wn * 32 * nj + l32) * 32 + ((kg ^ ((l32 >> 3) & 1)) << 4);
        sc_a_rd = ((wm * 128 + l32) * 2 + kg) * 4;
        sc_b_rd = kTile * 8 + ((wn * 32 * nj + l32) * 2 + kg) * 4;
    }
    // fragment `idx` of stage s in consumption order: 0 = a0, 1..NJ = b0.., NJ+1.. = a1..a3 (an A fragment is
    // two 16-byte reads: slot ^ 2 is the second block's half)
    template <int NJ>
    __device__ __forceinline__ void read_frag(int s, int idx, uint4 (&fa)[4][2], uint4 (&fb)[NJ]) const {
        const uint8_t* base = smem + (s & (kRing - 1)) * kA8Stage;
        if (idx == 0 || idx > NJ) {
            const int i = idx == 0 ? 0 : idx - NJ;
            fa[i][0] = *reinterpret_cast<const uint4*>(base + a_rd + i * 32 * 64);
            fa[i][1] = *reinterpret_cast<const uint4*>(base + (a_rd ^ 32) + i * 32 * 64);
        } else {
            fb[idx - 1] = *reinterpret_cast<const uint4*>(base + b_rd + (idx - 1) * 32 * 32);
        }
    }
    template <int NJ>
    __device__ __forceinline__ void read_scales(int g, int (&sa)[4], int (&sb)[NJ]) const {
        const uint8_t* sp = smem + kA8ScaleLds0 + (g & 1) * kScaleGroupLds;
#pragma unroll
        for (int i = 0; i < 4; ++i) sa[i] = *reinterpret_cast<const int*>(sp + sc_a_rd + i * 256);
#pragma unroll
        for (int j = 0; j < NJ; ++j) sb[j] = *reinterpret_cast<const int*>(sp + sc_b_rd + j * 256);
    }
};

template <int PAR, bool ZERO>
__device__ __forceinline__ void a8_mfma(v16f& acc, const uint4 (&a)[2], const uint4& b, int sa, int sb) {
    if constexpr (ZERO)
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag8(a[0], a[1]), frag(b), v16f{}, 0, 4, PAR, sa, PAR, sb);
    else
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag8(a[0], a[1]), frag(b), acc, 0, 4, PAR, sa, PAR, sb);
}

// Matrix instructions Q .. 2 NJ - 1 of the second half of a stage (tile rows 2 and 3), each followed by its
// share of the reads of stage s+1's fragments (4 + NJ), of the next group's scales (PAR 3) and of the 7 load
// parts of stage s+4.
template <int NJ, int PAR, bool NEXT, bool ISSUE, int Q>
__device__ __forceinline__ void a8_second_half(const A8Ctx& c, int s, v16f (&acc)[4][NJ], const uint4 (&a)[4][2],
                                               const uint4 (&b)[NJ], const int (&sa)[4], const int (&sb)[NJ],
                                               uint4 (&an)[4][2], uint4 (&bn)[NJ]) {
    if constexpr (Q < 2 * NJ) {
        constexpr int i = 2 + Q / NJ, j = Q % NJ;
        constexpr int kSlots = 2 * NJ, kFrags = 4 + NJ, kParts = 7;
        a8_mfma<PAR, false>(acc[i][j], a[i], b[j], sa[i], sb[j]);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (NEXT) {
#pragma unroll
            for (int f = Q * kFrags / kSlots; f < (Q + 1) * kFrags / kSlots; ++f) c.read_frag<NJ>(s + 1, f, an, bn);
        }
        if constexpr (ISSUE) {
            constexpr int p0 = Q * kParts / kSlots, p1 = (Q + 1) * kParts / kSlots;
            if constexpr (p0 <= 0 && 0 < p1) c.issue_part<0, PAR>(s + 4);
            if constexpr (p0 <= 1 && 1 < p1) c.issue_part<1, PAR>(s + 4);
            if constexpr (p0 <= 2 && 2 < p1) c.issue_part<2, PAR>(s + 4);
            if constexpr (p0 <= 3 && 3 < p1) c.issue_part<3, PAR>(s + 4);
            if constexpr (p0 <= 4 && 4 < p1) c.issue_part<4, PAR>(s + 4);
            if constexpr (p0 <= 5 && 5 < p1) c.issue_part<5, PAR>(s + 4);
            if constexpr (p0 <= 6 && 6 < p1) c.issue_part<6, PAR>(s + 4);
        }
        __builtin_amdgcn_sched_barrier(0);
        a8_second_half<NJ, PAR, NEXT, ISSUE, Q + 1>(c, s, acc, a, b, sa, sb, an, bn);
    }
}

// One stage = one K step.  PAR = s % 4 (scale byte); WAIT = loads that may stay in flight once stage s+1 has
// landed (-1: last stage); ISSUE: start stage s+4; FIRST: start the accumulators from zero.
// (a, b) hold stage s on entry; (an, bn) receive stage s+1.
template <int NJ, int PAR, int WAIT, bool ISSUE, bool FIRST>
__device__ __forceinline__ void a8_stage(const A8Ctx& c, int s, v16f (&acc)[4][NJ], const uint4 (&a)[4][2],
                                         const uint4 (&b)[NJ], uint4 (&an)[4][2], uint4 (&bn)[NJ], int (&sa)[4],
                                         int (&sb)[NJ]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) a8_mfma<PAR, FIRST>(acc[i][j], a[i], b[j], sa[i], sb[j]);
    __builtin_amdgcn_sched_barrier(0);
    int sna[4], snb[NJ];
    if constexpr (WAIT >= 0) {
        // every wave holds stage s in registers; once all have also seen stage s+1 land, slot s can be refilled
        wait_vmcnt<WAIT>();
        __syncthreads();
        if constexpr (PAR == 3) c.read_scales<NJ>((s + 1) >> 2, sna, snb);
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (FIRST) {
        // rows 2 and 3 also start from zero
#pragma unroll
        for (int i = 2; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[i][j] = v16f{};
    }
    a8_second_half<NJ, PAR, (WAIT >= 0), ISSUE, 0>(c, s, acc, a, b, sa, sb, an, bn);
    if constexpr (WAIT >= 0 && PAR == 3) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) sa[i] = sna[i];
#pragma unroll
        for (int j = 0; j < NJ; ++j) sb[j] = snb[j];
    }
}

template <int NJ, typename YT, bool GLU>
__device__ __forceinline__ void a8_run_tile(A8Ctx& c, const Tile& t, bool has_next, const Tile& next,
                                            YT* __restrict__ Y, int64_t ldy, int64_t part_stride) {
    const int lane = c.lane, wave = c.wave;
    const int wm = wave >> 1, wn = wave & 1;
    const int T = c.T, G = T >> 2;
    c.aim_reads(NJ, wm, wn, lane & 31);
    asm volatile("" : "+v"(c.a_rd), "+v"(c.b_rd), "+v"(c.sc_a_rd), "+v"(c.sc_b_rd));      // see run_tile

    v16f acc[4][NJ];
    uint4 a0[4][2], a1[4][2], b0[NJ], b1[NJ];
    int sa[4], sb[NJ];

    // per thread and stage: 6 loads, 4 more with the first stage of a K group, completing in issue order
    wait_vmcnt<18>();                                       // stages 1..3 may still be in flight
    __syncthreads();
    c.read_scales<NJ>(0, sa, sb);
#pragma unroll
    for (int f = 0; f < 4 + NJ; ++f) c.read_frag<NJ>(0, f, a0, b0);

    // stage s waits for stage s+1 and leaves stages s+2, s+3 in flight: 12 loads, 16 if one of them opens a group
    if (G >= 2) {
        a8_stage<NJ, 0, 12, true, true>(c, 0, acc, a0, b0, a1, b1, sa, sb);
        a8_stage<NJ, 1, 16, true, false>(c, 1, acc, a1, b1, a0, b0, sa, sb);
        a8_stage<NJ, 2, 16, true, false>(c, 2, acc, a0, b0, a1, b1, sa, sb);
        a8_stage<NJ, 3, 12, true, false>(c, 3, acc, a1, b1, a0, b0, sa, sb);
        for (int g = 1; g + 1 < G; ++g) {
            a8_stage<NJ, 0, 12, true, false>(c, 4 * g, acc, a0, b0, a1, b1, sa, sb);
            a8_stage<NJ, 1, 16, true, false>(c, 4 * g + 1, acc, a1, b1, a0, b0, sa, sb);
            a8_stage<NJ, 2, 16, true, false>(c, 4 * g + 2, acc, a0, b0, a1, b1, sa, sb);
            a8_stage<NJ, 3, 12, true, false>(c, 4 * g + 3, acc, a1, b1, a0, b0, sa, sb);
        }
        a8_stage<NJ, 0, 12, false, false>(c, T - 4, acc, a0, b0, a1, b1, sa, sb);
    } else {
        a8_stage<NJ, 0, 12, false, true>(c, 0, acc, a0, b0, a1, b1, sa, sb);
    }
    a8_stage<NJ, 1, 6, false, false>(c, T - 3, acc, a1, b1, a0, b0, sa, sb);
    a8_stage<NJ, 2, 0, false, false>(c, T - 2, acc, a0, b0, a1, b1, sa, sb);
    a8_stage<NJ, 3, -1, false, false>(c, T - 1, acc, a1, b1, a0, b0, sa, sb);

    __syncthreads();                                      // every wave is done with the stage ring
    if (has_next) {
        c.aim(next);
        c.issue_stage<0>(0);
        c.issue_stage<1>(1);
        c.issue_stage<2>(2);
        c.issue_stage<3>(3);
    }
    if constexpr (std::is_same_v<YT, partial_f32>) {
        store_partial<NJ>(acc, reinterpret_cast<float*>(Y) + t.part * part_stride, lane, wm, wn, t, (int)ldy);
    } else {
        store_tile<NJ, YT, GLU>(acc, const_cast<uint8_t*>(c.smem) + kA8EpilogueLds0 + wave * kEpilogueWaveLds, lane, wm,
                                wn, t, c.M, GLU ? c.N / 2 : c.N, Y, ldy);
    }
}

// Requires operand code arrays below 2 GiB (32-bit load offsets) and gridDim.x == pl.workers.
template <typename YT, bool GLU>
__global__ void __launch_bounds__(256, 1)
gemm_tiled_a8(const uint8_t* __restrict__ xc, const uint8_t* __restrict__ xs, const uint8_t* __restrict__ wc,
              const uint8_t* __restrict__ ws, int M, int N, int nb, TilePlan pl, YT* __restrict__ Y, int64_t ldy,
              int64_t part_stride) {
    extern __shared__ __align__(16) uint8_t smem[];
    typedef __attribute__((address_space(3))) uint8_t lds_byte;

    int cur, end;
    worker_share(pl, blockIdx.x, cur, end);
    TileWalk walk;
    walk_begin(pl, blockIdx.x, cur, end, walk);

    Tile t, next;
    if (!next_tile(pl, walk, t)) return;                  // workgroup-uniform

    const int lane = threadIdx.x & 63;
    A8Ctx c;
    c.xc = xc; c.wc = wc; c.xs = xs; c.ws = ws;
    c.M = M; c.N = N; c.smem = smem;
    c.row_group_bytes = (uint32_t)(4 * ((nb + 7) >> 3)) * 1024u;   // stages of 64 K elements (K zero-padded to 256)
    c.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    c.lane = lane;
    c.lds0 = (uint32_t)(uintptr_t)(lds_byte*)smem;
    c.lds_sc = c.lds0 + kA8ScaleLds0;
    c.kg = lane >> 5;

    c.aim(t);
    c.issue_stage<0>(0);
    c.issue_stage<1>(1);
    c.issue_stage<2>(2);
    c.issue_stage<3>(3);
    for (;;) {
        const bool has_next = next_tile(pl, walk, next);
        if constexpr (GLU) {
            if (t.nj == 4) a8_run_tile<4, YT, true>(c, t, has_next, next, Y, ldy, part_stride);
            else a8_run_tile<2, YT, true>(c, t, has_next, next, Y, ldy, part_stride);
        } else {
            switch (t.nj) {
                case 4: a8_run_tile<4, YT, false>(c, t, has_next, next, Y, ldy, part_stride); break;
                case 3: a8_run_tile<3, YT, false>(c, t, has_next, next, Y, ldy, part_stride); break;
                case 2: a8_run_tile<2, YT, false>(c, t, has_next, next, Y, ldy, part_stride); break;
                default: a8_run_tile<1, YT, false>(c, t, has_next, next, Y, ldy, part_stride); break;
            }
        }
        if (!has_next) break;
        t = next;
    }
}

// Sum of the K parts' partial blocks (store_partial order), in part order (fixed, so the result does not depend
// on timing), to Y.  One workgroup per 32x32 block: wave q sums piece q into an LDS tile, then the tile leaves
// row by row, four columns per lane.
template <typename YT>
__global__ void __launch_bounds__(256)
splitk_reduce(const float* __restrict__ P, int parts, int64_t part_stride, int col_blocks, int M, int N,
              YT* __restrict__ Y, int64_t ldy) {
    constexpr int kPitch = 32 + 4;
    __shared__ float tile[32 * kPitch];
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int rb = blockIdx.y, cb = blockIdx.x;
    const int l32 = lane & 31, kg = lane >> 5;
    const float* src = P + ((size_t)rb * col_blocks + cb) * kPartialBlockFloats + q * 256 + lane * 4;
    f32x4 a = *reinterpret_cast<const f32x4*>(src);
    for (int p = 1; p < parts; ++p) a += *reinterpret_cast<const f32x4*>(src + (size_t)p * part_stride);
#pragma unroll
    for (int r = 0; r < 4; ++r) tile[(8 * q + 4 * kg + r) * kPitch + l32] = a[r];
    __syncthreads();
    // 32 rows x 32 columns: thread -> (row, 4 columns)
    const int row = threadIdx.x >> 3, c0 = (threadIdx.x & 7) * 4;
    const int m = 32 * rb + row, n = 32 * cb + c0;
    if (m >= M || n >= N) return;
    const f32x4 v = *reinterpret_cast<const f32x4*>(tile + row * kPitch + c0);
    YT* dst = Y + (size_t)m * ldy + n;
    const bool whole = n + 4 <= N && (reinterpret_cast<uintptr_t>(dst) & (4 * sizeof(YT) - 1)) == 0;
    if (whole) {
        if constexpr (sizeof(YT) == 2) {
            const f32x2 lo = {v[0], v[1]}, hi = {v[2], v[3]};
            *reinterpret_cast<uint2*>(dst) = uint2{__builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2)),
                                                   __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2))};
        } else {
            *reinterpret_cast<f32x4*>(dst) = v;
        }
        return;
    }
    for (int i = 0; i < 4 && n + i < N; ++i) store_y<YT>(dst + i, v[i]);
}

// The same for row-major partial sums partial[part][M][N] (the small-M kernel): one thread per output element.
template <typename YT>
__global__ void __launch_bounds__(256)
splitk_reduce_rows(const float* __restrict__ P, int parts, int M, int N, YT* __restrict__ Y, int64_t ldy) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)M * N) return;
    const int m = (int)(e / N), n = (int)(e - (int64_t)m * N);
    float acc = P[e];
    for (int p = 1; p < parts; ++p) acc += P[(int64_t)p * M * N + e];
    store_y<YT>(Y + (int64_t)m * ldy + n, acc);
}

// A8: the activation codes are MXFP8 in the blocked 8-bit layout.  GLU: gated output (Y is M x N/2, N % 64 == 0).
// Partial sums of the K parts live in caller memory: `parts` (256-byte aligned, `parts_bytes` bytes; null: none).
// How many K parts a launch uses is a function of the shape, the device's compute units and parts_bytes only
// (gemm_plan), so the same call gives the same bits on every stream, eagerly or captured.
#ifndef BATQ_MID
#define BATQ_MID 1
#endif
// LDS slots of gemm_mid's weight strip (10: slower on every shape tried, 128 x 4096 x 14336 12.0 -> 12.8 us)
constexpr int kMidDepth = 6;
struct GemmPlan {
    TilePlan tiled;             // M > 64: the tiled kernels' plan, ksplit set
    size_t part_floats = 0;     // floats of one K part's partial sums
    int col_blocks = 0;         // 32-column blocks of the padded output (tiled kernels)
    int ksplit = 1;             // K parts used
    int want = 1;               // K parts the shape would like (workspace permitting)
    int rt = 4;                 // 4-bit tiled kernel: 32-row matrix tiles per wave (4: 4 waves, 2: 8 waves)
    bool mid = false;           // 4-bit, plain output, at most one gemm_mid workgroup per compute unit
    int mid_strips = 1;         // strips of a gemm_mid workgroup (tile of 128 rows x 64 or 128 columns)
    bool skinny = false, wide = false, narrow = false;
    int cols = 0;               // skinny: workgroups along N
};

// fits32: both code arrays are below 2 GiB (the tiled kernels and gemm_mid use 32-bit load offsets; M > 64 without
// it is the caller's case for gemm_direct).
inline GemmPlan gemm_plan(int M, int N, int nb, int cus, bool a8, bool glu, size_t parts_bytes, bool fits32 = true) {
    GemmPlan g;
    if (M > 32) {
        g.tiled = make_plan(M, N, nb, cus, glu);
        if (!glu) {
            g.col_blocks = 2 * g.tiled.strips_n;
            g.part_floats = (size_t)g.tiled.tiles_m * 8 * g.col_blocks * kPartialBlockFloats;
            g.want = choose_ksplit(g.tiled, 0, 0);
            g.ksplit = g.want > 1 ? choose_ksplit(g.tiled, g.part_floats * sizeof(float), parts_bytes) : 1;
        }
        g.tiled.ksplit = g.ksplit;
        // Eight waves where the workgroups get tiles three or four strips wide: their epilogues and LDS waits then
        // overlap with the other wave's matrix instructions (2048 x 4096 x 14336: 67.8 -> 64.5 us,
        // 8192 x 3584 x 18944: 345 -> 328, 1024 x 4096 x 14336: 38.7 -> 36.3).  Narrow tiles stay with four waves
        // (one strip per workgroup, 256 x 14336 x 4096: 40.0 us against 46.5 with eight waves, which then fetch
        // more of B than they use and read each A fragment for fewer instructions).
        const long units = (long)g.tiled.tiles_m * g.tiled.strips_n;
        const long per_worker = (units + g.tiled.workers - 1) / g.tiled.workers;
        g.rt = (!a8 && g.ksplit == 1 && per_worker * g.tiled.pair >= 3) ? 2 : 4;
        // gemm_mid where all its workgroups (128-row panels x strips x K parts) run at once.  Graph-replayed, weights
        // in HBM, tiled kernel -> gemm_mid: 128 x 4096 x 14336 14.9 -> 12.0 us, 300 x 4096 x 4096 12.8 -> 9.9,
        // 2048 x 4096 x 1024 12.5 -> 10.5, 256 x 14336 x 4096 without K parts 39.1 -> 29.0, 128 x 14336 x 4096 with
        // 4 K parts 19.8 -> 15.5, 256 x 8192 x 4096 with 2 K parts 19.9 -> 17.0.  With more workgroups than compute
        // units it loses (256 x 4096 x 14336: 16.6 -> 19.4, 512 x 14336 x 4096 with 4 K parts 30.7 -> 36.7); 256-row
        // panels, with two 32-row tiles per wave or with eight waves, lose everywhere (256 x 4096 x 14336: 18.1, 18.7).
        // From 33 rows on it also beats the small-M kernel (64 x 4096 x 14336: 12.9 -> 11.0 us).  Where single strips
        // are too many but pairs of strips fit, a workgroup takes two (tiled kernel -> that: 256 x 4096 x 14336
        // 17.1 -> 16.3 us, 200 rows 15.9 -> 15.4); where single strips fit they are the faster choice (128 x 4096 x
        // 14336: 12.0 us against 16.1 with pairs on half the compute units).
        if (BATQ_MID && !a8 && !glu && fits32 && g.rt == 4) {
            const long panels = (M + 127) / 128, strips = g.tiled.strips_n;
            const bool one = panels * strips * g.ksplit <= g.tiled.workers;
            const bool two = panels * ((strips + 1) / 2) * g.ksplit <= g.tiled.workers;
            g.mid = one || two;
            g.mid_strips = one ? 1 : 2;
        }
        if (M > 64 || g.mid) return g;
        g = GemmPlan();
    }
    g.skinny = true;
    // 64 columns per workgroup pay with two row tiles (the X codes are the larger share of a workgroup's
    // loads then) when they make one full round of workgroups: between three quarters of and all the compute
    // units (64 x 4096 x 14336: 15.4 -> 12.9 us; with one row tile, or a second partial round, it loses).  Not
    // for the 8-bit kernel, which would not fit its registers.
    const int cols64 = (N + 63) / 64;
    g.wide = !glu && !a8 && M > 32 && cols64 <= cus && 4 * cols64 >= 3 * cus;
    // 16 columns per workgroup where 32 would give at most half the compute units a workgroup (decode shapes with
    // N <= 4096 on 256 compute units; graph-replayed, 20 weight copies taking turns: 16 x 4096 x 4096 4.7 -> 4.5 us,
    // 16 x 14336 x 4096 11.2 -> 10.2 us, where it also replaces two K parts and their second kernel,
    // 32 x 8192 x 2048 7.0 -> 6.8).  (Four instead of two K groups in flight per wave, with a ring of register sets:
    // 16 x 14336 x 4096 back to 11.2 us; not in.)
    g.narrow = !glu && !g.wide && M <= 32 && 2 * ((N + 31) / 32) <= cus;
    g.cols = (glu || g.wide) ? cols64 : g.narrow ? (N + 15) / 16 : (N + 31) / 32;
    // Narrow N with a long K leaves half the compute units idle while every workgroup reads all of A: two
    // workgroup rows then take half of K each (64 x 14336 x 4096: 15.8 -> 12.0 us).  More parts, or shorter
    // K, lose more to the second kernel than they gain.
    g.part_floats = (size_t)M * N;
    g.want = (!glu && !g.wide && 2 * g.cols <= cus && scale_groups(nb) >= 48) ? 2 : 1;
    g.ksplit = (g.want > 1 && (size_t)g.want * g.part_floats * sizeof(float) <= parts_bytes) ? g.want : 1;
    return g;
}

template <typename YT, bool A8, bool GLU>
hipError_t launch_typed(const uint8_t* xc, const uint8_t* xs, const batq_weight* w, int M, YT* Y, int64_t ldy,
                        float* parts, size_t parts_bytes, hipStream_t stream) {
    const int N = w->N, nb = w->nb;
    const size_t xbytes = A8 ? code8_bytes_blocked(M, nb) : code_bytes_blocked(M, nb);
    const bool fits32 = xbytes < (1ull << 31) && code_bytes_blocked(N, nb) < (1ull << 31);
    if (M > 64 && !fits32) {
        if constexpr (GLU) return hipErrorNotSupported;       // callers check gemm_glu_supported first
        const dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
        gemm_direct<YT, A8><<<grid, block, 0, stream>>>(xc, xs, w->d_codes, w->d_scales, M, N, nb, Y, ldy);
        return hipGetLastError();
    }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const int cus = device_compute_units(dev, &e);
    if (e != hipSuccess) return e;
    const GemmPlan g = gemm_plan(M, N, nb, cus, A8, GLU, parts ? parts_bytes : 0, fits32);
    if (!g.skinny) {
        const TilePlan& pl = g.tiled;
        if (g.mid) {
            if constexpr (!A8 && !GLU) {
                const int ns = g.mid_strips;
                const dim3 grid((pl.strips_n + ns - 1) / ns, (M + 127) / 128, g.ksplit), block(256);
                if (g.ksplit > 1) {
                    partial_f32* const P = reinterpret_cast<partial_f32*>(parts);
                    if (ns == 2)
                        gemm_mid<partial_f32, 1, kMidDepth, 2><<<grid, block, 0, stream>>>(
                            xc, xs, w->d_codes, w->d_scales, M, N, nb, g.ksplit, P, (int64_t)g.col_blocks, (int64_t)g.part_floats);
                    else
                        gemm_mid<partial_f32, 1, kMidDepth, 1><<<grid, block, 0, stream>>>(
                            xc, xs, w->d_codes, w->d_scales, M, N, nb, g.ksplit, P, (int64_t)g.col_blocks, (int64_t)g.part_floats);
                    splitk_reduce<YT><<<dim3(g.col_blocks, (M + 31) / 32), dim3(256), 0, stream>>>(
                        parts, g.ksplit, (int64_t)g.part_floats, g.col_blocks, M, N, Y, ldy);
                } else if (ns == 2) {
                    gemm_mid<YT, 1, kMidDepth, 2><<<grid, block, 0, stream>>>(xc, xs, w->d_codes, w->d_scales, M, N, nb, 1, Y, ldy, 0);
                } else {
                    gemm_mid<YT, 1, kMidDepth, 1><<<grid, block, 0, stream>>>(xc, xs, w->d_codes, w->d_scales, M, N, nb, 1, Y, ldy, 0);
                }
            }
        } else if (g.ksplit > 1) {
            if constexpr (!GLU) {
                if constexpr (A8) {
                    e = ensure_dynamic_lds<&gemm_tiled_a8<partial_f32, false>>(dev, kA8Lds);
                    if (e != hipSuccess) return e;
                    gemm_tiled_a8<partial_f32, false><<<dim3(pl.workers), dim3(256), kA8Lds, stream>>>(
                        xc, xs, w->d_codes, w->d_scales, M, N, nb, pl, reinterpret_cast<partial_f32*>(parts),
                        (int64_t)g.col_blocks, (int64_t)g.part_floats);
                } else {
                    e = ensure_dynamic_lds<&gemm_tiled<partial_f32, false, 4>>(dev, kTiledLds);
                    if (e != hipSuccess) return e;
                    gemm_tiled<partial_f32, false, 4><<<dim3(pl.workers), dim3(256), kTiledLds, stream>>>(
                        xc, xs, w->d_codes, w->d_scales, M, N, nb, pl, reinterpret_cast<partial_f32*>(parts),
                        (int64_t)g.col_blocks, (int64_t)g.part_floats);
                }
                splitk_reduce<YT><<<dim3(g.col_blocks, (M + 31) / 32), dim3(256), 0, stream>>>(
                    parts, g.ksplit, (int64_t)g.part_floats, g.col_blocks, M, N, Y, ldy);
            }
        } else if constexpr (A8) {
            e = ensure_dynamic_lds<&gemm_tiled_a8<YT, GLU>>(dev, kA8Lds);
            if (e != hipSuccess) return e;
            gemm_tiled_a8<YT, GLU><<<dim3(pl.workers), dim3(256), kA8Lds, stream>>>(xc, xs, w->d_codes, w->d_scales,
                                                                                     M, N, nb, pl, Y, ldy, 0);
        } else if (g.rt == 2) {
            e = ensure_dynamic_lds<&gemm_tiled<YT, GLU, 2>>(dev, kTiledLds);
            if (e != hipSuccess) return e;
            gemm_tiled<YT, GLU, 2><<<dim3(pl.workers), dim3(512), kTiledLds, stream>>>(xc, xs, w->d_codes, w->d_scales, M,
                                                                                        N, nb, pl, Y, ldy, 0);
        } else {
            e = ensure_dynamic_lds<&gemm_tiled<YT, GLU, 4>>(dev, kTiledLds);
            if (e != hipSuccess) return e;
            gemm_tiled<YT, GLU, 4><<<dim3(pl.workers), dim3(256), kTiledLds, stream>>>(xc, xs, w->d_codes, w->d_scales, M,
                                                                                        N, nb, pl, Y, ldy, 0);
        }
    } else {
        const dim3 grid(g.cols, g.ksplit), block(kSkinnyWaves * 64);
        float* pp = g.ksplit > 1 ? parts : nullptr;
        if constexpr (GLU) {
            if (M <= 32)
                gemm_skinny<YT, 1, A8, true, false><<<grid, block, 0, stream>>>(xc, xs, w->d_codes, w->d_scales, M, N, nb, Y, ldy, pp);
            else
                gemm_skinny<YT, 2, A8, true, false><<<grid, block, 0, stream>>>(xc, xs, w->d_codes, w->d_scales, M, N, nb, Y, ldy, pp);
        } else if (g.wide) {
            if constexpr (!A8)
                gemm_skinny<YT, 2, false, false, true><<<grid, block, 0, stream>>>(xc, xs, w->d_codes, w->d_scales, M, N, nb, Y, ldy, pp);
        } else if (g.narrow) {
            gemm_skinny<YT, 1, A8, false, false, true><<<grid, block, 0, stream>>>(xc, xs, w->d_codes, w->d_scales, M, N, nb, Y, ldy, pp);
        } else {
            if (M <= 32)
                gemm_skinny<YT, 1, A8, false, false><<<grid, block, 0, stream>>>(xc, xs, w->d_codes, w->d_scales, M, N, nb, Y, ldy, pp);
            else
                gemm_skinny<YT, 2, A8, false, false><<<grid, block, 0, stream>>>(xc, xs, w->d_codes, w->d_scales, M, N, nb, Y, ldy, pp);
        }
        if (g.ksplit > 1) {
            const int64_t total = (int64_t)M * N;
            splitk_reduce_rows<YT><<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(parts, g.ksplit, M, N, Y, ldy);
        }
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_scales_to_internal(const uint8_t* canon, uint8_t* internal, int rows, int nb, hipStream_t stream) {
    const size_t total = (size_t)rows * scale_groups(nb) * 8;
    const int grid = (int)std::min<size_t>((total + 255) / 256, 4096);
    scales_to_internal<<<grid, 256, 0, stream>>>(canon, internal, rows, nb);
    return hipGetLastError();
}

hipError_t launch_scales_to_canonical(const uint8_t* internal, uint8_t* canon, int rows, int nb, hipStream_t stream) {
    const size_t total = (size_t)rows * nb;
    const int grid = (int)std::min<size_t>((total + 255) / 256, 4096);
    scales_to_canonical<<<grid, 256, 0, stream>>>(internal, canon, rows, nb);
    return hipGetLastError();
}

hipError_t launch_codes_to_blocked(const uint8_t* rowmajor, uint8_t* blocked, int rows, int nb, hipStream_t stream) {
    const size_t total = (size_t)rows * scale_groups(nb) * 8;
    const int grid = (int)std::min<size_t>((total + 255) / 256, 8192);
    codes_to_blocked<<<grid, 256, 0, stream>>>(rowmajor, blocked, rows, nb);
    return hipGetLastError();
}

hipError_t launch_codes_to_rowmajor(const uint8_t* blocked, uint8_t* rowmajor, int rows, int nb, hipStream_t stream) {
    const size_t total = (size_t)rows * nb;
    const int grid = (int)std::min<size_t>((total + 255) / 256, 8192);
    codes_to_rowmajor<<<grid, 256, 0, stream>>>(blocked, rowmajor, rows, nb);
    return hipGetLastError();
}

hipError_t launch_codes8_to_blocked(const uint8_t* rowmajor, uint8_t* blocked, int rows, int nb, hipStream_t stream) {
    const size_t total = (size_t)rows * scale_groups(nb) * 16;
    const int grid = (int)std::min<size_t>((total + 255) / 256, 8192);
    codes8_to_blocked<<<grid, 256, 0, stream>>>(rowmajor, blocked, rows, nb);
    return hipGetLastError();
}

hipError_t launch_codes8_to_rowmajor(const uint8_t* blocked, uint8_t* rowmajor, int rows, int nb, hipStream_t stream) {
    const size_t total = (size_t)rows * nb * 2;
    const int grid = (int)std::min<size_t>((total + 255) / 256, 8192);
    codes8_to_rowmajor<<<grid, 256, 0, stream>>>(blocked, rowmajor, rows, nb);
    return hipGetLastError();
}

int tile_schedule(int M, int N, int K, int compute_units, bool glu, bool allow_ksplit, int* out, int capacity) {
    const int nb = K / 32;
    if (M <= 64) return 0;                                      // the small-M kernels have no tile schedule
    const GemmPlan g = gemm_plan(M, N, nb, compute_units, false, glu, allow_ksplit ? ~size_t(0) : 0);
    const TilePlan& pl = g.tiled;
    int n = 0;
    for (int b = 0; b < pl.workers; ++b) {
        int cur, end;
        worker_share(pl, b, cur, end);
        TileWalk walk;
        walk_begin(pl, b, cur, end, walk);
        Tile t;
        while (next_tile(pl, walk, t)) {
            if (n < capacity) {
                int* o = out + (size_t)n * 7;
                o[0] = b; o[1] = t.m0; o[2] = t.n0; o[3] = t.nj; o[4] = t.part; o[5] = t.g0; o[6] = t.ng;
            }
            ++n;
        }
    }
    return n;
}

size_t gemm_workspace_bytes(const batq_weight* w, int M, bool a8, int cus) {
    if (M <= 0) return 0;
    const size_t xbytes = a8 ? code8_bytes_blocked(M, w->nb) : code_bytes_blocked(M, w->nb);
    const bool fits32 = xbytes < (1ull << 31) && code_bytes_blocked(w->N, w->nb) < (1ull << 31);
    if (M > 64 && !fits32) return 0;
    const GemmPlan g = gemm_plan(M, w->N, w->nb, cus, a8, false, 0, fits32);
    return g.want > 1 ? (size_t)g.want * g.part_floats * sizeof(float) : 0;
}

bool gemm_glu_supported(const batq_weight* w, int M, bool a8) {
    if (w->N % 64 != 0) return false;
    if (M <= 64) return true;
    const size_t xbytes = a8 ? code8_bytes_blocked(M, w->nb) : code_bytes_blocked(M, w->nb);
    return xbytes < (1ull << 31) && code_bytes_blocked(w->N, w->nb) < (1ull << 31);
}

template <bool GLU>
static hipError_t launch_gemm_as(const uint8_t* xcodes, const uint8_t* xscales_internal, const batq_weight* w, int M,
                                 void* Y, batq_dtype ydtype, int64_t ldy, bool a8, float* parts, size_t parts_bytes,
                                 hipStream_t stream) {
    if (ydtype == BATQ_BF16) {
        uint16_t* Yp = static_cast<uint16_t*>(Y);
        return a8 ? launch_typed<uint16_t, true, GLU>(xcodes, xscales_internal, w, M, Yp, ldy, parts, parts_bytes, stream)
                  : launch_typed<uint16_t, false, GLU>(xcodes, xscales_internal, w, M, Yp, ldy, parts, parts_bytes, stream);
    }
    float* Yp = static_cast<float*>(Y);
    return a8 ? launch_typed<float, true, GLU>(xcodes, xscales_internal, w, M, Yp, ldy, parts, parts_bytes, stream)
              : launch_typed<float, false, GLU>(xcodes, xscales_internal, w, M, Yp, ldy, parts, parts_bytes, stream);
}

hipError_t launch_gemm_mxfp4(const uint8_t* xcodes, const uint8_t* xscales_internal, const batq_weight* w, int M,
                             void* Y, batq_dtype ydtype, int64_t ldy, bool a8, bool glu, void* parts,
                             size_t parts_bytes, hipStream_t stream) {
    if (M == 0) return hipSuccess;
    float* pf = static_cast<float*>(parts);
    return glu ? launch_gemm_as<true>(xcodes, xscales_internal, w, M, Y, ydtype, ldy, a8, nullptr, 0, stream)
               : launch_gemm_as<false>(xcodes, xscales_internal, w, M, Y, ydtype, ldy, a8, pf, parts_bytes, stream);
}

// Partial-sum memory for callers that can pass no workspace and must not allocate: one array per device, part of
// the loaded code object (each device that runs the library holds its own copy until the process ends).  In host
// code the array's name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
// Nothing in it has to start at zero: every K part writes all the blocks the reduction reads.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t static_scratch(void** ptr) {
    static std::atomic<void*> address[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool cached = dev >= 0 && dev < kMaxDevices;
    void* p = cached ? address[dev].load(std::memory_order_acquire) : nullptr;
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // the current device's copy
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        if (cached) address[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    return hipSuccess;
}

}  // namespace batq
