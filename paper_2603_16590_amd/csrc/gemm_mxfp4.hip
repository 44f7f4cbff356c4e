// MXFP4 x MXFP4 GEMM (the low-bit product of Sec. 3.1: Q(XP) Q(P^-1 W)) on gfx950's
// block-scaled FP4 matrix instruction, fp32 accumulation.
//
// v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in FP4: lane l supplies, for matrix
// row (l % 32), the 32 consecutive K elements of MX block (l / 32) as 16 packed bytes, plus
// that block's E8M0 scale; so one 16-byte chunk of the code layout (code_layout.h) is exactly
// one operand fragment.  Accumulator register r of lane l is element
// (8*(r/4) + 4*(l/32) + r%4, l % 32) of the 32x32 tile.
//
// Two kernels:
//   gemm_tiled  - 256x256 output tile per workgroup (4 waves, each 128x128 = 4x4 matrix
//                 tiles held in 256 accumulator registers); codes and scales stream
//                 global -> LDS with LDS-direct loads through a 4-stage ring (XOR-swizzled
//                 16-byte slots); workgroup -> tile mapping grouped per XCD so that an XCD's
//                 L2 sees a compact sub-grid.
//   gemm_direct - one wave per 32x32 tile with operands straight from global memory, for
//                 small M.
#include <algorithm>

#include "batq_internal.h"
#include "code_layout.h"
#include "mxfp4_device.h"
#include "scale_layout.h"

namespace batq {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

template <typename YT>
__device__ __forceinline__ void store_y(YT* p, float v);
template <>
__device__ __forceinline__ void store_y<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_y<uint16_t>(uint16_t* p, float v) { *p = (uint16_t)float_to_bf16_bits(v); }

__device__ __forceinline__ v8i frag(const uint4 v) {
    return v8i{(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};
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

// ------------------------------------------------------------------------------------------
template <typename YT>
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
    for (int s = 0; s < steps; ++s) {
        const uint4 a = *reinterpret_cast<const uint4*>(xc + code_chunk_offset(am, 2 * s + kg, nb));
        const uint4 b = *reinterpret_cast<const uint4*>(wc + code_chunk_offset(bn, 2 * s + kg, nb));
        const int sa = xs[scale_index_internal(am, 2 * s + kg, M)];
        const int sb = ws[scale_index_internal(bn, 2 * s + kg, N)];
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag(a), frag(b), acc, 4, 4, 0, sa, 0, sb);
    }
    if (nb & 1) {
        // odd block count: the upper half-wave contributes an all-zero operand
        const int s = steps;
        uint4 a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
        int sa = 127, sb = 127;
        if (kg == 0) {
            a = *reinterpret_cast<const uint4*>(xc + code_chunk_offset(am, 2 * s, nb));
            b = *reinterpret_cast<const uint4*>(wc + code_chunk_offset(bn, 2 * s, nb));
            sa = xs[scale_index_internal(am, 2 * s, M)];
            sb = ws[scale_index_internal(bn, 2 * s, N)];
        }
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag(a), frag(b), acc, 4, 4, 0, sa, 0, sb);
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
// Tiled kernel.  256x256 output tile per workgroup of 4 waves (2x2, each wave 128x128 = 4x4
// matrix tiles in 256 accumulator registers).  K advances in stages of 128 elements (64 code
// bytes per row).  Codes and scales go global -> LDS with LDS-direct loads (no VGPR staging,
// no ds_write): a ring of 4 stage buffers keeps three stages in flight.  Scales of a whole
// 256-element K group (two stages) are fetched once per group into a 2-deep ring.
constexpr int kTile = 256;                 // output tile edge
constexpr int kStageBytes = 64;            // code bytes per row per stage (128 elements, 4 MX blocks)
constexpr int kOperandStage = kTile * kStageBytes;        // 16 KiB per operand per stage
constexpr int kStageLds = 2 * kOperandStage;               // A then B
constexpr int kRing = 4;                   // stage buffers
constexpr int kScaleGroupLds = 2 * kTile * 8;              // A then B scale bytes of one K group (4 KiB)
constexpr int kTiledLds = kRing * kStageLds + 2 * kScaleGroupLds;   // 136 KiB

// 16-byte slot swizzle inside a 64-byte LDS row: the 32 rows a fragment read touches, and the
// 16 rows x 4 slots an LDS-direct load writes, both spread over all banks.
__device__ __forceinline__ int slot_swizzle(int row) { return (row >> 2) & 3; }

// Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous range of tile
// ids, and order tile ids in bands of kBand tile-rows so that the range is a compact sub-grid.
__device__ __forceinline__ void tile_of_workgroup(int pid, int tiles_m, int tiles_n, int& tm, int& tn) {
    const int T = tiles_m * tiles_n;
    const int q = T >> 3, rem = T & 7;
    const int xcd = pid & 7, local = pid >> 3;
    int id = xcd * q + min(xcd, rem) + local;
    constexpr int kBand = 4;
    const int per_band = kBand * tiles_n;
    const int band = id / per_band;
    const int first_m = band * kBand;
    const int rows_in_band = min(kBand, tiles_m - first_m);
    id -= band * per_band;
    tm = first_m + id % rows_in_band;
    tn = id / rows_in_band;
}

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
// s_waitcnt vmcnt(N) only (expcnt and lgkmcnt left at their maxima), gfx9 encoding.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// One matrix instruction of the 4x4 grid of 32x32 tiles a wave owns.
template <int KK>
__device__ __forceinline__ void mfma_one(v16f& acc, const uint4& a, const uint4& b, int sa, int sb) {
    acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag(a), frag(b), acc, 4, 4, KK, sa, KK, sb);
}

// Scheduling hints: keep the instruction order written below (the wave runs alone on its
// SIMD, so LDS latency is hidden only by what the wave itself has queued on the matrix pipe).
#define BATQ_SCHED_MFMA(n) __builtin_amdgcn_sched_group_barrier(0x008, (n), 0)
#define BATQ_SCHED_DSRD(n) __builtin_amdgcn_sched_group_barrier(0x100, (n), 0)

struct TiledCtx {
    // global -> LDS
    const uint8_t* xc; const uint8_t* wc; const uint8_t* xs; const uint8_t* ws;
    uint32_t aoff[4], boff[4], sao[2], sbo[2];
    uint32_t lds0, lds_sc;
    int M, N, wave;
    // LDS -> registers
    const uint8_t* smem;
    int a_rd, b_rd, sc_a_rd, sc_b_rd, kg, fsw;

    // The loads of one stage, in a fixed order: part 0..7 = the 8 code pieces of this wave (A then B),
    // part 8 = the scales of the K group an even stage opens (4 dword loads).  Completion is counted
    // per thread in this order.
    __device__ __forceinline__ void issue_part(int s, int part) const {
        const uint32_t buf = lds0 + (uint32_t)(s & (kRing - 1)) * kStageLds + (uint32_t)wave * 4096;
        if (part < 4) {
            dma16(xc + (size_t)s * 1024, aoff[part], buf + part * 1024);        // one 1 KiB piece per 16 rows and stage
        } else if (part < 8) {
            dma16(wc + (size_t)s * 1024, boff[part - 4], buf + kOperandStage + (part - 4) * 1024);
        } else if ((s & 1) == 0) {
            const int g = s >> 1;
            const uint32_t sbuf = lds_sc + (uint32_t)(g & 1) * kScaleGroupLds + (uint32_t)wave * 512;
            const uint8_t* sag = xs + (size_t)g * M * 8;
            const uint8_t* sbg = ws + (size_t)g * N * 8;
#pragma unroll
            for (int j = 0; j < 2; ++j) dma4(sag, sao[j], sbuf + j * 256);
#pragma unroll
            for (int j = 0; j < 2; ++j) dma4(sbg, sbo[j], sbuf + kTile * 8 + j * 256);
        }
    }
    __device__ __forceinline__ void issue_stage(int s) const {
#pragma unroll
        for (int part = 0; part < 9; ++part) issue_part(s, part);
    }
    __device__ __forceinline__ void read_frags(int s, int half, uint4 (&fa)[4], uint4 (&fb)[4]) const {
        const uint8_t* base = smem + (s & (kRing - 1)) * kStageLds + (((2 * half + kg) ^ fsw) << 4);
        // in the order the matrix instructions consume them: a0, b0..b3, a1..a3
        fa[0] = *reinterpret_cast<const uint4*>(base + a_rd);
#pragma unroll
        for (int i = 0; i < 4; ++i) fb[i] = *reinterpret_cast<const uint4*>(base + b_rd + i * 32 * kStageBytes);
#pragma unroll
        for (int i = 1; i < 4; ++i) fa[i] = *reinterpret_cast<const uint4*>(base + a_rd + i * 32 * kStageBytes);
    }
    __device__ __forceinline__ void read_scales(int g, int (&sa)[4], int (&sb)[4]) const {
        const uint8_t* sp = smem + kRing * kStageLds + (g & 1) * kScaleGroupLds;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sa[i] = *reinterpret_cast<const int*>(sp + sc_a_rd + i * 256);
            sb[i] = *reinterpret_cast<const int*>(sp + sc_b_rd + i * 256);
        }
    }
};

// One K stage (two matrix-instruction K steps) of the software pipeline.
//   PAR    parity of the stage inside its K group (selects the scale bytes: op_sel 2 PAR, 2 PAR + 1)
//   WAIT   loads that may stay in flight once stage s+1 has landed (-1: there is no stage s+1)
//   ISSUE  start the loads of stage s+4 into the ring slot this stage frees
// On entry f0 holds the fragments of (s, first half); on exit those of (s+1, first half).
template <int PAR, int WAIT, bool ISSUE>
__device__ __forceinline__ void tiled_stage(const TiledCtx& c, int s, v16f (&acc)[4][4], uint4 (&a0)[4],
                                            uint4 (&b0)[4], int (&sa)[4], int (&sb)[4]) {
    uint4 a1[4], b1[4];
    // first half: fetch the second half's fragments underneath the 16 matrix instructions
    c.read_frags(s, 1, a1, b1);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) mfma_one<2 * PAR>(acc[i][j], a0[i], b0[j], sa[i], sb[j]);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        BATQ_SCHED_DSRD(1);
        BATQ_SCHED_MFMA(2);
    }
    // second half, part one
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) mfma_one<2 * PAR + 1>(acc[i][j], a1[i], b1[j], sa[i], sb[j]);
    BATQ_SCHED_MFMA(8);
    __builtin_amdgcn_sched_barrier(0);
    int sna[4], snb[4];
    if constexpr (WAIT >= 0) {
        // every wave has read stage s completely (its last fragments are in registers); once all
        // have also seen stage s+1 land, the slot of stage s can be refilled
        wait_vmcnt<WAIT>();
        __syncthreads();
        c.read_frags(s + 1, 0, a0, b0);
        if constexpr (PAR == 1) c.read_scales((s + 1) >> 1, sna, snb);
    }
    __builtin_amdgcn_sched_barrier(0);
    // second half, part two: covers the latency of the reads just issued; the loads of stage s+4
    // are issued one between every two matrix instructions, so the matrix pipe never waits for them
#pragma unroll
    for (int i = 2; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            mfma_one<2 * PAR + 1>(acc[i][j], a1[i], b1[j], sa[i], sb[j]);
            if constexpr (WAIT >= 0 && ISSUE) {
                __builtin_amdgcn_sched_barrier(0);
                c.issue_part(s + 4, (i - 2) * 4 + j);
                if (i == 3 && j == 3) c.issue_part(s + 4, 8);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    if constexpr (WAIT >= 0 && PAR == 1) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sa[i] = sna[i];
            sb[i] = snb[i];
        }
    }
}

// Requires operand code arrays below 2 GiB (32-bit load offsets).
template <typename YT>
__global__ void __launch_bounds__(256, 1)
gemm_tiled(const uint8_t* __restrict__ xc, const uint8_t* __restrict__ xs, const uint8_t* __restrict__ wc,
           const uint8_t* __restrict__ ws, int M, int N, int nb, int tiles_m, int tiles_n,
           YT* __restrict__ Y, int64_t ldy) {
    extern __shared__ __align__(16) uint8_t smem[];
    typedef __attribute__((address_space(3))) uint8_t lds_byte;

    int tm, tn;
    tile_of_workgroup(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int m0 = tm * kTile, n0 = tn * kTile;

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, kg = lane >> 5;
    const int G = (nb + 7) >> 3;            // K groups of 256 elements (K is zero-padded to them)
    const int T = 2 * G;                    // stages of 128 K elements

    TiledCtx c;
    c.xc = xc; c.wc = wc; c.xs = xs; c.ws = ws;
    c.M = M; c.N = N; c.wave = wave; c.smem = smem;
    c.lds0 = (uint32_t)(uintptr_t)(lds_byte*)smem;            // LDS byte address of the stage ring
    c.lds_sc = c.lds0 + kRing * kStageLds;                    // scale ring
    {
        // LDS-direct tile loads: wave w, load j (0..3) copies the 1 KiB piece of row group
        // (tile row / 16 + 4 w + j) into LDS rows 16 (4 w + j) .. + 15 of a stage buffer; the blocked
        // code layout already is the swizzled LDS image, so lane i just moves bytes 16 i .. 16 i + 15.
        const int rgA = (M + 15) >> 4, rgB = (N + 15) >> 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int rg = 4 * wave + j;
            c.aoff[j] = (uint32_t)min((m0 >> 4) + rg, rgA - 1) * (uint32_t)(T * 1024) + lane * 16;
            c.boff[j] = (uint32_t)min((n0 >> 4) + rg, rgB - 1) * (uint32_t)(T * 1024) + lane * 16;
        }
        // LDS-direct scale loads: per K group, A and B each 256 rows x 2 dwords; wave w loads dwords
        // 128 w .. 128 w + 127 of each (two pieces of 64).
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int d = 128 * wave + 64 * j + lane;
            c.sao[j] = ((uint32_t)min(m0 + (d >> 1), M - 1) * 2 + (d & 1)) * 4;
            c.sbo[j] = ((uint32_t)min(n0 + (d >> 1), N - 1) * 2 + (d & 1)) * 4;
        }
    }
    // fragment reads: lane reads slot ((2 half + kg) ^ f(row)) of row (wave row base + 32 i + l32)
    c.kg = kg;
    c.fsw = slot_swizzle(l32);
    c.a_rd = (wm * 128 + l32) * kStageBytes;
    c.b_rd = kOperandStage + (wn * 128 + l32) * kStageBytes;
    c.sc_a_rd = ((wm * 128 + l32) * 2 + kg) * 4;
    c.sc_b_rd = kTile * 8 + ((wn * 128 + l32) * 2 + kg) * 4;

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v16f{};
    uint4 fa[4], fb[4];
    int sa[4], sb[4];

    // Loads per thread: 8 per stage, plus 4 for the scales of a K group issued right after the
    // group's even stage; they complete in issue order.  In steady state stages s+2 and s+3
    // (8 + 8 + 4 = 20 loads) stay in flight while stage s+1 is awaited.
    c.issue_stage(0);
    c.issue_stage(1);
    if (T >= 4) {
        c.issue_stage(2);
        c.issue_stage(3);
        wait_vmcnt<28>();
    } else {
        wait_vmcnt<8>();
    }
    __syncthreads();
    c.read_scales(0, sa, sb);
    c.read_frags(0, 0, fa, fb);

    for (int g = 0; g + 2 < G; ++g) {
        tiled_stage<0, 20, true>(c, 2 * g, acc, fa, fb, sa, sb);
        tiled_stage<1, 20, true>(c, 2 * g + 1, acc, fa, fb, sa, sb);
    }
    if (G >= 2) {
        tiled_stage<0, 20, false>(c, T - 4, acc, fa, fb, sa, sb);
        tiled_stage<1, 8, false>(c, T - 3, acc, fa, fb, sa, sb);
    }
    tiled_stage<0, 0, false>(c, T - 2, acc, fa, fb, sa, sb);
    tiled_stage<1, -1, false>(c, T - 1, acc, fa, fb, sa, sb);

    // ---- epilogue: accumulators -> Y
    if constexpr (sizeof(YT) == 2) {
        // bf16: transpose through LDS so that every lane stores 16 contiguous bytes.
        // Needs the whole 256-column span inside N and 16-byte aligned rows (workgroup-uniform).
        const bool fast = n0 + kTile <= N && (ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(Y) & 15) == 0;
        if (fast) {
            __syncthreads();                                  // every wave is done with the stage ring
            uint8_t* ep = smem + wave * 32768;                // wave-private [128 rows][256 bytes]
            const int odd = lane & 1;
            // Element (i, j, rr) of this lane goes to row R = 32 i + 8 (rr / 2) + 2 (rr % 2) + (4 kg + odd)
            // and 16-byte chunk (4 j + l32 / 8) ^ swizzle(R); the swizzle only depends on the lane
            // (R & 1 = odd, (R >> 2) & 1 = kg), so it folds into four per-lane base pointers, one per j,
            // and everything else is an immediate offset.
            uint8_t* pj[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                pj[j] = ep + (4 * kg + odd) * 256 + ((4 * (j ^ (odd | (kg << 1))) + (l32 >> 3)) << 4) + ((l32 >> 1) & 3) * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int rr = 0; rr < 8; ++rr) {
                        // lanes pair up: the even lane keeps row r0 and both columns, the odd lane row r0 + 1
                        const float v0 = acc[i][j][2 * rr], v1 = acc[i][j][2 * rr + 1];
                        const float send = odd ? v0 : v1;
                        const float recv = __builtin_bit_cast(
                            float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, true));
                        f32x2 pr;
                        pr.x = odd ? recv : v0;
                        pr.y = odd ? v1 : recv;
                        const uint32_t packed = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
                        *reinterpret_cast<uint32_t*>(pj[j] + (32 * i + 8 * (rr >> 1) + 2 * (rr & 1)) * 256) = packed;
                    }
            // wave-private region: the wave's own LDS operations complete in order
            const int rsub = lane >> 4, c16 = lane & 15;
#pragma unroll 4
            for (int it = 0; it < 32; ++it) {
                const int R = 4 * it + rsub;
                const int chunk = c16 ^ (((R & 1) << 2) | (((R >> 2) & 1) << 3));
                const uint4 v = *reinterpret_cast<const uint4*>(ep + R * 256 + chunk * 16);
                const int row = m0 + wm * 128 + R;
                if (row < M)
                    *reinterpret_cast<uint4*>(Y + (size_t)row * ldy + n0 + wn * 128 + c16 * 8) = v;
            }
            return;
        }
    }
    const int col0 = n0 + wn * 128 + l32;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = m0 + wm * 128 + 32 * i + 8 * (r >> 2) + 4 * kg + (r & 3);
            if (row < M) {
                YT* yp = Y + (size_t)row * ldy;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int col = col0 + 32 * j;
                    if (col < N) store_y<YT>(yp + col, acc[i][j][r]);
                }
            }
        }
    }
}

template <typename YT>
hipError_t launch_typed(const uint8_t* xc, const uint8_t* xs, const batq_weight* w, int M, YT* Y, int64_t ldy,
                        hipStream_t stream) {
    const int N = w->N, nb = w->nb;
    const bool fits32 = code_bytes_blocked(M, nb) < (1ull << 31) && code_bytes_blocked(N, nb) < (1ull << 31);
    if (M > 64 && fits32) {
        static bool attr_set = false;
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_tiled<YT>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, kTiledLds);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        const int tiles_m = (M + kTile - 1) / kTile, tiles_n = (N + kTile - 1) / kTile;
        gemm_tiled<YT><<<dim3(tiles_m * tiles_n), dim3(256), kTiledLds, stream>>>(xc, xs, w->d_codes, w->d_scales, M,
                                                                                   N, nb, tiles_m, tiles_n, Y, ldy);
    } else {
        const dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
        gemm_direct<YT><<<grid, block, 0, stream>>>(xc, xs, w->d_codes, w->d_scales, M, N, nb, Y, ldy);
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

hipError_t launch_gemm_mxfp4(const uint8_t* xcodes, const uint8_t* xscales_internal, const batq_weight* w, int M,
                             void* Y, batq_dtype ydtype, int64_t ldy, hipStream_t stream) {
    if (M == 0) return hipSuccess;
    if (ydtype == BATQ_BF16)
        return launch_typed<uint16_t>(xcodes, xscales_internal, w, M, static_cast<uint16_t*>(Y), ldy, stream);
    return launch_typed<float>(xcodes, xscales_internal, w, M, static_cast<float*>(Y), ldy, stream);
}

}  // namespace batq
