// Fused online activation path: block-wise affine transform (Eq. 1-2, Global-and-Private
// Kronecker factors), block clipping (Eq. 3-4, symmetric form) and MXFP4 quantisation
// (Sec. 2: E2M1 elements, one UE8M0 scale per 32).  gfx950 only.
//
// Two kernels.
//
// Matrix-core kernel (`quant_act_mfma`, bf16 input with a transform).  The 12 multiply-adds
// per element of the Kronecker route would make the kernel VALU-bound on this chip (packed
// fp32 arithmetic is not used), so the 32x32 block product runs on the matrix pipe instead,
// at fp32 accuracy: bf16 inputs are exact, and the fp32 entries of T_k are split on the host
// into three bf16 terms (hi + mid + lo = 24 significant bits), so every product is exact in
// the fp32 accumulator.  Per 32-row tile and MX block:
//   D (32 out-cols x 32 rows) = T_k^T (32 x 32) * X_tile^T (32 x 32), six 32x32x16 bf16
//   matrix instructions (3 terms x 2 K-halves).  The K order of the instruction is mapped
//   to input columns so that a lane's operand is 32 contiguous bytes of one row of X, and
//   the output rows of T_k^T are permuted so that a lane ends with 16 consecutive output
//   columns of one row: amax needs one cross-lane exchange, and the 16 codes are 8 bytes of
//   the block's 16-byte chunk.
// Persistent workgroups (one per compute unit): the workgroups that share a 256-element K group keep
// its transform operands in LDS and split its 32-row tiles; X arrives by LDS-direct loads, code
// pieces and scale bytes leave as whole cache lines (details at the kernel).
//
// Register-level kernel (`quant_act_quad`; fp32 input, or no transform).  One quad of lanes
// owns one 32-element block
// of one row: lane q of the quad holds the 8 contiguous elements 8q..8q+7.  The Kronecker structure T_k = G (x) P_k splits the 32x32 block product into
//   - a product with the factor that acts on the contiguous index, done in the lane's own
//     registers, and
//   - a mix across the four lanes of the quad with the other factor, done with DPP
//     quad broadcasts,
// which is the vec identity of Sec. 3.1.1 (12 multiply-adds per element instead of 32).
// The block amax is a two-step DPP reduction inside the quad.  Every lane then emits its
// 8 codes as one dword into the GEMM's blocked code layout; lane 0 of the quad stores the
// scale byte (grouped scale layout).
#include <algorithm>

#include "batq_internal.h"
#include "mxfp4_device.h"
#include "code_layout.h"
#include "scale_layout.h"

namespace batq {
namespace {

template <int CTRL>
__device__ __forceinline__ float dpp_quad(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

__device__ __forceinline__ void load8(const float* p, float (&x)[8]) {
    const float4 a = reinterpret_cast<const float4*>(p)[0];
    const float4 b = reinterpret_cast<const float4*>(p)[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

__device__ __forceinline__ void load8(const uint16_t* p, float (&x)[8]) {
    const uint4 a = *reinterpret_cast<const uint4*>(p);
    x[0] = __uint_as_float(a.x << 16); x[1] = __uint_as_float(a.x & 0xFFFF0000u);
    x[2] = __uint_as_float(a.y << 16); x[3] = __uint_as_float(a.y & 0xFFFF0000u);
    x[4] = __uint_as_float(a.z << 16); x[5] = __uint_as_float(a.z & 0xFFFF0000u);
    x[6] = __uint_as_float(a.w << 16); x[7] = __uint_as_float(a.w & 0xFFFF0000u);
}

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
// two bf16 pairs (gate, up) -> the bf16 pair of their gated products
__device__ __forceinline__ uint32_t swiglu_pair(uint32_t g2, uint32_t u2) {
    const f32x2 h = {swiglu_f32(__uint_as_float(g2 << 16), __uint_as_float(u2 << 16)),
                     swiglu_f32(__uint_as_float(g2 & 0xFFFF0000u), __uint_as_float(u2 & 0xFFFF0000u))};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(h, bf16x2v));
}
// register form for the kernels that hold fp32 copies: x <- bf16(silu(x) * u)
__device__ __forceinline__ void swiglu8(float (&x)[8], const float (&u)[8]) {
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
        const f32x2 h = {swiglu_f32(x[i], u[i]), swiglu_f32(x[i + 1], u[i + 1])};
        const uint32_t b = __builtin_bit_cast(uint32_t, __builtin_convertvector(h, bf16x2v));
        x[i] = __uint_as_float(b << 16);
        x[i + 1] = __uint_as_float(b & 0xFFFF0000u);
    }
}

// Mix across the quad: out = sum over source lanes s of coef[s] * (value held by lane s).
#define BATQ_QUAD_MIX(out, v, c0, c1, c2, c3)            \
    do {                                                  \
        out = (c0) * dpp_quad<0x00>(v);                   \
        out = __builtin_fmaf((c1), dpp_quad<0x55>(v), out); \
        out = __builtin_fmaf((c2), dpp_quad<0xAA>(v), out); \
        out = __builtin_fmaf((c3), dpp_quad<0xFF>(v), out); \
    } while (0)

// GO = size of the outer factor (4 or 8); the inner factor is (32/GO) x (32/GO).  Block k uses
// G + k * g_stride and P + k * p_stride (a stride of 0 = one factor shared by all blocks), which covers
// the Global-and-Private form, the order Eq. 2 prints (private outer, shared inner) and the naive
// Kronecker product (both private).  clip_max != null selects the two-ratio clipping of Eq. 3-4
// (clip then holds the ratios on the block minimum).
// FP8 selects MXFP8 (E4M3) output, one byte per element in the blocked 8-bit code layout.
// U != null: X is the gate and U the up tensor of a gated activation; the input is bf16(silu(X) * U).
template <typename XT, int GO, bool TRANSFORM, bool FP8>
__global__ void __launch_bounds__(256)
quant_act_quad(const XT* __restrict__ X, int64_t ldx, const XT* __restrict__ U, int64_t ldu, int M, int nb,
               int row0, int srows, int rows_per_wg,
               const float* __restrict__ G, int g_stride, const float* __restrict__ P, int p_stride,
               const float* __restrict__ clip, const float* __restrict__ clip_max,
               const float* __restrict__ row_scale, uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
    constexpr int GI = 32 / GO;
    const int q = threadIdx.x & 3;
    int k = blockIdx.x * 64 + (threadIdx.x >> 2);
    const bool live = k < nb;
    // padding blocks of the last 8-block scale group get the neutral scale
    const bool pad = !live && k < scale_groups(nb) * 8;
    const int kpad = k;
    if (!live) k = nb - 1;               // keep the whole quad running for the DPP exchanges

    // factors, held in registers across the row loop
    float Pr[GI * GI];
    float Gc[GO == 4 ? 4 : 16];
    if constexpr (TRANSFORM) {
#pragma unroll
        for (int i = 0; i < GI * GI; ++i) Pr[i] = P[(size_t)k * p_stride + i];
        G += (size_t)k * g_stride;
        if constexpr (GO == 4) {
            // lane q produces row a' = q of the mixed result: needs G[a][q], a = 0..3
#pragma unroll
            for (int a = 0; a < 4; ++a) Gc[a] = G[a * 4 + q];
        } else {
            // lane q produces rows a' = 2q + h': needs G[2s+h][2q+h'], index (s, h, h')
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2) Gc[s * 4 + h * 2 + h2] = G[(2 * s + h) * 8 + 2 * q + h2];
        }
    }
    const float ck = clip[k];
    const float ck_max = clip_max ? clip_max[k] : 0.f;

    const int row_begin = blockIdx.y * rows_per_wg;
    const int row_end = min(M, row_begin + rows_per_wg);
    for (int row = row_begin; row < row_end; ++row) {
        float x[8], y[8];
        load8(X + (size_t)row * ldx + (size_t)k * 32 + q * 8, x);
        if (U) {
            float u[8];
            load8(U + (size_t)row * ldu + (size_t)k * 32 + q * 8, u);
            swiglu8(x, u);
        }
        if constexpr (TRANSFORM) {
            float v[8];
            if constexpr (GO == 4) {
                // private 8x8 factor on the contiguous index, in registers
#pragma unroll
                for (int c2 = 0; c2 < 8; ++c2) {
                    float acc = x[0] * Pr[c2];
#pragma unroll
                    for (int c = 1; c < 8; ++c) acc = __builtin_fmaf(x[c], Pr[c * 8 + c2], acc);
                    v[c2] = acc;
                }
                // shared 4x4 factor across the quad
#pragma unroll
                for (int c2 = 0; c2 < 8; ++c2) BATQ_QUAD_MIX(y[c2], v[c2], Gc[0], Gc[1], Gc[2], Gc[3]);
            } else {
                // private 4x4 factor on each of the lane's two rows
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int c2 = 0; c2 < 4; ++c2) {
                        float acc = x[4 * h] * Pr[c2];
#pragma unroll
                        for (int c = 1; c < 4; ++c) acc = __builtin_fmaf(x[4 * h + c], Pr[c * 4 + c2], acc);
                        v[4 * h + c2] = acc;
                    }
                // shared 8x8 factor: 8 source rows live in 4 lanes x 2 registers
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                    for (int c2 = 0; c2 < 4; ++c2) {
                        float lo, hi;
                        BATQ_QUAD_MIX(lo, v[c2], Gc[0 + h2], Gc[4 + h2], Gc[8 + h2], Gc[12 + h2]);
                        BATQ_QUAD_MIX(hi, v[4 + c2], Gc[2 + h2], Gc[6 + h2], Gc[10 + h2], Gc[14 + h2]);
                        y[4 * h2 + c2] = lo + hi;
                    }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) y[i] = x[i];
        }

        if (row_scale) {
            // fused row scaling (e.g. RMSNorm's 1/rms): the transformed row times row_scale[row]
            const float rs = row_scale[row];
#pragma unroll
            for (int i = 0; i < 8; ++i) y[i] *= rs;
        }
        float bound;
        if (clip_max) {
            // Eq. 3-4 as printed: block minimum and maximum over the quad, clamp to [r_min min, r_max max];
            // the largest magnitude left is that of the clamped minimum or of the clamped maximum
            float mn = y[0], mx = y[0];
#pragma unroll
            for (int i = 1; i < 8; ++i) {
                mn = __builtin_fminf(mn, y[i]);
                mx = __builtin_fmaxf(mx, y[i]);
            }
            mn = __builtin_fminf(mn, dpp_quad<0xB1>(mn));
            mn = __builtin_fminf(mn, dpp_quad<0x4E>(mn));
            mx = __builtin_fmaxf(mx, dpp_quad<0xB1>(mx));
            mx = __builtin_fmaxf(mx, dpp_quad<0x4E>(mx));
            const float lo = ck * mn, hi = ck_max * mx;
#pragma unroll
            for (int i = 0; i < 8; ++i) y[i] = clamp_lo_hi(y[i], lo, hi);
            bound = __builtin_fmaxf(__builtin_fabsf(clamp_lo_hi(mn, lo, hi)), __builtin_fabsf(clamp_lo_hi(mx, lo, hi)));
        } else {
            // block amax over the quad's 32 values
            float m = __builtin_fabsf(y[0]);
#pragma unroll
            for (int i = 1; i < 8; ++i) m = __builtin_fmaxf(m, __builtin_fabsf(y[i]));
            m = __builtin_fmaxf(m, dpp_quad<0xB1>(m));
            m = __builtin_fmaxf(m, dpp_quad<0x4E>(m));
            bound = ck * m;                             // one fp32 multiply
        }
        if constexpr (FP8) {
            // the lane's 8 codes are bytes 8 (q % 2) .. + 7 of 16-byte slot q / 2 of the block
            const uint32_t s = e8m0_of_bound_fp8(bound);
            const uint2 packed = encode8_fp8(y, bound, s, scale_operand(s));
            if (live) {
                *reinterpret_cast<uint2*>(codes + code8_slot_offset(row0 + row, k, q >> 1, nb) + (q & 1) * 8) = packed;
                if (q == 0) scales[scale_index_internal(row0 + row, k, srows)] = (uint8_t)s;
            } else if (pad) {
                *reinterpret_cast<uint2*>(codes + code8_slot_offset(row0 + row, kpad, q >> 1, nb) + (q & 1) * 8) = uint2{0u, 0u};
                if (q == 0) scales[scale_index_internal(row0 + row, kpad, srows)] = (uint8_t)127;
            }
        } else {
            const uint32_t s = e8m0_of_bound(bound);
            const uint32_t packed = encode8(y, bound, scale_operand(s));
            if (live) {
                *reinterpret_cast<uint32_t*>(codes + code_chunk_offset(row0 + row, k, nb) + q * 4) = packed;
                if (q == 0) scales[scale_index_internal(row0 + row, k, srows)] = (uint8_t)s;
            } else if (pad) {
                // padding blocks up to the next multiple of 8: zero codes, neutral scale
                *reinterpret_cast<uint32_t*>(codes + code_chunk_offset(row0 + row, kpad, nb) + q * 4) = 0u;
                if (q == 0) scales[scale_index_internal(row0 + row, kpad, srows)] = (uint8_t)127;
            }
        }
    }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Lane layout of the pre-split transform operand (built by the host, see batq_api.hip):
//   Tsplit[k][term][half][lane] = 8 bf16: T_k[16 (lane / 32) + 8 half + e][sigma(lane % 32)], e = 0..7,
//   sigma(m) = 16 ((m >> 2) & 1) + 4 (m >> 3) + (m & 3); terms 0, 1, 2 = hi, mid, lo.
constexpr int kTsplitBlock = 3 * 2 * 64 * 16;               // bytes of pre-split transform operand per MX block
constexpr int kXSlot = 32 * 256;        // one unit of X: 32 rows x 128 bf16
constexpr int kQuantLdsT = 8 * kTsplitBlock;

// LDS plan of the persistent workgroup (one per compute unit): transform operands of one K group, then per
// wave one X slot and the staging area for the code pieces of a unit (two 1 KiB pieces for 4-bit codes,
// four for 8-bit codes), then the unit counter.  8 waves: 64 KiB of X in flight per compute unit saturate the
// stream, and more waves only lengthen the last round of units (10 waves measured 5 % slower on cfg2, 1 % on
// cfg3 and cfg4).  With a gated input a wave's slot holds the unit of the gate and the unit of the up tensor
// (6 and 5 waves, about the same bytes in flight).
template <bool FP8, bool SWIGLU>
struct QuantPlan {
    static constexpr int kWaves = SWIGLU ? (FP8 ? 5 : 6) : 8;
    static constexpr int kSlot = SWIGLU ? 2 * kXSlot : kXSlot;
    static constexpr int kCodeStage = FP8 ? 4096 : 2048;
    static constexpr int kLdsX = kQuantLdsT;
    static constexpr int kLdsStage = kLdsX + kWaves * kSlot;
    static constexpr int kLdsCounter = kLdsStage + kWaves * kCodeStage;
    static constexpr int kLds = kLdsCounter + 16;           // 128 KiB / 144 KiB (gated: 156 KiB / 148 KiB)
};

// Persistent kernel.  Work comes in units of (32-row tile, half K group = 4 MX blocks = 256 bytes per
// row).  `wpg` workgroups share a K group and split its row tiles evenly, so a workgroup fetches the
// group's transform operands (48 KiB, kept in LDS) exactly once; its waves draw units from an LDS
// counter.  A wave's unit of X is fetched global -> LDS with LDS-direct loads (no registers are tied up
// while it is in flight), as rows of 16 chunks of 16 bytes, chunk c of row r at position c ^ (r & 7) so
// that the operand reads (all lanes the same chunk, 32 different rows) spread over the banks.  As soon
// as the unit is in registers the next one is requested into the same slot; the code pieces and scale
// bytes of a unit are written out one unit late, so that nothing waits on a store that was just issued
// (loads and stores share one completion counter).
// MINMAX selects the two-ratio clipping of Eq. 3-4 (clip = ratios on the block minimum, clip_max on the
// maximum) instead of one ratio on the block amax.
// FP8 selects MXFP8 (E4M3) output in the blocked 8-bit code layout (a unit then fills four pieces:
// two piece columns of 2 blocks each, times two 16-row groups).
// SWIGLU: X is the gate and U the up tensor of a gated activation; both units are fetched, and the operand
// the matrix pipe sees is bf16(silu(X) * U), formed in registers.
template <bool MINMAX, bool FP8, bool SWIGLU>
__global__ void __launch_bounds__((QuantPlan<FP8, SWIGLU>::kWaves * 64))
quant_act_mfma(const uint16_t* __restrict__ X, int64_t ldx, const uint16_t* __restrict__ U, int64_t ldu, int M,
               int nb, int srows, int wpg,
               const uint4* __restrict__ Tsplit, const float* __restrict__ outer, int outer_stride,
               const float* __restrict__ inner, int inner_stride, int gshift,
               const float* __restrict__ clip, const float* __restrict__ clip_max,
               const float* __restrict__ row_scale, uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
    extern __shared__ __align__(16) uint8_t qlds[];
    typedef __attribute__((address_space(3))) uint8_t lds_byte;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kg = lane >> 5;
    const int row_tiles = (M + 31) >> 5;
    const int groups = scale_groups(nb);
    using Plan = QuantPlan<FP8, SWIGLU>;
    constexpr int kQuantWaves = Plan::kWaves;
    const size_t piece_stride = (size_t)(FP8 ? code8_stages(nb) : code_stages(nb)) * 1024;

    uint8_t* const tlds = qlds;
    uint8_t* const xslot = qlds + Plan::kLdsX + wave * Plan::kSlot;
    uint8_t* const my = qlds + Plan::kLdsStage + wave * Plan::kCodeStage;
    uint32_t* const counter = reinterpret_cast<uint32_t*>(qlds + Plan::kLdsCounter);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_byte*)qlds;
    const uint32_t xslot_lds = lds_base + Plan::kLdsX + wave * Plan::kSlot;

    // `wpg` workgroups share a K group, each taking an equal range of its row tiles; with more groups
    // than workgroups (wpg = 1) a workgroup takes every (gridDim.x)-th group
    const int part = blockIdx.x % wpg;
    const int t_begin = (int)((int64_t)row_tiles * part / wpg), t_end = (int)((int64_t)row_tiles * (part + 1) / wpg);
    const int u_end = 2 * t_end;                            // units of a group: u = 2 tile + half
    auto grab = [&]() -> int {
        int v = 0;
        if (lane == 0) v = (int)__hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        return __builtin_amdgcn_readfirstlane(v);
    };
    auto request = [&](int g, int u) -> bool {              // false: nothing to fetch (a half group of padding)
        const int tile = u >> 1, half = u & 1;
        const int kb = 8 * g + 4 * half;                    // first MX block of the unit
        const int nreal = min(4, nb - kb);                  // blocks that exist (the rest of the group is padding)
        if (nreal <= 0) return false;
        const uint8_t* base = reinterpret_cast<const uint8_t*>(X) + ((size_t)tile * 32 * ldx + (size_t)kb * 32) * 2;
        const uint8_t* ubase =
            SWIGLU ? reinterpret_cast<const uint8_t*>(U) + ((size_t)tile * 32 * ldu + (size_t)kb * 32) * 2 : nullptr;
        const int rows_left = M - 1 - tile * 32;            // rows past the end repeat the last one: computed, not stored
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = 4 * j + (lane >> 4);
            int c = (lane & 15) ^ (r & 7);                  // the chunk that belongs at this lane's LDS position
            if (c >= 4 * nreal) c = 0;                      // never read past the end of the row
            const uint32_t voff = (uint32_t)min(r, rows_left) * (uint32_t)(ldx * 2) + (uint32_t)c * 16;
            // X is read exactly once: non-temporal, so it does not push the transform operands or
            // the pending output lines out of the L2
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                         :: "v"(voff), "s"(base), "s"(xslot_lds + (uint32_t)j * 1024) : "memory");
            if constexpr (SWIGLU) {
                const uint32_t uoff = (uint32_t)min(r, rows_left) * (uint32_t)(ldu * 2) + (uint32_t)c * 16;
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                             :: "v"(uoff), "s"(ubase), "s"(xslot_lds + (uint32_t)(kXSlot + j * 1024)) : "memory");
            }
        }
        return true;
    };

    const int r16 = l32 & 15;
    // this lane's row inside the staging area [piece column][row group][1 KiB]
    const int st_row = (l32 >> 4) * 1024 + r16 * 64;
    const int st_swz = (r16 >> 2) & 3;

    // stores of the unit finished last
    int pend_u = -1, pend_g = 0;
    uint32_t pend_sc = 0;
    auto flush = [&]() {
        if (pend_u < 0) return;
        const int tile = pend_u >> 1, half = pend_u & 1;
        // pieces (piece column pc of the unit, rows 0-15) and (pc, rows 16-31); the code array is padded to
        // whole 32-row tiles, so all of them exist.  Streamed out past the caches' keep-lists: nothing in
        // this kernel reads them again.
        constexpr int kCols = FP8 ? 2 : 1;                  // piece columns per unit
#pragma unroll
        for (int pc = 0; pc < kCols; ++pc)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const u32x4 v = *reinterpret_cast<const u32x4*>(my + (pc * 2 + p) * 1024 + lane * 16);
                __builtin_nontemporal_store(
                    v, reinterpret_cast<u32x4*>(codes + (size_t)(2 * tile + p) * piece_stride +
                                                (size_t)(kCols * (2 * pend_g + half) + pc) * 1024 + lane * 16));
            }
        // the unit's four scale bytes of the row's 8-byte word: even blocks at 2 half, 2 half + 1,
        // odd blocks at 4 + 2 half, 4 + 2 half + 1; lane kg writes pair kg
        const int row = tile * 32 + l32;
        if (row < M)
            *reinterpret_cast<uint16_t*>(scales + ((size_t)pend_g * srows + row) * 8 + 4 * kg + 2 * half) = (uint16_t)pend_sc;
        pend_u = -1;
    };

    for (int g = blockIdx.x / wpg; g < groups; g += gridDim.x / wpg) {
        const int k0 = g * 8;
        const int nblk = min(8, nb - k0);                   // real blocks in this group
        __syncthreads();                                    // every wave is done with the previous group's operands
        // the first units go to the waves by number (no barrier and no draw in front of a launch's first request: they
        // cost 0.5 us), the rest are drawn from the counter, which is set by the barrier below
        if (tid == 0) *counter = (uint32_t)(2 * t_begin + kQuantWaves);
        if (gshift) {
            // Kronecker form: only the factors are fetched (outer and inner factor of block k0 + kb, 320 bytes, by
            // wave kb % waves into its code staging area, which the flush leaves free), and the workgroup forms the
            // blocks' split operands itself below
            flush();
            const int go = 32 >> gshift, gi = 1 << gshift;
            for (int kb = wave; kb < nblk; kb += kQuantWaves) {
                const uint32_t dst = lds_base + Plan::kLdsStage + wave * Plan::kCodeStage + (kb / kQuantWaves) * 512;
                const float* ob = outer + (size_t)(k0 + kb) * outer_stride;
                const float* ib = inner + (size_t)(k0 + kb) * inner_stride;
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                             :: "v"((uint32_t)min(lane, go * go - 1) * 4u), "s"(ob), "s"(dst) : "memory");
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                             :: "v"((uint32_t)min(lane, gi * gi - 1) * 4u), "s"(ib), "s"(dst + 256) : "memory");
            }
        } else {
            // the group's transform operands go global -> LDS with LDS-direct loads (1 KiB per wave
            // instruction, lane i -> LDS base + 16 i)
            const uint8_t* src = reinterpret_cast<const uint8_t*>(Tsplit) + (size_t)k0 * kTsplitBlock;
            const int pieces = nblk * (kTsplitBlock / 1024);   // 6 per block
            for (int p = wave; p < pieces; p += kQuantWaves)
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                             :: "v"((uint32_t)(p * 1024 + lane * 16)), "s"(src), "s"(lds_base + (uint32_t)p * 1024) : "memory");
        }
        int my_u = 2 * t_begin + wave;
        // this wave's share of the operands has landed once only the unit's loads (8, or 16 with a gated input;
        // loads complete in order) are still out: the workgroup does not wait for everybody's first unit
        if (my_u < u_end && request(g, my_u)) __builtin_amdgcn_s_waitcnt(SWIGLU ? 0x4F70 : 0x0F78);     // vmcnt(16) : vmcnt(8)
        else __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0)
        __syncthreads();                                    // all operands have landed, the counter is set
        if (gshift) {
            // T_k = outer (x) inner, element by element the exact product of the two fp32 factors, split into three
            // bf16 terms (each the remainder rounded to fp32, then to bf16, nearest even) in the operand's lane order:
            // bit for bit what the host writes into the pre-split array (from the fp64 product), at 320 instead of
            // 6144 bytes fetched per block, while the first units' rows are on their way
            const int go = 32 >> gshift, gi = 1 << gshift;
            for (int item = tid; item < nblk * 128; item += kQuantWaves * 64) {
                const int kb = item >> 7, hf = (item >> 6) & 1, ln = item & 63;
                const float* fo = reinterpret_cast<const float*>(qlds + Plan::kLdsStage + (kb % kQuantWaves) * Plan::kCodeStage +
                                                                 (kb / kQuantWaves) * 512);
                const float* fi = fo + 64;
                const int m = ln & 31;
                const int oc = 16 * ((m >> 2) & 1) + 4 * (m >> 3) + (m & 3);
                const int a2 = oc >> gshift, c2 = oc & (gi - 1);
                const int in0 = 16 * (ln >> 5) + 8 * hf;
                uint32_t w[3][4];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int ic = in0 + e, a = ic >> gshift, c = ic & (gi - 1);
                    // p = o * i exactly = h + l (h the rounded product, l its error, from a fused multiply-add); the
                    // terms are b0 = bf16(h), b1 = bf16(fl(p - b0)), b2 = bf16(fl(p - b0 - b1)), where h - b0 and
                    // (h - b0) - b1 are exact in fp32 and one addition of l rounds each remainder correctly
                    const float o = fo[a * go + a2], iv = fi[c * gi + c2];
                    float h = o * iv;
                    asm volatile("" : "+v"(h));             // the rounded product itself: not to be fused into what follows
                    const float l = __builtin_fmaf(o, iv, -h);
                    uint32_t b[3];
                    b[0] = float_to_bf16_bits(h);
                    const float d0 = h - bf16_bits_to_float(b[0]);
                    b[1] = float_to_bf16_bits(d0 + l);
                    const float d1 = d0 - bf16_bits_to_float(b[1]);
                    b[2] = float_to_bf16_bits(d1 + l);
#pragma unroll
                    for (int term = 0; term < 3; ++term) {
                        if (e & 1) w[term][e >> 1] |= b[term] << 16;
                        else w[term][e >> 1] = b[term];
                    }
                }
#pragma unroll
                for (int term = 0; term < 3; ++term)
                    *reinterpret_cast<uint4*>(tlds + kb * kTsplitBlock + ((term * 2 + hf) * 64 + ln) * 16) =
                        uint4{w[term][0], w[term][1], w[term][2], w[term][3]};
            }
            __syncthreads();                                // the operands are complete, the staging areas free again
        }

        while (my_u < u_end) {
            const int u = my_u;
            const int half = u & 1;
            const int nreal = min(4, nb - (k0 + 4 * half));
            __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0): the unit has landed (older stores are long done)
            u32x4 x[4][2] = {};
            u32x4 up[SWIGLU ? 4 : 1][2] = {};
            if (nreal > 0) {
#pragma unroll
                for (int bb = 0; bb < 4; ++bb)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int c = 4 * bb + 2 * kg + h;
                        const int at = l32 * 256 + (((c & 8) | ((c ^ l32) & 7)) << 4);
                        x[bb][h] = *reinterpret_cast<const u32x4*>(xslot + at);
                        if constexpr (SWIGLU) up[bb][h] = *reinterpret_cast<const u32x4*>(xslot + kXSlot + at);
                    }
                // the slot is refilled next: its contents must be in registers first
#pragma unroll
                for (int bb = 0; bb < 4; ++bb)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        asm volatile("" : "+v"(x[bb][h]));
                        if constexpr (SWIGLU) asm volatile("" : "+v"(up[bb][h]));
                    }
            }
            my_u = grab();
            if (my_u < u_end) request(g, my_u);
            flush();
            if constexpr (SWIGLU) {
                if (nreal > 0) {
#pragma unroll
                    for (int bb = 0; bb < 4; ++bb)
#pragma unroll
                        for (int h = 0; h < 2; ++h)
#pragma unroll
                            for (int i = 0; i < 4; ++i) x[bb][h][i] = swiglu_pair(x[bb][h][i], up[bb][h][i]);
                }
            }

            // fused row scaling (e.g. RMSNorm's 1/rms): this lane's row of the tile
            const float rs = row_scale ? row_scale[min((u >> 1) * 32 + l32, M - 1)] : 1.0f;
            uint32_t sc4[4] = {127u, 127u, 127u, 127u};    // padding blocks keep the neutral scale
            // Quantisation of block bb of the unit in two steps, so that the four blocks of a unit can go through
            // each step together (the cross-lane exchange in between has a long latency).
            // Step 1: y = the transformed values (acc: element 16 kg + r of this lane's row, times the row
            // factor); returns this lane's partial extrema (amax in `a`, or minimum and maximum in `a`, `b2`).
            auto block_extrema = [&](const v16f& acc, float (&y)[16], float& a, float& b2) {
#pragma unroll
                for (int r = 0; r < 16; ++r) y[r] = acc[r];
                if (row_scale) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) y[r] *= rs;
                }
                if constexpr (MINMAX) {
                    a = y[0];
                    b2 = y[0];
#pragma unroll
                    for (int r = 1; r < 16; ++r) {
                        a = __builtin_fminf(a, y[r]);
                        b2 = __builtin_fmaxf(b2, y[r]);
                    }
                } else {
                    a = __builtin_fabsf(y[0]);
#pragma unroll
                    for (int r = 1; r < 16; ++r) a = __builtin_fmaxf(a, __builtin_fabsf(y[r]));
                    b2 = 0.f;
                }
            };
            // the other half of the block lives in lane ^ 32
            auto other_half = [&](float v) -> float {
                return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __builtin_bit_cast(int, v)));
            };
            // Step 2: block extrema (own and the other half's) -> clip, scale, codes into the staging area;
            // sc4[bb] = the block's scale byte.
            auto block_finish = [&](int bb, float (&y)[16], float a, float b2, float oa, float ob) {
                const int b = 4 * half + bb;                // block inside the K group
                float bound;
                if constexpr (MINMAX) {
                    const float mn = __builtin_fminf(a, oa), mx = __builtin_fmaxf(b2, ob);
                    const float lo = clip[k0 + b] * mn, hi = clip_max[k0 + b] * mx;
#pragma unroll
                    for (int r = 0; r < 16; ++r) y[r] = clamp_lo_hi(y[r], lo, hi);
                    // the largest magnitude left is that of the clamped minimum or of the clamped maximum
                    bound = __builtin_fmaxf(__builtin_fabsf(clamp_lo_hi(mn, lo, hi)),
                                            __builtin_fabsf(clamp_lo_hi(mx, lo, hi)));
                } else {
                    bound = clip[k0 + b] * __builtin_fmaxf(a, oa);      // one fp32 multiply
                }
                if constexpr (FP8) {
                    const uint32_t sb = e8m0_of_bound_fp8(bound);
                    const float sc = scale_operand(sb);
                    const uint2 out = encode8_fp8(y, bound, sb, sc), out2 = encode8_fp8(y + 8, bound, sb, sc);
                    sc4[bb] = sb;
                    // the lane's 16 codes are 16-byte slot 2 (bb % 2) + kg of its row in piece column bb / 2
                    *reinterpret_cast<uint4*>(my + (bb >> 1) * 2048 + st_row + (((2 * (bb & 1) + kg) ^ st_swz) << 4)) =
                        uint4{out.x, out.y, out2.x, out2.y};
                } else {
                    const uint32_t sb = e8m0_of_bound(bound);
                    const float sc = scale_operand(sb);
                    uint2 out;
                    out.x = encode8(y, bound, sc);
                    out.y = encode8(y + 8, bound, sc);
                    sc4[bb] = sb;
                    *reinterpret_cast<uint2*>(my + st_row + 8 * kg + ((bb ^ st_swz) << 4)) = out;
                }
            };
            auto quantise_block = [&](int bb, const v16f& acc) {
                float y[16], a, b2;
                block_extrema(acc, y, a, b2);
                const float oa = other_half(a), ob = MINMAX ? other_half(b2) : 0.f;
                block_finish(bb, y, a, b2, oa, ob);
            };
            auto zero_block = [&](int bb) {                 // padding block: zero codes
                if constexpr (FP8)
                    *reinterpret_cast<uint4*>(my + (bb >> 1) * 2048 + st_row + (((2 * (bb & 1) + kg) ^ st_swz) << 4)) =
                        uint4{0u, 0u, 0u, 0u};
                else
                    *reinterpret_cast<uint2*>(my + st_row + 8 * kg + ((bb ^ st_swz) << 4)) = uint2{0u, 0u};
            };
            if (nreal == 4) {
                // All four blocks at once: the 24 operand reads go out together, and the four accumulation
                // chains (3 terms x 2 K halves each, smallest terms first) are interleaved, so that neither the
                // LDS latency nor the latency of a matrix instruction's result is waited for block by block.
                uint4 tfr[4][6];
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) {
                    const uint4* tf = reinterpret_cast<const uint4*>(tlds + (4 * half + bb) * kTsplitBlock) + lane;
#pragma unroll
                    for (int i = 0; i < 6; ++i) tfr[bb][i] = tf[i * 64];
                }
                __builtin_amdgcn_sched_barrier(0);          // all 24 reads are issued before the first product
                v16f acc[4] = {};
#pragma unroll
                for (int t = 2; t >= 0; --t)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int bb = 0; bb < 4; ++bb)
                            acc[bb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tfr[bb][t * 2 + h]),
                                                                          __builtin_bit_cast(bf16x8, x[bb][h]), acc[bb], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                float y[4][16], a[4], b2[4], oa[4], ob[4];
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) block_extrema(acc[bb], y[bb], a[bb], b2[bb]);
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) {
                    oa[bb] = other_half(a[bb]);
                    ob[bb] = MINMAX ? other_half(b2[bb]) : 0.f;
                }
                __builtin_amdgcn_sched_barrier(0);          // the four exchanges are in flight together
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) block_finish(bb, y[bb], a[bb], b2[bb], oa[bb], ob[bb]);
            } else {
                // last, partly padded half group: block by block
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) {
                    if (bb < nreal) {
                        const uint4* tf = reinterpret_cast<const uint4*>(tlds + (4 * half + bb) * kTsplitBlock) + lane;
                        v16f acc = {};
#pragma unroll
                        for (int t = 2; t >= 0; --t)
#pragma unroll
                            for (int h = 0; h < 2; ++h)
                                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tf[(t * 2 + h) * 64]),
                                                                          __builtin_bit_cast(bf16x8, x[bb][h]), acc, 0, 0, 0);
                        quantise_block(bb, acc);
                    } else {
                        zero_block(bb);
                    }
                }
            }
            pend_u = u;
            pend_g = g;
            pend_sc = kg == 0 ? (sc4[0] | (sc4[2] << 8)) : (sc4[1] | (sc4[3] << 8));
        }
    }
    flush();
}

// The same arithmetic for few rows, and for rows that do not start on a 32-row tile of the destination (cache
// appends): one wave per (32-row tile of the call, MX block), operands straight from global memory into registers
// (no workgroup set-up, no LDS staging: with few rows that would cost more than the rows), codes and scale bytes
// stored row by row at any destination row.  Every floating-point step - the six matrix instructions of a block
// in the same order on the same pre-split operand, the row factor, the block extrema, the bound, the clamp and the
// convert - is the one quant_act_mfma takes, so a row gets the same codes and scale whichever of the two kernels
// quantises it, in whatever batch it arrives.
template <bool MINMAX, bool FP8, bool SWIGLU>
__global__ void __launch_bounds__(256)
quant_act_mfma_rows(const uint16_t* __restrict__ X, int64_t ldx, const uint16_t* __restrict__ U, int64_t ldu, int M,
                    int nb, int row0, int srows, const uint4* __restrict__ Tsplit, const float* __restrict__ clip,
                    const float* __restrict__ clip_max, const float* __restrict__ row_scale,
                    uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, kg = lane >> 5;
    const int nbp = scale_groups(nb) * 8;                   // blocks of a row, the padding of the last K group included
    const int tiles = (M + 31) >> 5;
    const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (unit >= tiles * nbp) return;                        // wave-uniform
    const int tile = unit / nbp, k = unit - tile * nbp;
    const int row = tile * 32 + l32;
    const bool live = row < M;
    const int drow = row0 + row;                            // destination row in arrays laid out for srows rows
    if (k >= nb) {
        // padding block: zero codes, neutral scale
        if (live) {
            if constexpr (FP8)
                *reinterpret_cast<uint4*>(codes + code8_slot_offset(drow, k, kg, nb)) = uint4{0u, 0u, 0u, 0u};
            else
                *reinterpret_cast<uint2*>(codes + code_chunk_offset(drow, k, nb) + 8 * kg) = uint2{0u, 0u};
            if (kg == 0) scales[scale_index_internal(drow, k, srows)] = (uint8_t)127;
        }
        return;
    }
    const int rr = min(row, M - 1);                         // rows past the end repeat the last one: computed, not stored
    // this lane's operand: elements 16 kg + 8 h .. + 7 of block k of its row
    const uint16_t* xp = X + (size_t)rr * ldx + (size_t)k * 32 + 16 * kg;
    u32x4 x[2], up[2] = {};
    x[0] = *reinterpret_cast<const u32x4*>(xp);
    x[1] = *reinterpret_cast<const u32x4*>(xp + 8);
    if constexpr (SWIGLU) {
        const uint16_t* upp = U + (size_t)rr * ldu + (size_t)k * 32 + 16 * kg;
        up[0] = *reinterpret_cast<const u32x4*>(upp);
        up[1] = *reinterpret_cast<const u32x4*>(upp + 8);
    }
    const uint4* tf = Tsplit + (size_t)k * (kTsplitBlock / 16) + lane;
    uint4 tfr[6];
#pragma unroll
    for (int i = 0; i < 6; ++i) tfr[i] = tf[i * 64];
    const float rs = row_scale ? row_scale[rr] : 1.0f;
    if constexpr (SWIGLU) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) x[h][i] = swiglu_pair(x[h][i], up[h][i]);
    }
    v16f acc = {};
#pragma unroll
    for (int t = 2; t >= 0; --t)
#pragma unroll
        for (int h = 0; h < 2; ++h)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tfr[t * 2 + h]),
                                                          __builtin_bit_cast(bf16x8, x[h]), acc, 0, 0, 0);
    float y[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) y[r] = acc[r];
    if (row_scale) {
#pragma unroll
        for (int r = 0; r < 16; ++r) y[r] *= rs;
    }
    auto other_half = [&](float v) -> float {
        return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __builtin_bit_cast(int, v)));
    };
    float bound;
    if constexpr (MINMAX) {
        float mn = y[0], mx = y[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) {
            mn = __builtin_fminf(mn, y[r]);
            mx = __builtin_fmaxf(mx, y[r]);
        }
        mn = __builtin_fminf(mn, other_half(mn));
        mx = __builtin_fmaxf(mx, other_half(mx));
        const float lo = clip[k] * mn, hi = clip_max[k] * mx;
#pragma unroll
        for (int r = 0; r < 16; ++r) y[r] = clamp_lo_hi(y[r], lo, hi);
        bound = __builtin_fmaxf(__builtin_fabsf(clamp_lo_hi(mn, lo, hi)), __builtin_fabsf(clamp_lo_hi(mx, lo, hi)));
    } else {
        float a = __builtin_fabsf(y[0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) a = __builtin_fmaxf(a, __builtin_fabsf(y[r]));
        bound = clip[k] * __builtin_fmaxf(a, other_half(a));    // one fp32 multiply
    }
    if constexpr (FP8) {
        const uint32_t sb = e8m0_of_bound_fp8(bound);
        const float sc = scale_operand(sb);
        const uint2 o0 = encode8_fp8(y, bound, sb, sc), o1 = encode8_fp8(y + 8, bound, sb, sc);
        if (live) {
            *reinterpret_cast<uint4*>(codes + code8_slot_offset(drow, k, kg, nb)) = uint4{o0.x, o0.y, o1.x, o1.y};
            if (kg == 0) scales[scale_index_internal(drow, k, srows)] = (uint8_t)sb;
        }
    } else {
        const uint32_t sb = e8m0_of_bound(bound);
        const float sc = scale_operand(sb);
        uint2 out;
        out.x = encode8(y, bound, sc);
        out.y = encode8(y + 8, bound, sc);
        if (live) {
            *reinterpret_cast<uint2*>(codes + code_chunk_offset(drow, k, nb) + 8 * kg) = out;
            if (kg == 0) scales[scale_index_internal(drow, k, srows)] = (uint8_t)sb;
        }
    }
}

// Destination rows of a call: the code and scale arrays are laid out for `srows` rows, and the M rows of X go to
// rows row0 .. row0 + M - 1 (a plain call: row0 = 0, srows = M).
struct RowWindow {
    int row0, srows;
};

template <bool MINMAX, bool FP8, bool SWIGLU>
hipError_t launch_mfma_as(const batq_transform* t, const uint16_t* X, int M, int64_t ldx, const uint16_t* U,
                          int64_t ldu, const float* row_scale, uint8_t* codes, uint8_t* scales, RowWindow win, int dev,
                          int cus, hipStream_t stream) {
    using Plan = QuantPlan<FP8, SWIGLU>;
    if (hipError_t e = ensure_dynamic_lds<&quant_act_mfma<MINMAX, FP8, SWIGLU>>(dev, Plan::kLds); e != hipSuccess) return e;
    // whole K groups per workgroup set: floor(compute units / groups) workgroups share a group
    const int nb = t->nb;
    const int groups = scale_groups(nb), row_tiles = (M + 31) / 32;
    const int wpg = std::max(1, std::min(cus / groups, row_tiles));
    const int wgs = wpg * std::min(groups, cus);
    // Kronecker forms: a workgroup can form the split operands of its K group from the factors (320 bytes fetched per
    // block) instead of fetching them (6 KiB per block, which every XCD pulls into its L2 once and every workgroup
    // into its LDS).  Forming them takes a workgroup ~1 us before its first unit, so it pays where a wave has three
    // or more units to work through (kernel trace, fetching -> forming: 4096 x 14336 28-33 -> 29 us and 128.7 ->
    // 118.2 MB fetched for 117.4 MB of input, 8192 x 3584 18.8 -> 18.0 us; 2048 x 4096, one unit per wave: 8.0 -> 9.1 us,
    // so that shape keeps fetching).  The bits of the operands, and so of the output, are the same either way.
    const int units_per_wg = 2 * ((row_tiles + wpg - 1) / wpg);
    const bool build_operands = t->form == BATQ_FORM_KRON && units_per_wg >= 3 * Plan::kWaves;
    // the window starts on a 32-row tile (the caller checks): whole 16-row code groups and 8-byte scale rows in
    const size_t code_group = (size_t)(FP8 ? code8_stages(nb) : code_stages(nb)) * 1024;
    quant_act_mfma<MINMAX, FP8, SWIGLU><<<dim3(wgs), dim3(Plan::kWaves * 64), Plan::kLds, stream>>>(
        X, ldx, U, ldu, M, nb, win.srows, wpg, reinterpret_cast<const uint4*>(t->d_Tsplit), t->d_outer, t->outer_stride,
        t->d_inner, t->inner_stride, build_operands ? (t->g_inner == 8 ? 3 : 2) : 0, t->d_clip,
        MINMAX ? t->d_clip_max : nullptr, row_scale, codes + (size_t)(win.row0 >> 4) * code_group,
        scales + (size_t)win.row0 * 8);
    return hipGetLastError();
}

template <bool SWIGLU>
hipError_t launch_mfma(const batq_transform* t, const uint16_t* X, int M, int64_t ldx, const uint16_t* U, int64_t ldu,
                       const float* row_scale, uint8_t* codes, uint8_t* scales, RowWindow win, bool fp8,
                       hipStream_t stream) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const int cus = device_compute_units(dev, &e);
    if (e != hipSuccess) return e;
    if (fp8)
        return t->minmax
                   ? launch_mfma_as<true, true, SWIGLU>(t, X, M, ldx, U, ldu, row_scale, codes, scales, win, dev, cus, stream)
                   : launch_mfma_as<false, true, SWIGLU>(t, X, M, ldx, U, ldu, row_scale, codes, scales, win, dev, cus, stream);
    return t->minmax
               ? launch_mfma_as<true, false, SWIGLU>(t, X, M, ldx, U, ldu, row_scale, codes, scales, win, dev, cus, stream)
               : launch_mfma_as<false, false, SWIGLU>(t, X, M, ldx, U, ldu, row_scale, codes, scales, win, dev, cus, stream);
}

template <bool SWIGLU>
hipError_t launch_mfma_rows(const batq_transform* t, const uint16_t* X, int M, int64_t ldx, const uint16_t* U, int64_t ldu,
                            const float* row_scale, uint8_t* codes, uint8_t* scales, RowWindow win, bool fp8,
                            hipStream_t stream) {
    const int nb = t->nb;
    const int64_t units = (int64_t)((M + 31) / 32) * scale_groups(nb) * 8;
    const dim3 grid((unsigned)((units + 3) / 4)), block(256);
    const uint4* ts = reinterpret_cast<const uint4*>(t->d_Tsplit);
    const float* cmax = t->minmax ? t->d_clip_max : nullptr;
#define BATQ_ROWS(MM, F8)                                                                                              \
    quant_act_mfma_rows<MM, F8, SWIGLU><<<grid, block, 0, stream>>>(X, ldx, U, ldu, M, nb, win.row0, win.srows, ts,    \
                                                                     t->d_clip, cmax, row_scale, codes, scales)
    if (fp8) {
        if (t->minmax) BATQ_ROWS(true, true);
        else BATQ_ROWS(false, true);
    } else {
        if (t->minmax) BATQ_ROWS(true, false);
        else BATQ_ROWS(false, false);
    }
#undef BATQ_ROWS
    return hipGetLastError();
}

template <typename XT, bool FP8>
hipError_t launch_quad(const batq_transform* t, const XT* X, int M, int64_t ldx, const XT* U, int64_t ldu,
                       const float* row_scale, uint8_t* codes, uint8_t* scales, RowWindow win, hipStream_t stream) {
    const int nb = t->nb;
    const int gx = (scale_groups(nb) * 8 + 63) / 64;
    // aim at >= 4 workgroups per CU while keeping the per-lane factor loads amortised
    int rows_per_wg = 16;
    while (rows_per_wg > 1 && (long)gx * ((M + rows_per_wg - 1) / rows_per_wg) < 2048) rows_per_wg >>= 1;
    while ((M + rows_per_wg - 1) / rows_per_wg > 65535) rows_per_wg <<= 1;      // grid.y limit
    const dim3 grid(gx, (M + rows_per_wg - 1) / rows_per_wg), block(256);
    const float* cmax = t->minmax ? t->d_clip_max : nullptr;
    if (!t->has_transform)
        quant_act_quad<XT, 4, false, FP8><<<grid, block, 0, stream>>>(X, ldx, U, ldu, M, nb, win.row0, win.srows, rows_per_wg, nullptr, 0, nullptr,
                                                                       0, t->d_clip, cmax, row_scale, codes, scales);
    else if (t->g_outer == 4)
        quant_act_quad<XT, 4, true, FP8><<<grid, block, 0, stream>>>(X, ldx, U, ldu, M, nb, win.row0, win.srows, rows_per_wg, t->d_outer,
                                                                      t->outer_stride, t->d_inner, t->inner_stride,
                                                                      t->d_clip, cmax, row_scale, codes, scales);
    else
        quant_act_quad<XT, 8, true, FP8><<<grid, block, 0, stream>>>(X, ldx, U, ldu, M, nb, win.row0, win.srows, rows_per_wg, t->d_outer,
                                                                      t->outer_stride, t->d_inner, t->inner_stride,
                                                                      t->d_clip, cmax, row_scale, codes, scales);
    return hipGetLastError();
}

// Dense 32x32 block per MX block with fp32 input (the form Sec. 3.1.1 calls the dense P_i): one thread
// per (row, block); T_k (fp32, 4 KiB) sits in LDS, the 32 products of an output element are
// accumulated with fp32 fused multiply-adds in input order.  Not a tuned path: bf16 inputs of every
// form take the matrix-core kernel.
template <typename XT, bool FP8>
__global__ void __launch_bounds__(256)
quant_act_dense(const XT* __restrict__ X, int64_t ldx, const XT* __restrict__ U, int64_t ldu, int M, int nb,
                int row0, int srows, const float* __restrict__ T,
                const float* __restrict__ clip, const float* __restrict__ clip_max,
                const float* __restrict__ row_scale, uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
    __shared__ float sT[32 * 32];
    const int k = blockIdx.x;                               // includes the padding blocks of the last K group
    const bool live = k < nb;
    if (live)
        for (int i = threadIdx.x; i < 1024; i += 256) sT[i] = T[(size_t)k * 1024 + i];
    __syncthreads();
    const int row = blockIdx.y * 256 + threadIdx.x;
    if (row >= M) return;
    if (!live) {
        if constexpr (FP8) {
            *reinterpret_cast<uint4*>(codes + code8_slot_offset(row0 + row, k, 0, nb)) = uint4{0u, 0u, 0u, 0u};
            *reinterpret_cast<uint4*>(codes + code8_slot_offset(row0 + row, k, 1, nb)) = uint4{0u, 0u, 0u, 0u};
        } else {
            *reinterpret_cast<uint4*>(codes + code_chunk_offset(row0 + row, k, nb)) = uint4{0u, 0u, 0u, 0u};
        }
        scales[scale_index_internal(row0 + row, k, srows)] = (uint8_t)127;
        return;
    }
    float x[32], y[32];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float(&xq)[8] = *reinterpret_cast<float(*)[8]>(x + 8 * q);
        load8(X + (size_t)row * ldx + (size_t)k * 32 + q * 8, xq);
        if (U) {                                            // gated input: bf16(silu(X) * U)
            float u[8];
            load8(U + (size_t)row * ldu + (size_t)k * 32 + q * 8, u);
            swiglu8(xq, u);
        }
    }
#pragma unroll 4
    for (int j2 = 0; j2 < 32; ++j2) {
        float acc = x[0] * sT[j2];
#pragma unroll
        for (int j = 1; j < 32; ++j) acc = __builtin_fmaf(x[j], sT[j * 32 + j2], acc);
        y[j2] = acc;
    }
    if (row_scale) {
        const float rs = row_scale[row];
#pragma unroll
        for (int j = 0; j < 32; ++j) y[j] *= rs;
    }
    float bound;
    if (clip_max) {
        float mn = y[0], mx = y[0];
#pragma unroll
        for (int j = 1; j < 32; ++j) {
            mn = __builtin_fminf(mn, y[j]);
            mx = __builtin_fmaxf(mx, y[j]);
        }
        const float lo = clip[k] * mn, hi = clip_max[k] * mx;
#pragma unroll
        for (int j = 0; j < 32; ++j) y[j] = clamp_lo_hi(y[j], lo, hi);
        bound = __builtin_fmaxf(__builtin_fabsf(clamp_lo_hi(mn, lo, hi)), __builtin_fabsf(clamp_lo_hi(mx, lo, hi)));
    } else {
        float m = __builtin_fabsf(y[0]);
#pragma unroll
        for (int j = 1; j < 32; ++j) m = __builtin_fmaxf(m, __builtin_fabsf(y[j]));
        bound = clip[k] * m;
    }
    if constexpr (FP8) {
        const uint32_t s = e8m0_of_bound_fp8(bound);
        const float sc = scale_operand(s);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint2 a = encode8_fp8(y + 16 * h, bound, s, sc), b = encode8_fp8(y + 16 * h + 8, bound, s, sc);
            *reinterpret_cast<uint4*>(codes + code8_slot_offset(row0 + row, k, h, nb)) = uint4{a.x, a.y, b.x, b.y};
        }
        scales[scale_index_internal(row0 + row, k, srows)] = (uint8_t)s;
    } else {
        const uint32_t s = e8m0_of_bound(bound);
        const float sc = scale_operand(s);
        uint4 out;
        out.x = encode8(y, bound, sc);
        out.y = encode8(y + 8, bound, sc);
        out.z = encode8(y + 16, bound, sc);
        out.w = encode8(y + 24, bound, sc);
        *reinterpret_cast<uint4*>(codes + code_chunk_offset(row0 + row, k, nb)) = out;
        scales[scale_index_internal(row0 + row, k, srows)] = (uint8_t)s;
    }
}

template <typename XT, bool FP8>
hipError_t launch_dense(const batq_transform* t, const XT* X, int M, int64_t ldx, const XT* U, int64_t ldu,
                        const float* row_scale, uint8_t* codes, uint8_t* scales, RowWindow win, hipStream_t stream) {
    const dim3 grid(scale_groups(t->nb) * 8, (M + 255) / 256), block(256);
    quant_act_dense<XT, FP8><<<grid, block, 0, stream>>>(X, ldx, U, ldu, M, t->nb, win.row0, win.srows, t->d_T, t->d_clip,
                                                          t->minmax ? t->d_clip_max : nullptr, row_scale, codes, scales);
    return hipGetLastError();
}

// bf16 rows with a transform always go through the matrix cores, with one arithmetic (see quant_act_mfma_rows).
// Which of the two kernels serves a row only changes the speed: the row-by-row kernel has no set-up but fetches
// 6 KiB of transform operand per 2 KiB of X, so it wins while the call is small (graph-replayed, rows x K:
// 16 x 4096 2.4 us against 4.6 us, 1024 x 4096 5.0 against 5.7, 384 x 14336 6.4 against 6.5, 2048 x 4096 7.7 against
// 7.3): it takes calls of up to 2^22 elements, and the rows in front of the first 32-row tile of a longer window.
constexpr int64_t kRowsKernelMaxElements = int64_t(1) << 22;

template <bool FP8>
hipError_t launch_quantize_as(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int64_t ldx,
                              const void* U, int64_t ldu, const float* row_scale, uint8_t* codes, uint8_t* scales,
                              RowWindow win, hipStream_t stream) {
    if (xdtype == BATQ_BF16) {
        auto Xp = static_cast<const uint16_t*>(X);
        auto Up = static_cast<const uint16_t*>(U);
        if (t->has_transform && t->d_Tsplit) {
            // the persistent kernel addresses a 32-row tile with 32-bit byte offsets and writes whole 32-row tiles of
            // codes, so its window must start on one
            const bool wide_ok = ldx < (int64_t(1) << 25) && ldu < (int64_t(1) << 25);
            const int head = std::min(M, (32 - (win.row0 & 31)) & 31);
            const int rest = M - head;
            const int by_rows = (!wide_ok || (int64_t)rest * t->K <= kRowsKernelMaxElements) ? M : head;
            if (by_rows > 0) {
                hipError_t e = Up ? launch_mfma_rows<true>(t, Xp, by_rows, ldx, Up, ldu, row_scale, codes, scales, win, FP8, stream)
                                  : launch_mfma_rows<false>(t, Xp, by_rows, ldx, nullptr, 0, row_scale, codes, scales, win, FP8, stream);
                if (e != hipSuccess || by_rows == M) return e;
            }
            const RowWindow tail{win.row0 + by_rows, win.srows};
            const uint16_t* Xt = Xp + (size_t)by_rows * ldx;
            const float* rst = row_scale ? row_scale + by_rows : nullptr;
            return Up ? launch_mfma<true>(t, Xt, M - by_rows, ldx, Up + (size_t)by_rows * ldu, ldu, rst, codes, scales, tail, FP8, stream)
                      : launch_mfma<false>(t, Xt, M - by_rows, ldx, nullptr, 0, rst, codes, scales, tail, FP8, stream);
        }
        if (t->form == BATQ_FORM_DENSE)
            return launch_dense<uint16_t, FP8>(t, Xp, M, ldx, Up, ldu, row_scale, codes, scales, win, stream);
        return launch_quad<uint16_t, FP8>(t, Xp, M, ldx, Up, ldu, row_scale, codes, scales, win, stream);
    }
    auto Xp = static_cast<const float*>(X);
    auto Up = static_cast<const float*>(U);
    if (t->form == BATQ_FORM_DENSE)
        return launch_dense<float, FP8>(t, Xp, M, ldx, Up, ldu, row_scale, codes, scales, win, stream);
    return launch_quad<float, FP8>(t, Xp, M, ldx, Up, ldu, row_scale, codes, scales, win, stream);
}

// 1 / sqrt(mean_j x_j^2 + eps) per row (RMSNorm's row factor), one wave per row, fp32 accumulation.
template <typename XT>
__global__ void __launch_bounds__(256)
row_rms_scale(const XT* __restrict__ X, int64_t ldx, int M, int K, float eps, float* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;                                   // wave-uniform
    float acc = 0.f;
    for (int c = lane * 8; c < K; c += 64 * 8) {            // K is a multiple of 32, so whole groups of 8
        float x[8];
        load8(X + (size_t)row * ldx + c, x);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc = __builtin_fmaf(x[i], x[i], acc);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) out[row] = 1.0f / __builtin_sqrtf(acc / (float)K + eps);
}

}  // namespace

hipError_t launch_quantize_act(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int K,
                               int64_t ldx, const void* U, int64_t ldu, const float* row_scale, uint8_t* codes,
                               uint8_t* scales, bool fp8, int row_offset, int layout_rows, hipStream_t stream) {
    (void)K;
    if (M == 0) return hipSuccess;
    const RowWindow win{row_offset, layout_rows > 0 ? layout_rows : M};
    return fp8 ? launch_quantize_as<true>(t, X, xdtype, M, ldx, U, ldu, row_scale, codes, scales, win, stream)
               : launch_quantize_as<false>(t, X, xdtype, M, ldx, U, ldu, row_scale, codes, scales, win, stream);
}

hipError_t launch_row_rms_scale(const void* X, batq_dtype xdtype, int M, int K, int64_t ldx, float eps, float* out,
                                hipStream_t stream) {
    if (M == 0) return hipSuccess;
    const dim3 grid((M + 3) / 4), block(256);
    if (xdtype == BATQ_BF16)
        row_rms_scale<uint16_t><<<grid, block, 0, stream>>>(static_cast<const uint16_t*>(X), ldx, M, K, eps, out);
    else
        row_rms_scale<float><<<grid, block, 0, stream>>>(static_cast<const float*>(X), ldx, M, K, eps, out);
    return hipGetLastError();
}

}  // namespace batq
