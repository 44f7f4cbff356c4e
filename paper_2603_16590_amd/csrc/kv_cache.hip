// Helpers for the key/value-cache placement of the transforms (Sec. 3.2, "Self-Attention Module": P_k and P_v
// transform the key and value cache head by head).  The cache itself is written by the activation quantiser
// (a head of 128 channels is 4 MX blocks, each with its own 32x32 transform); this file holds the two pieces
// around it:
//   dequantise     - blocked MXFP4 / MXFP8 codes + grouped E8M0 scales -> row-major bf16 / fp32, for an
//                    attention kernel that works on 16-bit keys and values;
//   transform_apply - x T_k, x T_k^-1 or x T_k^-T block by block without quantisation: the query takes
//                    T_k^-T so that (q T^-T)(k T)^T = q k^T, the attention output takes T_v^-1.
// gfx950 only.
#include "batq_internal.h"
#include "mxfp4_device.h"
#include "code_layout.h"
#include "scale_layout.h"

namespace batq {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void store16_through(void* p, const uint4& q) {
    batq::store16_through(p, batq_u32x4{q.x, q.y, q.z, q.w});
}

// 2^(byte - 127) as fp32; byte 0 is the subnormal 2^-127, byte 255 (the format's NaN) gives NaN.
__device__ __forceinline__ float e8m0_value(uint32_t byte) {
    if (byte == 0u) return __uint_as_float(0x00400000u);
    if (byte == 255u) return __uint_as_float(0x7FC00000u);
    return __uint_as_float(byte << 23);
}

// E2M1 nibble -> fp32 (exact): 0, 0.5, 1, 1.5, 2, 3, 4, 6 with the sign bit on top (also for zero).
__device__ __forceinline__ float e2m1_value(uint32_t c) {
    const uint32_t e = (c >> 1) & 3u, m = c & 1u;
    const uint32_t mag = e == 0u ? (m ? 0x3F000000u : 0u) : (((e + 126u) << 23) | (m << 22));
    return __uint_as_float(mag | ((c & 8u) << 28));
}

// E4M3 byte -> fp32 (exact): subnormals m 2^-9, normals (1 + m/8) 2^(e-7), 0x7F / 0xFF = NaN.
__device__ __forceinline__ float e4m3_value(uint32_t c) {
    const uint32_t e = (c >> 3) & 15u, m = c & 7u;
    uint32_t mag;
    if ((c & 0x7Fu) == 0x7Fu) mag = 0x7FC00000u;
    else if (e == 0u) mag = __float_as_uint((float)m * 0.001953125f);
    else mag = ((e + 120u) << 23) | (m << 20);
    return __uint_as_float(mag | ((c & 0x80u) << 24));
}

template <typename OT>
__device__ __forceinline__ void store8(OT* p, const float (&v)[8]);
template <>
__device__ __forceinline__ void store8<float>(float* p, const float (&v)[8]) {
    reinterpret_cast<float4*>(p)[0] = float4{v[0], v[1], v[2], v[3]};
    reinterpret_cast<float4*>(p)[1] = float4{v[4], v[5], v[6], v[7]};
}
template <>
__device__ __forceinline__ void store8<uint16_t>(uint16_t* p, const float (&v)[8]) {
    uint4 o;
    o.x = float_to_bf16_bits(v[0]) | (float_to_bf16_bits(v[1]) << 16);
    o.y = float_to_bf16_bits(v[2]) | (float_to_bf16_bits(v[3]) << 16);
    o.z = float_to_bf16_bits(v[4]) | (float_to_bf16_bits(v[5]) << 16);
    o.w = float_to_bf16_bits(v[6]) | (float_to_bf16_bits(v[7]) << 16);
    *reinterpret_cast<uint4*>(p) = o;
}

// One wave per (32-row tile, K group of 8 MX blocks): 4 (MXFP4) or 8 (MXFP8) pieces of 1 KiB.  Every lane
// converts 8 elements at a time (4 or 8 code bytes -> one 16-byte store of bf16, two of fp32), and the lanes are
// laid over a piece so that neighbours hold neighbouring elements of a row: one wave instruction reads
// 256 (512) contiguous code bytes and writes 4 (8) rows x 256 (128) contiguous output bytes.
// bf16 output uses the hardware converts (two codes -> two bf16, times 2^(scale byte - 127)); they are exact for
// every result in bf16's normal range, smaller ones are not specified here.  fp32 output is computed as
// code value x 2^(byte - 127), exact in fp32 (subnormals included; scale byte 255 and the E4M3 NaN codes give NaN).
template <typename OT, bool FP8>
__global__ void __launch_bounds__(256)
dequant_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales, int M, int nb, int row0,
               int srows, OT* __restrict__ out, int64_t ldo, bool big) {
    constexpr int kPerRow = FP8 ? 4 : 2;                   // pieces of a K group per 16-row group
    constexpr int kPieces = 2 * kPerRow;
    constexpr int kSub = FP8 ? 2 : 4;                       // wave instructions per piece
    constexpr int kRows = 16 / kSub;                        // piece rows per instruction
    constexpr bool kHw = sizeof(OT) == 2;                   // bf16 output
    const int lane = threadIdx.x & 63;
    const int groups = scale_groups(nb);
    const int64_t unit = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    // rows row0 .. row0 + M - 1 of arrays laid out for srows rows -> out rows 0 .. M - 1
    const int first_tile = row0 >> 5, last_tile = (row0 + M - 1) >> 5;
    const int tile = first_tile + (int)(unit / groups), g = (int)(unit % groups);
    if (tile > last_tile) return;                           // wave-uniform
    const size_t stages = (size_t)(FP8 ? code8_stages(nb) : code_stages(nb));
    // this lane inside an instruction's rows: row, 16-byte slot of the row, 8-element part of the slot
    const int lr = FP8 ? lane >> 3 : lane >> 4;
    const int pos = FP8 ? (lane >> 1) & 3 : (lane >> 2) & 3;
    const int part = FP8 ? lane & 1 : lane & 3;
    uint2 w[kPieces][kSub];
#pragma unroll
    for (int p = 0; p < kPieces; ++p) {
        const uint8_t* piece = codes + ((size_t)(2 * tile + p / kPerRow) * stages + (size_t)(g * kPerRow + p % kPerRow)) * 1024;
#pragma unroll
        for (int i = 0; i < kSub; ++i) {
            if constexpr (FP8) w[p][i] = *reinterpret_cast<const uint2*>(piece + i * 512 + lane * 8);
            else w[p][i] = uint2{*reinterpret_cast<const uint32_t*>(piece + i * 256 + lane * 4), 0u};
        }
    }
#pragma unroll
    for (int p = 0; p < kPieces; ++p)
#pragma unroll
        for (int i = 0; i < kSub; ++i) {
            const int r = i * kRows + lr;                   // row inside the piece
            const int slot = pos ^ ((r >> 2) & 3);          // undo the bank swizzle
            const int row = tile * 32 + (p / kPerRow) * 16 + r;
            const int k = g * 8 + (p % kPerRow) * (FP8 ? 2 : 4) + (FP8 ? slot >> 1 : slot);
            if (row < row0 || row >= row0 + M || k >= nb) continue;
            const uint32_t byte = scales[scale_index_internal(row, k, srows)];
            OT* o = out + (size_t)(row - row0) * ldo + (size_t)k * 32 + (FP8 ? (slot & 1) * 16 + part * 8 : part * 8);
            const uint2 d = w[p][i];
            if constexpr (kHw) {
                const float sc = scale_operand(byte);
                uint4 q;
                if constexpr (FP8) {
                    q.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(d.x, sc, false));
                    q.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(d.x, sc, true));
                    q.z = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(d.y, sc, false));
                    q.w = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(d.y, sc, true));
                } else {
                    q.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(d.x, sc, 0));
                    q.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(d.x, sc, 1));
                    q.z = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(d.x, sc, 2));
                    q.w = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(d.x, sc, 3));
                }
                // no reader in this kernel, and nothing should be left dirty in the L2s at its end: written
                // through (32768 x 1024: plain stores 14.1 us, non-temporal 12.9, through 11.1), or, for outputs
                // beyond the memory-side cache, non-temporal (131072 x 1024: 71 / 53 / 71 us)
                if (big) __builtin_nontemporal_store(u32x4{q.x, q.y, q.z, q.w}, reinterpret_cast<u32x4*>(o));
                else store16_through(o, q);
            } else {
                const float sc = e8m0_value(byte);
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if constexpr (FP8) v[e] = e4m3_value(((e < 4 ? d.x : d.y) >> (8 * (e & 3))) & 0xFFu) * sc;
                    else v[e] = e2m1_value((d.x >> (4 * e)) & 0xFu) * sc;
                }
                store8<OT>(o, v);
            }
        }
}

template <typename XT>
__device__ __forceinline__ double load_x(const XT* p);
template <>
__device__ __forceinline__ double load_x<float>(const float* p) { return (double)*p; }
template <>
__device__ __forceinline__ double load_x<uint16_t>(const uint16_t* p) { return (double)bf16_bits_to_float(*p); }

template <typename OT>
__device__ __forceinline__ void store_o(OT* p, float v);
template <>
__device__ __forceinline__ void store_o<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_o<uint16_t>(uint16_t* p, float v) { *p = (uint16_t)float_to_bf16_bits(v); }

// y = x B_k with B_k = Mat[k] (TRANSPOSED: Mat[k]^T), fp64 products and sums, one rounding to fp32 and, for
// bf16 output, one more to bf16.  One thread per (row, block); the block's matrix sits in LDS.
template <typename XT, typename OT, bool TRANSPOSED>
__global__ void __launch_bounds__(256)
apply_kernel(const XT* __restrict__ X, int64_t ldx, int M, const double* __restrict__ Mat, OT* __restrict__ out,
             int64_t ldo) {
    __shared__ double sB[32 * 33];
    const int k = blockIdx.x;
    for (int i = threadIdx.x; i < 1024; i += 256) {
        const int r = i >> 5, c = i & 31;
        // sB[j][j2] = B_k[j][j2]
        if constexpr (TRANSPOSED) sB[c * 33 + r] = Mat[(size_t)k * 1024 + i];
        else sB[r * 33 + c] = Mat[(size_t)k * 1024 + i];
    }
    __syncthreads();
    const int row = blockIdx.y * 256 + threadIdx.x;
    if (row >= M) return;
    double x[32];
#pragma unroll
    for (int j = 0; j < 32; ++j) x[j] = load_x<XT>(X + (size_t)row * ldx + (size_t)k * 32 + j);
    OT* o = out + (size_t)row * ldo + (size_t)k * 32;
#pragma unroll 4
    for (int j2 = 0; j2 < 32; ++j2) {
        double acc = 0.0;
#pragma unroll
        for (int j = 0; j < 32; ++j) acc = __builtin_fma(x[j], sB[j * 33 + j2], acc);
        store_o<OT>(o + j2, (float)acc);
    }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kSplitBlock = 3 * 2 * 64 * 16;               // bytes of split operand per MX block (see split_operand)
constexpr int kApplyWaves = 8;
constexpr int kApplySlot = 32 * 256;                        // a unit: 32 rows x 4 MX blocks of bf16
constexpr int kApplyLdsT = 4 * kSplitBlock;                 // 24 KiB
constexpr int kApplyLds = kApplyLdsT + kApplyWaves * 2 * kApplySlot;        // 152 KiB

// y = x B_k on the matrix cores for bf16 input: B_k comes pre-split into three bf16 terms (products with bf16
// inputs are then exact, sums are fp32: the arithmetic of the quantiser's transform).  A workgroup takes a
// unit column (4 MX blocks, operands in LDS) and a range of 32-row tiles that its waves go through in turn;
// a wave fetches its unit with LDS-direct loads (rows of 256 contiguous bytes, 16-byte chunk c of row r at
// position (c & 8) | ((c ^ r) & 7)), prefetching the next unit into its second slot, and sends the results
// back through the slot it has just emptied, so that the stores are rows of 256 contiguous bytes as well.
// The output rows are written through the L2 (8192 x 4096: plain stores 28.9 us, through 25.8).
template <typename OT>
__global__ void __launch_bounds__(kApplyWaves * 64)
apply_mfma(const uint16_t* __restrict__ X, int64_t ldx, int M, int nb, int tiles_per_wg,
           const uint4* __restrict__ split, OT* __restrict__ out, int64_t ldo) {
    extern __shared__ __align__(16) uint8_t alds[];
    typedef __attribute__((address_space(3))) uint8_t lds_byte;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, kg = lane >> 5;
    const int kb = 4 * blockIdx.x;                          // first MX block of the unit column
    const int nreal = min(4, nb - kb);
    const int row_tiles = (M + 31) >> 5;
    const int t_begin = blockIdx.y * tiles_per_wg, t_end = min(row_tiles, t_begin + tiles_per_wg);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_byte*)alds;
    uint8_t* const slots = alds + kApplyLdsT + wave * 2 * kApplySlot;
    const uint32_t slots_lds = lds_base + kApplyLdsT + wave * 2 * kApplySlot;

    {   // operands of the column's blocks: 6 pieces of 1 KiB per block
        const uint8_t* src = reinterpret_cast<const uint8_t*>(split) + (size_t)kb * kSplitBlock;
        const int pieces = nreal * (kSplitBlock / 1024);
        for (int p = wave; p < pieces; p += kApplyWaves)
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                         :: "v"((uint32_t)(p * 1024 + lane * 16)), "s"(src), "s"(lds_base + (uint32_t)p * 1024) : "memory");
    }
    auto request = [&](int tile, int slot) {
        const uint8_t* base = reinterpret_cast<const uint8_t*>(X) + ((size_t)tile * 32 * ldx + (size_t)kb * 32) * 2;
        const int rows_left = M - 1 - tile * 32;            // rows past the end repeat the last one: computed, not stored
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = 4 * j + (lane >> 4);
            int c = ((lane & 15) & 8) | (((lane & 15) ^ r) & 7);    // the chunk that belongs at this lane's LDS position
            if (c >= 4 * nreal) c = 0;                      // never read past the end of the row
            const uint32_t voff = (uint32_t)min(r, rows_left) * (uint32_t)(ldx * 2) + (uint32_t)c * 16;
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                         :: "v"(voff), "s"(base), "s"(slots_lds + (uint32_t)(slot * kApplySlot + j * 1024)) : "memory");
        }
    };
    int tile = t_begin + wave;
    if (tile < t_end) request(tile, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);                     // vmcnt(0): this wave's share of the operands
    __syncthreads();                                        // all operands have landed

    for (int it = 0; tile < t_end; tile += kApplyWaves, ++it) {
        uint8_t* const slot = slots + (it & 1) * kApplySlot;
        __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): the unit has landed, the last stores are out
        if (tile + kApplyWaves < t_end) request(tile + kApplyWaves, (it + 1) & 1);
        u32x4 x[4][2];
#pragma unroll
        for (int bb = 0; bb < 4; ++bb)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int c = 4 * bb + 2 * kg + h;
                x[bb][h] = *reinterpret_cast<const u32x4*>(slot + l32 * 256 + (((c & 8) | ((c ^ l32) & 7)) << 4));
            }
        // results go back into this slot: its contents must be in registers first
#pragma unroll
        for (int bb = 0; bb < 4; ++bb)
#pragma unroll
            for (int h = 0; h < 2; ++h) asm volatile("" : "+v"(x[bb][h]));
        v16f acc[4] = {};
#pragma unroll
        for (int bb = 0; bb < 4; ++bb) {
            if (bb >= nreal) break;
            const uint4* tf = reinterpret_cast<const uint4*>(alds + bb * kSplitBlock) + lane;
#pragma unroll
            for (int t = 2; t >= 0; --t)                    // smallest terms first
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    acc[bb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tf[(t * 2 + h) * 64]),
                                                                  __builtin_bit_cast(bf16x8, x[bb][h]), acc[bb], 0, 0, 0);
        }
        // acc[bb][r] = element 16 kg + r of block bb of this lane's row
        const int row0 = tile * 32;
        if constexpr (sizeof(OT) == 2) {
#pragma unroll
            for (int bb = 0; bb < 4; ++bb)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    uint4 q;
                    q.x = float_to_bf16_bits(acc[bb][8 * h + 0]) | (float_to_bf16_bits(acc[bb][8 * h + 1]) << 16);
                    q.y = float_to_bf16_bits(acc[bb][8 * h + 2]) | (float_to_bf16_bits(acc[bb][8 * h + 3]) << 16);
                    q.z = float_to_bf16_bits(acc[bb][8 * h + 4]) | (float_to_bf16_bits(acc[bb][8 * h + 5]) << 16);
                    q.w = float_to_bf16_bits(acc[bb][8 * h + 6]) | (float_to_bf16_bits(acc[bb][8 * h + 7]) << 16);
                    const int c = 4 * bb + 2 * kg + h;
                    *reinterpret_cast<uint4*>(slot + l32 * 256 + (((c & 8) | ((c ^ l32) & 7)) << 4)) = q;
                }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = 4 * j + (lane >> 4), pos = lane & 15;
                const int c = (pos & 8) | ((pos ^ r) & 7);
                const uint4 q = *reinterpret_cast<const uint4*>(slot + r * 256 + pos * 16);
                if (row0 + r < M && c < 4 * nreal)
                {
                    uint4* dst = reinterpret_cast<uint4*>(out + (size_t)(row0 + r) * ldo + (size_t)kb * 32 + c * 8);
                    store16_through(dst, q);
                }
            }
        } else {
            // fp32 output: two blocks (256 bytes per row) at a time through the same slot
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
                for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const v16f& a = acc[2 * pass + b2];
                        const int c = 8 * b2 + 4 * kg + q4;
                        *reinterpret_cast<float4*>(slot + l32 * 256 + (((c & 8) | ((c ^ l32) & 7)) << 4)) =
                            float4{a[4 * q4], a[4 * q4 + 1], a[4 * q4 + 2], a[4 * q4 + 3]};
                    }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int r = 4 * j + (lane >> 4), pos = lane & 15;
                    const int c = (pos & 8) | ((pos ^ r) & 7);
                    const float4 q = *reinterpret_cast<const float4*>(slot + r * 256 + pos * 16);
                    if (row0 + r < M && 2 * pass + (c >> 3) < nreal)
                        *reinterpret_cast<float4*>(out + (size_t)(row0 + r) * ldo + (size_t)(kb + 2 * pass) * 32 + c * 4) = q;
                }
            }
        }
    }
}

template <typename XT, typename OT>
__global__ void __launch_bounds__(256)
convert_kernel(const XT* __restrict__ X, int64_t ldx, int M, int K, OT* __restrict__ out, int64_t ldo) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)M * K) return;
    const int row = (int)(idx / K), c = (int)(idx - (int64_t)row * K);
    store_o<OT>(out + (size_t)row * ldo + c, (float)load_x<XT>(X + (size_t)row * ldx + c));
}

template <typename XT, typename OT>
hipError_t apply_typed(const batq_transform* t, const XT* X, int M, int64_t ldx, int mode, OT* out, int64_t ldo,
                       hipStream_t stream) {
    if (!t->has_transform) {
        const int64_t total = (int64_t)M * t->K;
        convert_kernel<XT, OT><<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(X, ldx, M, t->K, out, ldo);
        return hipGetLastError();
    }
    if constexpr (sizeof(XT) == 2) {
        const uint16_t* sp = mode == BATQ_APPLY_FORWARD ? t->d_Tsplit : mode == BATQ_APPLY_INVERSE ? t->d_TinvSplit : t->d_TinvTSplit;
        // 16-byte accesses, and a tile's rows are addressed with 32-bit byte offsets
        const bool fits = ((uintptr_t)X | (uintptr_t)out | (uintptr_t)(ldx * 2) | (uintptr_t)(ldo * (int64_t)sizeof(OT))) % 16 == 0 &&
                          ldx < (int64_t(1) << 25);
        if (sp && fits) {
            int dev = 0;
            if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
            if (hipError_t e = ensure_dynamic_lds<&apply_mfma<OT>>(dev, kApplyLds); e != hipSuccess) return e;
            const int units = (t->nb + 3) / 4, row_tiles = (M + 31) / 32;
            // about four workgroups per compute unit, at least 16 tiles each (the operands are fetched per workgroup)
            int tiles_per_wg = (int)(((int64_t)row_tiles * units + 1023) / 1024);
            if (tiles_per_wg < 16) tiles_per_wg = 16;
            const dim3 grid(units, (row_tiles + tiles_per_wg - 1) / tiles_per_wg), block(kApplyWaves * 64);
            apply_mfma<OT><<<grid, block, kApplyLds, stream>>>(X, ldx, M, t->nb, tiles_per_wg,
                                                               reinterpret_cast<const uint4*>(sp), out, ldo);
            return hipGetLastError();
        }
    }
    const dim3 grid(t->nb, (M + 255) / 256), block(256);
    if (mode == BATQ_APPLY_FORWARD)
        apply_kernel<XT, OT, false><<<grid, block, 0, stream>>>(X, ldx, M, t->d_Tf64, out, ldo);
    else if (mode == BATQ_APPLY_INVERSE)
        apply_kernel<XT, OT, false><<<grid, block, 0, stream>>>(X, ldx, M, t->d_Tinv, out, ldo);
    else
        apply_kernel<XT, OT, true><<<grid, block, 0, stream>>>(X, ldx, M, t->d_Tinv, out, ldo);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_dequantize(const uint8_t* codes, const uint8_t* scales, int M, int nb, bool fp8, void* out,
                             batq_dtype odtype, int64_t ldo, int row_offset, int layout_rows, hipStream_t stream) {
    if (M == 0) return hipSuccess;
    const int tiles = ((row_offset + M - 1) >> 5) - (row_offset >> 5) + 1;
    const int64_t units = (int64_t)tiles * scale_groups(nb);                // one wave each, four to a workgroup
    const dim3 grid((unsigned)((units + 3) / 4)), block(256);
    const bool big = (size_t)M * nb * 32 * (odtype == BATQ_BF16 ? 2 : 4) > (size_t(128) << 20);
    if (odtype == BATQ_BF16) {
        auto o = static_cast<uint16_t*>(out);
        if (fp8) dequant_kernel<uint16_t, true><<<grid, block, 0, stream>>>(codes, scales, M, nb, row_offset, layout_rows, o, ldo, big);
        else dequant_kernel<uint16_t, false><<<grid, block, 0, stream>>>(codes, scales, M, nb, row_offset, layout_rows, o, ldo, big);
    } else {
        auto o = static_cast<float*>(out);
        if (fp8) dequant_kernel<float, true><<<grid, block, 0, stream>>>(codes, scales, M, nb, row_offset, layout_rows, o, ldo, big);
        else dequant_kernel<float, false><<<grid, block, 0, stream>>>(codes, scales, M, nb, row_offset, layout_rows, o, ldo, big);
    }
    return hipGetLastError();
}

hipError_t launch_transform_apply(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int64_t ldx,
                                  int mode, void* out, batq_dtype odtype, int64_t ldo, hipStream_t stream) {
    if (M == 0) return hipSuccess;
    if (xdtype == BATQ_BF16) {
        auto x = static_cast<const uint16_t*>(X);
        return odtype == BATQ_BF16 ? apply_typed(t, x, M, ldx, mode, static_cast<uint16_t*>(out), ldo, stream)
                                   : apply_typed(t, x, M, ldx, mode, static_cast<float*>(out), ldo, stream);
    }
    auto x = static_cast<const float*>(X);
    return odtype == BATQ_BF16 ? apply_typed(t, x, M, ldx, mode, static_cast<uint16_t*>(out), ldo, stream)
                               : apply_typed(t, x, M, ldx, mode, static_cast<float*>(out), ldo, stream);
}

}  // namespace batq
