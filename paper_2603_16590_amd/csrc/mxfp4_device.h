// Device-side MX encoding helpers (Sec. 2 of the paper: E2M1 elements for MXFP4, E4M3 for MXFP8,
// one UE8M0 scale per 32 elements), written for gfx950's scaled fp32->fp4 / fp32->fp8 convert
// instructions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace batq {

// E8M0 byte of a block whose clipped bound is `bound` (>= 0, finite):
// E = floor(log2 bound) - 2 clamped below at -127, byte = E + 127.  For a normal fp32
// bound floor(log2) is the exponent field minus 127; zero and subnormal bounds have
// field 0 and clamp to byte 0.
__device__ __forceinline__ uint32_t e8m0_of_bound(float bound) {
    uint32_t field = __float_as_uint(bound) >> 23;
    return field > 2u ? field - 2u : 0u;
}

// The scale operand of the convert instruction is an fp32 whose exponent field is the
// E8M0 byte (a field of 0 is read as 2^-127).
__device__ __forceinline__ float scale_operand(uint32_t e8m0) { return __uint_as_float(e8m0 << 23); }

// Clamp to [-bound, bound] keeping the element's own sign bit (also for zeros): the median of
// (y, -b, b).  `b` must be positive for a zero to keep its sign, so a zero bound (an all-zero
// block, where nothing is clamped anyway) is replaced by the smallest positive fp32.
__device__ __forceinline__ float clamp_limit(float bound) {
    return __uint_as_float(max(__float_as_uint(bound), 1u));
}
__device__ __forceinline__ float clamp_keep_sign(float y, float b) { return __builtin_amdgcn_fmed3f(y, -b, b); }

// Two-sided clamp of Eq. 3-4 as printed: below lo -> lo, else above hi -> hi, else unchanged (in this
// order also when lo > hi, which ratios on an all-positive or all-negative block can produce).
__device__ __forceinline__ float clamp_lo_hi(float y, float lo, float hi) { return y < lo ? lo : (y > hi ? hi : y); }

// Eight fp32 values -> eight E2M1 codes in one dword, element 0 in bits 3:0.
// The hardware convert rounds to nearest even on the E2M1 grid, saturates at 6 and
// keeps the sign bit of results that round to zero.
__device__ __forceinline__ uint32_t encode8(const float* y, float bound, float sc) {
    const float b = clamp_limit(bound);
    uint32_t r = 0;
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, clamp_keep_sign(y[0], b), clamp_keep_sign(y[1], b), sc, 0);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, clamp_keep_sign(y[2], b), clamp_keep_sign(y[3], b), sc, 1);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, clamp_keep_sign(y[4], b), clamp_keep_sign(y[5], b), sc, 2);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, clamp_keep_sign(y[6], b), clamp_keep_sign(y[7], b), sc, 3);
    return r;
}

// ---- MXFP8 (E4M3 elements, the 8-bit activation format of Sec. 2): E = floor(log2 bound) - 8.
__device__ __forceinline__ uint32_t e8m0_of_bound_fp8(float bound) {
    uint32_t field = __float_as_uint(bound) >> 23;
    return field > 8u ? field - 8u : 0u;
}

typedef short batq_v2s __attribute__((ext_vector_type(2)));

// Eight fp32 values -> eight E4M3 codes in two dwords, element 0 in the lowest byte.  The hardware
// convert rounds to nearest even and keeps the sign of zero, but turns magnitudes from 480 * 2^E up
// into the NaN code, so the clamp limit is the smaller of the block's bound and 448 * 2^E
// (= 1.75 * 2^(byte - 119)).
__device__ __forceinline__ uint2 encode8_fp8(const float* y, float bound, uint32_t e8m0, float sc) {
    const float top = 1.75f * __uint_as_float((e8m0 + 8u) << 23);
    const float b = clamp_limit(__builtin_fminf(bound, top));
    batq_v2s lo = {0, 0}, hi = {0, 0};
    lo = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(lo, clamp_keep_sign(y[0], b), clamp_keep_sign(y[1], b), sc, false);
    lo = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(lo, clamp_keep_sign(y[2], b), clamp_keep_sign(y[3], b), sc, true);
    hi = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(hi, clamp_keep_sign(y[4], b), clamp_keep_sign(y[5], b), sc, false);
    hi = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(hi, clamp_keep_sign(y[6], b), clamp_keep_sign(y[7], b), sc, true);
    return uint2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
}

// Gated activation of the MLP (Sec. 3.2: its output is what P_down transforms): silu(g) * u =
// g u / (1 + 2^(-g log2 e)) in fp32 (hardware exp2 and reciprocal, about 2^-21 relative).  Magnitudes below
// 2^-100 may come out as zero.
__device__ __forceinline__ float swiglu_f32(float g, float u) {
    const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * g);
    return g * __builtin_amdgcn_rcpf(1.0f + e) * u;
}

// 16-byte store written through the L2 (device scope), for output that nobody reads in the same kernel: lines left
// dirty in the eight L2s would be written back when the kernel ends.  A store of more than 8 bytes reads its data
// registers after it has issued; the compiler keeps the next instructions from overwriting them for its own
// stores but cannot see inside an asm statement, so the two wait states are part of it.
typedef uint32_t batq_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store16_through(void* p, const batq_u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" :: "v"(p), "v"(v) : "memory");
}

// The same for an output larger than the memory-side cache can hold for whoever reads it next: also non-temporal,
// so that it does not push the operands out of that cache on its way.
__device__ __forceinline__ void store16_through_nt(void* p, const batq_u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" :: "v"(p), "v"(v) : "memory");
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

}  // namespace batq
