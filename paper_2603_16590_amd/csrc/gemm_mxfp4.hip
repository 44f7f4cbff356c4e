// MXFP4 x MXFP4 GEMM (the low-bit product of Sec. 3.1: Q(XP) Q(P^-1 W)) on gfx950's
// block-scaled FP4 matrix instruction, fp32 accumulation.
//
// v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in FP4: lane l supplies, for matrix
// row (l % 32), the 32 consecutive K elements of MX block (l / 32) as 16 packed bytes, plus
// that block's E8M0 scale; so one 128-bit read of the canonical [rows][K/2] code layout is
// exactly one operand fragment.  The accumulator register r of lane l is element
// (8*(r/4) + 4*(l/32) + r%4, l % 32) of the 32x32 tile.
#include "batq_internal.h"
#include "mxfp4_device.h"

namespace batq {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

template <typename YT>
__device__ __forceinline__ void store_y(YT* p, float v);
template <>
__device__ __forceinline__ void store_y<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_y<uint16_t>(uint16_t* p, float v) { *p = (uint16_t)float_to_bf16_bits(v); }

// Direct kernel: one wave per 32x32 output tile, operands straight from global memory.
// Used for small problems and as the reference path of the tiled kernel.
template <typename YT>
__global__ void __launch_bounds__(256)
gemm_direct(const uint8_t* __restrict__ xc, const uint8_t* __restrict__ xs, const uint8_t* __restrict__ wc,
            const uint8_t* __restrict__ ws, int M, int N, int nb, YT* __restrict__ Y, int64_t ldy) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m0 = blockIdx.y * 64 + (wave >> 1) * 32;
    const int n0 = blockIdx.x * 64 + (wave & 1) * 32;
    if (m0 >= M || n0 >= N) return;                       // wave-uniform
    const int i = lane & 31, kg = lane >> 5;
    const int am = min(m0 + i, M - 1), bn = min(n0 + i, N - 1);   // clamp: rows past the edge are computed, not stored
    const size_t Kh = (size_t)nb * 16;
    const uint8_t* ap = xc + (size_t)am * Kh + kg * 16;
    const uint8_t* bp = wc + (size_t)bn * Kh + kg * 16;
    const uint8_t* asp = xs + (size_t)am * nb + kg;
    const uint8_t* bsp = ws + (size_t)bn * nb + kg;
    v16f acc = {};
    const int steps = nb >> 1;
    for (int s = 0; s < steps; ++s) {
        const uint4 a = *reinterpret_cast<const uint4*>(ap + (size_t)s * 32);
        const uint4 b = *reinterpret_cast<const uint4*>(bp + (size_t)s * 32);
        const v8i av = {(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
        const v8i bv = {(int)b.x, (int)b.y, (int)b.z, (int)b.w, 0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, acc, 4, 4, 0, (int)asp[2 * s], 0, (int)bsp[2 * s]);
    }
    if (nb & 1) {
        // odd block count: the upper half-wave contributes an all-zero operand
        const int s = steps;
        uint4 a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
        int sa = 127, sb = 127;
        if (kg == 0) {
            a = *reinterpret_cast<const uint4*>(ap + (size_t)s * 32);
            b = *reinterpret_cast<const uint4*>(bp + (size_t)s * 32);
            sa = asp[2 * s];
            sb = bsp[2 * s];
        }
        const v8i av = {(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
        const v8i bv = {(int)b.x, (int)b.y, (int)b.z, (int)b.w, 0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, acc, 4, 4, 0, sa, 0, sb);
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

}  // namespace

hipError_t launch_gemm_mxfp4(const uint8_t* xcodes, const uint8_t* xscales, const batq_weight* w, int M,
                             void* Y, batq_dtype ydtype, int64_t ldy, hipStream_t stream) {
    if (M == 0) return hipSuccess;
    const dim3 grid((w->N + 63) / 64, (M + 63) / 64), block(256);
    if (ydtype == BATQ_BF16)
        gemm_direct<uint16_t><<<grid, block, 0, stream>>>(xcodes, xscales, w->d_codes, w->d_scales, M, w->N, w->nb,
                                                          static_cast<uint16_t*>(Y), ldy);
    else
        gemm_direct<float><<<grid, block, 0, stream>>>(xcodes, xscales, w->d_codes, w->d_scales, M, w->N, w->nb,
                                                       static_cast<float*>(Y), ldy);
    return hipGetLastError();
}

}  // namespace batq
