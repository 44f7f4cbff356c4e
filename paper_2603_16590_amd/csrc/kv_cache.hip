// Helpers for the key/value-cache placement of the transforms (Sec. 3.2, "Self-Attention Module": P_k and P_v
// transform the key and value cache head by head).  The cache itself is written by the activation quantiser
// (a head of 128 channels is 4 MX blocks, each with its own 32x32 transform); this file holds the two pieces
// around it:
//   dequantise     - blocked MXFP4 / MXFP8 codes + grouped E8M0 scales -> row-major bf16 / fp32, for an
//                    attention kernel that works on 16-bit keys and values;
//   transform_apply - x T_k, x T_k^-1 or x T_k^-T block by block without quantisation: the query takes
//                    T_k^-T so that (q T^-T)(k T)^T = q k^T, the attention output takes T_v^-1.
// Neither is on the timed path; both are written for exactness first.  gfx950 only.
#include "batq_internal.h"
#include "mxfp4_device.h"
#include "code_layout.h"
#include "scale_layout.h"

namespace batq {
namespace {

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

// One thread per (row, MX block, quarter of the block): consecutive threads write consecutive 8-element
// pieces of a row.  The product code value x 2^(byte - 127) is exact in fp32 (fp32 subnormals included);
// bf16 output rounds to nearest even, which only matters below 2^-126.
template <typename OT, bool FP8>
__global__ void __launch_bounds__(256)
dequant_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales, int M, int nb,
               OT* __restrict__ out, int64_t ldo) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)M * nb * 4) return;
    const int q = (int)(idx & 3);
    const int64_t blk = idx >> 2;
    const int row = (int)(blk / nb), k = (int)(blk - (int64_t)row * nb);
    const float sc = e8m0_value(scales[scale_index_internal(row, k, M)]);
    float v[8];
    if constexpr (FP8) {
        const uint2 w = *reinterpret_cast<const uint2*>(codes + code8_slot_offset(row, k, q >> 1, nb) + (q & 1) * 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[i] = e4m3_value((w.x >> (8 * i)) & 0xFFu) * sc;
            v[4 + i] = e4m3_value((w.y >> (8 * i)) & 0xFFu) * sc;
        }
    } else {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(codes + code_chunk_offset(row, k, nb) + q * 4);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = e2m1_value((w >> (4 * i)) & 0xFu) * sc;
    }
    store8<OT>(out + (size_t)row * ldo + (size_t)k * 32 + q * 8, v);
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
                             batq_dtype odtype, int64_t ldo, hipStream_t stream) {
    if (M == 0) return hipSuccess;
    const int64_t total = (int64_t)M * nb * 4;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (odtype == BATQ_BF16) {
        auto o = static_cast<uint16_t*>(out);
        if (fp8) dequant_kernel<uint16_t, true><<<grid, block, 0, stream>>>(codes, scales, M, nb, o, ldo);
        else dequant_kernel<uint16_t, false><<<grid, block, 0, stream>>>(codes, scales, M, nb, o, ldo);
    } else {
        auto o = static_cast<float*>(out);
        if (fp8) dequant_kernel<float, true><<<grid, block, 0, stream>>>(codes, scales, M, nb, o, ldo);
        else dequant_kernel<float, false><<<grid, block, 0, stream>>>(codes, scales, M, nb, o, ldo);
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
