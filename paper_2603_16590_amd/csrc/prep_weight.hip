// Offline weight preparation (Alg. 2, "Offline Fusion for Deployment"):
// W~ = P^-1 W per 32-row K-slab, optional block clip (Eq. 3-4, one ratio on the amax or two on min and
// max), MXFP4 along K (Sec. 2).
// Not on the timed path: written for accuracy (fp64 products with the host-inverted
// fp64 blocks, one rounding to fp32) rather than speed.  gfx950 only.
#include "batq_internal.h"
#include "mxfp4_device.h"
#include "code_layout.h"
#include "scale_layout.h"

namespace batq {
namespace {

template <typename WT>
__device__ __forceinline__ double load_w(const WT* p);
template <>
__device__ __forceinline__ double load_w<float>(const float* p) { return (double)*p; }
template <>
__device__ __forceinline__ double load_w<uint16_t>(const uint16_t* p) { return (double)bf16_bits_to_float(*p); }

// One thread per (K-block k, output column n).  blockIdx.y = k, blockIdx.x tiles N by 256.
// Codes go to the blocked code layout, scales to the grouped layout (padding of both is
// initialised by the caller).  Column n of W becomes row n of the prepared weight (N_out = N rows), or, with
// il_off >= 0, row 64 (n / 32) + il_off + n % 32 of a weight of N_out = 2 N rows: the gate (il_off 0) and up
// (il_off 32) projections of an MLP interleaved in groups of 32 columns for the GEMM's gated output.
template <typename WT, bool TRANSFORM>
__global__ void __launch_bounds__(256)
prep_weight_kernel(const WT* __restrict__ W, int64_t ldw, int w_is_KxN, int N, int N_out, int il_off, int nb,
                   const double* __restrict__ Tinv, const float* __restrict__ clip_w,
                   const float* __restrict__ clip_w_max, uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
    __shared__ double sT[TRANSFORM ? 32 * 32 : 1];
    const int k = blockIdx.y;
    if constexpr (TRANSFORM) {
        for (int i = threadIdx.x; i < 32 * 32; i += 256) sT[i] = Tinv[(size_t)k * 1024 + i];
        __syncthreads();
    }
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;

    double w[32];
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const size_t idx = w_is_KxN ? (size_t)(32 * k + j) * ldw + n : (size_t)n * ldw + 32 * k + j;
        w[j] = load_w<WT>(W + idx);
    }
    float y[32];
    if constexpr (TRANSFORM) {
#pragma unroll 4
        for (int j2 = 0; j2 < 32; ++j2) {
            double acc = 0.0;
#pragma unroll
            for (int j = 0; j < 32; ++j) acc = __builtin_fma(sT[j2 * 32 + j], w[j], acc);
            y[j2] = (float)acc;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 32; ++j) y[j] = (float)w[j];
    }
    float bound;
    if (clip_w_max) {
        // Eq. 3-4 as printed: clamp to [r_min * min, r_max * max]; the scale comes from what is left
        float mn = y[0], mx = y[0];
#pragma unroll
        for (int j = 1; j < 32; ++j) {
            mn = __builtin_fminf(mn, y[j]);
            mx = __builtin_fmaxf(mx, y[j]);
        }
        const float lo = clip_w[k] * mn, hi = clip_w_max[k] * mx;
        bound = 0.f;
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            y[j] = clamp_lo_hi(y[j], lo, hi);
            bound = __builtin_fmaxf(bound, __builtin_fabsf(y[j]));
        }
    } else {
        float m = 0.f;
#pragma unroll
        for (int j = 0; j < 32; ++j) m = __builtin_fmaxf(m, __builtin_fabsf(y[j]));
        bound = clip_w ? clip_w[k] * m : m;
    }
    const uint32_t s = e8m0_of_bound(bound);
    const float sc = scale_operand(s);
    uint4 out;
    out.x = encode8(y, bound, sc);
    out.y = encode8(y + 8, bound, sc);
    out.z = encode8(y + 16, bound, sc);
    out.w = encode8(y + 24, bound, sc);
    const int n_out = il_off >= 0 ? 64 * (n >> 5) + il_off + (n & 31) : n;
    *reinterpret_cast<uint4*>(codes + code_chunk_offset(n_out, k, nb)) = out;
    scales[scale_index_internal(n_out, k, N_out)] = (uint8_t)s;
}

}  // namespace

hipError_t launch_prepare_weight(const batq_transform* t, const void* W, batq_dtype wdtype, int K, int N,
                                 int64_t ldw, int w_is_KxN, int N_out, int il_off, const float* d_clip_w,
                                 const float* d_clip_w_max, uint8_t* codes, uint8_t* scales, hipStream_t stream) {
    const int nb = K / 32;
    const dim3 grid((N + 255) / 256, nb), block(256);
    if (wdtype == BATQ_BF16) {
        auto Wp = static_cast<const uint16_t*>(W);
        if (t->has_transform)
            prep_weight_kernel<uint16_t, true><<<grid, block, 0, stream>>>(Wp, ldw, w_is_KxN, N, N_out, il_off, nb, t->d_Tinv,
                                                                           d_clip_w, d_clip_w_max, codes, scales);
        else
            prep_weight_kernel<uint16_t, false><<<grid, block, 0, stream>>>(Wp, ldw, w_is_KxN, N, N_out, il_off, nb, nullptr,
                                                                            d_clip_w, d_clip_w_max, codes, scales);
    } else {
        auto Wp = static_cast<const float*>(W);
        if (t->has_transform)
            prep_weight_kernel<float, true><<<grid, block, 0, stream>>>(Wp, ldw, w_is_KxN, N, N_out, il_off, nb, t->d_Tinv,
                                                                        d_clip_w, d_clip_w_max, codes, scales);
        else
            prep_weight_kernel<float, false><<<grid, block, 0, stream>>>(Wp, ldw, w_is_KxN, N, N_out, il_off, nb, nullptr,
                                                                         d_clip_w, d_clip_w_max, codes, scales);
    }
    return hipGetLastError();
}

}  // namespace batq
