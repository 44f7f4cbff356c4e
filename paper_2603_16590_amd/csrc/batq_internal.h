// Internal declarations of libbatq: handle layouts and kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include "../../include/batq.h"

namespace batq {

constexpr int kBlock = 32;   // MXFP block size (Sec. 2, MXFP definition)

}  // namespace batq

// Learned parameters of one transform set, host-validated and resident on the device.
struct batq_transform {
    int K = 0, nb = 0;
    int form = BATQ_FORM_IDENTITY;
    int g_outer = 4, g_inner = 8;
    bool has_transform = false;   // form != identity
    bool minmax = false;          // two-ratio clipping (d_clip = ratios on the block minimum, d_clip_max on the maximum)
    // Kronecker forms: factors as given; stride = elements between consecutive blocks (0: shared)
    float* d_outer = nullptr;
    float* d_inner = nullptr;
    int outer_stride = 0, inner_stride = 0;
    float* d_T = nullptr;         // dense form: [nb][32][32] fp32 forward blocks
    float* d_clip = nullptr;      // [nb], 1.0 when no clipping
    float* d_clip_max = nullptr;  // [nb], only when minmax
    double* d_Tinv = nullptr;     // [nb][32][32] fp64 T_k^-1     (null when !has_transform)
    double* d_Tf64 = nullptr;     // [nb][32][32] fp64 T_k        (null when !has_transform)
    uint16_t* d_Tsplit = nullptr; // [nb][3][2][64][8] bf16 three-term split of T_k in MFMA operand order
    uint16_t* d_TinvSplit = nullptr;   // the same split of T_k^-1
    uint16_t* d_TinvTSplit = nullptr;  // and of T_k^-T
};

// Prepared (inverse-transformed, quantised) weights.
struct batq_weight {
    int K = 0, N = 0, nb = 0;
    int cus = 0;                  // compute units of the device the weight lives on
    uint8_t* d_codes = nullptr;   // blocked code layout (code_layout.h), rows and K zero-padded
    uint8_t* d_scales = nullptr;  // internal group-major layout (scale_layout.h), padded groups
};

namespace batq {

// Per-device facts the launch code needs, looked up once per device and safe to use from several host threads
// (the values are idempotent, so a race between two first calls only repeats the lookup).
constexpr int kMaxDevices = 64;

// Compute units of `dev` (hipDeviceAttributeMultiprocessorCount); 0 with *err set on failure.
inline int device_compute_units(int dev, hipError_t* err) {
    static std::atomic<int> cus[kMaxDevices];
    *err = hipSuccess;
    const bool cached = dev >= 0 && dev < kMaxDevices;
    int n = cached ? cus[dev].load(std::memory_order_relaxed) : 0;
    if (n > 0) return n;
    *err = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (*err != hipSuccess) return 0;
    if (cached) cus[dev].store(n, std::memory_order_relaxed);
    return n;
}

// Raises the dynamic-LDS limit of `Kernel` to `bytes` on the current device, once per device and kernel.
template <auto Kernel>
inline hipError_t ensure_dynamic_lds(int dev, int bytes) {
    static std::atomic<bool> done[kMaxDevices];
    const bool cached = dev >= 0 && dev < kMaxDevices;
    if (cached && done[dev].load(std::memory_order_acquire)) return hipSuccess;
    const hipError_t e =
        hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && cached) done[dev].store(true, std::memory_order_release);
    return e;
}

// Each launcher validates nothing: callers (the C ABI) have checked shapes already.
// Codes are written in the blocked layout of code_layout.h (fp8: MXFP8 codes in its 8-bit variant),
// scales in the grouped layout of scale_layout.h (padding blocks of the last K group included).
// row_scale: DEVICE fp32 [M] or null; each transformed row is multiplied by its factor before clipping.
// U: DEVICE tensor like X (same dtype, row stride ldu) or null; with U the input is bf16(silu(X) * U).
hipError_t launch_quantize_act(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int K,
                               int64_t ldx, const void* U, int64_t ldu, const float* row_scale, uint8_t* codes,
                               uint8_t* scales, bool fp8, int row_offset, int layout_rows, hipStream_t stream);
// Blocked codes (fp8: the 8-bit variant) + grouped scales -> row-major out (bf16 or fp32, row stride ldo).
hipError_t launch_dequantize(const uint8_t* codes, const uint8_t* scales, int M, int nb, bool fp8, void* out,
                             batq_dtype odtype, int64_t ldo, int row_offset, int layout_rows, hipStream_t stream);
// out = X T_k, X T_k^-1 or X T_k^-T block by block (mode = batq_apply_mode), no quantisation.
hipError_t launch_transform_apply(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int64_t ldx,
                                  int mode, void* out, batq_dtype odtype, int64_t ldo, hipStream_t stream);
hipError_t launch_row_rms_scale(const void* X, batq_dtype xdtype, int M, int K, int64_t ldx, float eps, float* out,
                                hipStream_t stream);
hipError_t launch_prepare_weight(const batq_transform* t, const void* W, batq_dtype wdtype, int K, int N,
                                 int64_t ldw, int w_is_KxN, int N_out, int il_off, const float* d_clip_w,
                                 const float* d_clip_w_max, uint8_t* codes, uint8_t* scales, hipStream_t stream);
// N_out / il_off: rows of the prepared weight and the interleave offset (-1: column n -> row n; 0 / 32: gate /
// up columns of an MLP interleaved in groups of 32, N_out = 2 N).
// d_clip_w_max != null selects the two-ratio clipping (d_clip_w then holds the ratios on the minimum).
// Weight scales are written in the internal layout (pad bytes must have been set to 127).
// xscales_internal: activation scales in the grouped layout.
// glu: gated output, Y = silu(gate) * up is M x N/2 for a weight with interleaved gate / up columns
// (gemm_glu_supported says whether the shapes allow it).
// parts / parts_bytes: DEVICE memory (256-byte aligned) for the partial sums of K parts, or null / 0; how many
// K parts run depends on the shape, the device and parts_bytes only (never on the stream or on earlier calls).
hipError_t launch_gemm_mxfp4(const uint8_t* xcodes, const uint8_t* xscales_internal, const batq_weight* w, int M,
                             void* Y, batq_dtype ydtype, int64_t ldy, bool a8, bool glu, void* parts,
                             size_t parts_bytes, hipStream_t stream);
// Partial-sum bytes with which the GEMM of M rows against `w` runs all the K parts it wants (0: it wants none).
size_t gemm_workspace_bytes(const batq_weight* w, int M, bool a8, int compute_units);
// The per-device partial-sum array of the allocation-free entry point (kStaticScratchBytes bytes, 256-byte
// aligned) on the current device; its address is looked up once per device.  64 KiB per compute unit is the
// most a GEMM's K parts ask for, so 16 MiB serves every shape on 256 compute units.
constexpr size_t kStaticScratchBytes = size_t(16) << 20;
hipError_t static_scratch(void** ptr);
bool gemm_glu_supported(const batq_weight* w, int M, bool a8);
// Host replay of the tiled kernels' work split: 7 ints per tile (workgroup, first row, first column, strips, K part,
// first K group, K groups) into out[capacity * 7]; returns the number of tiles.
int tile_schedule(int M, int N, int K, int compute_units, bool glu, bool allow_ksplit, int* out, int capacity);
hipError_t launch_codes8_to_blocked(const uint8_t* rowmajor, uint8_t* blocked, int rows, int nb, hipStream_t stream);
hipError_t launch_codes8_to_rowmajor(const uint8_t* blocked, uint8_t* rowmajor, int rows, int nb, hipStream_t stream);
hipError_t launch_codes_to_blocked(const uint8_t* rowmajor, uint8_t* blocked, int rows, int nb, hipStream_t stream);
hipError_t launch_codes_to_rowmajor(const uint8_t* blocked, uint8_t* rowmajor, int rows, int nb, hipStream_t stream);
hipError_t launch_scales_to_internal(const uint8_t* canon, uint8_t* internal, int rows, int nb, hipStream_t stream);
hipError_t launch_scales_to_canonical(const uint8_t* internal, uint8_t* canon, int rows, int nb, hipStream_t stream);

}  // namespace batq
