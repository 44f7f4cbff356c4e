// MXFP4 x MXFP4 GEMM (the low-bit product of Sec. 3.1: Q(XP) Q(P^-1 W)) on gfx950's
// block-scaled FP4 matrix instruction, fp32 accumulation.
//
// v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in FP4: lane l supplies, for matrix
// row (l % 32), the 32 consecutive K elements of MX block (l / 32) as 16 packed bytes, plus
// that block's E8M0 scale; so one 128-bit read of the [rows][K/2] code layout is exactly one
// operand fragment.  Accumulator register r of lane l is element
// (8*(r/4) + 4*(l/32) + r%4, l % 32) of the 32x32 tile.
//
// Two kernels:
//   gemm_tiled  - 256x256 output tile per workgroup (4 waves, each 128x128 = 4x4 matrix
//                 tiles held in 256 accumulator registers), K stage of 256 elements,
//                 operands staged through LDS (double buffered, XOR-swizzled 16-byte slots),
//                 scales read straight from the group-major internal layout, workgroup ->
//                 tile mapping grouped per XCD so that an XCD's L2 sees a compact sub-grid.
//   gemm_direct - one wave per 32x32 tile with operands straight from global memory, for
//                 problems too small to fill 256x256 tiles.
#include <algorithm>

#include "batq_internal.h"
#include "mxfp4_device.h"
#include "scale_layout.h"

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
    const size_t Kh = (size_t)nb * 16;
    const uint8_t* ap = xc + (size_t)am * Kh + kg * 16;
    const uint8_t* bp = wc + (size_t)bn * Kh + kg * 16;
    v16f acc = {};
    const int steps = nb >> 1;
    for (int s = 0; s < steps; ++s) {
        const uint4 a = *reinterpret_cast<const uint4*>(ap + (size_t)s * 32);
        const uint4 b = *reinterpret_cast<const uint4*>(bp + (size_t)s * 32);
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
            a = *reinterpret_cast<const uint4*>(ap + (size_t)s * 32);
            b = *reinterpret_cast<const uint4*>(bp + (size_t)s * 32);
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
constexpr int kTile = 256;            // output tile edge
constexpr int kStageBytes = 128;      // code bytes per row per K stage (256 elements, 8 MX blocks)
constexpr int kOperandStage = kTile * kStageBytes;   // 32 KiB per operand per stage
constexpr int kTiledLds = 4 * kOperandStage;         // A and B, double buffered

// 16-byte slot swizzle inside a 128-byte LDS row: conflict-free for both the row-strided
// fragment reads (32 rows, one slot) and the row-contiguous staging writes.
__device__ __forceinline__ int slot_swizzle(int row) { return (row & 7) ^ ((row >> 3) & 1); }

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

template <int KK>
__device__ __forceinline__ void mfma_kstep(v16f (&acc)[4][4], const uint4 (&a)[4], const uint4 (&b)[4],
                                           const int (&sa)[4], const int (&sb)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag(a[i]), frag(b[j]), acc[i][j], 4, 4, KK,
                                                                        sa[i], KK, sb[j]);
}

template <typename YT>
__global__ void __launch_bounds__(256, 1)
gemm_tiled(const uint8_t* __restrict__ xc, const uint8_t* __restrict__ xs, const uint8_t* __restrict__ wc,
           const uint8_t* __restrict__ ws, int M, int N, int nb, int tiles_m, int tiles_n,
           YT* __restrict__ Y, int64_t ldy) {
    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t* const As = smem;
    uint8_t* const Bs = smem + 2 * kOperandStage;

    int tm, tn;
    tile_of_workgroup(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int m0 = tm * kTile, n0 = tn * kTile;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, kg = lane >> 5;
    const uint32_t Kh = (uint32_t)nb * 16;
    const int stages = (nb + 7) >> 3;

    // ---- global -> LDS staging: thread t copies 16-byte chunk (t & 7) of rows (t >> 3) + 32 j
    const int lrow = t >> 3, lcc = t & 7;
    const int lds_w = lrow * kStageBytes + ((lcc ^ slot_swizzle(lrow)) << 4);
    uint32_t aoff[8], boff[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        aoff[j] = (uint32_t)min(m0 + lrow + 32 * j, M - 1) * Kh + lcc * 16;
        boff[j] = (uint32_t)min(n0 + lrow + 32 * j, N - 1) * Kh + lcc * 16;
    }
    uint4 ra[8], rb[8];
    auto load_stage = [&](int s) {
        const bool valid = s * 8 + lcc < nb;            // K tail: chunks past the last block are zero
        const uint32_t ko = (uint32_t)s * kStageBytes;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            ra[j] = valid ? *reinterpret_cast<const uint4*>(xc + aoff[j] + ko) : uint4{0, 0, 0, 0};
            rb[j] = valid ? *reinterpret_cast<const uint4*>(wc + boff[j] + ko) : uint4{0, 0, 0, 0};
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            *reinterpret_cast<uint4*>(As + buf * kOperandStage + lds_w + j * 32 * kStageBytes) = ra[j];
            *reinterpret_cast<uint4*>(Bs + buf * kOperandStage + lds_w + j * 32 * kStageBytes) = rb[j];
        }
    };

    // ---- fragment reads: lane reads slot (2 kk + kg) of row (wave row base + 32 i + l32)
    const int fsw = slot_swizzle(l32);
    const int a_rd = (wm * 128 + l32) * kStageBytes;
    const int b_rd = (wn * 128 + l32) * kStageBytes;
    // ---- scales: one dword per fragment per stage (four K steps, selected by op_sel)
    uint32_t sa_idx[4], sb_idx[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        sa_idx[i] = (uint32_t)min(m0 + wm * 128 + 32 * i + l32, M - 1) * 2 + kg;
        sb_idx[i] = (uint32_t)min(n0 + wn * 128 + 32 * i + l32, N - 1) * 2 + kg;
    }
    const uint32_t* xs32 = reinterpret_cast<const uint32_t*>(xs);
    const uint32_t* ws32 = reinterpret_cast<const uint32_t*>(ws);

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v16f{};

    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int s = 0; s < stages; ++s) {
        const int buf = s & 1;
        const bool more = s + 1 < stages;
        if (more) load_stage(s + 1);
        int sa[4], sb[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sa[i] = (int)xs32[(size_t)s * M * 2 + sa_idx[i]];
            sb[i] = (int)ws32[(size_t)s * N * 2 + sb_idx[i]];
        }
        const uint8_t* Ab = As + buf * kOperandStage + a_rd;
        const uint8_t* Bb = Bs + buf * kOperandStage + b_rd;
        uint4 fa[4], fb[4];
#define BATQ_LOAD_FRAGS(KK)                                                                                  \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                          \
        fa[i] = *reinterpret_cast<const uint4*>(Ab + i * 32 * kStageBytes + (((2 * (KK) + kg) ^ fsw) << 4)); \
        fb[i] = *reinterpret_cast<const uint4*>(Bb + i * 32 * kStageBytes + (((2 * (KK) + kg) ^ fsw) << 4)); \
    }
        BATQ_LOAD_FRAGS(0)
        mfma_kstep<0>(acc, fa, fb, sa, sb);
        BATQ_LOAD_FRAGS(1)
        mfma_kstep<1>(acc, fa, fb, sa, sb);
        BATQ_LOAD_FRAGS(2)
        mfma_kstep<2>(acc, fa, fb, sa, sb);
        BATQ_LOAD_FRAGS(3)
        mfma_kstep<3>(acc, fa, fb, sa, sb);
#undef BATQ_LOAD_FRAGS
        if (more) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: accumulators -> Y
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
    const bool fits32 = (size_t)M * nb * 16 < (1ull << 31) && (size_t)N * nb * 16 < (1ull << 31);
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

hipError_t launch_gemm_mxfp4(const uint8_t* xcodes, const uint8_t* xscales_internal, const batq_weight* w, int M,
                             void* Y, batq_dtype ydtype, int64_t ldy, hipStream_t stream) {
    if (M == 0) return hipSuccess;
    if (ydtype == BATQ_BF16)
        return launch_typed<uint16_t>(xcodes, xscales_internal, w, M, static_cast<uint16_t*>(Y), ldy, stream);
    return launch_typed<float>(xcodes, xscales_internal, w, M, static_cast<float*>(Y), ldy, stream);
}

}  // namespace batq
