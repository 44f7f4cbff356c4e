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
// A workgroup owns one 256-element K group and keeps its transform operands in LDS; each wave
// owns whole 32-row tiles (512 contiguous bytes per row), so there are no barriers in the
// steady state, and code pieces and scale words leave as whole cache lines.
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

// Mix across the quad: out = sum over source lanes s of coef[s] * (value held by lane s).
#define BATQ_QUAD_MIX(out, v, c0, c1, c2, c3)            \
    do {                                                  \
        out = (c0) * dpp_quad<0x00>(v);                   \
        out = __builtin_fmaf((c1), dpp_quad<0x55>(v), out); \
        out = __builtin_fmaf((c2), dpp_quad<0xAA>(v), out); \
        out = __builtin_fmaf((c3), dpp_quad<0xFF>(v), out); \
    } while (0)

// GO = size of the shared factor G (4 or 8); the private factor is (32/GO) x (32/GO).
// MODE 0: no transform; 1: transform.
template <typename XT, int GO, bool TRANSFORM>
__global__ void __launch_bounds__(256)
quant_act_quad(const XT* __restrict__ X, int64_t ldx, int M, int nb, int rows_per_wg,
               const float* __restrict__ G, const float* __restrict__ P, const float* __restrict__ clip,
               uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
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
        for (int i = 0; i < GI * GI; ++i) Pr[i] = P[(size_t)k * GI * GI + i];
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

    const int row0 = blockIdx.y * rows_per_wg;
    const int row1 = min(M, row0 + rows_per_wg);
    for (int row = row0; row < row1; ++row) {
        float x[8], y[8];
        load8(X + (size_t)row * ldx + (size_t)k * 32 + q * 8, x);
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

        // block amax over the quad's 32 values
        float m = __builtin_fabsf(y[0]);
#pragma unroll
        for (int i = 1; i < 8; ++i) m = __builtin_fmaxf(m, __builtin_fabsf(y[i]));
        m = __builtin_fmaxf(m, dpp_quad<0xB1>(m));
        m = __builtin_fmaxf(m, dpp_quad<0x4E>(m));

        const float bound = ck * m;                     // one fp32 multiply
        const uint32_t s = e8m0_of_bound(bound);
        const uint32_t packed = encode8(y, bound, scale_operand(s));
        if (live) {
            *reinterpret_cast<uint32_t*>(codes + code_chunk_offset(row, k, nb) + q * 4) = packed;
            if (q == 0) scales[scale_index_internal(row, k, M)] = (uint8_t)s;
        } else if (pad) {
            // padding blocks up to the next multiple of 8: zero codes, neutral scale
            *reinterpret_cast<uint32_t*>(codes + code_chunk_offset(row, kpad, nb) + q * 4) = 0u;
            if (q == 0) scales[scale_index_internal(row, kpad, M)] = (uint8_t)127;
        }
    }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Lane layout of the pre-split transform operand (built by the host, see batq_api.hip):
//   Tsplit[k][term][half][lane] = 8 bf16: T_k[16 (lane / 32) + 8 half + e][sigma(lane % 32)], e = 0..7,
//   sigma(m) = 16 ((m >> 2) & 1) + 4 (m >> 3) + (m & 3); terms 0, 1, 2 = hi, mid, lo.
constexpr int kQuantWaves = 8;          // waves per workgroup, each owning whole 32-row tiles
constexpr int kTsplitBlock = 3 * 2 * 64 * 16;               // bytes of pre-split transform operand per MX block

__global__ void __launch_bounds__(kQuantWaves * 64)
quant_act_mfma(const uint16_t* __restrict__ X, int64_t ldx, int M, int nb, int tiles_per_wave,
               const uint4* __restrict__ Tsplit, const float* __restrict__ clip,
               uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
    // A workgroup owns one 256-element K group (8 MX blocks = two 1 KiB piece columns of the code
    // layout and one 8-byte scale word per row).  Its transform operands (48 KiB) are fetched once
    // into LDS; after that every wave works alone, without workgroup barriers: it reads 32 rows x
    // 512 contiguous bytes of X, runs the 8 blocks through the matrix pipe one after the other,
    // collects its four finished code pieces in a private 4 KiB LDS area and writes them, and the
    // 32 scale words, as whole cache lines.
    __shared__ __align__(16) uint8_t tlds[8 * kTsplitBlock];
    __shared__ __align__(16) uint8_t cstage[kQuantWaves][4096];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = blockIdx.x;                               // K group
    const int k0 = g * 8;
    const int nblk = min(8, nb - k0);                       // real blocks in this group (rest is padding)
    const int l32 = lane & 31, kg = lane >> 5;
    const int row_tiles = (M + 31) >> 5;
    const size_t piece_stride = (size_t)code_stages(nb) * 1024;
    uint8_t* const my = cstage[wave];
    const int r16 = l32 & 15;
    // this lane's 8 code bytes of a block inside the wave's staging area [piece column][row group][1 KiB]
    const int st_base = (l32 >> 4) * 1024 + r16 * 64 + 8 * kg;
    const int st_swz = (r16 >> 2) & 3;

    // ---- per-wave work: units of (32-row tile, half K group = 4 blocks = 256 bytes per row); the
    // next unit is loaded into a second register set while the current one is processed
    const int wave_tile0 = (blockIdx.y * kQuantWaves + wave) * tiles_per_wave;
    const int ntiles = max(0, min(tiles_per_wave, row_tiles - wave_tile0));
    const int nunits = 2 * ntiles;
    auto load_unit = [&](int u, uint4 (&x)[4][2]) {
        const int rowc = min((wave_tile0 + (u >> 1)) * 32 + l32, M - 1);   // rows past the end: computed, not stored
        const uint4* xp = reinterpret_cast<const uint4*>(X + (size_t)rowc * ldx + (size_t)(k0 + 4 * (u & 1)) * 32 + 16 * kg);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            if (4 * (u & 1) + b < nblk) {                   // uniform
                x[b][0] = xp[4 * b];
                x[b][1] = xp[4 * b + 1];
            }
        }
    };
    uint4 xc[4][2], xn[4][2];
    if (nunits > 0) load_unit(0, xc);                       // in flight while the operands go to LDS
    {
        // the group's transform operands go global -> LDS with LDS-direct loads (1 KiB per wave
        // instruction, lane i -> LDS base + 16 i), all issued back to back
        typedef __attribute__((address_space(3))) uint8_t lds_byte;
        const uint32_t lds_t = (uint32_t)(uintptr_t)(lds_byte*)tlds;
        const uint8_t* src = reinterpret_cast<const uint8_t*>(Tsplit) + (size_t)k0 * kTsplitBlock;
        const int pieces = nblk * (kTsplitBlock / 1024);   // 6 per block
        for (int p = wave; p < pieces; p += kQuantWaves)
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                         :: "v"((uint32_t)(p * 1024 + lane * 16)), "s"(src), "s"(lds_t + (uint32_t)p * 1024) : "memory");
        __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): operands (and the first X unit) have landed
    }
    __syncthreads();

    uint32_t sc_lo = 0x7F7F7F7Fu, sc_hi = 0x7F7F7F7Fu;     // scale word of the row; padding blocks stay neutral
    for (int u = 0; u < nunits; ++u) {
        const int tile = wave_tile0 + (u >> 1);
        const int half = u & 1;
        if (u + 1 < nunits) load_unit(u + 1, xn);
#pragma unroll
        for (int bb = 0; bb < 4; ++bb) {
            const int b = 4 * half + bb;                    // block inside the K group
            uint2 out = {0u, 0u};                           // padding blocks: zero codes
            if (b < nblk) {
                const uint4* tf = reinterpret_cast<const uint4*>(tlds + b * kTsplitBlock) + lane;
                uint4 tfr[6];
#pragma unroll
                for (int i = 0; i < 6; ++i) tfr[i] = tf[i * 64];
                // two independent accumulation chains (one per K half), smallest terms first
                v16f acc0 = {}, acc1 = {};
#pragma unroll
                for (int t = 2; t >= 0; --t) {
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tfr[t * 2 + 0]),
                                                                   __builtin_bit_cast(bf16x8, xc[bb][0]), acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tfr[t * 2 + 1]),
                                                                   __builtin_bit_cast(bf16x8, xc[bb][1]), acc1, 0, 0, 0);
                }
                // y[r] = transformed element 16 kg + r of this lane's row
                float y[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) y[r] = acc0[r] + acc1[r];
                float m = __builtin_fabsf(y[0]);
#pragma unroll
                for (int r = 1; r < 16; ++r) m = __builtin_fmaxf(m, __builtin_fabsf(y[r]));
                // the other half of the block lives in lane ^ 32
                const float mo = __builtin_bit_cast(
                    float, __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __builtin_bit_cast(int, m)));
                m = __builtin_fmaxf(m, mo);
                const float bound = clip[k0 + b] * m;       // one fp32 multiply
                const uint32_t s = e8m0_of_bound(bound);
                const float sc = scale_operand(s);
                out.x = encode8(y, bound, sc);
                out.y = encode8(y + 8, bound, sc);
                // byte (b/2) + 4 (b%2) of the row's scale word
                const int sh = 8 * (b >> 1);
                if (b & 1) sc_hi = (sc_hi & ~(0xFFu << sh)) | (s << sh);
                else sc_lo = (sc_lo & ~(0xFFu << sh)) | (s << sh);
            }
            *reinterpret_cast<uint2*>(my + half * 2048 + st_base + ((bb ^ st_swz) << 4)) = out;
        }
        // the two finished pieces of this half: (column `half`, rows 0-15) and (column `half`, rows 16-31);
        // the code array is padded to whole 32-row tiles, so both always exist
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const uint4 v = *reinterpret_cast<const uint4*>(my + half * 2048 + p * 1024 + lane * 16);
            *reinterpret_cast<uint4*>(codes + (size_t)(2 * tile + p) * piece_stride + (size_t)(2 * g + half) * 1024 +
                                      lane * 16) = v;
        }
        if (half == 1) {
            const int row = tile * 32 + l32;
            if (kg == 0 && row < M)
                *reinterpret_cast<uint2*>(scales + ((size_t)g * M + row) * 8) = uint2{sc_lo, sc_hi};
            sc_lo = 0x7F7F7F7Fu;
            sc_hi = 0x7F7F7F7Fu;
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            xc[b][0] = xn[b][0];
            xc[b][1] = xn[b][1];
        }
    }
}

hipError_t launch_mfma(const batq_transform* t, const uint16_t* X, int M, int64_t ldx, uint8_t* codes,
                       uint8_t* scales, hipStream_t stream) {
    const int nb = t->nb;
    const int groups = scale_groups(nb);
    const int row_tiles = (M + 31) / 32;
    // a few 32-row tiles per wave amortise the 48 KiB operand fetch of a workgroup; small problems
    // keep one tile per wave so that the grid still covers the chip
    int tiles_per_wave = (int)std::min<long>(4, std::max<long>(1, (long)row_tiles * groups / (512L * kQuantWaves)));
    const int per_wg = kQuantWaves * tiles_per_wave;
    const dim3 grid(groups, (row_tiles + per_wg - 1) / per_wg), block(kQuantWaves * 64);
    quant_act_mfma<<<grid, block, 0, stream>>>(X, ldx, M, nb, tiles_per_wave,
                                               reinterpret_cast<const uint4*>(t->d_Tsplit), t->d_clip, codes, scales);
    return hipGetLastError();
}

template <typename XT>
hipError_t launch_quad(const batq_transform* t, const XT* X, int M, int64_t ldx, uint8_t* codes,
                       uint8_t* scales, hipStream_t stream) {
    const int nb = t->nb;
    const int gx = (scale_groups(nb) * 8 + 63) / 64;
    // aim at >= 4 workgroups per CU while keeping the per-lane factor loads amortised
    int rows_per_wg = 16;
    while (rows_per_wg > 1 && (long)gx * ((M + rows_per_wg - 1) / rows_per_wg) < 2048) rows_per_wg >>= 1;
    while ((M + rows_per_wg - 1) / rows_per_wg > 65535) rows_per_wg <<= 1;      // grid.y limit
    const dim3 grid(gx, (M + rows_per_wg - 1) / rows_per_wg), block(256);
    if (!t->has_transform)
        quant_act_quad<XT, 4, false><<<grid, block, 0, stream>>>(X, ldx, M, nb, rows_per_wg, nullptr, nullptr,
                                                                  t->d_clip, codes, scales);
    else if (t->g_outer == 4)
        quant_act_quad<XT, 4, true><<<grid, block, 0, stream>>>(X, ldx, M, nb, rows_per_wg, t->d_G, t->d_P,
                                                                 t->d_clip, codes, scales);
    else
        quant_act_quad<XT, 8, true><<<grid, block, 0, stream>>>(X, ldx, M, nb, rows_per_wg, t->d_G, t->d_P,
                                                                 t->d_clip, codes, scales);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_quantize_act(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int K,
                               int64_t ldx, uint8_t* codes, uint8_t* scales, hipStream_t stream) {
    (void)K;
    if (M == 0) return hipSuccess;
    if (xdtype == BATQ_BF16) {
        if (t->has_transform && t->d_Tsplit)
            return launch_mfma(t, static_cast<const uint16_t*>(X), M, ldx, codes, scales, stream);
        return launch_quad(t, static_cast<const uint16_t*>(X), M, ldx, codes, scales, stream);
    }
    return launch_quad(t, static_cast<const float*>(X), M, ldx, codes, scales, stream);
}

}  // namespace batq
