// batq_ceilings: measures, on the GPU it runs on, the practical ceilings that the two hot
// kernels of libbatq are judged against, next to the data-sheet peaks:
//   - the block-scaled FP4 matrix instruction issued back to back from registers (no memory
//     traffic at all), with constant and with random operand bits: the matrix pipe is
//     power-limited, so the sustainable rate depends on how many operand bits toggle;
//   - streaming HBM reads, a plain copy, and a read:write mix in the ratio of the activation
//     quantiser (2 bytes in, 0.53 bytes out per element), over buffers larger than the
//     last-level cache.
// The copy kernel doubles as the known-size reference for scaling hardware traffic counters.
// Prints one JSON object.  Standalone: uses nothing from the library.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

#define CK(x)                                                                        \
    do {                                                                             \
        hipError_t e_ = (x);                                                         \
        if (e_ != hipSuccess) {                                                      \
            fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            exit(1);                                                                 \
        }                                                                            \
    } while (0)

// 16 independent accumulators per wave, one wave per SIMD: the shape of the GEMM's inner loop.
__global__ void __launch_bounds__(256, 1)
mfma_loop(const v8i* __restrict__ a, const v8i* __restrict__ b, v16f* __restrict__ sink, int iters) {
    const int t = threadIdx.x & 63;
    const v8i A = a[t], B = b[t];
    v16f acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = v16f{};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, acc[i], 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][0];
    if (s == 12345.678f) sink[0] = acc[0];      // never true; keeps the loop alive
}

__global__ void __launch_bounds__(256)
batq_ceilings_copy(const uint4* __restrict__ in, uint4* __restrict__ out, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) out[i] = in[i];
}

__global__ void __launch_bounds__(256)
stream_read(const uint4* __restrict__ in, uint4* __restrict__ sink, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint4 acc = {0, 0, 0, 0};
    for (; i < n; i += stride) {
        const uint4 v = in[i];
        acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
    if (acc.x == 0x12345u && acc.y == 0x777u) sink[0] = acc;
}

// reads 64 bytes, writes 16 + 1 bytes per thread-iteration: the quantiser's 2 : 0.53 byte ratio
__global__ void __launch_bounds__(256)
stream_quant_mix(const uint4* __restrict__ in, uint4* __restrict__ out, uint8_t* __restrict__ out8, size_t nout) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < nout; i += stride) {
        const uint4 a = in[i], b = in[i + nout], c = in[i + 2 * nout], d = in[i + 3 * nout];
        uint4 r;
        r.x = a.x ^ b.x ^ c.x ^ d.x; r.y = a.y ^ b.y ^ c.y ^ d.y;
        r.z = a.z ^ b.z ^ c.z ^ d.z; r.w = a.w ^ b.w ^ c.w ^ d.w;
        out[i] = r;
        out8[i] = (uint8_t)r.x;
    }
}

int main() {
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    auto elapsed_ms = [&]() {
        float ms;
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        return (double)ms;
    };

    // ---- matrix pipe
    v8i *da, *db;
    v16f* dsink;
    CK(hipMalloc(&da, 64 * 32));
    CK(hipMalloc(&db, 64 * 32));
    CK(hipMalloc(&dsink, 4096));
    double mfma_tflops[2];
    const int blocks = prop.multiProcessorCount, iters = 4000;
    for (int pat = 0; pat < 2; ++pat) {
        std::vector<uint32_t> h(512);
        uint32_t lcg = 12345u;
        for (auto& x : h) {
            lcg = lcg * 1664525u + 1013904223u;
            x = pat == 0 ? 0x22222222u : lcg;
        }
        CK(hipMemcpy(da, h.data(), 2048, hipMemcpyHostToDevice));
        for (auto& x : h) {
            lcg = lcg * 1664525u + 1013904223u;
            x = pat == 0 ? 0x22222222u : lcg;
        }
        CK(hipMemcpy(db, h.data(), 2048, hipMemcpyHostToDevice));
        mfma_loop<<<blocks, 256>>>(da, db, dsink, 50);
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0));
        mfma_loop<<<blocks, 256>>>(da, db, dsink, iters);
        CK(hipEventRecord(e1));
        const double ms = elapsed_ms();
        mfma_tflops[pat] = (double)blocks * 4 * iters * 16 * 2.0 * 32 * 32 * 64 / ms / 1e9;
    }

    // ---- memory: six buffer pairs of 112 MiB in, 28 MiB + 1.75 MiB out (> 2x the 256 MB cache)
    const int NB = 6;
    const size_t rbytes = (size_t)112 << 20, wbytes = rbytes / 4;
    uint4 *in[NB], *out[NB];
    uint8_t* out8[NB];
    for (int i = 0; i < NB; ++i) {
        CK(hipMalloc(&in[i], rbytes));
        CK(hipMemset(in[i], i + 1, rbytes));
        CK(hipMalloc(&out[i], rbytes));
        CK(hipMemset(out[i], 0, rbytes));
        CK(hipMalloc(&out8[i], wbytes / 16));
    }
    auto time_loop = [&](auto launch) {
        launch(0);
        CK(hipDeviceSynchronize());
        const int reps = 12;
        CK(hipEventRecord(e0));
        for (int r = 0; r < reps; ++r) launch(r % NB);
        CK(hipEventRecord(e1));
        return elapsed_ms() / reps;
    };
    const double ms_read = time_loop([&](int b) { stream_read<<<4096, 256>>>(in[b], (uint4*)dsink, rbytes / 16); });
    const double ms_copy = time_loop([&](int b) { batq_ceilings_copy<<<8192, 256>>>(in[b], out[b], rbytes / 16); });
    const double ms_mix = time_loop(
        [&](int b) { stream_quant_mix<<<8192, 256>>>(in[b], out[b], out8[b], wbytes / 16); });
    const double mix_bytes = (double)rbytes + wbytes + wbytes / 16;

    printf("{\"device\": \"%s\", \"compute_units\": %d, "
           "\"mfma_fp4_32x32x64_tflops_const_operands\": %.0f, \"mfma_fp4_32x32x64_tflops_random_operands\": %.0f, "
           "\"hbm_stream_read_gbs\": %.0f, \"hbm_copy_gbs\": %.0f, \"copy_bytes_each_way\": %zu, "
           "\"hbm_quant_mix_gbs\": %.0f}\n",
           prop.gcnArchName, prop.multiProcessorCount, mfma_tflops[0], mfma_tflops[1], rbytes / ms_read / 1e6,
           2.0 * rbytes / ms_copy / 1e6, rbytes, mix_bytes / ms_mix / 1e6);
    return 0;
}
