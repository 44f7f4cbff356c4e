// C ABI of libbatq: argument validation, handle management, host-side fp64 inversion of
// the Kronecker factors (Alg. 2 uses A^-1 and B_i^-1 for the weight side).
#include <atomic>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "batq_internal.h"
#include "code_layout.h"
#include "scale_layout.h"

namespace {

#define BATQ_HIP(expr)                                   \
    do {                                                 \
        if ((expr) != hipSuccess) {                      \
            (void)hipGetLastError();                     \
            return BATQ_ERR_DEVICE;                      \
        }                                                \
    } while (0)

// In-place fp64 Gauss-Jordan inverse with partial pivoting of an n x n row-major matrix.
bool invert_small(const double* A, int n, double* inv) {
    std::vector<double> a(A, A + n * n);
    double amax = 0.0;
    for (double v : a) amax = std::fmax(amax, std::fabs(v));
    if (!(amax > 0.0) || !std::isfinite(amax)) return false;
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) inv[i * n + j] = (i == j) ? 1.0 : 0.0;
    for (int col = 0; col < n; ++col) {
        int piv = col;
        for (int r = col + 1; r < n; ++r)
            if (std::fabs(a[r * n + col]) > std::fabs(a[piv * n + col])) piv = r;
        if (!(std::fabs(a[piv * n + col]) >= 1e-12 * amax)) return false;
        if (piv != col)
            for (int j = 0; j < n; ++j) {
                std::swap(a[piv * n + j], a[col * n + j]);
                std::swap(inv[piv * n + j], inv[col * n + j]);
            }
        const double d = 1.0 / a[col * n + col];
        for (int j = 0; j < n; ++j) {
            a[col * n + j] *= d;
            inv[col * n + j] *= d;
        }
        for (int r = 0; r < n; ++r) {
            if (r == col) continue;
            const double f = a[r * n + col];
            if (f == 0.0) continue;
            for (int j = 0; j < n; ++j) {
                a[r * n + j] -= f * a[col * n + j];
                inv[r * n + j] -= f * inv[col * n + j];
            }
        }
    }
    return true;
}

uint16_t bf16_rne(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

float bf16_value(uint16_t b) {
    const uint32_t u = (uint32_t)b << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// A block-diagonal matrix B (Mat[k] = B_k as [in][out], or its transpose with `transposed`) split into three
// bf16 terms (hi, mid, lo) in the lane order of the 32x32x16 matrix instruction's first operand:
//   out[k][term][half][lane][e] = B_k[16 (lane / 32) + 8 half + e][sigma(lane % 32)],
//   sigma(m) = 16 ((m >> 2) & 1) + 4 (m >> 3) + (m & 3),
// so that a lane's 16 results of a product with a 32-row tile are 16 consecutive output columns of its row.
std::vector<uint16_t> split_operand(const std::vector<double>& Mat, int nb, bool transposed) {
    std::vector<uint16_t> out((size_t)nb * 3 * 2 * 64 * 8);
    for (int k = 0; k < nb; ++k)
        for (int half = 0; half < 2; ++half)
            for (int lane = 0; lane < 64; ++lane)
                for (int e = 0; e < 8; ++e) {
                    const int m = lane & 31;
                    const int out_col = 16 * ((m >> 2) & 1) + 4 * (m >> 3) + (m & 3);
                    const int in_col = 16 * (lane >> 5) + 8 * half + e;
                    double rest = transposed ? Mat[(size_t)k * 1024 + out_col * 32 + in_col]
                                             : Mat[(size_t)k * 1024 + in_col * 32 + out_col];
                    for (int term = 0; term < 3; ++term) {
                        const uint16_t b = bf16_rne((float)rest);
                        rest -= (double)bf16_value(b);
                        out[((((size_t)k * 3 + term) * 2 + half) * 64 + lane) * 8 + e] = b;
                    }
                }
    return out;
}

bool clip_ok(const float* c, int n) {
    for (int i = 0; i < n; ++i)
        if (!(c[i] > 0.0f && c[i] <= 1.0f)) return false;
    return true;
}

bool dtype_ok(batq_dtype d) { return d == BATQ_F32 || d == BATQ_BF16; }
size_t dtype_size(batq_dtype d) { return d == BATQ_BF16 ? 2 : 4; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// BATQ_OK if the current device is a gfx950; looked up once per device.
batq_status check_device() {
    static std::atomic<int> state[batq::kMaxDevices];   // 0 unknown, 1 ok, 2 bad
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return BATQ_ERR_DEVICE;
    }
    const bool cached = dev >= 0 && dev < batq::kMaxDevices;
    int st = cached ? state[dev].load(std::memory_order_relaxed) : 0;
    if (st == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) {
            (void)hipGetLastError();
            return BATQ_ERR_DEVICE;
        }
        st = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 2;
        if (cached) state[dev].store(st, std::memory_order_relaxed);
    }
    return st == 1 ? BATQ_OK : BATQ_ERR_DEVICE;
}

template <typename T>
batq_status upload(T** dst, const T* src, size_t count) {
    if (hipMalloc(reinterpret_cast<void**>(dst), count * sizeof(T)) != hipSuccess) {
        (void)hipGetLastError();
        *dst = nullptr;
        return BATQ_ERR_ALLOC;
    }
    BATQ_HIP(hipMemcpy(*dst, src, count * sizeof(T), hipMemcpyHostToDevice));
    return BATQ_OK;
}

void free_transform(batq_transform* t) {
    if (!t) return;
    if (t->d_outer) (void)hipFree(t->d_outer);
    if (t->d_inner) (void)hipFree(t->d_inner);
    if (t->d_T) (void)hipFree(t->d_T);
    if (t->d_clip) (void)hipFree(t->d_clip);
    if (t->d_clip_max) (void)hipFree(t->d_clip_max);
    if (t->d_Tinv) (void)hipFree(t->d_Tinv);
    if (t->d_Tf64) (void)hipFree(t->d_Tf64);
    if (t->d_Tsplit) (void)hipFree(t->d_Tsplit);
    if (t->d_TinvSplit) (void)hipFree(t->d_TinvSplit);
    if (t->d_TinvTSplit) (void)hipFree(t->d_TinvTSplit);
    delete t;
}

void free_weight(batq_weight* w) {
    if (!w) return;
    if (w->d_codes) (void)hipFree(w->d_codes);
    if (w->d_scales) (void)hipFree(w->d_scales);
    delete w;
}

batq_status alloc_weight(batq_weight** out, int K, int N) {
    batq_weight* w = new (std::nothrow) batq_weight;
    if (!w) return BATQ_ERR_ALLOC;
    w->K = K;
    w->N = N;
    w->nb = K / 32;
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) w->cus = batq::device_compute_units(dev, &e);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            delete w;
            return BATQ_ERR_DEVICE;
        }
    }
    {
        void* unused = nullptr;                             // first use of the device: resolve the static scratch array
        if (batq::static_scratch(&unused) != hipSuccess) (void)hipGetLastError();
    }
    if (hipMalloc(reinterpret_cast<void**>(&w->d_codes), batq::code_bytes_blocked(N, K / 32)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void**>(&w->d_scales), batq::scale_bytes_internal(N, K / 32)) != hipSuccess) {
        (void)hipGetLastError();
        free_weight(w);
        return BATQ_ERR_ALLOC;
    }
    *out = w;
    return BATQ_OK;
}

}  // namespace

extern "C" {

const char* batq_status_string(batq_status s) {
    switch (s) {
        case BATQ_OK: return "ok";
        case BATQ_ERR_NULL: return "null pointer";
        case BATQ_ERR_SHAPE: return "bad shape, stride or alignment";
        case BATQ_ERR_DTYPE: return "unknown dtype";
        case BATQ_ERR_UNSUPPORTED: return "unsupported Kronecker split";
        case BATQ_ERR_SINGULAR: return "transform factor is singular";
        case BATQ_ERR_CLIP_RANGE: return "clip ratio outside (0, 1]";
        case BATQ_ERR_WORKSPACE: return "workspace too small";
        case BATQ_ERR_ALLOC: return "allocation failed";
        case BATQ_ERR_DEVICE: return "HIP error or device is not gfx950";
        case BATQ_ERR_MISMATCH: return "transform and weight disagree on K";
    }
    return "unknown status";
}

const char* batq_version(void) { return "0.1"; }

batq_status batq_transform_create_ex(batq_transform** out, const batq_transform_desc* d) {
    if (!out || !d) return BATQ_ERR_NULL;
    const int K = d->K;
    if (K <= 0 || K % 32 != 0) return BATQ_ERR_SHAPE;
    const int nb = K / 32;
    const int form = d->form;
    if (form != BATQ_FORM_IDENTITY && form != BATQ_FORM_KRON && form != BATQ_FORM_DENSE) return BATQ_ERR_UNSUPPORTED;
    const int go = d->g_outer, gi = d->g_inner;
    if (form == BATQ_FORM_KRON) {
        if (!((go == 4 && gi == 8) || (go == 8 && gi == 4))) return BATQ_ERR_UNSUPPORTED;
        if (!d->outer || !d->inner) return BATQ_ERR_NULL;
    }
    if (form == BATQ_FORM_DENSE && !d->dense) return BATQ_ERR_NULL;
    if ((d->clip_min == nullptr) != (d->clip_max == nullptr)) return BATQ_ERR_NULL;
    if (d->clip && d->clip_min) return BATQ_ERR_UNSUPPORTED;
    if (d->clip && !clip_ok(d->clip, nb)) return BATQ_ERR_CLIP_RANGE;
    if (d->clip_min && (!clip_ok(d->clip_min, nb) || !clip_ok(d->clip_max, nb))) return BATQ_ERR_CLIP_RANGE;

    // host fp64: the dense forward blocks T_k, their inverses (from the inverted factors for the
    // Kronecker forms, T_k^-1 = O_k^-1 (x) I_k^-1), and T_k split into three bf16 terms in the lane
    // order of the activation kernel's matrix-instruction operand
    std::vector<double> T, Tinv;
    std::vector<float> Tf;
    std::vector<uint16_t> Tsplit, TinvSplit, TinvTSplit;
    if (form != BATQ_FORM_IDENTITY) {
        T.resize((size_t)nb * 1024);
        Tinv.resize((size_t)nb * 1024);
        if (form == BATQ_FORM_KRON) {
            std::vector<double> Od(go * go), Oinv(go * go), Id(gi * gi), Iinv(gi * gi);
            for (int k = 0; k < nb; ++k) {
                const float* O = d->outer + (d->outer_per_block ? (size_t)k * go * go : 0);
                const float* I = d->inner + (d->inner_per_block ? (size_t)k * gi * gi : 0);
                if (k == 0 || d->outer_per_block) {
                    for (int i = 0; i < go * go; ++i) Od[i] = O[i];
                    if (!invert_small(Od.data(), go, Oinv.data())) return BATQ_ERR_SINGULAR;
                }
                if (k == 0 || d->inner_per_block) {
                    for (int i = 0; i < gi * gi; ++i) Id[i] = I[i];
                    if (!invert_small(Id.data(), gi, Iinv.data())) return BATQ_ERR_SINGULAR;
                }
                double* Tk = T.data() + (size_t)k * 1024;
                double* Tik = Tinv.data() + (size_t)k * 1024;
                for (int a = 0; a < go; ++a)
                    for (int c = 0; c < gi; ++c)
                        for (int a2 = 0; a2 < go; ++a2)
                            for (int c2 = 0; c2 < gi; ++c2) {
                                Tk[(a * gi + c) * 32 + a2 * gi + c2] = Od[a * go + a2] * Id[c * gi + c2];
                                Tik[(a * gi + c) * 32 + a2 * gi + c2] = Oinv[a * go + a2] * Iinv[c * gi + c2];
                            }
            }
        } else {
            Tf.assign(d->dense, d->dense + (size_t)nb * 1024);
            for (size_t i = 0; i < T.size(); ++i) T[i] = d->dense[i];
            for (int k = 0; k < nb; ++k)
                if (!invert_small(T.data() + (size_t)k * 1024, 32, Tinv.data() + (size_t)k * 1024))
                    return BATQ_ERR_SINGULAR;
        }
        Tsplit = split_operand(T, nb, false);
        TinvSplit = split_operand(Tinv, nb, false);
        TinvTSplit = split_operand(Tinv, nb, true);
    }

    batq_status st = check_device();
    if (st != BATQ_OK) return st;
    batq_transform* t = new (std::nothrow) batq_transform;
    if (!t) return BATQ_ERR_ALLOC;
    t->K = K;
    t->nb = nb;
    t->form = form;
    t->has_transform = form != BATQ_FORM_IDENTITY;
    t->minmax = d->clip_min != nullptr;
    std::vector<float> clip(nb, 1.0f);
    if (d->clip) std::memcpy(clip.data(), d->clip, sizeof(float) * nb);
    if (d->clip_min) std::memcpy(clip.data(), d->clip_min, sizeof(float) * nb);
    st = upload(&t->d_clip, clip.data(), (size_t)nb);
    if (st == BATQ_OK && d->clip_max) st = upload(&t->d_clip_max, d->clip_max, (size_t)nb);
    if (st == BATQ_OK && form == BATQ_FORM_KRON) {
        t->g_outer = go;
        t->g_inner = gi;
        t->outer_stride = d->outer_per_block ? go * go : 0;
        t->inner_stride = d->inner_per_block ? gi * gi : 0;
        st = upload(&t->d_outer, d->outer, (size_t)(d->outer_per_block ? nb : 1) * go * go);
        if (st == BATQ_OK) st = upload(&t->d_inner, d->inner, (size_t)(d->inner_per_block ? nb : 1) * gi * gi);
    }
    if (st == BATQ_OK && form == BATQ_FORM_DENSE) st = upload(&t->d_T, Tf.data(), Tf.size());
    if (st == BATQ_OK && t->has_transform) {
        st = upload(&t->d_Tinv, Tinv.data(), Tinv.size());
        if (st == BATQ_OK) st = upload(&t->d_Tf64, T.data(), T.size());
        if (st == BATQ_OK) st = upload(&t->d_Tsplit, Tsplit.data(), Tsplit.size());
        if (st == BATQ_OK) st = upload(&t->d_TinvSplit, TinvSplit.data(), TinvSplit.size());
        if (st == BATQ_OK) st = upload(&t->d_TinvTSplit, TinvTSplit.data(), TinvTSplit.size());
    }
    if (st != BATQ_OK) {
        free_transform(t);
        return st;
    }
    *out = t;
    return BATQ_OK;
}

batq_status batq_transform_create(batq_transform** out, int K, int g_outer, int g_inner, const float* G,
                                  const float* P, const float* clip_a) {
    if (!out) return BATQ_ERR_NULL;
    if (K <= 0 || K % 32 != 0) return BATQ_ERR_SHAPE;
    if (!((g_outer == 4 && g_inner == 8) || (g_outer == 8 && g_inner == 4))) return BATQ_ERR_UNSUPPORTED;
    if ((G == nullptr) != (P == nullptr)) return BATQ_ERR_NULL;
    batq_transform_desc d = {};
    d.K = K;
    d.form = G ? BATQ_FORM_KRON : BATQ_FORM_IDENTITY;
    d.g_outer = g_outer;
    d.g_inner = g_inner;
    d.outer = G;
    d.outer_per_block = 0;
    d.inner = P;
    d.inner_per_block = 1;
    d.clip = clip_a;
    return batq_transform_create_ex(out, &d);
}

batq_status batq_transform_destroy(batq_transform* t) {
    if (!t) return BATQ_ERR_NULL;
    free_transform(t);
    return BATQ_OK;
}

}  // extern "C"

namespace {

// clip_a / clip_b: symmetric ratios in clip_a (clip_b null), or the ratios on the block minimum and
// maximum (two_ratio).
// W_up != null: W is the gate projection and W_up the up projection (same shape and layout); the prepared
// weight has 2 N rows, gate and up interleaved in groups of 32.
batq_status prepare_weight_impl(batq_weight** out, const batq_transform* t, const void* W, const void* W_up,
                                batq_dtype wdtype, int K, int N, int64_t ldw, int w_is_KxN, const float* clip_a,
                                const float* clip_b, bool two_ratio, void* stream) {
    if (!out || !t || !W) return BATQ_ERR_NULL;
    if (W_up && N % 32 != 0) return BATQ_ERR_SHAPE;
    const int N_out = W_up ? 2 * N : N;
    if (two_ratio && (!clip_a || !clip_b)) return BATQ_ERR_NULL;
    if (!dtype_ok(wdtype)) return BATQ_ERR_DTYPE;
    if (K <= 0 || N <= 0 || K % 32 != 0) return BATQ_ERR_SHAPE;
    if (ldw < (w_is_KxN ? N : K)) return BATQ_ERR_SHAPE;
    if (t->K != K) return BATQ_ERR_MISMATCH;
    const int nb = K / 32;
    if (clip_a && !clip_ok(clip_a, nb)) return BATQ_ERR_CLIP_RANGE;
    if (clip_b && !clip_ok(clip_b, nb)) return BATQ_ERR_CLIP_RANGE;
    batq_status st = check_device();
    if (st != BATQ_OK) return st;

    hipStream_t s = static_cast<hipStream_t>(stream);
    batq_weight* w = nullptr;
    st = alloc_weight(&w, K, N_out);
    if (st != BATQ_OK) return st;
    float* d_clip_a = nullptr;
    float* d_clip_b = nullptr;
    if (clip_a) st = upload(&d_clip_a, clip_a, (size_t)nb);
    if (st == BATQ_OK && clip_b) st = upload(&d_clip_b, clip_b, (size_t)nb);
    if (st != BATQ_OK) {
        if (d_clip_a) (void)hipFree(d_clip_a);
        free_weight(w);
        return st;
    }
    // padding: zero codes (rows up to a multiple of 16, K up to a multiple of 256), neutral scales
    hipError_t e = hipMemsetAsync(w->d_scales, 127, batq::scale_bytes_internal(N_out, nb), s);
    if (e == hipSuccess) e = hipMemsetAsync(w->d_codes, 0, batq::code_bytes_blocked(N_out, nb), s);
    if (e == hipSuccess)
        e = batq::launch_prepare_weight(t, W, wdtype, K, N, ldw, w_is_KxN, N_out, W_up ? 0 : -1, d_clip_a, d_clip_b,
                                        w->d_codes, w->d_scales, s);
    if (e == hipSuccess && W_up)
        e = batq::launch_prepare_weight(t, W_up, wdtype, K, N, ldw, w_is_KxN, N_out, 32, d_clip_a, d_clip_b,
                                        w->d_codes, w->d_scales, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (d_clip_a) (void)hipFree(d_clip_a);
    if (d_clip_b) (void)hipFree(d_clip_b);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        free_weight(w);
        return BATQ_ERR_DEVICE;
    }
    *out = w;
    return BATQ_OK;
}

}  // namespace

extern "C" {

batq_status batq_prepare_weight(batq_weight** out, const batq_transform* t, const void* W, batq_dtype wdtype,
                                int K, int N, int64_t ldw, int w_is_KxN, const float* clip_w, void* stream) {
    return prepare_weight_impl(out, t, W, nullptr, wdtype, K, N, ldw, w_is_KxN, clip_w, nullptr, false, stream);
}

batq_status batq_prepare_weight_gate_up(batq_weight** out, const batq_transform* t, const void* W_gate,
                                        const void* W_up, batq_dtype wdtype, int K, int F, int64_t ldw,
                                        int w_is_KxN, const float* clip_w, void* stream) {
    if (!W_up) return BATQ_ERR_NULL;
    return prepare_weight_impl(out, t, W_gate, W_up, wdtype, K, F, ldw, w_is_KxN, clip_w, nullptr, false, stream);
}

batq_status batq_prepare_weight_minmax(batq_weight** out, const batq_transform* t, const void* W,
                                       batq_dtype wdtype, int K, int N, int64_t ldw, int w_is_KxN,
                                       const float* clip_w_min, const float* clip_w_max, void* stream) {
    return prepare_weight_impl(out, t, W, nullptr, wdtype, K, N, ldw, w_is_KxN, clip_w_min, clip_w_max, true, stream);
}

batq_status batq_weight_export(const batq_weight* w, uint8_t* codes, uint8_t* scales, void* stream) {
    if (!w || !codes || !scales) return BATQ_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    BATQ_HIP(batq::launch_codes_to_rowmajor(w->d_codes, codes, w->N, w->nb, s));
    BATQ_HIP(batq::launch_scales_to_canonical(w->d_scales, scales, w->N, w->nb, s));
    return BATQ_OK;
}

batq_status batq_weight_import(batq_weight** out, const uint8_t* codes, const uint8_t* scales, int K, int N,
                               void* stream) {
    if (!out || !codes || !scales) return BATQ_ERR_NULL;
    if (K <= 0 || N <= 0 || K % 32 != 0) return BATQ_ERR_SHAPE;
    batq_status st = check_device();
    if (st != BATQ_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    batq_weight* w = nullptr;
    st = alloc_weight(&w, K, N);
    if (st != BATQ_OK) return st;
    hipError_t e = hipMemsetAsync(w->d_codes, 0, batq::code_bytes_blocked(N, K / 32), s);
    if (e == hipSuccess) e = batq::launch_codes_to_blocked(codes, w->d_codes, N, K / 32, s);
    if (e == hipSuccess) e = batq::launch_scales_to_internal(scales, w->d_scales, N, K / 32, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        free_weight(w);
        return BATQ_ERR_DEVICE;
    }
    *out = w;
    return BATQ_OK;
}

batq_status batq_weight_shape(const batq_weight* w, int* K, int* N) {
    if (!w || !K || !N) return BATQ_ERR_NULL;
    *K = w->K;
    *N = w->N;
    return BATQ_OK;
}

batq_status batq_weight_destroy(batq_weight* w) {
    if (!w) return BATQ_ERR_NULL;
    free_weight(w);
    return BATQ_OK;
}

}  // extern "C"

namespace {

// The optional inputs of the online path: per-row factors and the up tensor of a gated activation.
struct ActExtras {
    const float* row_scale = nullptr;
    const void* up = nullptr;
    int64_t ld_up = 0;
    // destination window of a cache append: the arrays are laid out for `layout_rows` rows (0: for M) and the
    // M rows go to rows row_offset .. row_offset + M - 1
    int row_offset = 0, layout_rows = 0;
};

// Gated input: bf16 only (the rounding of silu(gate) * up is to bf16), up laid out like X.
batq_status check_extras(const ActExtras& ex, batq_dtype xdtype, int K) {
    if ((reinterpret_cast<uintptr_t>(ex.row_scale) & 3u) != 0) return BATQ_ERR_SHAPE;
    if (ex.up) {
        if (xdtype != BATQ_BF16) return BATQ_ERR_DTYPE;
        if (ex.ld_up < K || !aligned16(ex.up) || (ex.ld_up * 2) % 16 != 0) return BATQ_ERR_SHAPE;
    }
    return BATQ_OK;
}

batq_status quantize_impl(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int K, int64_t ldx,
                          const ActExtras& ex, uint8_t* codes, uint8_t* scales, bool fp8, void* stream) {
    if (!t) return BATQ_ERR_NULL;
    if (!dtype_ok(xdtype)) return BATQ_ERR_DTYPE;
    if (M < 0 || K <= 0 || K % 32 != 0 || ldx < K) return BATQ_ERR_SHAPE;
    if (t->K != K) return BATQ_ERR_MISMATCH;
    if (M == 0) return BATQ_OK;          // nothing to do; empty tensors may carry null pointers
    if (!X || !codes || !scales) return BATQ_ERR_NULL;
    // rows are read with 128-bit loads and codes written as dwords
    if (!aligned16(X) || (ldx * (int64_t)dtype_size(xdtype)) % 16 != 0 || !aligned16(codes) ||
        (reinterpret_cast<uintptr_t>(scales) & 7u) != 0)
        return BATQ_ERR_SHAPE;
    if (batq_status st = check_extras(ex, xdtype, K); st != BATQ_OK) return st;
    if (batq::launch_quantize_act(t, X, xdtype, M, K, ldx, ex.up, ex.ld_up, ex.row_scale, codes, scales, fp8,
                                  ex.row_offset, ex.layout_rows, static_cast<hipStream_t>(stream)) != hipSuccess) {
        (void)hipGetLastError();
        return BATQ_ERR_DEVICE;
    }
    return BATQ_OK;
}

// Partial sums of the GEMM's K parts start on a 256-byte boundary.
constexpr size_t kPartsAlign = 256;
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// glu: Y = silu(gate) * up, M x N/2, for a weight prepared by batq_prepare_weight_gate_up
// parts / parts_bytes: caller memory for the partial sums of K parts (null / 0: none, every tile runs over all of K)
batq_status gemm_impl(const uint8_t* xcodes, const uint8_t* xscales, const batq_weight* w, int M, void* Y,
                      batq_dtype ydtype, int64_t ldy, bool a8, bool glu, void* parts, size_t parts_bytes,
                      void* stream) {
    if (!w) return BATQ_ERR_NULL;
    if (!dtype_ok(ydtype)) return BATQ_ERR_DTYPE;
    if (M < 0 || ldy < (glu ? w->N / 2 : w->N)) return BATQ_ERR_SHAPE;
    if (glu && !batq::gemm_glu_supported(w, M, a8)) return w->N % 64 != 0 ? BATQ_ERR_SHAPE : BATQ_ERR_UNSUPPORTED;
    if (M == 0) return BATQ_OK;
    if (!xcodes || !xscales || !Y) return BATQ_ERR_NULL;
    if (!aligned16(xcodes) || (reinterpret_cast<uintptr_t>(xscales) & 7u) != 0) return BATQ_ERR_SHAPE;
    if (parts_bytes > 0 && !parts) return BATQ_ERR_NULL;
    if (parts && (reinterpret_cast<uintptr_t>(parts) & (kPartsAlign - 1)) != 0) return BATQ_ERR_SHAPE;
    if (batq::launch_gemm_mxfp4(xcodes, xscales, w, M, Y, ydtype, ldy, a8, glu, parts, parts ? parts_bytes : 0,
                                static_cast<hipStream_t>(stream)) != hipSuccess) {
        (void)hipGetLastError();
        return BATQ_ERR_DEVICE;
    }
    return BATQ_OK;
}

size_t workspace_impl(int M, int K, bool a8) {
    if (M <= 0 || K <= 0 || K % 32 != 0) return 0;
    // activation codes (blocked layout, a multiple of 1 KiB) followed by their grouped scales
    return (a8 ? batq::code8_bytes_blocked(M, K / 32) : batq::code_bytes_blocked(M, K / 32)) +
           batq::scale_bytes_internal(M, K / 32);
}

batq_status linear_impl(const batq_transform* t, const batq_weight* w, const void* X, batq_dtype xdtype, int M,
                        int64_t ldx, const ActExtras& ex, void* Y, batq_dtype ydtype, int64_t ldy, void* workspace,
                        size_t workspace_bytes, bool a8, bool glu, void* stream) {
    if (!t || !w) return BATQ_ERR_NULL;
    if (!dtype_ok(xdtype) || !dtype_ok(ydtype)) return BATQ_ERR_DTYPE;
    if (t->K != w->K) return BATQ_ERR_MISMATCH;
    if (M < 0 || ldx < t->K || ldy < (glu ? w->N / 2 : w->N)) return BATQ_ERR_SHAPE;
    if (glu && !batq::gemm_glu_supported(w, M, a8)) return w->N % 64 != 0 ? BATQ_ERR_SHAPE : BATQ_ERR_UNSUPPORTED;
    if (M == 0) return BATQ_OK;
    if (!X || !Y || !workspace) return BATQ_ERR_NULL;
    if (workspace_bytes < workspace_impl(M, t->K, a8)) return BATQ_ERR_WORKSPACE;
    if (!aligned16(X) || (ldx * (int64_t)dtype_size(xdtype)) % 16 != 0 ||
        (reinterpret_cast<uintptr_t>(workspace) & (kPartsAlign - 1)) != 0)
        return BATQ_ERR_SHAPE;
    if (batq_status st = check_extras(ex, xdtype, t->K); st != BATQ_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* codes = static_cast<uint8_t*>(workspace);
    uint8_t* scales = codes + (a8 ? batq::code8_bytes_blocked(M, t->nb) : batq::code_bytes_blocked(M, t->nb));
    // what the workspace holds beyond the codes and scales serves the partial sums of the GEMM's K parts
    const size_t parts_at = align_up(workspace_impl(M, t->K, a8), kPartsAlign);
    uint8_t* parts = workspace_bytes > parts_at ? codes + parts_at : nullptr;
    const size_t parts_bytes = parts ? workspace_bytes - parts_at : 0;
    hipError_t e = batq::launch_quantize_act(t, X, xdtype, M, t->K, ldx, ex.up, ex.ld_up, ex.row_scale, codes, scales,
                                             a8, 0, 0, s);
    if (e == hipSuccess) e = batq::launch_gemm_mxfp4(codes, scales, w, M, Y, ydtype, ldy, a8, glu, parts, parts_bytes, s);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return BATQ_ERR_DEVICE;
    }
    return BATQ_OK;
}

}  // namespace

extern "C" {

batq_status batq_quantize_act(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int K,
                              int64_t ldx, uint8_t* codes, uint8_t* scales, void* stream) {
    return quantize_impl(t, X, xdtype, M, K, ldx, ActExtras{}, codes, scales, false, stream);
}

batq_status batq_quantize_act_mxfp8(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int K,
                                    int64_t ldx, uint8_t* codes8, uint8_t* scales, void* stream) {
    return quantize_impl(t, X, xdtype, M, K, ldx, ActExtras{}, codes8, scales, true, stream);
}

size_t batq_code8_bytes(int rows, int K) {
    if (rows <= 0 || K <= 0 || K % 32 != 0) return 0;
    return batq::code8_bytes_blocked(rows, K / 32);
}

size_t batq_code8_slot_offset(int row, int k, int half, int K) { return batq::code8_slot_offset(row, k, half, K / 32); }

batq_status batq_codes8_to_rowmajor(const uint8_t* blocked, uint8_t* rowmajor, int rows, int K, void* stream) {
    if (rows < 0 || K <= 0 || K % 32 != 0) return BATQ_ERR_SHAPE;
    if (rows == 0) return BATQ_OK;
    if (!blocked || !rowmajor) return BATQ_ERR_NULL;
    if (!aligned16(blocked) || !aligned16(rowmajor)) return BATQ_ERR_SHAPE;
    BATQ_HIP(batq::launch_codes8_to_rowmajor(blocked, rowmajor, rows, K / 32, static_cast<hipStream_t>(stream)));
    return BATQ_OK;
}

batq_status batq_codes8_from_rowmajor(const uint8_t* rowmajor, uint8_t* blocked, int rows, int K, void* stream) {
    if (rows < 0 || K <= 0 || K % 32 != 0) return BATQ_ERR_SHAPE;
    if (rows == 0) return BATQ_OK;
    if (!blocked || !rowmajor) return BATQ_ERR_NULL;
    if (!aligned16(blocked) || !aligned16(rowmajor)) return BATQ_ERR_SHAPE;
    BATQ_HIP(batq::launch_codes8_to_blocked(rowmajor, blocked, rows, K / 32, static_cast<hipStream_t>(stream)));
    return BATQ_OK;
}

size_t batq_code_bytes(int rows, int K) {
    if (rows <= 0 || K <= 0 || K % 32 != 0) return 0;
    return batq::code_bytes_blocked(rows, K / 32);
}

size_t batq_code_chunk_offset(int row, int k, int K) { return batq::code_chunk_offset(row, k, K / 32); }

batq_status batq_codes_to_rowmajor(const uint8_t* blocked, uint8_t* rowmajor, int rows, int K, void* stream) {
    if (rows < 0 || K <= 0 || K % 32 != 0) return BATQ_ERR_SHAPE;
    if (rows == 0) return BATQ_OK;
    if (!blocked || !rowmajor) return BATQ_ERR_NULL;
    if (!aligned16(blocked) || !aligned16(rowmajor)) return BATQ_ERR_SHAPE;
    BATQ_HIP(batq::launch_codes_to_rowmajor(blocked, rowmajor, rows, K / 32, static_cast<hipStream_t>(stream)));
    return BATQ_OK;
}

batq_status batq_codes_from_rowmajor(const uint8_t* rowmajor, uint8_t* blocked, int rows, int K, void* stream) {
    if (rows < 0 || K <= 0 || K % 32 != 0) return BATQ_ERR_SHAPE;
    if (rows == 0) return BATQ_OK;
    if (!blocked || !rowmajor) return BATQ_ERR_NULL;
    if (!aligned16(blocked) || !aligned16(rowmajor)) return BATQ_ERR_SHAPE;
    BATQ_HIP(batq::launch_codes_to_blocked(rowmajor, blocked, rows, K / 32, static_cast<hipStream_t>(stream)));
    return BATQ_OK;
}

size_t batq_scale_bytes(int rows, int K) {
    if (rows <= 0 || K <= 0 || K % 32 != 0) return 0;
    return batq::scale_bytes_internal(rows, K / 32);
}

size_t batq_scale_index(int row, int k, int rows) { return batq::scale_index_internal(row, k, rows); }

batq_status batq_scales_to_rowmajor(const uint8_t* grouped, uint8_t* rowmajor, int rows, int K, void* stream) {
    if (rows < 0 || K <= 0 || K % 32 != 0) return BATQ_ERR_SHAPE;
    if (rows == 0) return BATQ_OK;
    if (!grouped || !rowmajor) return BATQ_ERR_NULL;
    BATQ_HIP(batq::launch_scales_to_canonical(grouped, rowmajor, rows, K / 32, static_cast<hipStream_t>(stream)));
    return BATQ_OK;
}

batq_status batq_scales_from_rowmajor(const uint8_t* rowmajor, uint8_t* grouped, int rows, int K, void* stream) {
    if (rows < 0 || K <= 0 || K % 32 != 0) return BATQ_ERR_SHAPE;
    if (rows == 0) return BATQ_OK;
    if (!grouped || !rowmajor) return BATQ_ERR_NULL;
    BATQ_HIP(batq::launch_scales_to_internal(rowmajor, grouped, rows, K / 32, static_cast<hipStream_t>(stream)));
    return BATQ_OK;
}

batq_status batq_gemm_mxfp4(const uint8_t* xcodes, const uint8_t* xscales, const batq_weight* w, int M, void* Y,
                            batq_dtype ydtype, int64_t ldy, void* stream) {
    return gemm_impl(xcodes, xscales, w, M, Y, ydtype, ldy, false, false, nullptr, 0, stream);
}

batq_status batq_gemm_a8w4(const uint8_t* xcodes8, const uint8_t* xscales, const batq_weight* w, int M, void* Y,
                           batq_dtype ydtype, int64_t ldy, void* stream) {
    return gemm_impl(xcodes8, xscales, w, M, Y, ydtype, ldy, true, false, nullptr, 0, stream);
}

size_t batq_gemm_workspace(const batq_weight* w, int M, int act_bits) {
    if (!w || M <= 0 || (act_bits != 0 && act_bits != 4 && act_bits != 8)) return 0;
    return batq::gemm_workspace_bytes(w, M, act_bits == 8, w->cus);
}

batq_status batq_gemm_mxfp4_ws(const uint8_t* xcodes, const uint8_t* xscales, const batq_weight* w, int M, void* Y,
                               batq_dtype ydtype, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_impl(xcodes, xscales, w, M, Y, ydtype, ldy, false, false, workspace, workspace_bytes, stream);
}

batq_status batq_gemm_a8w4_ws(const uint8_t* xcodes8, const uint8_t* xscales, const batq_weight* w, int M, void* Y,
                              batq_dtype ydtype, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_impl(xcodes8, xscales, w, M, Y, ydtype, ldy, true, false, workspace, workspace_bytes, stream);
}

batq_status batq_gemm_mxfp4_noalloc(const uint8_t* xcodes, const uint8_t* xscales, const batq_weight* w, int M,
                                    void* Y, batq_dtype ydtype, int64_t ldy, void* stream) {
    if (!w) return BATQ_ERR_NULL;
    const size_t need = M > 0 ? batq::gemm_workspace_bytes(w, M, false, w->cus) : 0;
    if (need > batq::kStaticScratchBytes) return BATQ_ERR_WORKSPACE;
    void* parts = nullptr;
    if (need > 0 && batq::static_scratch(&parts) != hipSuccess) {
        (void)hipGetLastError();
        return BATQ_ERR_DEVICE;
    }
    return gemm_impl(xcodes, xscales, w, M, Y, ydtype, ldy, false, false, parts, need, stream);
}

size_t batq_linear_workspace(int M, int K) { return workspace_impl(M, K, false); }
size_t batq_linear_a8w4_workspace(int M, int K) { return workspace_impl(M, K, true); }

size_t batq_linear_workspace_for(const batq_weight* w, int M, int act_bits) {
    if (!w || M <= 0 || (act_bits != 0 && act_bits != 4 && act_bits != 8)) return 0;
    const size_t base = workspace_impl(M, w->K, act_bits == 8);
    const size_t parts = batq::gemm_workspace_bytes(w, M, act_bits == 8, w->cus);
    return parts ? align_up(base, kPartsAlign) + parts : base;
}

batq_status batq_linear(const batq_transform* t, const batq_weight* w, const void* X, batq_dtype xdtype, int M,
                        int64_t ldx, void* Y, batq_dtype ydtype, int64_t ldy, void* workspace,
                        size_t workspace_bytes, void* stream) {
    return linear_impl(t, w, X, xdtype, M, ldx, ActExtras{}, Y, ydtype, ldy, workspace, workspace_bytes, false, false, stream);
}

batq_status batq_linear_a8w4(const batq_transform* t, const batq_weight* w, const void* X, batq_dtype xdtype, int M,
                             int64_t ldx, void* Y, batq_dtype ydtype, int64_t ldy, void* workspace,
                             size_t workspace_bytes, void* stream) {
    return linear_impl(t, w, X, xdtype, M, ldx, ActExtras{}, Y, ydtype, ldy, workspace, workspace_bytes, true, false, stream);
}

// ---- options form of the online calls
static bool act_options_ok(const batq_act_options* opt, bool* a8, ActExtras* ex) {
    *a8 = false;
    *ex = ActExtras{};
    if (!opt) return true;
    if (opt->act_bits != 0 && opt->act_bits != 4 && opt->act_bits != 8) return false;
    *a8 = opt->act_bits == 8;
    ex->row_scale = opt->row_scale;
    ex->up = opt->up;
    ex->ld_up = opt->ld_up;
    return true;
}

batq_status batq_quantize_act_ex(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int K,
                                 int64_t ldx, const batq_act_options* opt, uint8_t* codes, uint8_t* scales,
                                 void* stream) {
    bool a8;
    ActExtras ex;
    if (!act_options_ok(opt, &a8, &ex)) return BATQ_ERR_UNSUPPORTED;
    return quantize_impl(t, X, xdtype, M, K, ldx, ex, codes, scales, a8, stream);
}

batq_status batq_linear_ex(const batq_transform* t, const batq_weight* w, const void* X, batq_dtype xdtype, int M,
                           int64_t ldx, const batq_act_options* opt, void* Y, batq_dtype ydtype, int64_t ldy,
                           void* workspace, size_t workspace_bytes, void* stream) {
    bool a8;
    ActExtras ex;
    if (!act_options_ok(opt, &a8, &ex)) return BATQ_ERR_UNSUPPORTED;
    return linear_impl(t, w, X, xdtype, M, ldx, ex, Y, ydtype, ldy, workspace, workspace_bytes, a8, false, stream);
}

batq_status batq_gemm_glu(const uint8_t* xcodes, const uint8_t* xscales, const batq_weight* w, int M, int act_bits,
                          void* H, batq_dtype hdtype, int64_t ldh, void* stream) {
    if (act_bits != 0 && act_bits != 4 && act_bits != 8) return BATQ_ERR_UNSUPPORTED;
    return gemm_impl(xcodes, xscales, w, M, H, hdtype, ldh, act_bits == 8, true, nullptr, 0, stream);
}

batq_status batq_linear_glu(const batq_transform* t, const batq_weight* w, const void* X, batq_dtype xdtype, int M,
                            int64_t ldx, const batq_act_options* opt, void* H, batq_dtype hdtype, int64_t ldh,
                            void* workspace, size_t workspace_bytes, void* stream) {
    bool a8;
    ActExtras ex;
    if (!act_options_ok(opt, &a8, &ex)) return BATQ_ERR_UNSUPPORTED;
    return linear_impl(t, w, X, xdtype, M, ldx, ex, H, hdtype, ldh, workspace, workspace_bytes, a8, true, stream);
}

int batq_debug_tile_schedule(int M, int N, int K, int compute_units, int glu, int allow_ksplit, int* tiles,
                             int capacity) {
    if (M <= 64 || N <= 0 || K <= 0 || K % 32 != 0 || compute_units < 8 || capacity < 0 || (capacity > 0 && !tiles))
        return -1;
    if (glu && N % 64 != 0) return -1;
    return batq::tile_schedule(M, N, K, compute_units, glu != 0, allow_ksplit != 0, tiles, capacity);
}

static batq_status dequantize_impl(const uint8_t* codes, const uint8_t* scales, int64_t layout_rows, int64_t row_offset,
                                   int M, int K, int bits, void* out, batq_dtype odtype, int64_t ldo, void* stream) {
    if (bits != 4 && bits != 8) return BATQ_ERR_UNSUPPORTED;
    if (!dtype_ok(odtype)) return BATQ_ERR_DTYPE;
    if (M < 0 || K <= 0 || K % 32 != 0 || ldo < K) return BATQ_ERR_SHAPE;
    if (row_offset < 0 || layout_rows < row_offset + M || layout_rows > INT32_MAX) return BATQ_ERR_SHAPE;
    if (M == 0) return BATQ_OK;
    if (!codes || !scales || !out) return BATQ_ERR_NULL;
    if (!aligned16(codes) || !aligned16(out) || (ldo * (int64_t)dtype_size(odtype)) % 16 != 0) return BATQ_ERR_SHAPE;
    batq_status st = check_device();
    if (st != BATQ_OK) return st;
    BATQ_HIP(batq::launch_dequantize(codes, scales, M, K / 32, bits == 8, out, odtype, ldo, (int)row_offset,
                                     (int)layout_rows, static_cast<hipStream_t>(stream)));
    return BATQ_OK;
}

batq_status batq_dequantize(const uint8_t* codes, const uint8_t* scales, int M, int K, int bits, void* out,
                            batq_dtype odtype, int64_t ldo, void* stream) {
    return dequantize_impl(codes, scales, M, 0, M, K, bits, out, odtype, ldo, stream);
}

batq_status batq_kv_dequantize(const uint8_t* codes, const uint8_t* scales, int64_t capacity_rows, int64_t row_offset,
                               int M, int K, int bits, void* out, batq_dtype odtype, int64_t ldo, void* stream) {
    if (capacity_rows < 1) return BATQ_ERR_SHAPE;
    return dequantize_impl(codes, scales, capacity_rows, row_offset, M, K, bits, out, odtype, ldo, stream);
}

batq_status batq_kv_append(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int K, int64_t ldx,
                           int act_bits, uint8_t* codes, uint8_t* scales, int64_t row_offset, int64_t capacity_rows,
                           void* stream) {
    if (act_bits != 4 && act_bits != 8) return BATQ_ERR_UNSUPPORTED;
    if (M < 0 || capacity_rows < 1 || capacity_rows > INT32_MAX || row_offset < 0 || row_offset + M > capacity_rows)
        return BATQ_ERR_SHAPE;
    ActExtras ex;
    ex.row_offset = (int)row_offset;
    ex.layout_rows = (int)capacity_rows;
    return quantize_impl(t, X, xdtype, M, K, ldx, ex, codes, scales, act_bits == 8, stream);
}

batq_status batq_transform_apply(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int K,
                                 int64_t ldx, batq_apply_mode mode, void* out, batq_dtype odtype, int64_t ldo,
                                 void* stream) {
    if (!t) return BATQ_ERR_NULL;
    if (!dtype_ok(xdtype) || !dtype_ok(odtype)) return BATQ_ERR_DTYPE;
    if (mode != BATQ_APPLY_FORWARD && mode != BATQ_APPLY_INVERSE && mode != BATQ_APPLY_INVERSE_T)
        return BATQ_ERR_UNSUPPORTED;
    if (M < 0 || K <= 0 || K % 32 != 0 || ldx < K || ldo < K) return BATQ_ERR_SHAPE;
    if (t->K != K) return BATQ_ERR_MISMATCH;
    if (M == 0) return BATQ_OK;
    if (!X || !out) return BATQ_ERR_NULL;
    if (X == out) return BATQ_ERR_SHAPE;                  // not in place: a block's outputs need all its inputs
    BATQ_HIP(batq::launch_transform_apply(t, X, xdtype, M, ldx, (int)mode, out, odtype, ldo,
                                          static_cast<hipStream_t>(stream)));
    return BATQ_OK;
}

batq_status batq_row_rms_scale(const void* X, batq_dtype xdtype, int M, int K, int64_t ldx, float eps,
                               float* row_scale, void* stream) {
    if (!dtype_ok(xdtype)) return BATQ_ERR_DTYPE;
    if (M < 0 || K <= 0 || K % 32 != 0 || ldx < K || !(eps >= 0.0f)) return BATQ_ERR_SHAPE;
    if (M == 0) return BATQ_OK;
    if (!X || !row_scale) return BATQ_ERR_NULL;
    if (!aligned16(X) || (ldx * (int64_t)dtype_size(xdtype)) % 16 != 0) return BATQ_ERR_SHAPE;
    batq_status st = check_device();
    if (st != BATQ_OK) return st;
    BATQ_HIP(batq::launch_row_rms_scale(X, xdtype, M, K, ldx, eps, row_scale, static_cast<hipStream_t>(stream)));
    return BATQ_OK;
}

}  // extern "C"
