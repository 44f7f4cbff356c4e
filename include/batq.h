/*
 * libbatq - W4A4 MXFP4 linear layer with block-wise affine transforms (BATQuant)
 * for AMD MI355X (gfx950).  C ABI.
 *
 * The layer computes  Y = Q(X P) * Q(P^-1 W)  (Sec. 3.1 of the paper, where it is
 * written with W stored out x in):
 *   - P = diag(T_0 .. T_{K/32-1}) is block-diagonal with one 32x32 block per MXFP
 *     block of the reduction dimension (Eq. 1);
 *   - each block is a Kronecker product of a factor shared by all blocks and a
 *     factor private to the block (Eq. 2, "Global and Private Kronecker");
 *   - after the transform each 32-block is clipped at a learned fraction of its
 *     own absolute maximum (Eq. 3-4, symmetric form) and quantised to MXFP4:
 *     E2M1 elements {0,.5,1,1.5,2,3,4,6} with sign, one UE8M0 power-of-two scale
 *     per 32 elements (Sec. 2, MXFP definition);
 *   - the weight side P^-1 W is computed and quantised once, offline (Alg. 2,
 *     "Offline Fusion"); the activation side runs online, fused with the quantiser.
 *
 * Notation used here: X is M x K (tokens x in-features), W is K x N (in x out),
 * Y is M x N.  Block k covers columns 32k .. 32k+31 of X (rows of W).
 *   T_k = G (x) P_k,  T_k[a*gi + c, a2*gi + c2] = G[a][a2] * P_k[c][c2],
 *   G: g_outer x g_outer shared ("global"), P_k: g_inner x g_inner ("private"),
 *   g_outer * g_inner = 32.  A row vector x_k is mapped to x_k T_k.
 *
 * Quantised tensors.  A 4-bit code is S|E1 E0|M (bit 3 = sign); a scale byte is E8M0,
 * value 2^(s-127), and 255 is never produced.  The 32 codes of one MX block form a 16-byte
 * chunk: element j of the block in byte j/2, even j in bits 3:0, odd j in bits 7:4.
 * Row-major order (weight export / import, and the conversion helpers):
 *     codes [rows][K/2], scales [rows][K/32].
 * Device order (what batq_quantize_act writes and batq_gemm_mxfp4 reads), chosen so that
 * the GEMM moves operands with contiguous 1 KiB loads that already are its LDS image, and
 * reads scales as the matrix instruction consumes them:
 *     codes   batq_code_bytes(rows, K) bytes; the chunk of block k of `row` starts at
 *             batq_code_chunk_offset(row, k, K)
 *               = ((row/16) * S + k/4) * 1024 + (row%16) * 64 + (((k%4) ^ ((row%16)/4)) * 16),
 *             S = 2 * ceil(K/256); rows are padded to a multiple of 32 (pad rows hold
 *             unspecified bytes) and K to a multiple of 256 with zero codes;
 *     scales  batq_scale_bytes(rows, K) bytes; block k of `row` at batq_scale_index(row, k, rows)
 *               = ((k/8) * rows + row) * 8 + (k%8)/2 + 4 * (k%2)
 *             (groups of 8 blocks, group-major, even blocks of a group first); a last
 *             partial group is padded with the neutral scale 127.
 * Quantiser definition (symmetric clip): bound = fl32(clip_k * max_j |y_j|); elements beyond +-bound
 * are replaced by +-bound; E = clamp(floor(log2 bound) - 2, -127, 127) (E = -127 for
 * a zero block); code = round-to-nearest on the E2M1 grid of y * 2^-E, ties to the
 * code with even mantissa bit, saturating at 6; the sign bit is always the sign bit
 * of the input element (also for results that round to zero).
 *
 * Conventions
 *   - Every function returns a batq_status; nothing throws, aborts or prints.
 *   - Pointers documented HOST are read on the host during the call; pointers
 *     documented DEVICE must be device memory on the current HIP device and stay
 *     valid until the stream has passed the call.  The caller owns every tensor it
 *     passes; the library owns only what is inside its handles.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Online calls (batq_quantize_act*, batq_gemm_*, batq_linear*, the cache calls) only
 *     enqueue kernels: no host synchronisation, no allocation, no state kept between
 *     calls.  Which kernels run is a function of the call's arguments and the device
 *     alone, so a call gives the same bits on any stream, eagerly or while the stream
 *     is captured into a graph.  Scratch memory comes from the caller (`workspace`).
 *   - Argument errors are detected on the host before anything is launched and
 *     leave all outputs untouched.  Non-finite inputs are outside the contract.
 *   - Calls are thread-safe; a handle may be used by several threads at once (online
 *     calls only read it), but not destroyed while in use.
 */
#ifndef BATQ_H
#define BATQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BATQ_OK = 0,
    BATQ_ERR_NULL = 1,        /* a required pointer is NULL                                  */
    BATQ_ERR_SHAPE = 2,       /* K % 32 != 0, a size <= 0, or a leading dimension too small  */
    BATQ_ERR_DTYPE = 3,       /* unknown batq_dtype                                          */
    BATQ_ERR_UNSUPPORTED = 4, /* (g_outer, g_inner) not one of (4,8), (8,4), or unknown form    */
    BATQ_ERR_SINGULAR = 5,    /* G or some P_k is not invertible                             */
    BATQ_ERR_CLIP_RANGE = 6,  /* a clip ratio is not in (0, 1]                               */
    BATQ_ERR_WORKSPACE = 7,   /* workspace smaller than batq_linear_workspace()              */
    BATQ_ERR_ALLOC = 8,       /* host or device allocation failed                            */
    BATQ_ERR_DEVICE = 9,      /* a HIP call failed, or the device is not gfx950              */
    BATQ_ERR_MISMATCH = 10    /* transform and weight were built for different K             */
} batq_status;

typedef enum { BATQ_F32 = 0, BATQ_BF16 = 1 } batq_dtype;

/* Static, NUL-terminated description of a status code. */
const char* batq_status_string(batq_status s);

/* Library version, "major.minor". Static storage. */
const char* batq_version(void);

/* ------------------------------------------------------------------------------------
 * Transform object: the learned parameters of one transform set (Alg. 2's Theta):
 * the shared factor, the private factors and the activation clip ratios.
 *   K        in-features, multiple of 32
 *   g_outer  size of the shared factor G, g_inner size of each private factor P_k;
 *            (4,8) or (8,4)
 *   G        HOST [g_outer*g_outer] row-major fp32; NULL = no transform (T_k = I),
 *            in which case P must be NULL too
 *   P        HOST [K/32][g_inner*g_inner] row-major fp32
 *   clip_a   HOST [K/32] clip ratios in (0,1] applied to the block amax of the
 *            transformed activations; NULL = 1.0 (no clipping)
 * The library copies everything (to the device too); the caller may free its arrays
 * on return.  The factors are inverted on the host in fp64; a pivot below
 * 1e-12 * max|entry| gives BATQ_ERR_SINGULAR.  Synchronises with the device.
 */
typedef struct batq_transform batq_transform;
batq_status batq_transform_create(batq_transform** out, int K, int g_outer, int g_inner,
                                  const float* G, const float* P, const float* clip_a);
batq_status batq_transform_destroy(batq_transform* t);

/* General form of the transform set.  Besides the Global-and-Private product above, Sec. 3.1.1
 * discusses a dense 32x32 matrix per block, the naive Kronecker product with both factors
 * private, and Eq. 2 prints the product in the order private (x) global; Eq. 3-4 print the
 * clipping with two ratios, on the block minimum and on the block maximum.
 *   form      BATQ_FORM_IDENTITY: T_k = I.  BATQ_FORM_KRON: T_k = O_k (x) I_k,
 *             T_k[a*gi + c, a2*gi + c2] = O_k[a][a2] * I_k[c][c2], (g_outer, g_inner) = (4,8) or (8,4).
 *             BATQ_FORM_DENSE: T_k given.  A row vector x_k is mapped to x_k T_k in every form.
 *   outer     HOST row-major fp32: [g_outer^2] if outer_per_block == 0 (one factor shared by all
 *             blocks), else [K/32][g_outer^2] (one per block)
 *   inner     likewise with g_inner
 *   dense     HOST [K/32][32][32] row-major fp32
 *   clip      HOST [K/32] ratios in (0,1] on the block amax (symmetric form), or NULL
 *   clip_min, clip_max   HOST [K/32] ratios in (0,1]: the block is clamped to
 *             [fl32(clip_min_k * min_j y_j), fl32(clip_max_k * max_j y_j)] and the shared scale is taken
 *             from the largest magnitude that is left.  Both or neither; not together with `clip`.
 * Everything is copied; blocks (or factors) are inverted on the host in fp64 with the same
 * singularity rule as batq_transform_create, which is the special case
 * {KRON, outer = G shared, inner = P per block, clip = clip_a}. */
typedef enum { BATQ_FORM_IDENTITY = 0, BATQ_FORM_KRON = 1, BATQ_FORM_DENSE = 2 } batq_form;
typedef struct {
    int K;
    int form;
    int g_outer, g_inner;
    const float* outer;
    int outer_per_block;
    const float* inner;
    int inner_per_block;
    const float* dense;
    const float* clip;
    const float* clip_min;
    const float* clip_max;
} batq_transform_desc;
batq_status batq_transform_create_ex(batq_transform** out, const batq_transform_desc* desc);

/* ------------------------------------------------------------------------------------
 * Offline weight preparation (Alg. 2, "Offline Fusion for Deployment"):
 * W~ = P^-1 W (each 32-row K-slab of W multiplied from the left by T_k^-1, fp64
 * accumulation, rounded once to fp32), optional block clip, MXFP4 along K.
 *   t        transform the weights pair with (its K must equal K)
 *   W        DEVICE, read-only; w_is_KxN != 0: row-major K x N with row stride ldw
 *            (>= N); w_is_KxN == 0: row-major N x K (the paper's out x in) with row
 *            stride ldw (>= K).  ldw counts elements.
 *   clip_w   HOST [K/32] ratios in (0,1] or NULL (= 1.0)
 * The result is an opaque handle owning device memory in the GEMM's internal layout.
 * Synchronises `stream` before returning (offline call).
 */
typedef struct batq_weight batq_weight;
batq_status batq_prepare_weight(batq_weight** out, const batq_transform* t,
                                const void* W, batq_dtype wdtype, int K, int N, int64_t ldw,
                                int w_is_KxN, const float* clip_w, void* stream);
/* The same with the two-ratio clipping of Eq. 3-4 on the weight side: each block of each output
 * column is clamped to [clip_w_min_k * min, clip_w_max_k * max] before MXFP4.  Both HOST [K/32]. */
batq_status batq_prepare_weight_minmax(batq_weight** out, const batq_transform* t,
                                       const void* W, batq_dtype wdtype, int K, int N, int64_t ldw,
                                       int w_is_KxN, const float* clip_w_min, const float* clip_w_max,
                                       void* stream);
/* Copy the prepared weights out in the canonical layout: codes DEVICE [N][K/2],
 * scales DEVICE [N][K/32].  Enqueued on `stream`. */
batq_status batq_weight_export(const batq_weight* w, uint8_t* codes, uint8_t* scales, void* stream);
/* Build a weight handle from canonical codes/scales (DEVICE), e.g. a stored checkpoint. */
batq_status batq_weight_import(batq_weight** out, const uint8_t* codes, const uint8_t* scales,
                               int K, int N, void* stream);
batq_status batq_weight_shape(const batq_weight* w, int* K, int* N);
batq_status batq_weight_destroy(batq_weight* w);

/* ------------------------------------------------------------------------------------
 * Online step 1: fused transform (Eq. 1-2) + block clip (Eq. 3-4) + MXFP4 (Sec. 2).
 *   X       DEVICE M x K row-major, row stride ldx elements (>= K), fp32 or bf16;
 *           the products and sums of the transform are carried in fp32 (bf16 is
 *           storage only; nothing is rounded to bf16 before the quantiser)
 *   codes   DEVICE, batq_code_bytes(M, K) bytes, device order, out
 *   scales  DEVICE, batq_scale_bytes(M, K) bytes, device order, out
 * X and codes must be 16-byte aligned, scales 8-byte aligned, and ldx * sizeof(element) a
 * multiple of 16.  M == 0 is a no-op.  A transform created with G == NULL quantises X as is.
 */
batq_status batq_quantize_act(const batq_transform* t, const void* X, batq_dtype xdtype,
                              int M, int K, int64_t ldx,
                              uint8_t* codes, uint8_t* scales, void* stream);

/* Layout helpers (Sec. 2: 32-element blocks with one UE8M0 scale; the orders are this library's).
 * Sizes return 0 for invalid arguments.  The four conversions run on the device (both
 * pointers DEVICE, 16-byte aligned for codes), enqueued on `stream`; converting to device
 * order also writes the zero / neutral padding of K. */
size_t batq_code_bytes(int rows, int K);
size_t batq_code_chunk_offset(int row, int k, int K);
size_t batq_scale_bytes(int rows, int K);
size_t batq_scale_index(int row, int k, int rows);
batq_status batq_codes_to_rowmajor(const uint8_t* device_order, uint8_t* rowmajor, int rows, int K, void* stream);
batq_status batq_codes_from_rowmajor(const uint8_t* rowmajor, uint8_t* device_order, int rows, int K, void* stream);
batq_status batq_scales_to_rowmajor(const uint8_t* device_order, uint8_t* rowmajor, int rows, int K, void* stream);
batq_status batq_scales_from_rowmajor(const uint8_t* rowmajor, uint8_t* device_order, int rows, int K, void* stream);

/* Online step 2 alone: MXFP4 x MXFP4 GEMM on activation codes and scales in device order,
 * as batq_quantize_act writes them.
 *   Y[m][n] = sum_k 2^(xs[m][k]-127) 2^(ws[n][k]-127) sum_{j<32} val(xq[m][32k+j]) val(wq[n][32k+j])
 * with fp32 accumulation; Y DEVICE M x N row-major, row stride ldy (>= N), fp32 or
 * bf16 (round-to-nearest-even). */
batq_status batq_gemm_mxfp4(const uint8_t* xcodes, const uint8_t* xscales, const batq_weight* w,
                            int M, void* Y, batq_dtype ydtype, int64_t ldy, void* stream);
/* The same with scratch memory for K parts.  Shapes with few output tiles and a long K (down projections at a
 * few hundred rows; at most 64 rows against a narrow N) are faster when K is cut into parts whose fp32 partial
 * sums are added by a second kernel, in part order (deterministic).  batq_gemm_workspace(w, M, act_bits) is the
 * number of bytes with which the GEMM of M rows against `w` uses all the parts it wants (0: the shape wants
 * none; act_bits 4 or 0 for batq_gemm_mxfp4_ws, 8 for batq_gemm_a8w4_ws).  `workspace` is DEVICE memory, 256-byte
 * aligned, or NULL with workspace_bytes 0; a smaller workspace gives fewer parts, none gives the plain call.
 * The number of parts, and with it the fp32 rounding of Y, depends on (M, w, workspace_bytes, device) only. */
size_t batq_gemm_workspace(const batq_weight* w, int M, int act_bits);
batq_status batq_gemm_mxfp4_ws(const uint8_t* xcodes, const uint8_t* xscales, const batq_weight* w,
                               int M, void* Y, batq_dtype ydtype, int64_t ldy,
                               void* workspace, size_t workspace_bytes, void* stream);

/* For callers that can neither pass a workspace nor let the library allocate (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): batq_gemm_mxfp4_ws with the K-part sums in a 16 MiB array that
 * is part of the library's device code (one copy per GPU that runs the library, held until the process ends).
 * Same result, bit for bit, as batq_gemm_mxfp4_ws with a workspace of batq_gemm_workspace(w, M, 4) bytes.
 * BATQ_ERR_WORKSPACE if the shape asks for more than 16 MiB (no shape does on 256 compute units: the K parts
 * ask for at most 64 KiB per compute unit).  Calls no allocating routine.  All calls on one GPU share that
 * GPU's array, which keeps the last call's contents (nothing in it needs clearing): calls that overlap on one GPU
 * - different streams, or graphs replayed side by side - race on it and must be serialised by the caller. */
batq_status batq_gemm_mxfp4_noalloc(const uint8_t* xcodes, const uint8_t* xscales, const batq_weight* w,
                                    int M, void* Y, batq_dtype ydtype, int64_t ldy, void* stream);

/* Online steps 1+2: Y = Q(X P) Q(P^-1 W) (the objective of Sec. 3.1).
 * `workspace` is DEVICE memory (256-byte aligned) of at least batq_linear_workspace(M, K)
 * bytes (= batq_code_bytes(M, K) + batq_scale_bytes(M, K)).  It holds the activation codes
 * (at offset 0) followed by their scales, both in device order, between the two kernels.
 * What it holds beyond that (from the next 256-byte boundary on) serves the GEMM's K parts as in
 * batq_gemm_mxfp4_ws: batq_linear_workspace_for(w, M, act_bits) is the size with which every call of
 * the batq_linear family on M rows against `w` runs as fast as it can (>= batq_linear_workspace). */
size_t batq_linear_workspace(int M, int K);
size_t batq_linear_workspace_for(const batq_weight* w, int M, int act_bits);
batq_status batq_linear(const batq_transform* t, const batq_weight* w,
                        const void* X, batq_dtype xdtype, int M, int64_t ldx,
                        void* Y, batq_dtype ydtype, int64_t ldy,
                        void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------
 * W4A8: MXFP8 activations (E4M3 elements, the 8-bit variant Sec. 2 adopts) against the same MXFP4
 * weights.  Same transform, clipping and scale layout as above; the shared exponent is
 * E = clamp(floor(log2 bound) - 8, -127, 127), elements round to nearest even on the E4M3 grid
 * (1 sign, 4 exponent bits with bias 7, 3 mantissa bits) and saturate at 448; the code 0x7F / 0xFF
 * (NaN) is never produced.  One byte per element.
 * Device order of 8-bit codes: batq_code8_bytes(rows, K) bytes in the same 1 KiB pieces of 16 rows x
 * 64 bytes as the 4-bit codes, a piece now covering 2 MX blocks; elements 16h .. 16h+15 (h = 0, 1) of
 * block k of `row` are the 16 bytes at batq_code8_slot_offset(row, k, h, K)
 *   = ((row/16) * S8 + k/2) * 1024 + (row%16) * 64 + (((2*(k%2) + h) ^ ((row%16)/4)) * 16),
 * S8 = 4 * ceil(K/256); rows padded to 32, K zero-padded to 256.  Row-major order: [rows][K].
 * Alignment and error rules as for the 4-bit calls. */
batq_status batq_quantize_act_mxfp8(const batq_transform* t, const void* X, batq_dtype xdtype,
                                    int M, int K, int64_t ldx,
                                    uint8_t* codes8, uint8_t* scales, void* stream);
size_t batq_code8_bytes(int rows, int K);
size_t batq_code8_slot_offset(int row, int k, int half, int K);
batq_status batq_codes8_to_rowmajor(const uint8_t* device_order, uint8_t* rowmajor, int rows, int K, void* stream);
batq_status batq_codes8_from_rowmajor(const uint8_t* rowmajor, uint8_t* device_order, int rows, int K, void* stream);
/* Y[m][n] = sum_k 2^(xs[m][k]-127) 2^(ws[n][k]-127) sum_{j<32} e4m3(xq8[m][32k+j]) val(wq[n][32k+j]) */
batq_status batq_gemm_a8w4(const uint8_t* xcodes8, const uint8_t* xscales, const batq_weight* w,
                           int M, void* Y, batq_dtype ydtype, int64_t ldy, void* stream);
batq_status batq_gemm_a8w4_ws(const uint8_t* xcodes8, const uint8_t* xscales, const batq_weight* w,
                              int M, void* Y, batq_dtype ydtype, int64_t ldy,
                              void* workspace, size_t workspace_bytes, void* stream);
size_t batq_linear_a8w4_workspace(int M, int K);
batq_status batq_linear_a8w4(const batq_transform* t, const batq_weight* w,
                             const void* X, batq_dtype xdtype, int M, int64_t ldx,
                             void* Y, batq_dtype ydtype, int64_t ldy,
                             void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------
 * Options form of the online calls, for fusing the step before the quantiser (Sec. 3.2 places the
 * transforms behind the normalisation layers):
 *   act_bits   4 (or 0): MXFP4 activations; 8: MXFP8 (the *_mxfp8 / *_a8w4 calls above)
 *   row_scale  DEVICE fp32 [M] (4-byte aligned) or NULL: every transformed row is multiplied by
 *              row_scale[m] (one fp32 multiply per element) before clipping and quantisation.  With
 *              row_scale = 1/rms(x_m) (batq_row_rms_scale) and the norm weight folded into the
 *              transform blocks, T'_k = diag(gamma_k) T_k (dense form), this is RMSNorm -> transform
 *              -> quantise in one pass over X:  RMSNorm(x) T = r (x diag(gamma)) T.
 *   up, ld_up  DEVICE bf16 [M][K] with row stride ld_up elements (16-byte aligned rows), or NULL.  With
 *              `up`, X is the gate of a gated activation (the producer of the down projection's
 *              input, which Sec. 3.2 puts P_down in front of) and the quantiser's input is
 *              h = bf16(silu(X) * up): the product in fp32 (about 2^-21 relative; magnitudes below
 *              2^-100 may come out as zero), rounded once to bf16 as an unfused model would store
 *              it.  X must then be BATQ_BF16 (else BATQ_ERR_DTYPE); gate and up may be the two
 *              halves of one [M][2K] tensor (ldx = ld_up = 2K).
 * A NULL `opt` is the plain call; zero-initialise the struct and set what is needed.  The workspace of batq_linear_ex is batq_linear_workspace or
 * batq_linear_a8w4_workspace according to act_bits. */
typedef struct {
    int act_bits;
    const float* row_scale;
    const void* up;
    int64_t ld_up;
} batq_act_options;
batq_status batq_quantize_act_ex(const batq_transform* t, const void* X, batq_dtype xdtype,
                                 int M, int K, int64_t ldx, const batq_act_options* opt,
                                 uint8_t* codes, uint8_t* scales, void* stream);
batq_status batq_linear_ex(const batq_transform* t, const batq_weight* w,
                           const void* X, batq_dtype xdtype, int M, int64_t ldx,
                           const batq_act_options* opt,
                           void* Y, batq_dtype ydtype, int64_t ldy,
                           void* workspace, size_t workspace_bytes, void* stream);
/* row_scale[m] = 1 / sqrt(mean_j X[m][j]^2 + eps), fp32 accumulation; X as for batq_quantize_act. */
batq_status batq_row_rms_scale(const void* X, batq_dtype xdtype, int M, int K, int64_t ldx, float eps,
                               float* row_scale, void* stream);

/* ------------------------------------------------------------------------------------
 * Gate and up projection as one GEMM with the gated activation in its epilogue (Sec. 3.2, "MLP Module": P_up
 * sits in front of up_proj and gate_proj, which therefore share their quantised input).
 *
 * batq_prepare_weight_gate_up: like batq_prepare_weight for two matrices of the same shape (K x F or F x K,
 *   same dtype, leading dimension and clip ratios): the prepared weight has N = 2 F columns, gate and up
 *   interleaved in groups of 32 (column 64 p + j = gate column 32 p + j, column 64 p + 32 + j = up column
 *   32 p + j, j < 32).  F must be a multiple of 32.  batq_weight_export / batq_gemm_mxfp4 see the 2 F columns in
 *   this order.
 * batq_gemm_glu: H[m][f] = silu(g) * u with g, u the fp32 sums of batq_gemm_mxfp4 (act_bits 4 or 0) or
 *   batq_gemm_a8w4 (act_bits 8) for the gate and up column of f; the product is formed in fp32 (about 2^-21
 *   relative) and rounded once to the output type.  H is M x N/2 (DEVICE, row stride ldh >= N/2 elements).  The
 *   weight's N must be a multiple of 64 (BATQ_ERR_SHAPE); with M > 64, operand code arrays of 2 GiB or more
 *   are not supported (BATQ_ERR_UNSUPPORTED).  K parts are not used.
 * batq_linear_glu: batq_linear_ex (same options and workspace) followed by the gated epilogue. */
batq_status batq_prepare_weight_gate_up(batq_weight** out, const batq_transform* t, const void* W_gate,
                                        const void* W_up, batq_dtype wdtype, int K, int F, int64_t ldw,
                                        int w_is_KxN, const float* clip_w, void* stream);
batq_status batq_gemm_glu(const uint8_t* xcodes, const uint8_t* xscales, const batq_weight* w, int M,
                          int act_bits, void* H, batq_dtype hdtype, int64_t ldh, void* stream);
batq_status batq_linear_glu(const batq_transform* t, const batq_weight* w, const void* X, batq_dtype xdtype,
                            int M, int64_t ldx, const batq_act_options* opt, void* H, batq_dtype hdtype,
                            int64_t ldh, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------
 * Key/value cache (Sec. 3.2, "Self-Attention Module": P_k and P_v transform the key and value cache head by
 * head).  A cache row is written with batq_quantize_act[_ex] on the [tokens][kv_heads * head_dim] key or value
 * tensor: the blocks of a head (head_dim / 32 of them) each carry their own T_k, act_bits 4 or 8 gives KV4 or
 * KV8.  The two calls below are the pieces around it for an attention kernel that works on 16-bit tensors.
 *
 * batq_dequantize: codes (DEVICE, device order of the given width) and scales (DEVICE, grouped order) of `M`
 *   rows -> out[m][j] = value(code) * 2^(scale - 127), row-major with row stride ldo elements (16-byte aligned
 *   rows), bf16 or fp32.  fp32 output is exact (subnormal results included; scale byte 255 and the E4M3 NaN
 *   codes give NaN); bf16 output uses the hardware's scaled converts and is exact for every result in bf16's
 *   normal range (results below 2^-126 are not specified).  bits = 4 or 8, else BATQ_ERR_UNSUPPORTED.
 *
 * batq_transform_apply: out = X T_k (FORWARD), X T_k^-1 (INVERSE) or X T_k^-T (INVERSE_T) block by block, no
 *   clipping or quantisation.  bf16 input with 16-byte aligned X, out and row pitches runs on the matrix
 *   cores with the arithmetic of the quantiser's transform (the handle's fp64 block split into three bf16
 *   terms, exact products, fp32 sums: within 2^-20 sum_j |x_j| |B_jk| of the exact result; FORWARD gives
 *   bit for bit the values batq_quantize_act quantises).  Any other input (fp32, unaligned) takes a slow
 *   reference route: products and sums in fp64, one rounding to fp32.  bf16 output adds one rounding.  The
 *   query side of a transformed key cache takes INVERSE_T ((q T^-T)(k T)^T = q k^T), the attention output
 *   over a transformed value cache takes INVERSE (or folds T_v^-1 into the output projection).  X and out
 *   as for batq_quantize_act (DEVICE, row strides in elements); not in place (BATQ_ERR_SHAPE).
 *
 * A cache that grows: batq_kv_append quantises M new token rows of X exactly as batq_quantize_act (act_bits 4) or
 *   batq_quantize_act_mxfp8 (act_bits 8) would, but into rows row_offset .. row_offset + M - 1 of code and scale
 *   arrays (DEVICE, caller-owned) that are laid out for capacity_rows rows: batq_code_bytes / batq_code8_bytes and
 *   batq_scale_bytes of (capacity_rows, K).  Rows are independent, and a row's codes and scale do not depend on
 *   the append that brought it: any sequence of appends leaves exactly the bytes one call over all rows writes
 *   (bf16 rows always take the matrix-core arithmetic, fp32 rows the register-level kernel).  Of a bf16 append of
 *   more than 2^22 / K rows the part from the first multiple of 32 on is written in whole 32-row tiles of codes: the
 *   code rows after the appended block up to the next multiple of 32 (not yet part of the cache) then hold
 *   unspecified values; other appends write their own rows only.
 *   BATQ_ERR_SHAPE if the window does not fit.
 *   batq_kv_dequantize reads rows row_offset .. row_offset + M - 1 of such arrays into out rows 0 .. M - 1
 *   (otherwise as batq_dequantize).  Both are asynchronous on `stream` and allocate nothing. */
typedef enum { BATQ_APPLY_FORWARD = 0, BATQ_APPLY_INVERSE = 1, BATQ_APPLY_INVERSE_T = 2 } batq_apply_mode;
batq_status batq_dequantize(const uint8_t* codes, const uint8_t* scales, int M, int K, int bits,
                            void* out, batq_dtype odtype, int64_t ldo, void* stream);
batq_status batq_transform_apply(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int K,
                                 int64_t ldx, batq_apply_mode mode, void* out, batq_dtype odtype, int64_t ldo,
                                 void* stream);
batq_status batq_kv_append(const batq_transform* t, const void* X, batq_dtype xdtype, int M, int K, int64_t ldx,
                           int act_bits, uint8_t* codes, uint8_t* scales, int64_t row_offset, int64_t capacity_rows,
                           void* stream);
batq_status batq_kv_dequantize(const uint8_t* codes, const uint8_t* scales, int64_t capacity_rows, int64_t row_offset,
                               int M, int K, int bits, void* out, batq_dtype odtype, int64_t ldo, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BATQ_H */
