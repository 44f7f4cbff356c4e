"""CPU oracle for the BATQuant W4A4 MXFP4 linear layer.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 NumPy statement of what the hot path computes, written from
the paper's equations and the MX format definition it cites.  Only the tests,
the smoke check and the benchmark's ``cpu_baseline`` leg may call it; the
product path never does and shares no code with it.

What each function follows (notation: X is M x K tokens x in-features, W is
K x N in x out, Y = X W; the paper writes the same layer as Y = X W^T with W
out x in, Sec. 3.1):

* ``kron_blocks``      - Eq. 2 (P_i as a Kronecker product of a shared and a
                         private factor), in the factor order T_k = G (x) P_k
                         with G global and P_k private.
* ``kron_blocks_general`` - the other forms Sec. 3.1.1 discusses: either factor
                         shared or private (the order Eq. 2 prints, private (x)
                         global; the naive Kronecker with both private); a dense
                         P_i is passed to the ``*_blocks`` functions directly.
* ``transform``        - Eq. 1 (block-diagonal P applied block by block).
* ``clip_blocks``      - Eq. 3-4 specialised to one symmetric ratio on the
                         block's absolute maximum; ``clip_blocks_minmax`` is
                         Eq. 3-4 as printed (two ratios on block min and max);
                         ``mxfp4_quantize_minmax`` quantises what it leaves.
* ``mxfp4_quantize``   - Sec. 2 "Microscaling Floating-Point Definition":
                         E2M1 elements, 32 per block, one UE8M0 scale; shared
                         exponent floor(log2 amax) - 2, round-to-nearest-even,
                         saturation at +-6.
* ``mxfp8_quantize``   - the same definition for MXFP8 with E4M3 elements, the
                         variant Sec. 2 adopts for 8-bit activations (W4A8):
                         shared exponent floor(log2 amax) - 8, saturation at
                         +-448; ``gemm_a8w4`` multiplies such activations with
                         MXFP4 weights.
* ``rmsnorm`` / ``fold_norm_weight`` / ``row_rms_scale`` - the normalisation layer
                         the transforms sit behind (Sec. 3.2, placement of P_qkv and
                         P_up) and the identity that lets it be fused:
                         RMSNorm(x) T = r (x diag(gamma)) T.
* ``silu`` / ``swiglu`` / ``swiglu_bf16`` - the gated activation whose output is the input of the
                         down projection (Sec. 3.2, placement of P_down): silu(gate) * up
                         as a plain definition, and its rounding to the bf16 tensor a model
                         hands to the layer.
* ``inverse_transpose_blocks`` / ``apply_blocks`` - the key/value-cache placement of Sec. 3.2
                         (P_k, P_v head by head): keys are stored as Q(k T), the query side
                         takes q T^-T so that (q T^-T)(k T)^T = q k^T; values are stored as
                         Q(v T) and the attention output takes T^-1.
* ``prepare_weight``   - Alg. 2 "Offline Fusion" (inverse transform of W,
                         clip, quantise).
* ``gemm`` / ``linear``- the objective of Sec. 3.1, Q(XP) Q(P^-1 W^T).

Every intermediate is fp64 except the two places where the definition fixes
fp32: the transformed tensor is rounded once to fp32 before the quantiser, and
the clip bound is one fp32 product ratio * amax.

Pins (tests/test_oracle_*.py): the E2M1 grid printed in Sec. 2; hand-computed
blocks in tests/golden/; idempotence and error bounds of the quantiser;
numpy.kron and the vec identity of Sec. 3.1.1; (X T)(T^-1 W) = X W;
permutation / power-of-two / Hadamard special transforms; brute-force triple
loop for the GEMM; Table 1 parameter counts.  The model-level accuracy tables
of the paper are not reproducible here: parity unpinned against those.
"""
from __future__ import annotations

import numpy as np

BLOCK = 32
# Sec. 2: the positive E2M1 values; code = index, bit 3 of a 4-bit code is the sign.
E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float64)
E2M1_EMAX = 2          # 6 = 1.5 * 2**2
E8M0_BIAS = 127


# --------------------------------------------------------------------------- bf16 helpers
def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16 value (ties to even); result returned as fp32.

    Rounds straight from the input precision (fp64 or fp32), by comparing with
    the two neighbouring bf16 values, so there is no double rounding.
    """
    x = np.asarray(x, dtype=np.float64)
    f = x.astype(np.float32)
    u = f.view(np.uint32)
    lo_bits = u & np.uint32(0xFFFF0000)          # bf16 neighbour towards zero of the fp32 rounding
    lo = lo_bits.view(np.float32).astype(np.float64)
    # the fp32 rounding may have moved past x; step back one bf16 ulp when |lo| > |x|
    back = np.abs(lo) > np.abs(x)
    lo_bits = np.where(back, lo_bits - np.uint32(0x10000), lo_bits).astype(np.uint32)
    lo = lo_bits.view(np.float32).astype(np.float64)
    hi_bits = (lo_bits + np.uint32(0x10000)).astype(np.uint32)
    hi = hi_bits.view(np.float32).astype(np.float64)
    dl = np.abs(x - lo)
    dh = np.abs(hi - x)
    even_lo = ((lo_bits >> np.uint32(16)) & np.uint32(1)) == 0
    take_lo = (dl < dh) | ((dl == dh) & even_lo)
    out = np.where(take_lo, lo_bits, hi_bits).astype(np.uint32)
    return out.view(np.float32)


# --------------------------------------------------------------------------- transform
def kron_blocks(G: np.ndarray, P: np.ndarray) -> np.ndarray:
    """Dense T_k = G (x) P_k for every block, fp64, shape [nb, g, g] (Eq. 2).

    T_k[a*gi + c, a2*gi + c2] = G[a, a2] * P_k[c, c2], with G go x go shared by
    all blocks and P_k gi x gi private, go*gi = 32.
    """
    G = np.asarray(G, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    go, gi = G.shape[0], P.shape[1]
    assert G.shape == (go, go) and P.shape[1:] == (gi, gi) and go * gi == BLOCK
    nb = P.shape[0]
    T = np.empty((nb, BLOCK, BLOCK), dtype=np.float64)
    for a in range(go):
        for c in range(gi):
            for a2 in range(go):
                for c2 in range(gi):
                    T[:, a * gi + c, a2 * gi + c2] = G[a, a2] * P[:, c, c2]
    return T


def kron_blocks_private_outer(B: np.ndarray, A: np.ndarray) -> np.ndarray:
    """Dense P_i = B_i (x) A, the factor order Eq. 2 prints (private (x) global)."""
    B = np.asarray(B, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    g2, g1 = B.shape[1], A.shape[0]
    assert g1 * g2 == BLOCK
    nb = B.shape[0]
    T = np.empty((nb, BLOCK, BLOCK), dtype=np.float64)
    for b in range(g2):
        for a in range(g1):
            for b2 in range(g2):
                for a2 in range(g1):
                    T[:, b * g1 + a, b2 * g1 + a2] = B[:, b, b2] * A[a, a2]
    return T


def kron_blocks_general(outer: np.ndarray, inner: np.ndarray, nb: int) -> np.ndarray:
    """Dense T_k = O_k (x) I_k, fp64 [nb, 32, 32]; a factor given as one matrix is shared by all blocks.

    T_k[a*gi + c, a2*gi + c2] = O_k[a, a2] * I_k[c, c2].  Shared outer + per-block inner is the
    Global-and-Private form; per-block outer + shared inner is the order Eq. 2 prints; both
    per-block is the naive Kronecker decomposition of Sec. 3.1.1.
    """
    O = np.asarray(outer, dtype=np.float64)
    I = np.asarray(inner, dtype=np.float64)
    go, gi = O.shape[-1], I.shape[-1]
    assert go * gi == BLOCK and O.shape[-2] == go and I.shape[-2] == gi
    T = np.empty((nb, BLOCK, BLOCK), dtype=np.float64)
    for k in range(nb):
        Ok = O if O.ndim == 2 else O[k]
        Ik = I if I.ndim == 2 else I[k]
        for a in range(go):
            for a2 in range(go):
                T[k, a * gi:(a + 1) * gi, a2 * gi:(a2 + 1) * gi] = Ok[a, a2] * Ik
    return T


def apply_blocks(X: np.ndarray, T: np.ndarray) -> np.ndarray:
    """Eq. 1: y_k = x_k T_k for every 32-wide block k of every row; fp64 in, fp64 out."""
    X = np.asarray(X, dtype=np.float64)
    M, K = X.shape
    nb = K // BLOCK
    assert K % BLOCK == 0 and T.shape == (nb, BLOCK, BLOCK)
    Xb = X.reshape(M, nb, BLOCK).transpose(1, 0, 2)          # [nb, M, 32]
    Yb = np.matmul(Xb, T)                                    # [nb, M, 32]
    return np.ascontiguousarray(Yb.transpose(1, 0, 2)).reshape(M, K)


def transform(X: np.ndarray, G, P) -> np.ndarray:
    """Transformed activations rounded once to fp32; identity when G is None."""
    if G is None:
        return np.asarray(X, dtype=np.float64).astype(np.float32)
    return apply_blocks(X, kron_blocks(G, P)).astype(np.float32)


# --------------------------------------------------------------------------- clipping
def clip_blocks(Xt32: np.ndarray, clip) -> tuple[np.ndarray, np.ndarray]:
    """Symmetric block clip: bound a' = fl32(c_k * amax_k), x clamped to [-a', a'].

    Returns (clipped fp32 [R, nb, 32], a' fp32 [R, nb]).  ``clip`` None means 1.
    """
    X = np.asarray(Xt32, dtype=np.float32)
    R, K = X.shape
    nb = K // BLOCK
    Xb = X.reshape(R, nb, BLOCK)
    amax = np.max(np.abs(Xb), axis=2)                        # fp32, exact
    if clip is None:
        bound = amax
    else:
        c = np.asarray(clip, dtype=np.float32).reshape(1, nb)
        bound = (c * amax).astype(np.float32)                # one fp32 multiply
    b = np.broadcast_to(bound[:, :, None], Xb.shape)
    # an element beyond the bound is replaced by the bound with the element's sign;
    # every other element (signed zeros included) passes through unchanged
    return np.where(np.abs(Xb) > b, np.copysign(b, Xb), Xb), bound


def clip_blocks_minmax(Xt32: np.ndarray, r_min, r_max) -> np.ndarray:
    """Eq. 3-4 as printed: clip(x, r_min*min(x), r_max*max(x)) per block (fp32 bounds)."""
    X = np.asarray(Xt32, dtype=np.float32)
    R, K = X.shape
    nb = K // BLOCK
    Xb = X.reshape(R, nb, BLOCK)
    lo = (np.asarray(r_min, np.float32).reshape(1, nb) * Xb.min(axis=2)).astype(np.float32)
    hi = (np.asarray(r_max, np.float32).reshape(1, nb) * Xb.max(axis=2)).astype(np.float32)
    lo = np.broadcast_to(lo[:, :, None], Xb.shape)
    hi = np.broadcast_to(hi[:, :, None], Xb.shape)
    return np.where(Xb < lo, lo, np.where(Xb > hi, hi, Xb))


# --------------------------------------------------------------------------- MXFP4 quantiser
def shared_exponent(bound: np.ndarray) -> np.ndarray:
    """E = floor(log2 bound) - 2 clamped to [-127, 127]; E = -127 for a zero block."""
    b = np.asarray(bound, dtype=np.float64)
    m, e = np.frexp(b)                                       # b = m * 2**e, m in [0.5, 1)
    E = np.where(b > 0, e - 1 - E2M1_EMAX, -E8M0_BIAS)
    return np.clip(E, -127, 127).astype(np.int64)


def e2m1_encode(v: np.ndarray, negative: np.ndarray) -> np.ndarray:
    """Nearest E2M1 magnitude code of |v| (ties to the even code, saturating), sign in bit 3."""
    mag = np.abs(np.asarray(v, dtype=np.float64))
    d = np.abs(mag[..., None] - E2M1_GRID)                   # distance to each grid value
    dmin = d.min(axis=-1, keepdims=True)
    cand = d == dmin                                         # one or two neighbours
    idx = np.arange(8)
    first = np.where(cand, idx, 99).min(axis=-1)
    last = np.where(cand, idx, -1).max(axis=-1)
    code = np.where(first == last, first, np.where(first % 2 == 0, first, last))
    return (code | (np.asarray(negative, dtype=np.int64) << 3)).astype(np.uint8)


def quantize_clipped(Xc: np.ndarray, bound: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """Clipped fp32 blocks [R, nb, 32] + bounds [R, nb] -> (codes u8 [R, nb, 32], scales u8 [R, nb])."""
    E = shared_exponent(bound)
    v = np.asarray(Xc, dtype=np.float64) * np.exp2(-E.astype(np.float64))[:, :, None]   # exact
    codes = e2m1_encode(v, np.signbit(Xc))
    return codes, (E + E8M0_BIAS).astype(np.uint8)


# --------------------------------------------------------------------------- MXFP8 (E4M3) activations
E4M3_EMAX = 8          # largest E4M3 value 448 = 1.75 * 2**8
E4M3_MAX = 448.0


def e4m3_value(code: np.ndarray) -> np.ndarray:
    """Value of an 8-bit S|EEEE|MMM code, exponent bias 7; S.1111.111 (NaN) is never produced and
    decodes to NaN."""
    c = np.asarray(code, dtype=np.int64)
    e, m = (c >> 3) & 15, c & 7
    mag = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * np.exp2(e - 7.0))
    mag = np.where((c & 0x7F) == 0x7F, np.nan, mag)
    return np.where(c & 0x80, -mag, mag)


_E4M3_GRID = e4m3_value(np.arange(127))     # the 127 finite non-negative values, ascending, index = code


def e4m3_encode(v: np.ndarray, negative: np.ndarray) -> np.ndarray:
    """Nearest E4M3 magnitude code of |v| (ties to the even code, saturating at 448), sign in bit 7."""
    mag = np.minimum(np.abs(np.asarray(v, dtype=np.float64)), E4M3_MAX)
    hi = np.clip(np.searchsorted(_E4M3_GRID, mag, side="left"), 1, 126)      # first grid value >= mag
    lo = hi - 1
    dl, dh = mag - _E4M3_GRID[lo], _E4M3_GRID[hi] - mag
    code = np.where(dl < dh, lo, np.where(dh < dl, hi, np.where(lo % 2 == 0, lo, hi)))
    code = np.where(mag == 0, 0, code)
    return (code | (np.asarray(negative, dtype=np.int64) << 7)).astype(np.uint8)


def mxfp8_quantize(Xt32: np.ndarray, clip=None) -> tuple[np.ndarray, np.ndarray]:
    """fp32 [R, K] -> (E4M3 codes u8 [R, K], E8M0 scales u8 [R, K/32]): symmetric clip as for MXFP4,
    shared exponent E = floor(log2 bound) - 8 clamped to [-127, 127], round to nearest even, saturate."""
    Xc, bound = clip_blocks(Xt32, clip)
    b = np.asarray(bound, dtype=np.float64)
    _, e = np.frexp(b)
    E = np.clip(np.where(b > 0, e - 1 - E4M3_EMAX, -E8M0_BIAS), -127, 127).astype(np.int64)
    v = np.asarray(Xc, dtype=np.float64) * np.exp2(-E.astype(np.float64))[:, :, None]     # exact
    codes = e4m3_encode(v, np.signbit(Xc))
    return codes.reshape(Xc.shape[0], -1), (E + E8M0_BIAS).astype(np.uint8)


def dequantize_fp8(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """(E4M3 codes [R, K], scales [R, K/32]) -> fp64 [R, K]."""
    s = np.exp2(np.asarray(scales, dtype=np.float64) - E8M0_BIAS)
    return e4m3_value(codes) * np.repeat(s, BLOCK, axis=1)


def quantize_act_fp8(X: np.ndarray, T, clip=None, chunk: int = 512) -> tuple[np.ndarray, np.ndarray]:
    """Online activation path with MXFP8 output for dense blocks T [nb, 32, 32] (None = identity)."""
    X = np.asarray(X)
    cs, ss = [], []
    for r0 in range(0, X.shape[0], chunk):
        Xr = X[r0:r0 + chunk]
        Xt = np.asarray(Xr, np.float64).astype(np.float32) if T is None else apply_blocks(Xr, T).astype(np.float32)
        c, s_ = mxfp8_quantize(Xt, clip)
        cs.append(c)
        ss.append(s_)
    if not cs:
        return (np.zeros((0, X.shape[1]), np.uint8), np.zeros((0, X.shape[1] // BLOCK), np.uint8))
    return np.concatenate(cs), np.concatenate(ss)


def gemm_a8w4(xcodes8, xscales, wcodes, wscales) -> np.ndarray:
    """Y[m, n] = sum_k dq8(x)[m, k] * dq4(w)[n, k] in fp64 (MXFP8 activations, MXFP4 weights)."""
    return dequantize_fp8(xcodes8, xscales) @ dequantize(wcodes, wscales).T


def pack_codes(codes: np.ndarray) -> np.ndarray:
    """[R, nb, 32] 4-bit codes -> [R, K/2] bytes, even element in the low nibble."""
    R = codes.shape[0]
    c = codes.reshape(R, -1)
    return (c[:, 0::2] | (c[:, 1::2] << 4)).astype(np.uint8)


def unpack_codes(packed: np.ndarray) -> np.ndarray:
    """[R, K/2] bytes -> [R, K] 4-bit codes."""
    R, Kh = packed.shape
    out = np.empty((R, Kh * 2), dtype=np.uint8)
    out[:, 0::2] = packed & 0xF
    out[:, 1::2] = packed >> 4
    return out


def mxfp4_quantize(Xt32: np.ndarray, clip=None) -> tuple[np.ndarray, np.ndarray]:
    """fp32 [R, K] -> (packed codes u8 [R, K/2], E8M0 scales u8 [R, K/32]): clip, scale, round, pack."""
    Xc, bound = clip_blocks(Xt32, clip)
    codes, scales = quantize_clipped(Xc, bound)
    return pack_codes(codes), scales


def mxfp4_quantize_minmax(Xt32: np.ndarray, r_min, r_max) -> tuple[np.ndarray, np.ndarray]:
    """As ``mxfp4_quantize`` with the clipping of Eq. 3-4 as printed: x clamped to
    [fl32(r_min * min), fl32(r_max * max)] per block; the shared scale comes from the largest
    magnitude that is left."""
    Xc = clip_blocks_minmax(Xt32, r_min, r_max)
    bound = np.max(np.abs(Xc), axis=2).astype(np.float32)
    codes, scales = quantize_clipped(Xc, bound)
    return pack_codes(codes), scales


def rmsnorm(X: np.ndarray, gamma: np.ndarray, eps: float) -> np.ndarray:
    """RMSNorm as a plain definition, fp64: x_j * gamma_j / sqrt(mean_j x_j^2 + eps)."""
    X = np.asarray(X, dtype=np.float64)
    return X / np.sqrt(np.mean(X * X, axis=1, keepdims=True) + eps) * np.asarray(gamma, dtype=np.float64)[None, :]


def row_rms_scale(X: np.ndarray, eps: float) -> np.ndarray:
    """r_m = 1 / sqrt(mean_j x_mj^2 + eps), fp64."""
    X = np.asarray(X, dtype=np.float64)
    return 1.0 / np.sqrt(np.mean(X * X, axis=1) + eps)


def fold_norm_weight(T: np.ndarray, gamma: np.ndarray) -> np.ndarray:
    """T'_k = diag(gamma_k) T_k: the norm weight moved into the transform blocks."""
    T = np.asarray(T, dtype=np.float64)
    return T * np.asarray(gamma, dtype=np.float64).reshape(T.shape[0], BLOCK, 1)


def silu(x: np.ndarray) -> np.ndarray:
    """x * sigmoid(x) = x / (1 + exp(-x)), fp64."""
    x = np.asarray(x, dtype=np.float64)
    with np.errstate(over="ignore"):
        return x / (1.0 + np.exp(-x))


def swiglu(gate: np.ndarray, up: np.ndarray) -> np.ndarray:
    """silu(gate) * up element by element, fp64."""
    return silu(gate) * np.asarray(up, dtype=np.float64)


def swiglu_bf16(gate: np.ndarray, up: np.ndarray) -> np.ndarray:
    """The gated activation as the bf16 tensor the down projection receives: one rounding of the
    fp64 product to bf16 (returned as fp32)."""
    return bf16_round(swiglu(gate, up))


def quantize_act_blocks(X: np.ndarray, T, clip=None, clip_min=None, clip_max=None,
                        chunk: int = 512, row_scale=None, fp8: bool = False) -> tuple[np.ndarray, np.ndarray]:
    """Online activation path for dense blocks T [nb, 32, 32] (None = identity): optional row factors,
    Eq. 1, then either the symmetric clip (``clip``) or the two-ratio clip of Eq. 3-4 (``clip_min``,
    ``clip_max``), then MXFP4 (MXFP8 with ``fp8``)."""
    X = np.asarray(X)
    assert (clip_min is None) == (clip_max is None) and (clip is None or clip_min is None)
    assert not (fp8 and clip_min is not None)
    cs, ss = [], []
    for r0 in range(0, X.shape[0], chunk):
        Xr = np.asarray(X[r0:r0 + chunk], dtype=np.float64)
        if row_scale is not None:                       # each row times its factor (e.g. RMSNorm's 1/rms)
            Xr = Xr * np.asarray(row_scale, dtype=np.float64)[r0:r0 + chunk, None]
        Xt = Xr.astype(np.float32) if T is None else apply_blocks(Xr, T).astype(np.float32)
        if fp8:
            c, s = mxfp8_quantize(Xt, clip)
        else:
            c, s = mxfp4_quantize(Xt, clip) if clip_min is None else mxfp4_quantize_minmax(Xt, clip_min, clip_max)
        cs.append(c)
        ss.append(s)
    if not cs:
        return (np.zeros((0, X.shape[1] // (1 if fp8 else 2)), np.uint8), np.zeros((0, X.shape[1] // BLOCK), np.uint8))
    return np.concatenate(cs), np.concatenate(ss)


def quantize_act(X: np.ndarray, G, P, clip, chunk: int = 512) -> tuple[np.ndarray, np.ndarray]:
    """Online activation path: transform (Eq. 1-2), clip (Eq. 3-4), MXFP4 (Sec. 2)."""
    X = np.asarray(X)
    T = None if G is None else kron_blocks(G, P)
    cs, ss = [], []
    for r0 in range(0, X.shape[0], chunk):
        Xr = X[r0:r0 + chunk]
        Xt = np.asarray(Xr, np.float64).astype(np.float32) if T is None else apply_blocks(Xr, T).astype(np.float32)
        c, s = mxfp4_quantize(Xt, clip)
        cs.append(c)
        ss.append(s)
    if not cs:
        return (np.zeros((0, X.shape[1] // 2), np.uint8), np.zeros((0, X.shape[1] // BLOCK), np.uint8))
    return np.concatenate(cs), np.concatenate(ss)


def dequantize(packed: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """(codes, scales) -> fp64 [R, K]: sign * grid[code & 7] * 2**(scale - 127)."""
    c = unpack_codes(np.asarray(packed, dtype=np.uint8))
    val = E2M1_GRID[c & 7] * np.where(c & 8, -1.0, 1.0)
    s = np.exp2(np.asarray(scales, dtype=np.float64) - E8M0_BIAS)
    return val * np.repeat(s, BLOCK, axis=1)


# --------------------------------------------------------------------------- weights
def invert(Tk: np.ndarray) -> np.ndarray:
    """fp64 Gauss-Jordan inverse with partial pivoting of one square matrix."""
    n = Tk.shape[0]
    A = np.concatenate([np.array(Tk, dtype=np.float64), np.eye(n)], axis=1)
    for col in range(n):
        piv = col + int(np.argmax(np.abs(A[col:, col])))
        if abs(A[piv, col]) < 1e-12 * max(1.0, float(np.abs(Tk).max())):
            raise np.linalg.LinAlgError("singular transform block")
        if piv != col:
            A[[col, piv]] = A[[piv, col]]
        A[col] /= A[col, col]
        for r in range(n):
            if r != col:
                A[r] -= A[r, col] * A[col]
    return A[:, n:]


def inverse_transpose_blocks(T: np.ndarray) -> np.ndarray:
    """T_k^-T for every block: the query-side companion of a key transform, (q T^-T)(k T)^T = q k^T."""
    T = np.asarray(T, dtype=np.float64)
    return np.stack([invert(T[k]).T for k in range(T.shape[0])])


def inverse_blocks(T: np.ndarray) -> np.ndarray:
    """T_k^-1 for every block (undoes a value transform on the attention output)."""
    T = np.asarray(T, dtype=np.float64)
    return np.stack([invert(T[k]) for k in range(T.shape[0])])


def inverse_transform_weight(W: np.ndarray, G, P) -> np.ndarray:
    """W~ = P^-1 W: each 32-row K-slab of W (K x N) is multiplied from the left by T_k^-1; fp64."""
    W = np.asarray(W, dtype=np.float64)
    K, N = W.shape
    nb = K // BLOCK
    if G is None:
        return W
    T = kron_blocks(G, P)
    out = np.empty_like(W)
    for k in range(nb):
        out[k * BLOCK:(k + 1) * BLOCK] = invert(T[k]) @ W[k * BLOCK:(k + 1) * BLOCK]
    return out


def prepare_weight(W: np.ndarray, G, P, clip_w=None, chunk: int = 1024) -> tuple[np.ndarray, np.ndarray]:
    """Offline weight path (Alg. 2, offline fusion): inverse transform, fp32, clip, MXFP4 along K.

    W is K x N.  Returns canonical (codes [N, K/2], scales [N, K/32]).
    """
    Wt = inverse_transform_weight(W, G, P).astype(np.float32)            # [K, N]
    cs, ss = [], []
    for n0 in range(0, Wt.shape[1], chunk):
        c, s = mxfp4_quantize(np.ascontiguousarray(Wt[:, n0:n0 + chunk].T), clip_w)
        cs.append(c)
        ss.append(s)
    return np.concatenate(cs), np.concatenate(ss)


def prepare_weight_blocks(W: np.ndarray, T, clip_w=None, clip_min=None, clip_max=None,
                          chunk: int = 1024) -> tuple[np.ndarray, np.ndarray]:
    """Offline weight path for dense blocks T [nb, 32, 32] (None = identity): each 32-row K-slab of W
    (K x N) multiplied from the left by T_k^-1 in fp64, one rounding to fp32, clip (symmetric or the two
    ratios of Eq. 3-4), MXFP4 along K.  Returns canonical (codes [N, K/2], scales [N, K/32])."""
    W = np.asarray(W, dtype=np.float64)
    assert (clip_min is None) == (clip_max is None) and (clip_w is None or clip_min is None)
    if T is None:
        Wt = W.astype(np.float32)
    else:
        Wt = np.empty(W.shape, dtype=np.float32)
        for k in range(W.shape[0] // BLOCK):
            Wt[k * BLOCK:(k + 1) * BLOCK] = (invert(T[k]) @ W[k * BLOCK:(k + 1) * BLOCK]).astype(np.float32)
    cs, ss = [], []
    for n0 in range(0, Wt.shape[1], chunk):
        Wn = np.ascontiguousarray(Wt[:, n0:n0 + chunk].T)
        c, s = mxfp4_quantize(Wn, clip_w) if clip_min is None else mxfp4_quantize_minmax(Wn, clip_min, clip_max)
        cs.append(c)
        ss.append(s)
    return np.concatenate(cs), np.concatenate(ss)


# --------------------------------------------------------------------------- GEMM / linear
def gemm(xcodes, xscales, wcodes, wscales) -> np.ndarray:
    """Y[m, n] = sum_k dq(x)[m, k] * dq(w)[n, k] in fp64."""
    return dequantize(xcodes, xscales) @ dequantize(wcodes, wscales).T


def linear(X, W, G, P, clip, clip_w=None) -> np.ndarray:
    """Q(X P) Q(P^-1 W) end to end, fp64 output."""
    xc, xs = quantize_act(X, G, P, clip)
    wc, ws = prepare_weight(W, G, P, clip_w)
    return gemm(xc, xs, wc, ws)


# --------------------------------------------------------------------------- Table 1
def param_count(N: int, g: int, g1: int, g2: int, method: str) -> int:
    """Number of learnable entries of P for a hidden size N (Table 1)."""
    k = N // g
    if method == "flatquant":          # two sqrt(N) x sqrt(N) Kronecker factors
        r = int(round(N ** 0.5))
        return 2 * r * r
    if method == "dense":
        return N * g
    if method == "naive_kron":
        return k * (g1 * g1 + g2 * g2)
    if method == "gpk":
        return g1 * g1 + k * g2 * g2
    raise ValueError(method)
