"""GPU parity for the key/value-cache helpers: dequantise (bit-exact) and the unquantised block transforms
(forward, inverse, inverse transpose), and the cache path they form with the quantiser."""
import numpy as np
import pytest

import batq_inputs as bi
from oracle import batq_oracle as o
from gpu_util import (require_gpu, to_dev, y_to_f32, rowmajor_to_blocked, rowmajor_to_blocked8, rowmajor_to_grouped,
                      assert_same_quantisation)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    require_gpu()
    import paper_2603_16590_amd as b
    return b


@pytest.mark.parametrize("M,K", [(1, 32), (37, 96), (130, 1024 + 64), (513, 256)])
@pytest.mark.parametrize("bits", [4, 8])
def test_dequantise_is_bit_exact(B, M, K, bits):
    import torch
    rng = np.random.default_rng(M * 3 + K + bits)
    nb = K // 32
    if bits == 4:
        codes = rng.integers(0, 256, (M, K // 2), dtype=np.uint8)
        dev_codes = torch.from_numpy(rowmajor_to_blocked(codes)).cuda()
    else:
        codes = rng.integers(0, 256, (M, K), dtype=np.uint8)
        codes[(codes & 0x7F) == 0x7F] = 0x21                       # NaN codes are tested below
        dev_codes = torch.from_numpy(rowmajor_to_blocked8(codes)).cuda()
    # fp32 output: every scale byte whose products are finite fp32 numbers, subnormal results included
    scales = rng.integers(0, 246 if bits == 4 else 240, (M, nb), dtype=np.uint8)
    scales[0, 0] = 0
    dev_scales = torch.from_numpy(rowmajor_to_grouped(scales)).cuda()
    ref = (o.dequantize if bits == 4 else o.dequantize_fp8)(codes, scales)
    got = B.batq_dequantize(dev_codes, dev_scales, M, K, bits, torch.float32)
    torch.cuda.synchronize()
    g = got.cpu().numpy()
    assert np.array_equal(g.astype(np.float64), ref)                # exact values
    assert np.array_equal(np.signbit(g), np.signbit(ref))           # and the sign of zeros
    # bf16 output: exact for everything in bf16's normal range
    scales_b = rng.integers(20, 240, (M, nb), dtype=np.uint8)
    dev_scales_b = torch.from_numpy(rowmajor_to_grouped(scales_b)).cuda()
    ref_b = (o.dequantize if bits == 4 else o.dequantize_fp8)(codes, scales_b)
    out = torch.zeros((M, K + 8), dtype=torch.bfloat16, device="cuda")     # strided output rows
    B.batq_dequantize(dev_codes, dev_scales_b, M, K, bits, out=out[:, :K])
    torch.cuda.synchronize()
    assert np.array_equal(y_to_f32(out[:, :K]).astype(np.float64), ref_b)
    assert bool((out[:, K:] == 0).all())


def test_dequantise_nan_codes_and_errors(B):
    import torch
    codes = np.zeros((2, 32), np.uint8)
    codes[0, 3] = 0x7F
    codes[1, 5] = 0xFF
    scales = np.full((2, 1), 127, np.uint8)
    got = B.batq_dequantize(torch.from_numpy(rowmajor_to_blocked8(codes)).cuda(),
                            torch.from_numpy(rowmajor_to_grouped(scales)).cuda(), 2, 32, 8, torch.float32)
    torch.cuda.synchronize()
    g = got.cpu().numpy()
    assert np.isnan(g[0, 3]) and np.isnan(g[1, 5]) and np.count_nonzero(np.isnan(g)) == 2
    c = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    s = torch.zeros(64, dtype=torch.uint8, device="cuda")
    outp = torch.zeros((2, 32), device="cuda")
    assert B.lib.batq_dequantize(c.data_ptr(), s.data_ptr(), 2, 32, 6, outp.data_ptr(), 0, 32, None) == 4
    assert B.lib.batq_dequantize(c.data_ptr(), s.data_ptr(), 2, 48, 4, outp.data_ptr(), 0, 48, None) == 2
    assert B.lib.batq_dequantize(c.data_ptr(), s.data_ptr(), 2, 32, 4, outp.data_ptr(), 0, 16, None) == 2
    assert B.lib.batq_dequantize(None, s.data_ptr(), 2, 32, 4, outp.data_ptr(), 0, 32, None) == 1


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_transform_apply_all_modes(B, dtype):
    import torch
    rng = np.random.default_rng(11)
    M, K = 75, 32 * 7
    nb = K // 32
    w = bi.make_small(M, K, 8, seed=5, dtype=dtype)
    T = o.kron_blocks(w.G, w.P)
    X = to_dev(w.X, dtype)
    Xf = w.X_f32().astype(np.float64)
    t = B.Transform(K, w.G, w.P, None)
    mats = {B.APPLY_FORWARD: T, B.APPLY_INVERSE: o.inverse_blocks(T), B.APPLY_INVERSE_T: o.inverse_transpose_blocks(T)}
    for mode, Mat in mats.items():
        ref = o.apply_blocks(Xf, Mat)
        absref = o.apply_blocks(np.abs(Xf), np.abs(Mat))
        got = B.batq_transform_apply(t, X, mode, torch.float32)
        torch.cuda.synchronize()
        # fp32 input: fp64 sums, one rounding to fp32; the library inverts its own fp64 blocks (Gauss-Jordan), so
        # the inverse modes carry its 1e-13-level difference from the oracle's inverse.  bf16 input goes
        # through the matrix cores: exact products of bf16 terms, six chained fp32 accumulations
        tol = 1e-11 if dtype == "f32" else 2.0 ** -20
        assert np.all(np.abs(got.cpu().numpy() - ref) <= 2.0 ** -24 * np.abs(ref) + tol * absref), mode
        gb = B.batq_transform_apply(t, X, mode, torch.bfloat16)
        torch.cuda.synchronize()
        refb = o.bf16_round(ref).astype(np.float64)
        ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(refb), 1e-300))) - 7)
        assert np.all(np.abs(y_to_f32(gb) - refb) <= ulp * 1.0001), mode
    # a dense-form handle gives the same, the identity handle converts
    td = B.Transform.general(K, dense=T.astype(np.float32))
    a = B.batq_transform_apply(t, X, B.APPLY_INVERSE_T, torch.float32)
    b = B.batq_transform_apply(td, X, B.APPLY_INVERSE_T, torch.float32)
    ti = B.Transform(K, None, None, None)
    c = B.batq_transform_apply(ti, X, B.APPLY_FORWARD, torch.float32)
    torch.cuda.synchronize()
    assert np.allclose(a.cpu().numpy(), b.cpu().numpy(), rtol=1e-5, atol=1e-6)
    assert np.array_equal(c.cpu().numpy(), w.X_f32())
    # in place is refused
    assert B.lib.batq_transform_apply(t.handle, X.data_ptr(), 1 if dtype == "bf16" else 0, M, K, K, 0, X.data_ptr(),
                                      1 if dtype == "bf16" else 0, K, None) == 2


@pytest.mark.parametrize("M,K", [(1, 32), (33, 32 * 5), (700, 32 * 13), (2049, 1024)])
@pytest.mark.parametrize("odt", ["bf16", "f32"])
def test_transform_apply_matrix_core_path(B, M, K, odt):
    """bf16 input at sizes with ragged row tiles and a ragged last unit column (K / 32 not a multiple of 4),
    strided input and output rows; every element against the oracle."""
    import torch
    w = bi.make_small(M, K, 8, seed=M + K, dtype="bf16")
    T = o.kron_blocks(w.G, w.P)
    Xf = w.X_f32().astype(np.float64)
    t = B.Transform(K, w.G, w.P, None)
    Xp = torch.zeros((M, K + 24), dtype=torch.bfloat16, device="cuda")
    Xp[:, :K] = to_dev(w.X, "bf16")
    tdt = torch.bfloat16 if odt == "bf16" else torch.float32
    for mode, Mat in ((B.APPLY_FORWARD, T), (B.APPLY_INVERSE, o.inverse_blocks(T)),
                      (B.APPLY_INVERSE_T, o.inverse_transpose_blocks(T))):
        ref = o.apply_blocks(Xf, Mat)
        absref = o.apply_blocks(np.abs(Xf), np.abs(Mat))
        out = torch.full((M, K + 8), 7.0, dtype=tdt, device="cuda")
        B.batq_transform_apply(t, Xp[:, :K], mode, out=out[:, :K])
        torch.cuda.synchronize()
        got = y_to_f32(out[:, :K]).astype(np.float64) if odt == "bf16" else out[:, :K].cpu().numpy().astype(np.float64)
        assert bool((out[:, K:] == 7.0).all())                      # nothing written past the row
        if odt == "f32":
            assert np.all(np.abs(got - ref) <= 2.0 ** -24 * np.abs(ref) + 2.0 ** -20 * absref), mode
        else:
            # one bf16 rounding of a value that is within 2^-20 absref of the reference
            assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 2.0 ** -19 * absref), mode


def test_transform_apply_forward_is_the_quantisers_transform(B):
    """x T_k from the apply call (fp32 out), quantised by the identity transform's kernel, gives the codes and
    scales the fused call produces: both use the same matrix-core arithmetic."""
    import torch
    M, K = 300, 1024
    w = bi.make_small(M, K, 8, seed=3, dtype="bf16")
    t = B.Transform(K, w.G, w.P, w.clip)
    tid = B.Transform(K, None, None, w.clip)
    X = to_dev(w.X, "bf16")
    y = B.batq_transform_apply(t, X, B.APPLY_FORWARD, torch.float32)
    c0, s0 = B.batq_quantize_act(t, X)
    c1, s1 = B.batq_quantize_act(tid, y)
    torch.cuda.synchronize()
    assert torch.equal(B.batq_codes_to_rowmajor(c0, M, K), B.batq_codes_to_rowmajor(c1, M, K))
    assert torch.equal(B.batq_scales_to_rowmajor(s0, M, K), B.batq_scales_to_rowmajor(s1, M, K))


@pytest.mark.parametrize("bits", [4, 8])
def test_quantised_cache_keeps_attention_scores(B, bits):
    """Keys stored as Q(k T_k), queries taken through T_k^-T, values stored as Q(v T_v) and the output through
    T_v^-1: against the oracle's same pipeline (tie-level differences only), and against exact attention
    (quantisation error only)."""
    import torch
    rng = np.random.default_rng(bits)
    heads, hd, nq, nk = 4, 128, 9, 70
    D = heads * hd
    nb = D // 32
    Tk = (np.eye(32)[None] + 0.08 * rng.standard_normal((nb, 32, 32))).astype(np.float32)
    Tv = (np.eye(32)[None] + 0.08 * rng.standard_normal((nb, 32, 32))).astype(np.float32)
    qb, kb, vb = (bi.f32_to_bf16_bits(rng.standard_normal((n, D)).astype(np.float32)) for n in (nq, nk, nk))
    q, k, v = (bi.bf16_bits_to_f32(x).astype(np.float64) for x in (qb, kb, vb))
    tk, tv = B.Transform.general(D, dense=Tk), B.Transform.general(D, dense=Tv)
    kc, ks = B.batq_quantize_act_ex(tk, to_dev(kb, "bf16"), act_bits=bits)
    vc, vs = B.batq_quantize_act_ex(tv, to_dev(vb, "bf16"), act_bits=bits)
    kd = B.batq_dequantize(kc, ks, nk, D, bits, torch.float32)
    vd = B.batq_dequantize(vc, vs, nk, D, bits, torch.float32)
    qt = B.batq_transform_apply(tk, to_dev(qb, "bf16"), B.APPLY_INVERSE_T, torch.float32)
    torch.cuda.synchronize()

    def attend(qq, kk, vv):
        out = np.empty((nq, D))
        for h in range(heads):
            sl = slice(h * hd, (h + 1) * hd)
            a = qq[:, sl] @ kk[:, sl].T / np.sqrt(hd)
            a = np.exp(a - a.max(axis=1, keepdims=True))
            out[:, sl] = (a / a.sum(axis=1, keepdims=True)) @ vv[:, sl]
        return out

    got_t = attend(qt.cpu().numpy().astype(np.float64), kd.cpu().numpy().astype(np.float64),
                   vd.cpu().numpy().astype(np.float64))
    got = B.batq_transform_apply(tv, torch.from_numpy(got_t.astype(np.float32)).cuda(), B.APPLY_INVERSE, torch.float32)
    torch.cuda.synchronize()
    got = got.cpu().numpy().astype(np.float64)
    # oracle pipeline
    fp8 = bits == 8
    okc, oks = o.quantize_act_blocks(k, Tk.astype(np.float64), None, fp8=fp8)
    ovc, ovs = o.quantize_act_blocks(v, Tv.astype(np.float64), None, fp8=fp8)
    dq = o.dequantize_fp8 if fp8 else o.dequantize
    ref_t = attend(o.apply_blocks(q, o.inverse_transpose_blocks(Tk)), dq(okc, oks), dq(ovc, ovs))
    ref = o.apply_blocks(ref_t, o.inverse_blocks(Tv))
    exact = attend(q, k, v)
    rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert rel < 5e-3, rel
    relq = np.linalg.norm(got - exact) / np.linalg.norm(exact)
    assert relq < (0.05 if fp8 else 0.35), relq


@pytest.mark.parametrize("bits", [4, 8])
def test_cache_shape_of_the_benchmark_on_sampled_rows(B, bits):
    """The shapes bench.py times (cache of 32768 tokens x 1024 channels, query of 8192 x 4096): sampled rows of
    the dequantised cache against the oracle's dequantisation of the same codes, sampled rows of the transform
    against the oracle."""
    import torch
    rng = np.random.default_rng(40 + bits)
    Mk, Kk = 32768, 1024
    G, P, clip = bi.make_factors(Kk // 32, rng, rng, rng, 0.7)
    t = B.Transform(Kk, G, P, clip)
    X = torch.randn((Mk, Kk), device="cuda", generator=torch.Generator(device="cuda").manual_seed(bits)).to(torch.bfloat16)
    codes, scales = B.batq_quantize_act_ex(t, X, act_bits=bits)
    out = B.batq_dequantize(codes, scales, Mk, Kk, bits)
    rm_codes = (B.batq_codes8_to_rowmajor if bits == 8 else B.batq_codes_to_rowmajor)(codes, Mk, Kk)
    rm_scales = B.batq_scales_to_rowmajor(scales, Mk, Kk)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([rng.integers(0, Mk, 200), [0, 15, 16, 31, 32, Mk - 33, Mk - 1]]))
    ref = (o.dequantize_fp8 if bits == 8 else o.dequantize)(rm_codes[rows].cpu().numpy(), rm_scales[rows].cpu().numpy())
    assert np.array_equal(y_to_f32(out[rows]).astype(np.float64), ref)
    if bits == 4:
        Mq, Kq = 8192, 4096
        Gq, Pq, _ = bi.make_factors(Kq // 32, rng, rng, rng, 0.7)
        tq = B.Transform(Kq, Gq, Pq, None)
        Q = torch.randn((Mq, Kq), device="cuda", generator=torch.Generator(device="cuda").manual_seed(9)).to(torch.bfloat16)
        got = B.batq_transform_apply(tq, Q, B.APPLY_INVERSE_T, torch.float32)
        torch.cuda.synchronize()
        rq = np.unique(np.concatenate([rng.integers(0, Mq, 64), [0, 31, 32, Mq - 1]]))
        Xf = Q[rq].float().cpu().numpy().astype(np.float64)
        Mat = o.inverse_transpose_blocks(o.kron_blocks(Gq, Pq))
        ref = o.apply_blocks(Xf, Mat)
        absref = o.apply_blocks(np.abs(Xf), np.abs(Mat))
        g = got[rq].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(g - ref) <= 2.0 ** -24 * np.abs(ref) + 2.0 ** -20 * absref)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("form", ["kron", "dense"])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_cache_filled_by_appends_equals_one_call(B, bits, form, dtype):
    """A cache laid out for `cap` rows and filled by appends of many sizes (a prefill from row 0, single decode
    rows, unaligned and aligned chunks, a large aligned chunk in the middle) holds what one call over all rows
    writes, byte for byte: a row's codes do not depend on the append that brought it (bf16 rows always take the
    matrix-core arithmetic, row by row or in 32-row tiles; fp32 rows one register-level kernel).  Windows of the cache
    dequantise to the oracle's values bit for bit."""
    import torch
    cap, K = 600, 1024 + 32                                         # ragged last tile, ragged last K group
    nb = K // 32
    w = bi.make_small(cap, K, 8, seed=bits, dtype=dtype)
    if form == "kron":
        t = B.Transform(K, w.G, w.P, w.clip)
    else:
        t = B.Transform.general(K, dense=o.kron_blocks(w.G, w.P).astype(np.float32), clip=w.clip)
    X = to_dev(w.X, dtype)
    c_ref, s_ref = B.batq_quantize_act_ex(t, X, act_bits=bits)
    nbytes = B.batq_code8_bytes(cap, K) if bits == 8 else B.batq_code_bytes(cap, K)
    codes = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device="cuda")
    scales = torch.full((B.batq_scale_bytes(cap, K),), 0x5A, dtype=torch.uint8, device="cuda")
    at = 0
    for m in (200, 1, 1, 22, 300, 3, 64, 9):                        # starts: 0, 200, 201, 202, 224, 524, 527, 591
        B.batq_kv_append(t, X[at:at + m], codes, scales, at, cap, bits)
        at += m
    assert at == cap
    torch.cuda.synchronize()
    to_rm = B.batq_codes8_to_rowmajor if bits == 8 else B.batq_codes_to_rowmajor
    assert_same_quantisation(B, codes, scales, c_ref, s_ref, cap, K, bits)
    # the padding blocks of the last K group carry zero codes and the neutral scale in every row
    Kp = (nb + 7) // 8 * 256
    rm_codes = to_rm(codes, cap, K).cpu().numpy()
    rm_scales = B.batq_scales_to_rowmajor(scales, cap, K).cpu().numpy()
    dq = o.dequantize_fp8 if bits == 8 else o.dequantize
    for row0, m in ((0, cap), (37, 150), (31, 1), (599, 1), (224, 300)):
        ref = dq(rm_codes[row0:row0 + m], rm_scales[row0:row0 + m])
        got = B.batq_kv_dequantize(codes, scales, cap, row0, m, K, bits, torch.float32)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy().astype(np.float64), ref), (row0, m)
        gb = B.batq_kv_dequantize(codes, scales, cap, row0, m, K, bits)
        torch.cuda.synchronize()
        assert np.array_equal(y_to_f32(gb).astype(np.float64), o.bf16_round(ref).astype(np.float64)), (row0, m)
    assert Kp >= K
    # windows that do not fit, and widths that do not exist
    x1 = X[:4]
    lib = B.lib
    args = (t.handle, x1.data_ptr(), 1 if dtype == "bf16" else 0, 4, K, K)
    assert lib.batq_kv_append(*args, bits, codes.data_ptr(), scales.data_ptr(), cap - 3, cap, None) == 2
    assert lib.batq_kv_append(*args, bits, codes.data_ptr(), scales.data_ptr(), -1, cap, None) == 2
    assert lib.batq_kv_append(*args, 5, codes.data_ptr(), scales.data_ptr(), 0, cap, None) == 4
    outp = torch.zeros((4, K), device="cuda")
    assert lib.batq_kv_dequantize(codes.data_ptr(), scales.data_ptr(), cap, cap - 3, 4, K, bits, outp.data_ptr(), 0, K,
                                  None) == 2
