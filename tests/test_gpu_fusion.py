"""GPU parity for the fused RMSNorm -> transform -> quantise path (row factors + folded norm weight)."""
import zlib

import numpy as np
import pytest

import batq_inputs as bi
from oracle import batq_oracle as o
from gpu_util import (require_gpu, to_dev, unpack, code_value_mismatch, TIE_POINTS, grouped_to_rowmajor,
                      blocked_to_rowmajor, blocked8_to_rowmajor, y_to_f32)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    require_gpu()
    import paper_2603_16590_amd as b
    return b


def _x(rng, M, K, dtype):
    X = rng.standard_normal((M, K)) * np.exp(0.7 * rng.standard_normal((M, 1)))
    X[:, rng.integers(0, K, max(1, K // 100))] *= 25.0
    if dtype == "bf16":
        bits = bi.f32_to_bf16_bits(X.astype(np.float32))
        return bits, bi.bf16_bits_to_f32(bits)
    Xf = X.astype(np.float32)
    return Xf, Xf


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_row_rms_scale(B, dtype):
    import torch
    rng = np.random.default_rng(1)
    for M, K in ((1, 32), (37, 96), (130, 4096 + 64)):
        Xs, Xf = _x(rng, M, K, dtype)
        r = B.batq_row_rms_scale(to_dev(Xs, dtype), 1e-6)
        torch.cuda.synchronize()
        ref = o.row_rms_scale(Xf, 1e-6)
        assert np.allclose(r.cpu().numpy(), ref, rtol=2e-6, atol=0)


def test_rowscale_bit_exact_without_transform(B):
    # identity transform, fp32 input: one fp32 multiply per element, same as the oracle's rounded product
    import torch
    rng = np.random.default_rng(2)
    M, K = 70, 32 * 9
    Xs, Xf = _x(rng, M, K, "f32")
    rs = rng.uniform(0.05, 20.0, M).astype(np.float32)
    for bits in (4, 8):
        t = B.Transform(K, None, None, None)
        c, s = B.batq_quantize_act_ex(t, to_dev(Xs, "f32"), act_bits=bits, row_scale=torch.from_numpy(rs).cuda())
        torch.cuda.synchronize()
        gs = grouped_to_rowmajor(s.cpu().numpy(), M, K // 32)
        oc, os_ = o.quantize_act_blocks(Xf, None, None, row_scale=rs, fp8=(bits == 8))
        gc = (blocked8_to_rowmajor if bits == 8 else blocked_to_rowmajor)(c.cpu().numpy(), M, K // 32)
        assert np.array_equal(gs, os_), bits
        assert np.array_equal(gc, oc), bits


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_fused_rmsnorm_transform_quantise(B, dtype):
    import torch
    rng = np.random.default_rng(zlib.crc32(dtype.encode()))
    M, K = 300, 32 * 24
    nb = K // 32
    Xs, Xf = _x(rng, M, K, dtype)
    gamma = rng.uniform(0.5, 1.5, K).astype(np.float32)
    G = (np.eye(4) + 0.05 * rng.standard_normal((4, 4))).astype(np.float32)
    P = (np.eye(8)[None] + 0.05 * rng.standard_normal((nb, 8, 8))).astype(np.float32)
    clip = rng.uniform(0.85, 1.0, nb).astype(np.float32)
    # T'_k = diag(gamma_k) (G (x) P_k), handed over as dense fp32 blocks (what the library receives)
    Tf32 = o.fold_norm_weight(o.kron_blocks(G, P), gamma).astype(np.float32)
    t = B.Transform.general(K, dense=Tf32, clip=clip)
    X = to_dev(Xs, dtype)
    r = B.batq_row_rms_scale(X, 1e-6)
    c, s = B.batq_quantize_act_ex(t, X, act_bits=4, row_scale=r)
    torch.cuda.synchronize()
    gc = blocked_to_rowmajor(c.cpu().numpy(), M, nb)
    gs = grouped_to_rowmajor(s.cpu().numpy(), M, nb)
    # oracle: the same row factors the GPU used (their own accuracy is tested above), fp64 transform
    rr = r.cpu().numpy().astype(np.float64)
    Yt = o.apply_blocks(Xf.astype(np.float64) * rr[:, None], Tf32.astype(np.float64))
    oc, os_ = o.mxfp4_quantize(Yt.astype(np.float32), clip)
    scale_bad = gs != os_
    mism = code_value_mismatch(gc, oc).reshape(M, nb, 32)
    frac = np.where(scale_bad, 32, mism.sum(axis=2)).sum() / mism.size
    assert frac <= 1e-3, frac
    Xc, bound = o.clip_blocks(Yt.astype(np.float32), clip)
    E = os_.astype(np.int64) - 127
    v = np.abs(Xc.astype(np.float64)) / np.exp2(E)[:, :, None]
    dist = np.abs(v[..., None] - TIE_POINTS).min(axis=-1)
    sel = mism & ~scale_bad[:, :, None]
    assert np.all(dist[sel] < 1e-4)
    # and it is the quantisation of the normalised activations: compare with the unfused oracle pipeline
    uc, us = o.mxfp4_quantize(o.apply_blocks(o.rmsnorm(Xf, gamma, 1e-6), o.kron_blocks(G, P)).astype(np.float32), clip)
    assert np.mean(code_value_mismatch(gc, uc)) < 5e-3 and np.mean(gs != us) < 1e-3


def test_linear_ex_with_row_scale_and_both_widths(B):
    import torch
    rng = np.random.default_rng(9)
    M, K, N = 200, 32 * 16, 288
    nb = K // 32
    Xs, Xf = _x(rng, M, K, "bf16")
    W = (0.02 * rng.standard_normal((K, N))).astype(np.float32)
    T = (np.eye(32)[None] + 0.05 * rng.standard_normal((nb, 32, 32))).astype(np.float32)
    t = B.Transform.general(K, dense=T)
    wh = B.batq_prepare_weight(t, to_dev(W, "f32"))
    X = to_dev(Xs, "bf16")
    r = B.batq_row_rms_scale(X, 1e-6)
    for bits in (4, 8):
        Y = B.batq_linear_ex(t, wh, X, act_bits=bits, row_scale=r, out_dtype=torch.float32)
        c, s = B.batq_quantize_act_ex(t, X, act_bits=bits, row_scale=r)
        Y2 = (B.batq_gemm_a8w4 if bits == 8 else B.batq_gemm_mxfp4)(c, s, wh, M, torch.float32)
        torch.cuda.synchronize()
        assert torch.equal(Y, Y2)
    # argument errors of the options form
    import ctypes as C
    from paper_2603_16590_amd.binding import ActOptions
    o_bad = ActOptions(); o_bad.act_bits = 6
    work = torch.empty(B.batq_linear_a8w4_workspace(M, K), dtype=torch.uint8, device="cuda")
    Yz = torch.zeros((M, N), device="cuda")
    assert B.lib.batq_linear_ex(t.handle, wh.handle, X.data_ptr(), 1, M, K, C.byref(o_bad), Yz.data_ptr(), 0, N,
                                work.data_ptr(), work.numel(), None) == 4
    o_odd = ActOptions(); o_odd.act_bits = 4; o_odd.row_scale = r.data_ptr() + 2
    assert B.lib.batq_linear_ex(t.handle, wh.handle, X.data_ptr(), 1, M, K, C.byref(o_odd), Yz.data_ptr(), 0, N,
                                work.data_ptr(), work.numel(), None) == 2
    torch.cuda.synchronize()
    assert bool((Yz == 0).all())
