"""GPU parity for the gate/up GEMM with the gated activation in its epilogue (silu(gate) * up)."""
import numpy as np
import pytest

import batq_inputs as bi
from oracle import batq_oracle as o
from gpu_util import (require_gpu, to_dev, y_to_f32, rowmajor_to_blocked, rowmajor_to_blocked8, rowmajor_to_grouped)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    require_gpu()
    import paper_2603_16590_amd as b
    return b


def _interleave(a, b):
    """rows of a (gate) and b (up) in groups of 32: 64 p + j <- a[32 p + j], 64 p + 32 + j <- b[32 p + j]"""
    F = a.shape[0]
    out = np.empty((2 * F,) + a.shape[1:], dtype=a.dtype)
    for p in range(F // 32):
        out[64 * p:64 * p + 32] = a[32 * p:32 * p + 32]
        out[64 * p + 32:64 * p + 64] = b[32 * p:32 * p + 32]
    return out


def test_gate_up_weight_is_the_interleave_of_the_two(B):
    import torch
    rng = np.random.default_rng(1)
    K, F = 32 * 6, 96
    w = bi.make_small(8, K, F, seed=3, dtype="f32")
    t = B.Transform(K, w.G, w.P, None)
    Wg = (0.02 * rng.standard_normal((K, F))).astype(np.float32)
    Wu = (0.02 * rng.standard_normal((K, F))).astype(np.float32)
    clip_w = rng.uniform(0.8, 1.0, K // 32).astype(np.float32)
    for kxn in (True, False):
        dg, du = (to_dev(Wg if kxn else np.ascontiguousarray(Wg.T), "f32"),
                  to_dev(Wu if kxn else np.ascontiguousarray(Wu.T), "f32"))
        wgu = B.batq_prepare_weight_gate_up(t, dg, du, kxn, clip_w)
        assert (wgu.K, wgu.N) == (K, 2 * F)
        c, s = wgu.export()
        torch.cuda.synchronize()
        ocg, osg = o.prepare_weight(Wg, w.G, w.P, clip_w)
        ocu, osu = o.prepare_weight(Wu, w.G, w.P, clip_w)
        assert np.array_equal(s.cpu().numpy(), _interleave(osg, osu))
        assert np.array_equal(c.cpu().numpy(), _interleave(ocg, ocu))
    # F must be a multiple of 32
    assert B.lib.batq_prepare_weight_gate_up(None, t.handle, dg.data_ptr(), du.data_ptr(), 0, K, 40, 40, 1, None,
                                             None) in (1, 2)


def _rand_codes(rng, R, K, bits):
    if bits == 4:
        return rng.integers(0, 256, size=(R, K // 2), dtype=np.uint8)
    c = rng.integers(0, 256, size=(R, K), dtype=np.uint8)
    c[(c & 0x7F) == 0x7F] = 0x3C                                  # no NaN codes
    return c


@pytest.mark.parametrize("M,K,F", [(1, 64, 32), (20, 96, 64), (33, 1024, 96), (64, 12288 + 32, 160), (65, 160, 32),
                                   (300, 2048 + 64, 288), (700, 512, 1440), (520, 512, 5632), (300, 768, 8192 + 96)])
@pytest.mark.parametrize("bits", [4, 8])
def test_gemm_glu_random_codes(B, M, K, F, bits):
    import torch
    rng = np.random.default_rng(M * 7 + K + F + bits)
    N = 2 * F
    xc = _rand_codes(rng, M, K, bits)
    xs = rng.integers(124, 130, size=(M, K // 32), dtype=np.uint8)
    wc = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    ws = rng.integers(124, 130, size=(N, K // 32), dtype=np.uint8)
    wh = B.batq_weight_import(torch.from_numpy(wc).cuda(), torch.from_numpy(ws).cuda(), K, N)
    dxc = torch.from_numpy(rowmajor_to_blocked8(xc) if bits == 8 else rowmajor_to_blocked(xc)).cuda()
    dxs = torch.from_numpy(rowmajor_to_grouped(xs)).cuda()
    dq_x = o.dequantize_fp8(xc, xs) if bits == 8 else o.dequantize(xc, xs)
    dq_w = o.dequantize(wc, ws)
    Yref = dq_x @ dq_w.T                                           # all 2 F columns, interleaved order
    absY = np.abs(dq_x) @ np.abs(dq_w).T
    cols = np.arange(F)
    gcol = 64 * (cols // 32) + cols % 32
    g, u = Yref[:, gcol], Yref[:, gcol + 32]
    ref = o.swiglu(g, u)
    # error of the fp32 sums (the 8-bit instruction's alignment window included) carried through the
    # derivative of silu(g) u, plus the fp32 evaluation of the product
    eps = 2e-4 if bits == 8 else 1e-6
    tol = 1.1 * np.abs(u) * eps * absY[:, gcol] + np.abs(o.silu(g)) * eps * absY[:, gcol + 32] + \
        2.0 ** -20 * (2.0 + np.abs(g)) * np.abs(ref)
    H = B.batq_gemm_glu(dxc, dxs, wh, M, bits, torch.float32)
    torch.cuda.synchronize()
    got = H.cpu().numpy().astype(np.float64)
    bad = np.argwhere(np.abs(got - ref) > tol + 1e-30)
    assert bad.size == 0, f"{len(bad)} wrong elements, first at {bad[0]}"
    # the plain GEMM on the same weight gives the two halves this is made of
    Y = (B.batq_gemm_a8w4 if bits == 8 else B.batq_gemm_mxfp4)(dxc, dxs, wh, M, torch.float32)
    torch.cuda.synchronize()
    Yn = Y.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - o.swiglu(Yn[:, gcol], Yn[:, gcol + 32])) <= 2.0 ** -20 * (2.0 + np.abs(g)) * np.abs(ref) + tol)
    # bf16 output into a strided tensor: one bf16 rounding on top
    Hb = torch.zeros((M, F + 8), dtype=torch.bfloat16, device="cuda")
    B.batq_gemm_glu(dxc, dxs, wh, M, bits, H=Hb[:, :F])
    torch.cuda.synchronize()
    refb = o.bf16_round(ref).astype(np.float64)
    ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(refb), 1e-300))) - 7)
    assert np.all(np.abs(y_to_f32(Hb[:, :F]) - refb) <= ulp * 1.0001 + tol)
    assert bool((Hb[:, F:] == 0).all())


def test_linear_glu_is_quantise_then_gemm_glu_and_errors(B):
    import torch
    rng = np.random.default_rng(5)
    M, K, F = 200, 32 * 16, 160
    w = bi.make_small(M, K, 8, seed=9, dtype="bf16")
    t = B.Transform(K, w.G, w.P, w.clip)
    Wg = (0.02 * rng.standard_normal((K, F))).astype(np.float32)
    Wu = (0.02 * rng.standard_normal((K, F))).astype(np.float32)
    wgu = B.batq_prepare_weight_gate_up(t, to_dev(Wg, "f32"), to_dev(Wu, "f32"))
    X = to_dev(w.X, "bf16")
    for bits in (4, 8):
        H = B.batq_linear_glu(t, wgu, X, act_bits=bits, out_dtype=torch.float32)
        c, s = B.batq_quantize_act_ex(t, X, act_bits=bits)
        H2 = B.batq_gemm_glu(c, s, wgu, M, bits, torch.float32)
        torch.cuda.synchronize()
        assert torch.equal(H, H2)
        # the oracle's layer: quantised gate and up projections, then the gated product
        xc, xs = o.quantize_act_blocks(w.X_f32(), o.kron_blocks(w.G, w.P), w.clip, fp8=(bits == 8))
        gm = o.gemm_a8w4 if bits == 8 else o.gemm
        ref = o.swiglu(gm(xc, xs, *o.prepare_weight(Wg, w.G, w.P)), gm(xc, xs, *o.prepare_weight(Wu, w.G, w.P)))
        rel = np.linalg.norm(H.cpu().numpy() - ref) / np.linalg.norm(ref)
        assert rel < 0.02, (bits, rel)
    # a weight whose column count is not a multiple of 64 cannot be gate/up
    wodd = B.batq_prepare_weight(t, to_dev(np.zeros((K, 96), np.float32), "f32"))
    Hz = torch.zeros((M, 48), device="cuda")
    c, s = B.batq_quantize_act(t, X)
    assert B.lib.batq_gemm_glu(c.data_ptr(), s.data_ptr(), wodd.handle, M, 4, Hz.data_ptr(), 0, 48, None) == 2
    assert B.lib.batq_gemm_glu(c.data_ptr(), s.data_ptr(), wgu.handle, M, 5, Hz.data_ptr(), 0, F, None) == 4
    assert B.lib.batq_gemm_glu(c.data_ptr(), s.data_ptr(), wgu.handle, M, 4, Hz.data_ptr(), 0, F - 1, None) == 2
    torch.cuda.synchronize()
    assert bool((Hz == 0).all())
