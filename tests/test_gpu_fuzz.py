"""Seeded random combinations of the options of the online calls against the oracle: every transform form,
both activation widths, both input types, the three clipping modes, row factors, gated input; and random GEMM
shapes with both output types and the gated epilogue.  Loose bars (rounding ties flip single codes): the point
is that no combination of paths is wrong, the tight bars are in the dedicated tests."""
import numpy as np
import pytest

import batq_inputs as bi
from oracle import batq_oracle as o
from gpu_util import (require_gpu, to_dev, y_to_f32, code_value_mismatch, grouped_to_rowmajor, blocked_to_rowmajor,
                      blocked8_to_rowmajor, rowmajor_to_blocked, rowmajor_to_blocked8, rowmajor_to_grouped,
                      assert_same_quantisation)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    require_gpu()
    import paper_2603_16590_amd as b
    return b


def _transform(B, rng, K, form):
    nb = K // 32
    eye = lambda n: np.eye(n)[None]
    if form == "identity":
        return None, {}
    if form == "dense":
        T = eye(32) + 0.05 * rng.standard_normal((nb, 32, 32))
        return T, dict(dense=T.astype(np.float32))
    go, gi = (4, 8) if rng.integers(0, 2) else (8, 4)
    outer_pb = form in ("private_outer", "naive")
    inner_pb = form in ("gpk", "naive")
    outer = (eye(go) if outer_pb else np.eye(go)) + 0.05 * rng.standard_normal((nb, go, go) if outer_pb else (go, go))
    inner = (eye(gi) if inner_pb else np.eye(gi)) + 0.05 * rng.standard_normal((nb, gi, gi) if inner_pb else (gi, gi))
    outer, inner = outer.astype(np.float32), inner.astype(np.float32)
    return o.kron_blocks_general(outer, inner, nb), dict(outer=outer, inner=inner)


@pytest.mark.parametrize("case", range(28))
def test_quantiser_option_combinations(B, case):
    import torch
    rng = np.random.default_rng(9000 + case)
    M = int(rng.choice([1, 7, 33, 64, 129, 200, 390]))
    K = 32 * int(rng.integers(1, 40))
    nb = K // 32
    form = ["identity", "gpk", "private_outer", "naive", "dense"][case % 5]
    bits = 8 if rng.integers(0, 3) == 0 else 4
    gated = bool(rng.integers(0, 3) == 0)
    dtype = "bf16" if gated or rng.integers(0, 2) else "f32"
    clipmode = "none" if form == "identity" and rng.integers(0, 2) else ["sym", "minmax", "none"][int(rng.integers(0, 3))]
    if bits == 8 and clipmode == "minmax":
        clipmode = "sym"
    use_rs = bool(rng.integers(0, 2))
    T, targs = _transform(B, rng, K, form)
    clip = cmin = cmax = None
    if clipmode == "sym":
        clip = rng.uniform(0.7, 1.0, nb).astype(np.float32)
        targs["clip"] = clip
    elif clipmode == "minmax":
        cmin, cmax = rng.uniform(0.7, 1.0, nb).astype(np.float32), rng.uniform(0.7, 1.0, nb).astype(np.float32)
        targs.update(clip_min=cmin, clip_max=cmax)
    t = B.Transform.general(K, **targs)
    X = rng.standard_normal((M, K)) * np.exp(0.5 * rng.standard_normal((M, 1)))
    X[:, rng.integers(0, K, max(1, K // 60))] *= 15.0
    U = rng.standard_normal((M, K))
    if dtype == "bf16":
        Xs, Us = bi.f32_to_bf16_bits(X.astype(np.float32)), bi.f32_to_bf16_bits(U.astype(np.float32))
        Xf, Uf = bi.bf16_bits_to_f32(Xs).astype(np.float64), bi.bf16_bits_to_f32(Us).astype(np.float64)
    else:
        Xs = X.astype(np.float32)
        Xf = Xs.astype(np.float64)
    rs = rng.uniform(0.2, 5.0, M).astype(np.float32) if use_rs else None
    c, s = B.batq_quantize_act_ex(t, to_dev(Xs, dtype), act_bits=bits,
                                  row_scale=None if rs is None else torch.from_numpy(rs).cuda(),
                                  up=to_dev(Us, dtype) if gated else None)
    torch.cuda.synchronize()
    gs = grouped_to_rowmajor(s.cpu().numpy(), M, nb)
    gc = (blocked8_to_rowmajor if bits == 8 else blocked_to_rowmajor)(c.cpu().numpy(), M, nb)
    inp = o.swiglu_bf16(Xf, Uf) if gated else Xf
    oc, os_ = o.quantize_act_blocks(inp, T, clip, cmin, cmax, row_scale=rs, fp8=(bits == 8))
    what = (case, M, K, form, bits, dtype, clipmode, use_rs, gated)
    assert np.mean(gs != os_) <= 4e-3, what
    if bits == 8:
        bad = (gc != oc) & ~(((gc | oc) & 0x7F) == 0)
        assert np.mean(bad) <= 2e-2, what                      # E4M3 steps are fine: fp32-vs-fp64 ties are frequent
        near = np.abs((gc & 0x7F).astype(int) - (oc & 0x7F).astype(int)) <= 1
        assert np.mean(near | (gs != os_).repeat(32, axis=1)) >= 0.999, what
    else:
        assert np.mean(code_value_mismatch(gc, oc)) <= 6e-3, what


@pytest.mark.parametrize("case", range(16))
def test_gemm_option_combinations(B, case):
    import torch
    rng = np.random.default_rng(7000 + case)
    M = int(rng.choice([1, 16, 33, 64, 65, 130, 257, 400]))
    K = 32 * int(rng.integers(1, 70))
    glu = bool(case % 2)
    N = 64 * int(rng.integers(1, 12)) if glu else int(rng.integers(1, 700))
    bits = 8 if case % 4 >= 2 else 4
    out_bf16 = bool(rng.integers(0, 2))
    wc = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    ws = rng.integers(124, 130, size=(N, K // 32), dtype=np.uint8)
    xs = rng.integers(124, 130, size=(M, K // 32), dtype=np.uint8)
    if bits == 8:
        e = rng.integers(5, 9, size=(M, K)); m = rng.integers(0, 8, size=(M, K)); sg = rng.integers(0, 2, size=(M, K))
        xc = ((sg << 7) | (e << 3) | m).astype(np.uint8)          # exponents within 4 binades: exact K-step sums
        dxc = torch.from_numpy(rowmajor_to_blocked8(xc)).cuda()
        dq_x = o.dequantize_fp8(xc, xs)
    else:
        xc = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
        dxc = torch.from_numpy(rowmajor_to_blocked(xc)).cuda()
        dq_x = o.dequantize(xc, xs)
    wh = B.batq_weight_import(torch.from_numpy(wc).cuda(), torch.from_numpy(ws).cuda(), K, N)
    dxs = torch.from_numpy(rowmajor_to_grouped(xs)).cuda()
    dq_w = o.dequantize(wc, ws)
    Yref = dq_x @ dq_w.T
    absY = np.abs(dq_x) @ np.abs(dq_w).T
    odt = torch.bfloat16 if out_bf16 else torch.float32
    if glu:
        F = N // 2
        cols = np.arange(F)
        gcol = 64 * (cols // 32) + cols % 32
        g, u = Yref[:, gcol], Yref[:, gcol + 32]
        ref = o.swiglu(g, u)
        tol = 1.1 * np.abs(u) * 2e-6 * absY[:, gcol] + np.abs(o.silu(g)) * 2e-6 * absY[:, gcol + 32] + \
            2.0 ** -20 * (2.0 + np.abs(g)) * np.abs(ref)
        got = y_to_f32(B.batq_gemm_glu(dxc, dxs, wh, M, bits, odt)).astype(np.float64)
    else:
        ref = Yref
        tol = 2e-6 * absY
        got = y_to_f32((B.batq_gemm_a8w4 if bits == 8 else B.batq_gemm_mxfp4)(dxc, dxs, wh, M, odt)).astype(np.float64)
    torch.cuda.synchronize()
    if out_bf16:
        refb = o.bf16_round(ref).astype(np.float64)
        ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(refb), 1e-300))) - 7)
        assert np.all(np.abs(got - refb) <= ulp * 1.0001 + tol), (case, M, K, N, bits, glu)
    else:
        assert np.all(np.abs(got - ref) <= tol + 1e-30), (case, M, K, N, bits, glu)


@pytest.mark.parametrize("case", range(17))
def test_gemm_kernel_choice_combinations(B, case):
    """Random (M, K, N, workspace) over the ranges in which the library switches between its 4-bit GEMM kernels (small-M,
    one tile per workgroup, tiled with four or eight waves, with and without K parts): every element against the
    oracle, and the same bits when the call is repeated."""
    import torch
    rng = np.random.default_rng(7700 + case)
    M = int(rng.choice([20, 33, 48, 64, 65, 100, 128, 129, 200, 300, 520, 700]))
    K = 32 * int(rng.integers(4, 130)) if case % 3 else 256 * int(rng.integers(24, 60))
    N = int(rng.integers(60, 16000)) if case % 2 else 64 * int(rng.integers(1, 120))
    if case >= 14:                                     # many strips per workgroup: the eight-wave tiled kernel
        M, K, N = int(rng.integers(520, 1100)), 32 * int(rng.integers(4, 40)), int(rng.integers(14000, 26000))
    if M * N * K > 2.5e10:
        N = max(64, int(2.5e10 / (M * K)))
    out_bf16 = bool(rng.integers(0, 2))
    wc = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    ws = rng.integers(124, 130, size=(N, K // 32), dtype=np.uint8)
    xc = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    xs = rng.integers(124, 130, size=(M, K // 32), dtype=np.uint8)
    wh = B.batq_weight_import(torch.from_numpy(wc).cuda(), torch.from_numpy(ws).cuda(), K, N)
    dxc = torch.from_numpy(rowmajor_to_blocked(xc)).cuda()
    dxs = torch.from_numpy(rowmajor_to_grouped(xs)).cuda()
    dq_x, dq_w = o.dequantize(xc, xs), o.dequantize(wc, ws)
    ref = dq_x @ dq_w.T
    tol = 2e-6 * (np.abs(dq_x) @ np.abs(dq_w).T)
    need = B.batq_gemm_workspace(wh, M)
    frac = [0.0, 0.4, 1.0][int(rng.integers(0, 3))]
    work = torch.empty(max(256, int(need * frac)), dtype=torch.uint8, device="cuda") if need and frac > 0 else None
    odt = torch.bfloat16 if out_bf16 else torch.float32
    Y = B.batq_gemm_mxfp4(dxc, dxs, wh, M, odt, workspace=work)
    Y2 = B.batq_gemm_mxfp4(dxc, dxs, wh, M, odt, workspace=work)
    torch.cuda.synchronize()
    what = (case, M, K, N, need, frac, out_bf16)
    assert torch.equal(Y, Y2), what
    got = y_to_f32(Y).astype(np.float64)
    if out_bf16:
        refb = o.bf16_round(ref).astype(np.float64)
        ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(refb), 1e-300))) - 7)
        bad = np.argwhere(np.abs(got - refb) > ulp * 1.0001 + tol)
    else:
        bad = np.argwhere(np.abs(got - ref) > tol + 1e-30)
    assert bad.size == 0, (what, len(bad), bad[:3].tolist())


@pytest.mark.parametrize("case", range(10))
def test_cache_append_chunkings(B, case):
    """Random capacities, forms, widths and chunkings of the appends (fp32 and bf16 rows): the filled cache holds
    the one-call result, byte for byte."""
    import torch
    rng = np.random.default_rng(9000 + case)
    K = 32 * int(rng.integers(1, 41))
    cap = int(rng.integers(1, 700))
    bits = int(rng.choice([4, 8]))
    form = str(rng.choice(["identity", "gpk", "private_outer", "naive", "dense"]))
    dtype = "bf16" if rng.integers(0, 3) else "f32"
    _, kw = _transform(B, rng, K, form)
    clip = rng.uniform(0.8, 1.0, K // 32).astype(np.float32)
    t = B.Transform.general(K, clip=clip, **kw) if kw else B.Transform(K, None, None, clip)
    w = bi.make_small(cap, K, 8, seed=case, dtype=dtype)
    X = to_dev(w.X, dtype)
    c_ref, s_ref = B.batq_quantize_act_ex(t, X, act_bits=bits)
    nbytes = B.batq_code8_bytes(cap, K) if bits == 8 else B.batq_code_bytes(cap, K)
    codes = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")
    scales = torch.full((B.batq_scale_bytes(cap, K),), 0xA5, dtype=torch.uint8, device="cuda")
    at = 0
    while at < cap:
        m = int(min(cap - at, rng.choice([1, 1, 2, 7, 31, 32, 33, 129, 160, 300])))
        B.batq_kv_append(t, X[at:at + m], codes, scales, at, cap, bits)
        at += m
    torch.cuda.synchronize()
    assert_same_quantisation(B, codes, scales, c_ref, s_ref, cap, K, bits,
                             what=(cap, K, bits, form, dtype))
