"""GPU parity: MXFP4 x MXFP4 GEMM and the whole batq_linear path against the fp64 oracle.

Bar: relative Frobenius error <= 1e-3 against the oracle's fp64 product of the same
dequantised operands (the codes and scales the GPU itself produced).  A bf16 output is
compared with the oracle's result rounded to bf16 (bf16 rounding alone is ~1.7e-3 relative,
so the unrounded fp64 result cannot be the reference for it) and may differ by one bf16 ulp
where the fp32 accumulation order moves a value across a rounding boundary.
"""
import numpy as np
import pytest

import batq_inputs as bi
from oracle import batq_oracle as o
from gpu_util import require_gpu, to_dev, y_to_f32, sample_rows, grouped_to_rowmajor, rowmajor_to_grouped, blocked_to_rowmajor, rowmajor_to_blocked

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    require_gpu()
    import paper_2603_16590_amd as b
    return b


def _relfro(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / max(np.linalg.norm(b), 1e-300))


def _rand_q(rng, R, K, lo=118, hi=136):
    import torch
    codes = rng.integers(0, 256, size=(R, K // 2), dtype=np.uint8)
    scales = rng.integers(lo, hi, size=(R, K // 32), dtype=np.uint8)
    # device side: activation scales travel in the grouped order, weight import takes row-major
    return codes, scales, torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda()


def _xs(scales):
    import torch
    return torch.from_numpy(rowmajor_to_grouped(scales)).cuda()


def _xc(codes):
    import torch
    return torch.from_numpy(rowmajor_to_blocked(codes)).cuda()


def test_single_block_is_exact(B):
    # K = 32: every product and the 32-term sum are exact in fp32, so the result equals the oracle's
    import torch
    rng = np.random.default_rng(0)
    xc, xs, dxc, dxs = _rand_q(rng, 40, 32)
    wc, ws, dwc, dws = _rand_q(rng, 50, 32)
    wh = B.batq_weight_import(dwc, dws, 32, 50)
    Y = B.batq_gemm_mxfp4(_xc(xc), _xs(xs), wh, xc.shape[0], torch.float32)
    torch.cuda.synchronize()
    ref = o.gemm(xc, xs, wc, ws)
    assert np.array_equal(y_to_f32(Y).astype(np.float64), ref)


@pytest.mark.parametrize("M,K,N", [(1, 64, 1), (37, 96, 70), (64, 128, 64), (65, 160, 129), (130, 1024, 96),
                                   (16, 4096, 256), (300, 2048 + 64, 520), (257, 256, 300), (513, 96, 257), (700, 32, 70),
                                   (16, 512, 1000), (32, 768, 4096), (5, 256, 17), (20, 1024 + 96, 4090)])
def test_small_shapes_random_codes(B, M, K, N):
    """(The last four: up to 32 rows and at most 4096 columns, where a workgroup of the small-M kernel takes 16 instead
    of 32 columns: N a multiple of 16 but not of 32, the full 4096, fewer than 32, and a ragged last group of 10.)"""
    import torch
    rng = np.random.default_rng(M * 7 + K + N)
    xc, xs, dxc, dxs = _rand_q(rng, M, K)
    wc, ws, dwc, dws = _rand_q(rng, N, K)
    wh = B.batq_weight_import(dwc, dws, K, N)
    ref = o.gemm(xc, xs, wc, ws)
    Y = B.batq_gemm_mxfp4(_xc(xc), _xs(xs), wh, xc.shape[0], torch.float32)
    torch.cuda.synchronize()
    assert _relfro(y_to_f32(Y), ref) <= 1e-5
    # element-wise: fp32 accumulation of nb exact block terms
    tol = 1e-6 * (np.abs(o.dequantize(xc, xs)) @ np.abs(o.dequantize(wc, ws)).T)
    assert np.all(np.abs(y_to_f32(Y) - ref) <= tol + 1e-30)
    Yb = B.batq_gemm_mxfp4(_xc(xc), _xs(xs), wh, xc.shape[0], torch.bfloat16)
    torch.cuda.synchronize()
    refb = o.bf16_round(ref).astype(np.float64)
    got = y_to_f32(Yb).astype(np.float64)
    assert _relfro(got, refb) <= 1e-3
    # one bf16 ulp, plus the fp32 accumulation error where the sum cancels
    ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(refb), 1e-300))) - 7)
    assert np.all(np.abs(got - refb) <= ulp * 1.0001 + tol)


def _check_every_element(B, M, K, N, workspace_fraction=None):
    """Random codes, every output element against the oracle, fp32 and bf16 output.  workspace_fraction: None for
    the plain call, else the share of batq_gemm_workspace() handed to the call with a workspace."""
    import torch
    rng = np.random.default_rng(M + K + N)
    xc, xs, dxc, dxs = _rand_q(rng, M, K, lo=122, hi=132)
    wc, ws, dwc, dws = _rand_q(rng, N, K, lo=122, hi=132)
    wh = B.batq_weight_import(dwc, dws, K, N)
    ref = o.gemm(xc, xs, wc, ws)
    dxc_b, dxs_g = _xc(xc), _xs(xs)
    work = None
    if workspace_fraction is not None:
        need = B.batq_gemm_workspace(wh, M)
        assert need > 0, "the shape was chosen to want K parts"
        work = torch.empty(max(256, int(need * workspace_fraction)), dtype=torch.uint8, device="cuda")
    Y = B.batq_gemm_mxfp4(dxc_b, dxs_g, wh, M, torch.float32, workspace=work)
    torch.cuda.synchronize()
    got = y_to_f32(Y)
    tol = 1e-6 * (np.abs(o.dequantize(xc, xs)) @ np.abs(o.dequantize(wc, ws)).T)
    bad = np.argwhere(np.abs(got - ref) > tol + 1e-30)
    assert bad.size == 0, f"{len(bad)} wrong elements, first at {bad[0]}"
    Yb = B.batq_gemm_mxfp4(dxc_b, dxs_g, wh, M, torch.bfloat16, workspace=work)
    torch.cuda.synchronize()
    refb = o.bf16_round(ref).astype(np.float64)
    gotb = y_to_f32(Yb).astype(np.float64)
    ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(refb), 1e-300))) - 7)
    bad = np.argwhere(np.abs(gotb - refb) > ulp * 1.0001 + tol)
    assert bad.size == 0, f"{len(bad)} wrong bf16 elements, first at {bad[0]}"
    return wh, dxc_b, dxs_g, Y


@pytest.mark.parametrize("M,K,N", [(768, 512, 30000), (4096, 256, 2098), (1500, 768, 9000), (2100, 1024 + 32, 7000),
                                   (520, 2048 + 96, 16000)])
def test_tile_schedule_shapes(B, M, K, N):
    """Shapes that give the persistent workgroups of the tiled kernel three or more strips each (the eight-wave
    kernel), in several tiles of every width (64 .. 256 columns), with ragged last row panels and column strips,
    2 to 18 K stages and every column-band count; every output element is checked."""
    _check_every_element(B, M, K, N)


@pytest.mark.parametrize("M,K,N", [(200, 2048, 14336), (300, 1536 + 32, 5000), (256, 768, 24000), (100, 512, 9000 + 24),
                                   (512, 1024, 14336), (256, 512, 12840), (130, 640, 16320)])
def test_narrow_tile_shapes(B, M, K, N):
    """Few rows and many columns: every workgroup gets one or two strips.  Where 128-row panels x strips, or x pairs
    of strips (200 x 14336, 256 x 12840 with its odd, ragged last strip, 130 x 16320 = exactly one workgroup per
    compute unit), fit the compute units that is one 128 x 64 or 128 x 128 tile each (the kernel that loads X
    fragments straight to registers), otherwise tiles of the four-wave tiled kernel one or two strips wide (their own
    stage schedule); 4 to 16 K stages, ragged rows and a ragged last strip; every element."""
    import torch
    rng = np.random.default_rng(M * 7 + K + N)
    xc, xs, dxc, dxs = _rand_q(rng, M, K, lo=122, hi=132)
    wc, ws, dwc, dws = _rand_q(rng, N, K, lo=122, hi=132)
    wh = B.batq_weight_import(dwc, dws, K, N)
    ref = o.gemm(xc, xs, wc, ws)
    Y = B.batq_gemm_mxfp4(_xc(xc), _xs(xs), wh, M, torch.float32)
    torch.cuda.synchronize()
    tol = 1e-6 * (np.abs(o.dequantize(xc, xs)) @ np.abs(o.dequantize(wc, ws)).T)
    bad = np.argwhere(np.abs(y_to_f32(Y) - ref) > tol + 1e-30)
    assert bad.size == 0, f"{len(bad)} wrong elements, first at {bad[0]}"
    Yb = B.batq_gemm_mxfp4(_xc(xc), _xs(xs), wh, M, torch.bfloat16)
    torch.cuda.synchronize()
    refb = o.bf16_round(ref).astype(np.float64)
    ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(refb), 1e-300))) - 7)
    bad = np.argwhere(np.abs(y_to_f32(Yb).astype(np.float64) - refb) > ulp * 1.0001 + tol)
    assert bad.size == 0, f"{len(bad)} wrong bf16 elements, first at {bad[0]}"


@pytest.mark.parametrize("M,K,N", [(130, 8192, 320), (300, 8192 + 32, 200), (256, 8192 + 256, 1000), (97, 6144, 64),
                                   (65, 12288 + 64, 2100), (520, 16384, 136), (64, 12288 + 32, 2070), (7, 16384, 96),
                                   (384, 8192 + 256, 3264 + 30)])
def test_split_k_shapes(B, M, K, N):
    """Few strips and a long K: with a workspace the kernels cut K into 2 to 8 parts (partial tiles summed in a
    second kernel), with ragged panels, strips and part lengths (the last shape: two K parts of the kernel with one
    128 x 128 tile per workgroup, whose last workgroup has a single, ragged strip).  Every output element is checked for the plain
    call, the full workspace and a third of it (fewer parts); the result is a function of the arguments: the same
    bits on the current stream, on a side stream and from launches that overlap (each with its own workspace)."""
    import torch
    _check_every_element(B, M, K, N)
    _check_every_element(B, M, K, N, workspace_fraction=0.34)
    wh, dxc_b, dxs_g, Y0 = _check_every_element(B, M, K, N, workspace_fraction=1.0)
    need = B.batq_gemm_workspace(wh, M)
    works = [torch.empty(need, dtype=torch.uint8, device="cuda") for _ in range(3)]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        Y1 = B.batq_gemm_mxfp4(dxc_b, dxs_g, wh, M, torch.float32, workspace=works[0])
        Y2 = B.batq_gemm_mxfp4(dxc_b, dxs_g, wh, M, torch.float32, workspace=works[1])
    Y3 = B.batq_gemm_mxfp4(dxc_b, dxs_g, wh, M, torch.float32, workspace=works[2])   # overlaps with the side stream
    torch.cuda.synchronize()
    assert torch.equal(Y0, Y1) and torch.equal(Y0, Y2) and torch.equal(Y0, Y3)
    # a larger workspace than asked for changes nothing
    big = torch.empty(2 * need + 4096, dtype=torch.uint8, device="cuda")
    Y4 = B.batq_gemm_mxfp4(dxc_b, dxs_g, wh, M, torch.float32, workspace=big)
    torch.cuda.synchronize()
    assert torch.equal(Y0, Y4)


def test_gemm_workspace_arguments(B):
    import torch
    rng = np.random.default_rng(12)
    xc, xs, dxc, dxs = _rand_q(rng, 130, 8192)
    wc, ws, dwc, dws = _rand_q(rng, 320, 8192)
    wh = B.batq_weight_import(dwc, dws, 8192, 320)
    assert B.batq_gemm_workspace(wh, 130) > 0 and B.batq_gemm_workspace(wh, 130) % 256 == 0
    assert B.batq_gemm_workspace(wh, 0) == 0 and B.batq_gemm_workspace(wh, 130, 5) == 0
    assert B.batq_linear_workspace_for(wh, 130) > B.batq_linear_workspace(130, 8192)
    wide = B.batq_weight_import(torch.zeros((9000, 64), dtype=torch.uint8, device="cuda"),
                                torch.full((9000, 4), 127, dtype=torch.uint8, device="cuda"), 128, 9000)
    assert B.batq_gemm_workspace(wide, 130) == 0
    assert B.batq_linear_workspace_for(wide, 130) == B.batq_linear_workspace(130, 128)
    Y = torch.empty((130, 320), device="cuda")
    work = torch.empty(B.batq_gemm_workspace(wh, 130) + 256, dtype=torch.uint8, device="cuda")
    args = (_xc(xc).data_ptr(), _xs(xs).data_ptr(), wh.handle, 130, Y.data_ptr(), B.F32, 320)
    assert B.lib.batq_gemm_mxfp4_ws(*args, None, 1024, None) == 1                    # bytes without memory
    assert B.lib.batq_gemm_mxfp4_ws(*args, work.data_ptr() + 16, 1024, None) == 2    # not 256-byte aligned
    assert B.lib.batq_gemm_mxfp4_ws(*args, None, 0, None) == 0                       # the plain call


def test_extreme_scales(B):
    import torch
    rng = np.random.default_rng(5)
    xc, xs, dxc, dxs = _rand_q(rng, 33, 64, lo=0, hi=40)
    wc, ws, dwc, dws = _rand_q(rng, 34, 64, lo=200, hi=255)
    wh = B.batq_weight_import(dwc, dws, 64, 34)
    Y = B.batq_gemm_mxfp4(_xc(xc), _xs(xs), wh, xc.shape[0], torch.float32)
    torch.cuda.synchronize()
    ref = o.gemm(xc, xs, wc, ws)
    assert _relfro(y_to_f32(Y), ref) <= 1e-5


def test_strided_output_and_empty(B):
    import torch
    rng = np.random.default_rng(6)
    xc, xs, dxc, dxs = _rand_q(rng, 20, 64)
    wc, ws, dwc, dws = _rand_q(rng, 24, 64)
    wh = B.batq_weight_import(dwc, dws, 64, 24)
    wide = torch.full((20, 40), 7.0, device="cuda")
    B.batq_gemm_mxfp4(_xc(xc), _xs(xs), wh, 20, Y=wide[:, :24])
    torch.cuda.synchronize()
    assert _relfro(wide[:, :24].cpu().numpy(), o.gemm(xc, xs, wc, ws)) <= 1e-5
    assert bool((wide[:, 24:] == 7.0).all())
    Y0 = B.batq_gemm_mxfp4(_xc(xc)[:0], _xs(xs)[:0], wh, 0, torch.float32)
    assert Y0.shape == (0, 24)


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_linear_all_configs(B, cfg):
    """batq_linear at full size: every output element against the oracle GEMM of the operands the GPU
    produced, and sampled rows and columns end to end against the pure-oracle layer."""
    import torch
    w = bi.make_workload(cfg)
    t = B.Transform(w.K, w.G, w.P, w.clip)
    wh = B.batq_prepare_weight(t, to_dev(w.W, w.dtype))
    X = to_dev(w.X, w.dtype)
    ws_bytes = B.batq_linear_workspace(w.M, w.K)
    assert ws_bytes == B.batq_code_bytes(w.M, w.K) + B.batq_scale_bytes(w.M, w.K)
    assert B.batq_linear_workspace_for(wh, w.M) >= ws_bytes
    work = torch.empty(B.batq_linear_workspace_for(wh, w.M), dtype=torch.uint8, device="cuda")
    out_dtype = torch.bfloat16 if w.out_dtype == "bf16" else torch.float32
    Y = B.batq_linear(t, wh, X, out_dtype, workspace=work)
    Y32 = B.batq_linear(t, wh, X, torch.float32, workspace=work)
    # the two-call route (quantise, then GEMM on the codes it wrote) is the same arithmetic
    xc_d, xs_d = B.batq_quantize_act(t, X)
    Y32b = B.batq_gemm_mxfp4(xc_d, xs_d, wh, w.M, torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(Y32, Y32b)
    # same codes in the workspace (rows past M of the last 32-row tile are unspecified)
    assert np.array_equal(blocked_to_rowmajor(work[: xc_d.numel()].cpu().numpy(), w.M, w.K // 32),
                          blocked_to_rowmajor(xc_d.cpu().numpy(), w.M, w.K // 32))
    # every element of Y (config 4: the first and last 512 rows, all columns) against the oracle's fp64 product
    # of the operands the GPU produced, 512 rows at a time
    xcodes = blocked_to_rowmajor(xc_d.cpu().numpy(), w.M, w.K // 32)
    xscales = grouped_to_rowmajor(xs_d.cpu().numpy(), w.M, w.K // 32)
    wc, wsc = wh.export()
    torch.cuda.synchronize()
    wc, wsc = wc.cpu().numpy(), wsc.cpu().numpy()
    Wdq = o.dequantize(wc, wsc)
    chunks = [(at, min(at + 512, w.M)) for at in range(0, w.M, 512)]
    if cfg == 4:
        chunks = [chunks[0], chunks[-1]]
    num = den = numb = denb = 0.0
    for r0, r1 in chunks:
        Xdq = o.dequantize(xcodes[r0:r1], xscales[r0:r1])
        ref = Xdq @ Wdq.T                                        # = o.gemm on these rows
        tol = 1e-6 * (np.abs(Xdq) @ np.abs(Wdq).T)
        got = Y32[r0:r1].cpu().numpy().astype(np.float64)
        bad = np.argwhere(np.abs(got - ref) > tol + 1e-30)
        assert bad.size == 0, f"rows {r0}..{r1}: {len(bad)} wrong fp32 elements, first at {bad[0]}"
        num += float(np.sum((got - ref) ** 2))
        den += float(np.sum(ref ** 2))
        if w.out_dtype == "bf16":
            refb = o.bf16_round(ref).astype(np.float64)
            gotb = Y[r0:r1].float().cpu().numpy().astype(np.float64)
            ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(refb), 1e-300))) - 7)
            bad = np.argwhere(np.abs(gotb - refb) > ulp * 1.0001 + tol)
            assert bad.size == 0, f"rows {r0}..{r1}: {len(bad)} wrong bf16 elements, first at {bad[0]}"
            numb += float(np.sum((gotb - refb) ** 2))
            denb += float(np.sum(refb ** 2))
    e32 = float(np.sqrt(num / den))
    assert e32 <= 1e-3 and e32 <= 1e-5, e32
    if w.out_dtype == "bf16":
        assert float(np.sqrt(numb / denb)) <= 1e-3
    del Wdq
    # end to end on sampled rows and columns: the oracle quantises the same rows and columns itself; only
    # tie-level code differences remain
    rows = sample_rows(w.M, 96, seed=cfg)
    cols = sample_rows(w.N, 768, seed=cfg + 10)
    sub = lambda T: T[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].float().cpu().numpy()
    oxc, oxs = o.quantize_act(w.X_f32()[rows], w.G, w.P, w.clip)
    owc, ows = o.prepare_weight(w.W_f32()[:, cols], w.G, w.P)
    ref_e2e = o.gemm(oxc, oxs, owc, ows)
    e2e = _relfro(sub(Y32), ref_e2e)
    print(f"cfg {cfg}: fp32-out err {e32:.2e} over {sum(b - a for a, b in chunks)} rows x {w.N} columns, end-to-end err {e2e:.2e}")
    assert e2e <= 2e-3, e2e


def test_linear_argument_errors(B):
    import torch
    w = bi.make_small(8, 64, 16, seed=1, dtype="bf16")
    t = B.Transform(w.K, w.G, w.P, w.clip)
    wh = B.batq_prepare_weight(t, to_dev(w.W, "bf16"))
    X = to_dev(w.X, "bf16")
    Y = torch.zeros((8, 16), device="cuda")
    work = torch.empty(B.batq_linear_workspace(8, 64), dtype=torch.uint8, device="cuda")
    lib = B.lib
    assert lib.batq_linear(t.handle, wh.handle, X.data_ptr(), 1, 8, 64, Y.data_ptr(), 0, 16, work.data_ptr(),
                           work.numel() - 1, None) == 7
    assert lib.batq_linear(t.handle, wh.handle, X.data_ptr(), 1, 8, 64, Y.data_ptr(), 0, 8, work.data_ptr(),
                           work.numel(), None) == 2
    assert lib.batq_linear(t.handle, wh.handle, X.data_ptr(), 1, 8, 64, Y.data_ptr(), 0, 16, None,
                           work.numel(), None) == 1
    t2 = B.Transform(96, None, None, None)
    assert lib.batq_linear(t2.handle, wh.handle, X.data_ptr(), 1, 8, 96, Y.data_ptr(), 0, 16, work.data_ptr(),
                           work.numel(), None) == 10
    xc, xs = B.batq_quantize_act(t, X)
    assert lib.batq_gemm_mxfp4(xc.data_ptr(), xs.data_ptr(), wh.handle, 8, Y.data_ptr(), 0, 8, None) == 2
    assert lib.batq_gemm_mxfp4(xc.data_ptr(), None, wh.handle, 8, Y.data_ptr(), 0, 16, None) == 1
    assert lib.batq_gemm_mxfp4(xc.data_ptr(), xs.data_ptr(), wh.handle, 8, Y.data_ptr(), 5, 16, None) == 3
    torch.cuda.synchronize()
    assert bool((Y == 0).all())


@pytest.mark.parametrize("M,K,N", [(16, 256, 14336 + 40), (33, 512, 13000), (64, 96, 12288 + 17), (50, 2048, 16384)])
def test_small_m_wide_n(B, M, K, N):
    """33 to 64 rows and an N for which the small-M kernel gives a workgroup 64 columns (12288 <= N <= 16384 on
    256 compute units): every element, ragged last column groups included; and its neighbours."""
    test_tile_schedule_shapes(B, M, K, N)


def test_weight_codes_of_two_gib(B):
    """Maximum sizes: a weight whose code array reaches 2 GiB cannot be addressed with the tiled kernel's 32-bit
    offsets; rows > 64 then take the direct kernel, rows <= 64 the small-M kernel with 64-bit addressing.
    Sampled output columns against the oracle."""
    import torch
    K, N = 65536, 65536
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    dwc = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda", generator=g)
    dws = torch.randint(122, 132, (N, K // 32), dtype=torch.uint8, device="cuda", generator=g)
    wh = B.batq_weight_import(dwc, dws, K, N)
    cols = np.concatenate([[0, 1, 31, 32, N - 1, N - 33], sample_rows(N, 42, seed=3)])
    wc = dwc[torch.from_numpy(cols).cuda()].cpu().numpy()
    ws = dws[torch.from_numpy(cols).cuda()].cpu().numpy()
    del dwc, dws
    rng = np.random.default_rng(12)
    for M in (65, 40):
        xc, xs, _, _ = _rand_q(rng, M, K, lo=122, hi=132)
        Y = B.batq_gemm_mxfp4(_xc(xc), _xs(xs), wh, M, torch.float32)
        torch.cuda.synchronize()
        got = Y[:, torch.from_numpy(cols).cuda()].cpu().numpy()
        ref = o.gemm(xc, xs, wc, ws)
        tol = 1e-6 * (np.abs(o.dequantize(xc, xs)) @ np.abs(o.dequantize(wc, ws)).T)
        assert np.all(np.abs(got - ref) <= tol + 1e-30), M
        assert bool(torch.isfinite(Y).all())
