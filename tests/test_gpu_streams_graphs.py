"""The online calls only enqueue kernels (no allocation, no host synchronisation): they must work on a
non-default stream and inside a captured HIP graph, replayed several times with eager work in between."""
import numpy as np
import pytest

import batq_inputs as bi
from oracle import batq_oracle as o
from gpu_util import require_gpu, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    require_gpu()
    import paper_2603_16590_amd as b
    return b


def _setup(B, M, K, N, seed):
    w = bi.make_small(M, K, N, seed=seed, dtype="bf16")
    t = B.Transform(w.K, w.G, w.P, w.clip)
    wh = B.batq_prepare_weight(t, to_dev(w.W, "bf16"))
    return w, t, wh


@pytest.mark.parametrize("M", [16, 384])
def test_linear_on_a_side_stream(B, M):
    import torch
    w, t, wh = _setup(B, M, 32 * 20, 320, seed=M)
    X = to_dev(w.X, "bf16")
    ref = B.batq_linear(t, wh, X, torch.bfloat16)
    ref8 = B.batq_linear_a8w4(t, wh, X, torch.bfloat16)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    work = torch.empty(B.batq_linear_workspace_for(wh, M, 8), dtype=torch.uint8, device="cuda")
    Y = torch.empty_like(ref)
    Y8 = torch.empty_like(ref)
    with torch.cuda.stream(side):
        B.batq_linear(t, wh, X, Y=Y, workspace=work)
        B.batq_linear_a8w4(t, wh, X, Y=Y8, workspace=work)
    side.synchronize()
    assert torch.equal(Y, ref) and torch.equal(Y8, ref8)


@pytest.mark.parametrize("M", [16, 384])
def test_linear_inside_a_captured_graph(B, M):
    import torch
    w, t, wh = _setup(B, M, 32 * 20, 320, seed=100 + M)
    rng = np.random.default_rng(M)
    X = to_dev(w.X, "bf16")
    work = torch.empty(B.batq_linear_workspace(M, w.K), dtype=torch.uint8, device="cuda")
    Y = torch.empty((M, w.N), dtype=torch.bfloat16, device="cuda")
    B.batq_linear(t, wh, X, Y=Y, workspace=work)              # first call outside the capture (one-time set-up)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.batq_linear(t, wh, X, Y=Y, workspace=work)
    for rep in range(4):
        # new input in place, eager reference, some unrelated eager work, then the replay
        Xn = bi.f32_to_bf16_bits((rng.standard_normal((M, w.K)) * (rep + 1)).astype(np.float32))
        X.copy_(to_dev(Xn, "bf16"))
        ref = B.batq_linear(t, wh, X, torch.bfloat16)
        junk = (torch.randn(257, 129, device="cuda") @ torch.randn(129, 65, device="cuda")).sum()
        torch.cuda.synchronize()
        Y.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, ref), rep
        assert bool(torch.isfinite(junk))


def _split_k_problem(B, seed=5):
    import torch
    M, K, N = 130, 8192, 320
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    wc = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda", generator=g)
    ws = torch.randint(122, 132, (N, K // 32), dtype=torch.uint8, device="cuda", generator=g)
    wh = B.batq_weight_import(wc, ws, K, N)
    xsr = torch.randint(122, 132, (M, K // 32), dtype=torch.uint8, device="cuda", generator=g)
    xr = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda", generator=g)
    ref = o.gemm(xr.cpu().numpy(), xsr.cpu().numpy(), wc.cpu().numpy(), ws.cpu().numpy())
    tol = 1e-6 * (np.abs(o.dequantize(xr.cpu().numpy(), xsr.cpu().numpy())) @
                  np.abs(o.dequantize(wc.cpu().numpy(), ws.cpu().numpy())).T)
    return M, wh, B.batq_codes_from_rowmajor(xr), B.batq_scales_from_rowmajor(xsr), ref, tol


def test_split_k_gemm_in_graphs(B):
    """A long-K, few-strip GEMM with a workspace cuts K into parts.  The kernels a call enqueues depend on its
    arguments only, so a capture records the same kernels as an eager call, on a stream that has never run the
    shape as on one that has, and every replay gives the eager bits."""
    import torch
    M, wh, xc, xs, ref64, tol = _split_k_problem(B)
    need = B.batq_gemm_workspace(wh, M)
    assert need > 0
    work = torch.empty(need, dtype=torch.uint8, device="cuda")
    ref = B.batq_gemm_mxfp4(xc, xs, wh, M, torch.float32, workspace=work)       # eager, current stream
    torch.cuda.synchronize()
    assert np.all(np.abs(ref.cpu().numpy().astype(np.float64) - ref64) <= tol + 1e-30)
    for warm in (False, True):
        st = torch.cuda.Stream()
        Y = torch.zeros_like(ref)
        if warm:
            with torch.cuda.stream(st):
                B.batq_gemm_mxfp4(xc, xs, wh, M, Y=Y, workspace=work)
            st.synchronize()
            assert torch.equal(Y, ref)
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr, stream=st):
            B.batq_gemm_mxfp4(xc, xs, wh, M, Y=Y, workspace=work)
        for rep in range(3):
            Y.zero_()
            junk = torch.randn(300, 300, device="cuda") @ torch.randn(300, 300, device="cuda")
            torch.cuda.synchronize()
            gr.replay()
            torch.cuda.synchronize()
            assert torch.equal(Y, ref), (warm, rep)
            assert bool(torch.isfinite(junk).all())


def test_split_k_graph_replay_beside_eager_launches(B):
    """A graph captured on stream A, replayed on stream B while eager K-part GEMMs run on A: each call owns the
    workspace it was given, so nothing is shared between the two and both give the reference bits."""
    import torch
    M, wh, xc, xs, ref64, tol = _split_k_problem(B, seed=6)
    need = B.batq_gemm_workspace(wh, M)
    work_g = torch.empty(need, dtype=torch.uint8, device="cuda")
    work_e = torch.empty(need, dtype=torch.uint8, device="cuda")
    ref = B.batq_gemm_mxfp4(xc, xs, wh, M, torch.float32, workspace=work_e)
    torch.cuda.synchronize()
    assert np.all(np.abs(ref.cpu().numpy().astype(np.float64) - ref64) <= tol + 1e-30)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    Yg = torch.zeros_like(ref)
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr, stream=sa):
        B.batq_gemm_mxfp4(xc, xs, wh, M, Y=Yg, workspace=work_g)
    Ye = [torch.zeros_like(ref) for _ in range(6)]
    for rep in range(3):
        Yg.zero_()
        for y in Ye:
            y.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(sa):
            for y in Ye[:3]:
                B.batq_gemm_mxfp4(xc, xs, wh, M, Y=y, workspace=work_e)
        with torch.cuda.stream(sb):
            gr.replay()
        with torch.cuda.stream(sa):
            for y in Ye[3:]:
                B.batq_gemm_mxfp4(xc, xs, wh, M, Y=y, workspace=work_e)
        torch.cuda.synchronize()
        assert torch.equal(Yg, ref), rep
        for y in Ye:
            assert torch.equal(y, ref), rep


def test_cache_calls_inside_a_captured_graph(B):
    """A decode step on the cache (append one row, read the window back, transform the query) captured once and
    replayed at a moving position is not possible (the position is a launch argument), so the graph holds the step
    for one position and its replays must give the eager result every time, with eager appends in between."""
    import torch
    D, cap = 32 * 12, 200
    w = bi.make_small(cap, D, 8, seed=4, dtype="bf16")
    t = B.Transform(D, w.G, w.P, w.clip)
    X = to_dev(w.X, "bf16")
    codes = torch.zeros(B.batq_code8_bytes(cap, D), dtype=torch.uint8, device="cuda")
    scales = torch.zeros(B.batq_scale_bytes(cap, D), dtype=torch.uint8, device="cuda")
    B.batq_kv_append(t, X[:150], codes, scales, 0, cap, 8)          # prefill on the matrix cores
    q = X[150:154]
    # eager reference for the step at position 150
    c_ref, s_ref = codes.clone(), scales.clone()
    B.batq_kv_append(t, X[150:151], c_ref, s_ref, 150, cap, 8)
    win_ref = B.batq_kv_dequantize(c_ref, s_ref, cap, 0, 151, D, 8)
    q_ref = B.batq_transform_apply(t, q, B.APPLY_INVERSE_T)
    torch.cuda.synchronize()
    win = torch.empty_like(win_ref)
    qt = torch.empty_like(q_ref)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):                                    # first calls outside the capture
        B.batq_kv_append(t, X[150:151], codes, scales, 150, cap, 8)
        B.batq_kv_dequantize(codes, scales, cap, 0, 151, D, 8, out=win)
        B.batq_transform_apply(t, q, B.APPLY_INVERSE_T, out=qt)
    side.synchronize()
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr, stream=side):
        B.batq_kv_append(t, X[150:151], codes, scales, 150, cap, 8)
        B.batq_kv_dequantize(codes, scales, cap, 0, 151, D, 8, out=win)
        B.batq_transform_apply(t, q, B.APPLY_INVERSE_T, out=qt)
    for rep in range(3):
        win.zero_()
        qt.zero_()
        B.batq_kv_append(t, X[160 + rep:161 + rep], codes, scales, 160 + rep, cap, 8)      # eager work in between
        torch.cuda.synchronize()
        gr.replay()
        torch.cuda.synchronize()
        assert torch.equal(win, win_ref), rep
        assert torch.equal(qt, q_ref), rep
