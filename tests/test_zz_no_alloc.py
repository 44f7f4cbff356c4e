"""The allocation-free GEMM entry point (partial sums of the K parts in a device array that belongs to the library)
against the entry point that takes the same memory as a caller workspace: identical bits, on two calls in a row,
the second on a smaller input, and on a shape of the small-M kernel."""
import numpy as np
import pytest

from gpu_util import require_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    require_gpu()
    import paper_2603_16590_amd as b
    return b


def _problem(B, M, K, N, seed):
    import torch
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    wc = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda", generator=g)
    ws = torch.randint(122, 132, (N, K // 32), dtype=torch.uint8, device="cuda", generator=g)
    wh = B.batq_weight_import(wc, ws, K, N)
    xc = B.batq_codes_from_rowmajor(torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda", generator=g))
    xs = B.batq_scales_from_rowmajor(torch.randint(122, 132, (M, K // 32), dtype=torch.uint8, device="cuda", generator=g))
    return wh, xc, xs


def _noalloc(B, xc, xs, wh, M, Y):
    import torch
    st = B.lib.batq_gemm_mxfp4_noalloc(xc.data_ptr(), xs.data_ptr(), wh.handle, M, Y.data_ptr(),
                                       B.BF16 if Y.dtype == torch.bfloat16 else B.F32, Y.stride(0),
                                       torch.cuda.current_stream().cuda_stream)
    assert st == 0, B.STATUS_NAMES.get(st, st)


def test_noalloc_gemm_equals_the_workspace_entry_point(B):
    import torch
    # (M, K, N): K parts at 16 MiB, the most any shape asks for; fewer rows and columns; 40 rows (K parts in the
    # one-tile-per-workgroup kernel) followed by 31 (two K parts in the small-M kernel); a shape without K parts
    cases = [(300, 14336, 4096), (130, 8192, 320), (40, 16384, 96), (200, 512, 3000)]
    for n, (M, K, N) in enumerate(cases):
        wh, xc, xs = _problem(B, M, K, N, seed=20 + n)
        need = B.batq_gemm_workspace(wh, M)
        assert need <= 16 << 20
        assert (need > 0) == (n < 3)
        for dt in (torch.float32, torch.bfloat16):
            work = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
            ref = B.batq_gemm_mxfp4(xc, xs, wh, M, dt, workspace=work if need else None)
            Y = torch.zeros((M, N), dtype=dt, device="cuda")
            _noalloc(B, xc, xs, wh, M, Y)
            torch.cuda.synchronize()
            assert torch.equal(Y, ref), (M, K, N, dt)
            # a second call right behind it on fewer rows of the same operands: the array still holds the first
            # call's sums, and nothing of them may show
            M2 = M - 37 if M > 64 else M - 9
            need2 = B.batq_gemm_workspace(wh, M2)
            xc2 = B.batq_codes_from_rowmajor(B.batq_codes_to_rowmajor(xc, M, K)[:M2].contiguous())
            xs2 = B.batq_scales_from_rowmajor(B.batq_scales_to_rowmajor(xs, M, K)[:M2].contiguous())
            work2 = torch.empty(max(need2, 256), dtype=torch.uint8, device="cuda")
            ref2 = B.batq_gemm_mxfp4(xc2, xs2, wh, M2, dt, workspace=work2 if need2 else None)
            Y1 = torch.zeros((M, N), dtype=dt, device="cuda")
            Y2 = torch.zeros((M2, N), dtype=dt, device="cuda")
            _noalloc(B, xc, xs, wh, M, Y1)
            _noalloc(B, xc2, xs2, wh, M2, Y2)
            torch.cuda.synchronize()
            assert torch.equal(Y1, ref), (M, K, N, dt)
            assert torch.equal(Y2, ref2), (M2, K, N, dt)
            # (the smaller call may run on another kernel with another summation order: compared with the first
            # call's rows only to rounding)
            assert torch.allclose(Y2.float(), ref[:M2].float(), rtol=2e-2 if dt == torch.bfloat16 else 1e-4,
                                  atol=1e-2 * float(ref.float().abs().max()) if dt == torch.bfloat16 else 1e-4 * float(ref.abs().max()))


def test_noalloc_gemm_argument_errors(B):
    import torch
    wh, xc, xs = _problem(B, 130, 8192, 320, seed=3)
    Y = torch.zeros((130, 320), device="cuda")
    lib = B.lib
    assert lib.batq_gemm_mxfp4_noalloc(xc.data_ptr(), xs.data_ptr(), None, 130, Y.data_ptr(), 0, 320, None) == 1
    assert lib.batq_gemm_mxfp4_noalloc(xc.data_ptr(), None, wh.handle, 130, Y.data_ptr(), 0, 320, None) == 1
    assert lib.batq_gemm_mxfp4_noalloc(xc.data_ptr(), xs.data_ptr(), wh.handle, 130, Y.data_ptr(), 0, 100, None) == 2
    assert lib.batq_gemm_mxfp4_noalloc(xc.data_ptr(), xs.data_ptr(), wh.handle, 130, Y.data_ptr(), 7, 320, None) == 3
    assert lib.batq_gemm_mxfp4_noalloc(xc.data_ptr(), xs.data_ptr(), wh.handle, 0, Y.data_ptr(), 0, 320, None) == 0
    torch.cuda.synchronize()
    assert bool((Y == 0).all())
