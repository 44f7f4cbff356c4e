"""GPU parity: batq_prepare_weight (inverse transform + clip + MXFP4 along K) against the oracle."""
import numpy as np
import pytest

import batq_inputs as bi
from oracle import batq_oracle as o
from gpu_util import require_gpu, to_dev, code_value_mismatch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    require_gpu()
    import paper_2603_16590_amd as b
    return b


def _export(B, wh):
    import torch
    c, s = wh.export()
    torch.cuda.synchronize()
    return c.cpu().numpy(), s.cpu().numpy()


def _compare(gc, gs, oc, os_, tol=1e-4):
    # fp64 products on both sides; only the summation order differs, so codes agree except
    # where a value sits within an fp64 rounding of a tie
    scale_bad = gs != os_
    mism = code_value_mismatch(gc, oc).reshape(gs.shape[0], gs.shape[1], 32)
    n_bad = int(np.where(scale_bad, 32, mism.sum(axis=2)).sum())
    assert n_bad / mism.size <= tol, n_bad / mism.size
    return n_bad


@pytest.mark.parametrize("cfg", [0, 1])
def test_prepare_weight_full(B, cfg):
    w = bi.make_workload(cfg)
    t = B.Transform(w.K, w.G, w.P, w.clip)
    wh = B.batq_prepare_weight(t, to_dev(w.W, w.dtype))
    gc, gs = _export(B, wh)
    assert gc.shape == (w.N, w.K // 2) and gs.shape == (w.N, w.K // 32)
    oc, os_ = o.prepare_weight(w.W_f32(), w.G, w.P)
    n_bad = _compare(gc, gs, oc, os_)
    print(f"cfg {cfg}: {n_bad} differing weight codes of {gc.size * 2}")


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_prepare_weight_large_sampled_columns(B, cfg):
    w = bi.make_workload(cfg, rows=1)
    t = B.Transform(w.K, w.G, w.P, w.clip)
    wh = B.batq_prepare_weight(t, to_dev(w.W, w.dtype))
    gc, gs = _export(B, wh)
    rng = np.random.default_rng(cfg)
    cols = np.sort(np.concatenate([[0, w.N - 1], rng.choice(np.arange(1, w.N - 1), 254, replace=False)]))
    oc, os_ = o.prepare_weight(w.W_f32()[:, cols], w.G, w.P)
    _compare(gc[cols], gs[cols], oc, os_)


def test_layouts_clip_and_dtypes(B):
    import torch
    w = bi.make_small(8, 160, 77, seed=4, dtype="f32")
    t = B.Transform(w.K, w.G, w.P, w.clip)
    clip_w = np.random.default_rng(1).uniform(0.6, 1.0, w.nb).astype(np.float32)
    oc, os_ = o.prepare_weight(w.W, w.G, w.P, clip_w)
    Wd = to_dev(w.W, "f32")
    # K x N
    gc, gs = _export(B, B.batq_prepare_weight(t, Wd, True, clip_w))
    _compare(gc, gs, oc, os_, tol=0)
    # N x K (the paper's out x in storage)
    gc, gs = _export(B, B.batq_prepare_weight(t, Wd.t().contiguous(), False, clip_w))
    _compare(gc, gs, oc, os_, tol=0)
    # strided rows
    wide = torch.zeros((w.K, 128), device="cuda")
    wide[:, :77] = Wd
    gc, gs = _export(B, B.batq_prepare_weight(t, wide[:, :77], True, clip_w))
    _compare(gc, gs, oc, os_, tol=0)
    # bf16 storage
    wb = bi.make_small(8, 160, 77, seed=4, dtype="bf16")
    oc, os_ = o.prepare_weight(wb.W_f32(), wb.G, wb.P, None)
    gc, gs = _export(B, B.batq_prepare_weight(t, to_dev(wb.W, "bf16")))
    _compare(gc, gs, oc, os_, tol=0)
    # no transform: plain RTN of W, bit-exact
    t0 = B.Transform(w.K, None, None, None)
    oc, os_ = o.prepare_weight(w.W, None, None, clip_w)
    gc, gs = _export(B, B.batq_prepare_weight(t0, Wd, True, clip_w))
    assert np.array_equal(gc, oc) and np.array_equal(gs, os_)


def test_import_export_round_trip(B):
    import torch
    rng = np.random.default_rng(3)
    codes = torch.from_numpy(rng.integers(0, 256, size=(70, 48), dtype=np.uint8)).cuda()
    scales = torch.from_numpy(rng.integers(100, 140, size=(70, 3), dtype=np.uint8)).cuda()
    wh = B.batq_weight_import(codes, scales, 96, 70)
    assert (wh.K, wh.N) == (96, 70)
    c, s = wh.export()
    torch.cuda.synchronize()
    assert torch.equal(c, codes) and torch.equal(s, scales)


def test_weight_argument_errors(B):
    import ctypes as C
    w = bi.make_small(4, 64, 16, seed=1, dtype="f32")
    t = B.Transform(w.K, w.G, w.P, None)
    Wd = to_dev(w.W, "f32")
    h = C.c_void_p()
    lib = B.lib
    assert lib.batq_prepare_weight(C.byref(h), t.handle, Wd.data_ptr(), 0, 96, 16, 16, 1, None, None) == 10
    assert lib.batq_prepare_weight(C.byref(h), t.handle, Wd.data_ptr(), 0, 64, 16, 8, 1, None, None) == 2
    assert lib.batq_prepare_weight(C.byref(h), t.handle, None, 0, 64, 16, 16, 1, None, None) == 1
    bad = np.array([0.5, 0.0], np.float32)
    assert lib.batq_prepare_weight(C.byref(h), t.handle, Wd.data_ptr(), 0, 64, 16, 16, 1,
                                   bad.ctypes.data_as(C.POINTER(C.c_float)), None) == 6
