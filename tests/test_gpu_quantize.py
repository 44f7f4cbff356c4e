"""GPU parity: batq_quantize_act (fused transform + clip + MXFP4) against the CPU oracle.

Bars: codes and scales bit-exact when the GPU quantiser is fed the oracle's
transformed fp32 tensor; end to end at most 0.1% of codes differ in value and
every difference sits at a rounding tie.
"""
import numpy as np
import pytest

import batq_inputs as bi
from oracle import batq_oracle as o
from gpu_util import require_gpu, to_dev, unpack, code_value_mismatch, sample_rows, TIE_POINTS, grouped_to_rowmajor, blocked_to_rowmajor

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    require_gpu()
    import paper_2603_16590_amd as b
    return b


def _run(B, t, Xdev):
    import torch
    c, s = B.batq_quantize_act(t, Xdev)
    torch.cuda.synchronize()
    M, K = Xdev.shape
    assert s.numel() == B.batq_scale_bytes(M, K) == ((K // 32 + 7) // 8) * 8 * M
    assert c.numel() == B.batq_code_bytes(M, K) == ((M + 31) // 32) * 32 * ((K + 255) // 256) * 128
    return blocked_to_rowmajor(c.cpu().numpy(), M, K // 32), grouped_to_rowmajor(s.cpu().numpy(), M, K // 32)


# ------------------------------------------------------------------ T1: quantiser alone, bit-exact
@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_quantiser_bit_exact_on_oracle_transformed_input(B, cfg):
    rows = {0: None, 1: None, 2: 512, 3: 256, 4: 512}[cfg]
    w = bi.make_workload(cfg, rows=rows, with_weight=False)
    Xt = o.transform(w.X_f32(), w.G, w.P)                       # oracle's fp32 transformed tensor
    t = B.Transform(w.K, None, None, w.clip)
    gc, gs = _run(B, t, to_dev(Xt, "f32"))
    oc, os_ = o.mxfp4_quantize(Xt, w.clip)
    assert np.array_equal(gs, os_)
    assert np.array_equal(gc, oc)


def test_exhaustive_bf16_patterns_bit_exact(B):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = bi.bf16_bits_to_f32(bits)
    bits = bits[np.isfinite(f)]
    rng = np.random.default_rng(7)
    variants = [np.sort(bits), bits.copy(), rng.permutation(bits)]
    # group by exponent so that every mantissa/sign pattern meets a block scale close to it
    f_ok = bi.bf16_bits_to_f32(bits)
    order = np.lexsort((rng.random(bits.size), np.abs(f_ok)))
    variants.append(bits[order])
    t = B.Transform(32 * 8, None, None, None)
    for v in variants:
        n = (v.size // 256) * 256
        Xb = v[:n].reshape(-1, 256)
        gc, gs = _run(B, t, to_dev(Xb, "bf16"))
        oc, os_ = o.mxfp4_quantize(bi.bf16_bits_to_f32(Xb), None)
        assert np.array_equal(gs, os_)
        assert np.array_equal(gc, oc)


def test_edge_blocks_bit_exact(B):
    K = 64
    rows = []
    z = np.zeros(K, np.float32); rows.append(z)                                    # all-zero blocks
    nz = np.zeros(K, np.float32); nz[::3] = -0.0; rows.append(nz)                  # signed zeros only
    d = np.zeros(K, np.float32); d[:8] = np.float32(1e-41) * np.arange(1, 9); d[9] = -1e-42; rows.append(d)   # subnormal block
    e = np.zeros(K, np.float32); e[0] = 2.0 ** -126; e[1] = -(2.0 ** -127); e[2] = 1.5 * 2.0 ** -125; rows.append(e)
    h = np.zeros(K, np.float32); h[0] = 3.0e38; h[1] = -1.7e38; h[2] = 1e30; h[40] = -3.4e38; rows.append(h)  # near fp32 max
    p = np.zeros(K, np.float32); p[:7] = TIE_POINTS * 4; p[7] = 24.0; p[32:39] = -TIE_POINTS / 8; p[39] = 0.75; rows.append(p)
    X = np.stack(rows)
    for clip in (None, np.array([0.6, 1.0], np.float32), np.array([1.0, 0.33], np.float32)):
        t = B.Transform(K, None, None, clip)
        gc, gs = _run(B, t, to_dev(X, "f32"))
        oc, os_ = o.mxfp4_quantize(X, clip)
        assert np.array_equal(gs, os_), clip
        assert np.array_equal(gc, oc), clip


# ------------------------------------------------------------------ T2: end to end with the transform
def _check_end_to_end(w, gc, gs, rows_idx, g_outer=4, g_inner=8, chunk=256):
    """Every code and scale of the given rows against the oracle; returns the fraction of differing codes.
    Rows are processed `chunk` at a time (the oracle's fp64 intermediates of a whole workload are large)."""
    rows_idx = np.asarray(rows_idx)
    T = o.kron_blocks(w.G, w.P)
    Xf = w.X_f32()
    n_bad = n_all = 0
    for at in range(0, len(rows_idx), chunk):
        ridx = rows_idx[at:at + chunk]
        n, total = _check_rows(w, T, gc[ridx], gs[ridx], Xf[ridx])
        n_bad += n
        n_all += total
    frac = n_bad / max(n_all, 1)
    assert frac <= 1e-3, f"{frac:.2e} of codes differ"
    return frac


def _check_rows(w, T, gc, gs, Xrows):
    Yt = o.apply_blocks(Xrows, T)                                # fp64, before the fp32 rounding
    oc, os_ = o.mxfp4_quantize(Yt.astype(np.float32), w.clip)
    R, nb = os_.shape
    scale_bad = gs != os_
    mism_blocks = code_value_mismatch(gc, oc).reshape(R, nb, 32)
    # a block whose scale differs counts all 32 elements as mismatched
    n_bad = int(np.where(scale_bad, 32, mism_blocks.sum(axis=2)).sum())
    sel = mism_blocks & ~scale_bad[:, :, None]
    if sel.any():
        # every differing element (in blocks with equal scale) sits at a rounding tie: its exact scaled
        # magnitude is within a few fp32 ulps (relative to the block range) of a tie point
        _, bound = o.clip_blocks(Yt.astype(np.float32), w.clip)
        E = os_.astype(np.int64) - 127
        r, k, j = np.nonzero(sel)
        v = np.minimum(np.abs(Yt.reshape(R, nb, 32)[r, k, j]), bound[r, k].astype(np.float64)) / np.exp2(E[r, k])
        dist = np.abs(v[:, None] - TIE_POINTS).min(axis=-1)
        assert np.all(dist < 1e-4), dist.max()
        # and the two codes are neighbours
        g, oo = unpack(gc).reshape(R, nb, 32)[r, k, j], unpack(oc).reshape(R, nb, 32)[r, k, j]
        assert np.all(np.abs((g & 7).astype(int) - (oo & 7).astype(int)) <= 1)
    # a scale difference can only come from a bound within rounding of a power of two (or of 5/4 of one)
    if scale_bad.any():
        _, bound = o.clip_blocks(Yt.astype(np.float32), w.clip)
        b = bound[scale_bad].astype(np.float64)
        m, _ = np.frexp(b)
        assert np.all(np.minimum(np.abs(m - 0.5), np.abs(m - 1.0)) < 1e-5)
    return n_bad, mism_blocks.size


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_fused_transform_quantise_full_configs(B, cfg):
    """The five workloads at full size, every row, code and scale against the oracle."""
    w = bi.make_workload(cfg, with_weight=False)
    t = B.Transform(w.K, w.G, w.P, w.clip)
    gc, gs = _run(B, t, to_dev(w.X, w.dtype))
    assert gc.shape == (w.M, w.K // 2) and gs.shape == (w.M, w.K // 32)
    frac = _check_end_to_end(w, gc, gs, np.arange(w.M))
    print(f"cfg {cfg}: code mismatch fraction {frac:.2e} on all {w.M} rows")


@pytest.mark.parametrize("M,K", [(1, 32), (3, 64), (37, 96), (65, 2080), (130, 4096 + 32), (17, 6144)])
def test_ragged_shapes_and_both_dtypes(B, M, K):
    for dtype in ("bf16", "f32"):
        w = bi.make_small(M, K, 8, seed=M + K, dtype=dtype)
        t = B.Transform(K, w.G, w.P, w.clip)
        gc, gs = _run(B, t, to_dev(w.X, dtype))
        _check_end_to_end(w, gc, gs, np.arange(M))


def test_empty_input_is_a_noop(B):
    import torch
    t = B.Transform(64, None, None, None)
    X = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    c, s = B.batq_quantize_act(t, X)
    assert c.numel() == 0 and s.numel() == 0


def test_strided_rows(B):
    import torch
    w = bi.make_small(33, 128, 8, seed=5, dtype="bf16")
    t = B.Transform(w.K, w.G, w.P, w.clip)
    wide = torch.zeros((33, 256), dtype=torch.bfloat16, device="cuda")
    wide[:, :128] = to_dev(w.X, "bf16")
    gc, gs = _run(B, t, wide[:, :128])
    gc2, gs2 = _run(B, t, to_dev(w.X, "bf16"))
    assert np.array_equal(gc, gc2) and np.array_equal(gs, gs2)


def test_global8_private4_split(B):
    w = bi.make_small(48, 256, 8, seed=9, dtype="bf16", g_outer=8, g_inner=4)
    assert w.G.shape == (8, 8) and w.P.shape == (8, 4, 4)
    t = B.Transform(w.K, w.G, w.P, w.clip, g_outer=8, g_inner=4)
    gc, gs = _run(B, t, to_dev(w.X, "bf16"))
    _check_end_to_end(w, gc, gs, np.arange(w.M))


def test_special_transforms_are_bit_exact(B):
    w = bi.make_workload(0)
    nb = w.nb
    rng = np.random.default_rng(17)
    I8 = np.tile(np.eye(8, dtype=np.float32), (nb, 1, 1))
    # identity == plain RTN
    t = B.Transform(w.K, np.eye(4, dtype=np.float32), I8, w.clip)
    gc, gs = _run(B, t, to_dev(w.X, "f32"))
    oc, os_ = o.mxfp4_quantize(w.X, w.clip)
    assert np.array_equal(gc, oc) and np.array_equal(gs, os_)
    # permutations (exact arithmetic: one non-zero product per output)
    G = np.eye(4, dtype=np.float32)[rng.permutation(4)]
    P = np.stack([np.eye(8, dtype=np.float32)[rng.permutation(8)] for _ in range(nb)])
    t = B.Transform(w.K, G, P, w.clip)
    gc, gs = _run(B, t, to_dev(w.X, "f32"))
    oc, os_ = o.quantize_act(w.X, G, P, w.clip)
    assert np.array_equal(gc, oc) and np.array_equal(gs, os_)
    # power-of-two scaling moves only the scale byte
    t = B.Transform(w.K, np.eye(4, dtype=np.float32) * 8, I8, w.clip)
    gc2, gs2 = _run(B, t, to_dev(w.X, "f32"))
    oc0, os0 = o.mxfp4_quantize(w.X, w.clip)
    assert np.array_equal(gc2, oc0) and np.array_equal(gs2.astype(int), os0.astype(int) + 3)
    # block Hadamard (the block-rotation baseline as a special case): end-to-end bar
    H2 = np.array([[1.0, 1.0], [1.0, -1.0]])
    w.G = (np.kron(H2, H2) / 2).astype(np.float32)
    w.P = np.tile((np.kron(H2, np.kron(H2, H2)) / np.sqrt(8.0)).astype(np.float32), (nb, 1, 1))
    t = B.Transform(w.K, w.G, w.P, w.clip)
    gc, gs = _run(B, t, to_dev(w.X, "f32"))
    _check_end_to_end(w, gc, gs, np.arange(w.M))


def test_scale_order_helpers(B):
    import torch
    rng = np.random.default_rng(2)
    for rows, nb in ((5, 3), (64, 8), (33, 21)):
        rm = rng.integers(0, 255, size=(rows, nb), dtype=np.uint8)
        g = B.batq_scales_from_rowmajor(torch.from_numpy(rm).cuda())
        torch.cuda.synchronize()
        assert np.array_equal(grouped_to_rowmajor(g.cpu().numpy(), rows, nb), rm)
        back = B.batq_scales_to_rowmajor(g, rows, nb * 32)
        torch.cuda.synchronize()
        assert np.array_equal(back.cpu().numpy(), rm)
        for (r, k) in ((0, 0), (rows - 1, nb - 1), (rows // 2, nb // 2)):
            assert B.lib.batq_scale_index(r, k, rows) == ((k // 8) * rows + r) * 8 + (k % 8) // 2 + 4 * (k % 2)


def test_code_order_helpers(B):
    import torch
    from gpu_util import rowmajor_to_blocked
    rng = np.random.default_rng(4)
    for rows, nb in ((5, 3), (64, 8), (33, 21), (16, 4)):
        rm = rng.integers(0, 256, size=(rows, nb * 16), dtype=np.uint8)
        d = B.batq_codes_from_rowmajor(torch.from_numpy(rm).cuda())
        torch.cuda.synchronize()
        assert np.array_equal(blocked_to_rowmajor(d.cpu().numpy(), rows, nb), rm)
        back = B.batq_codes_to_rowmajor(d, rows, nb * 32)
        torch.cuda.synchronize()
        assert np.array_equal(back.cpu().numpy(), rm)
        S = 2 * ((nb + 7) // 8)
        for (r, k) in ((0, 0), (rows - 1, nb - 1), (rows // 2, nb // 2)):
            exp = ((r // 16) * S + k // 4) * 1024 + (r % 16) * 64 + (((k % 4) ^ ((r % 16) // 4)) * 16)
            assert B.lib.batq_code_chunk_offset(r, k, nb * 32) == exp


def test_deterministic(B):
    w = bi.make_workload(1, with_weight=False)
    t = B.Transform(w.K, w.G, w.P, w.clip)
    X = to_dev(w.X, "bf16")
    a = _run(B, t, X)
    b = _run(B, t, X)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_argument_errors_leave_outputs_untouched(B):
    import torch
    t = B.Transform(64, None, None, None)
    X = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    codes = torch.full((B.batq_code_bytes(4, 64),), 0xAB, dtype=torch.uint8, device="cuda")
    scales = torch.full((4 * 8,), 0xCD, dtype=torch.uint8, device="cuda")
    lib = B.lib
    assert lib.batq_quantize_act(t.handle, X.data_ptr(), 1, 4, 96, 96, codes.data_ptr(), scales.data_ptr(), None) == 10
    assert lib.batq_quantize_act(t.handle, X.data_ptr(), 1, 4, 64, 32, codes.data_ptr(), scales.data_ptr(), None) == 2
    assert lib.batq_quantize_act(t.handle, X.data_ptr(), 7, 4, 64, 64, codes.data_ptr(), scales.data_ptr(), None) == 3
    assert lib.batq_quantize_act(t.handle, X.data_ptr() + 2, 1, 4, 64, 64, codes.data_ptr(), scales.data_ptr(), None) == 2
    assert lib.batq_quantize_act(t.handle, None, 1, 4, 64, 64, codes.data_ptr(), scales.data_ptr(), None) == 1
    torch.cuda.synchronize()
    assert bool((codes == 0xAB).all()) and bool((scales == 0xCD).all())


def test_row_stride_beyond_the_matrix_core_kernels_offsets(B):
    """A bf16 input whose row stride is 2^25 elements or more cannot be addressed with the persistent matrix-core
    kernel's 32-bit tile offsets: such calls take the row-by-row matrix-core kernel (64-bit addresses) whatever the
    row count, with the same arithmetic - the codes of the contiguous call, byte for byte."""
    import torch
    M, K, ld = 5, 32 * 9, 1 << 25
    w = bi.make_small(M, K, 8, seed=77, dtype="bf16")
    big = torch.zeros((M, ld), dtype=torch.bfloat16, device="cuda")
    big[:, :K] = to_dev(w.X, "bf16")
    T = o.kron_blocks(w.G, w.P)
    for t in (B.Transform(K, w.G, w.P, w.clip), B.Transform.general(K, dense=T.astype(np.float32), clip=w.clip)):
        c, s = B.batq_quantize_act(t, big[:, :K])
        c0, s0 = B.batq_quantize_act(t, to_dev(w.X, "bf16"))
        torch.cuda.synchronize()
        gc = blocked_to_rowmajor(c.cpu().numpy(), M, K // 32)
        gs = grouped_to_rowmajor(s.cpu().numpy(), M, K // 32)
        oc, os_ = o.quantize_act_blocks(w.X_f32(), T, w.clip)
        assert np.mean(gs != os_) <= 0.01 and np.mean(code_value_mismatch(gc, oc)) <= 1e-3
        # and the same codes and scales as the contiguous call
        g0 = blocked_to_rowmajor(c0.cpu().numpy(), M, K // 32)
        assert np.array_equal(gc, g0) and torch.equal(s, s0)


@pytest.mark.parametrize("bits", [4, 8])
def test_a_rows_codes_do_not_depend_on_the_batch(B, bits):
    """Sec. 3.2 writes the key/value cache token by token and evaluates whole sequences: the same bf16 row must get
    the same codes and scale in a 1-row, a 16-row, a 129-row and a 2100-row call.  The whole call (more than 2^22
    elements) runs on the persistent matrix-core kernel, the small ones on the row-by-row kernel; the two share one
    arithmetic.  Checked with every option of the online call, and for an append whose window starts off a 32-row
    tile (its first rows take the row-by-row kernel, the rest the persistent one)."""
    import torch
    M, K = 2100, 32 * 65
    assert M * K > 1 << 22
    w = bi.make_small(M, K, 8, seed=31 + bits, dtype="bf16")
    rng = np.random.default_rng(bits)
    rs = torch.from_numpy(rng.uniform(0.5, 2.0, M).astype(np.float32)).cuda()
    X = to_dev(w.X, "bf16")
    Uup = to_dev(bi.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)), "bf16")
    to_rm = B.batq_codes8_to_rowmajor if bits == 8 else B.batq_codes_to_rowmajor
    transforms = [B.Transform(K, w.G, w.P, w.clip),
                  B.Transform.general(K, dense=o.kron_blocks(w.G, w.P).astype(np.float32),
                                      clip_min=w.clip, clip_max=np.minimum(1.0, w.clip + 0.05).astype(np.float32))]
    for t in transforms:
        for opts in ({}, {"row_scale": rs}, {"up": Uup}):
            def run(r0, r1):
                kw = {k: v[r0:r1] for k, v in opts.items()}
                c, s = B.batq_quantize_act_ex(t, X[r0:r1], act_bits=bits, **kw)
                return to_rm(c, r1 - r0, K), B.batq_scales_to_rowmajor(s, r1 - r0, K)
            c_all, s_all = run(0, M)
            for r0, r1 in ((0, 1), (2099, 2100), (3, 19), (64, 193), (130, 131), (500, 628), (200, 1000)):
                c, s = run(r0, r1)
                torch.cuda.synchronize()
                assert torch.equal(c, c_all[r0:r1]) and torch.equal(s, s_all[r0:r1]), (bits, list(opts), r0, r1)
        # one long append at row 7 of a cache laid out for more rows
        cap = M + 40
        codes = torch.zeros(B.batq_code8_bytes(cap, K) if bits == 8 else B.batq_code_bytes(cap, K), dtype=torch.uint8, device="cuda")
        scales = torch.zeros(B.batq_scale_bytes(cap, K), dtype=torch.uint8, device="cuda")
        B.batq_kv_append(t, X, codes, scales, 7, cap, bits)
        c_ref, s_ref = B.batq_quantize_act_ex(t, X, act_bits=bits)
        torch.cuda.synchronize()
        assert torch.equal(to_rm(codes, cap, K)[7:7 + M], to_rm(c_ref, M, K))
        assert torch.equal(B.batq_scales_to_rowmajor(scales, cap, K)[7:7 + M], B.batq_scales_to_rowmajor(s_ref, M, K))
