"""Pins for the oracle's RMSNorm pieces and the identity behind fusing the norm into the quantiser."""
import numpy as np

from oracle import batq_oracle as o


def test_rmsnorm_is_the_textbook_definition():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((5, 64))
    g = rng.uniform(0.5, 1.5, 64)
    Y = o.rmsnorm(X, g, 1e-6)
    for m in range(5):
        ms = sum(float(v) ** 2 for v in X[m]) / 64
        for j in range(64):
            assert abs(Y[m, j] - X[m, j] * g[j] / (ms + 1e-6) ** 0.5) < 1e-14
    # unit weight, no eps: every row ends with mean square 1
    Z = o.rmsnorm(X, np.ones(64), 0.0)
    assert np.allclose(np.mean(Z * Z, axis=1), 1.0, rtol=0, atol=1e-14)
    # scale invariance of the normalised row (eps = 0)
    assert np.allclose(o.rmsnorm(3.7 * X, g, 0.0), Y * 0 + o.rmsnorm(X, g, 0.0), rtol=0, atol=1e-13)


def test_norm_then_transform_equals_rowscale_times_folded_transform():
    # RMSNorm(x) T = r (x diag(gamma)) T = r x T'  with T'_k = diag(gamma_k) T_k
    rng = np.random.default_rng(2)
    nb = 3
    X = rng.standard_normal((7, 32 * nb))
    g = rng.uniform(0.5, 1.5, 32 * nb)
    T = np.eye(32)[None] + 0.05 * rng.standard_normal((nb, 32, 32))
    lhs = o.apply_blocks(o.rmsnorm(X, g, 1e-5), T)
    r = o.row_rms_scale(X, 1e-5)
    rhs = o.apply_blocks(X, o.fold_norm_weight(T, g)) * r[:, None]
    assert np.allclose(lhs, rhs, rtol=0, atol=1e-13)
    Tf = o.fold_norm_weight(T, g)
    for k in range(nb):
        assert np.array_equal(Tf[k], np.diag(g[32 * k:32 * k + 32]) @ T[k])


def test_fused_path_quantises_the_normalised_activations():
    rng = np.random.default_rng(3)
    nb = 4
    X = (rng.standard_normal((9, 32 * nb)) * 5).astype(np.float32)
    g = rng.uniform(0.5, 1.5, 32 * nb)
    T = np.eye(32)[None] + 0.05 * rng.standard_normal((nb, 32, 32))
    clip = rng.uniform(0.8, 1.0, nb).astype(np.float32)
    # unfused: normalise (fp64), transform, quantise
    a = o.mxfp4_quantize(o.apply_blocks(o.rmsnorm(X, g, 1e-6), T).astype(np.float32), clip)
    # fused: row factors and folded blocks through the blocks path
    b = o.quantize_act_blocks(X, o.fold_norm_weight(T, g), clip, row_scale=o.row_rms_scale(X, 1e-6))
    # the two orders of fp64 operations agree to rounding: identical except at fp32-rounding ties
    assert np.mean(a[0] != b[0]) < 0.01 and np.array_equal(a[1], b[1])
    # row factors of one are the plain path, also for 8-bit output
    assert all(np.array_equal(u, v) for u, v in zip(o.quantize_act_blocks(X, T, clip, row_scale=np.ones(9)),
                                                    o.quantize_act_blocks(X, T, clip)))
    assert all(np.array_equal(u, v) for u, v in zip(o.quantize_act_blocks(X, T, clip, fp8=True),
                                                    o.quantize_act_fp8(X, T, clip)))
    # a power-of-two row factor moves the scale bytes and leaves the codes alone
    c2 = o.quantize_act_blocks(X, T, None, row_scale=np.full(9, 4.0))
    c1 = o.quantize_act_blocks(X, T, None)
    assert np.array_equal(c2[0], c1[0]) and np.array_equal(c2[1].astype(int), c1[1].astype(int) + 2)


# ---------------------------------------------------------------- gated activation (input of the down projection)
def test_silu_closed_forms_and_library():
    import math
    import torch
    assert o.silu(np.array([0.0]))[0] == 0.0
    # sigmoid(ln 3) = 3/4
    assert abs(o.silu(np.array([math.log(3.0)]))[0] - 0.75 * math.log(3.0)) < 1e-15
    # silu(x) - silu(-x) = x  (sigmoid(x) + sigmoid(-x) = 1)
    x = np.linspace(-30, 30, 1001)
    assert np.allclose(o.silu(x) - o.silu(-x), x, rtol=0, atol=1e-14)
    # the minimum: the stationary point solves x = -1 - exp(x), and there silu(x) = x + 1
    lo, hi = -2.0, -1.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if mid + 1.0 + math.exp(mid) > 0:
            hi = mid
        else:
            lo = mid
    xs = 0.5 * (lo + hi)
    assert abs(o.silu(np.array([xs]))[0] - (xs + 1.0)) < 1e-14
    assert np.all(o.silu(x) >= xs + 1.0 - 1e-15)
    # tails: -> x for large x, -> x exp(x) for very negative x; no overflow warnings or NaN
    assert o.silu(np.array([800.0]))[0] == 800.0
    assert abs(o.silu(np.array([-40.0]))[0] / (-40.0 * math.exp(-40.0)) - 1.0) < 1e-15
    assert o.silu(np.array([-800.0]))[0] == 0.0
    # library routine (fp64 CPU)
    xr = np.random.default_rng(3).standard_normal(500) * 4
    ref = torch.nn.functional.silu(torch.from_numpy(xr)).numpy()
    assert np.allclose(o.silu(xr), ref, rtol=1e-15, atol=1e-300)


def test_swiglu_is_silu_gate_times_up_and_rounds_once():
    import torch
    rng = np.random.default_rng(4)
    g = rng.standard_normal((6, 64)) * 2
    u = rng.standard_normal((6, 64))
    h = o.swiglu(g, u)
    for m in range(6):
        for j in range(64):
            gv, uv = float(g[m, j]), float(u[m, j])
            assert abs(h[m, j] - gv / (1.0 + np.exp(-gv)) * uv) <= 1e-15 * abs(h[m, j]) + 1e-300
    # not symmetric in its arguments: silu acts on the first
    assert not np.allclose(o.swiglu(g, u), o.swiglu(u, g))
    hb = o.swiglu_bf16(g, u)
    assert hb.dtype == np.float32 and np.all((hb.view(np.uint32) & 0xFFFF) == 0)
    # nearest bf16 value of the fp64 product: no farther than half a bf16 ulp (8 significant bits: 2^-8 relative at most)
    assert np.all(np.abs(hb.astype(np.float64) - h) <= np.abs(h) * 2.0 ** -8)
    # where the product is an fp32 number, the library's fp32 -> bf16 conversion agrees
    h32 = h.astype(np.float32)
    lib = torch.from_numpy(h32).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(o.bf16_round(h32), lib)
    # one rounding, not fp64 -> fp32 -> bf16: just above a bf16 tie must round up
    x = np.array([1.0 + 2.0 ** -8 + 2.0 ** -40])
    assert o.bf16_round(x)[0] == np.float32(1.0 + 2.0 ** -7)
    assert o.bf16_round(np.array([1.0 + 2.0 ** -8]))[0] == np.float32(1.0)              # tie -> even
    assert o.bf16_round(np.array([1.0 + 3 * 2.0 ** -8]))[0] == np.float32(1.0 + 2.0 ** -6)


def test_swiglu_feeds_the_quantiser_like_a_materialised_tensor():
    rng = np.random.default_rng(5)
    nb = 2
    g = rng.standard_normal((9, 32 * nb)) * 2
    u = rng.standard_normal((9, 32 * nb))
    T = np.eye(32)[None] + 0.05 * rng.standard_normal((nb, 32, 32))
    clip = rng.uniform(0.85, 1.0, nb).astype(np.float32)
    c1, s1 = o.quantize_act_blocks(o.swiglu_bf16(g, u), T, clip)
    H = np.empty((9, 32 * nb), dtype=np.float32)
    for m in range(9):
        for j in range(32 * nb):
            H[m, j] = o.bf16_round(np.array([o.silu(np.array([g[m, j]]))[0] * u[m, j]]))[0]
    c2, s2 = o.quantize_act_blocks(H, T, clip)
    assert np.array_equal(c1, c2) and np.array_equal(s1, s2)
    # zero gate or zero up gives an all-zero block: neutral codes, lowest scale byte
    cz, sz = o.quantize_act_blocks(o.swiglu_bf16(np.zeros((1, 32)), u[:1, :32]), T[:1], clip[:1])
    assert np.all(cz == 0) and np.all(sz == 0)
