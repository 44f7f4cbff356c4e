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
