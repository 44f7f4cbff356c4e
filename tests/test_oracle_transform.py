"""Pins for the oracle's block-wise affine transform and weight preparation.

Eq. 1 (block-diagonal P), Eq. 2 (Kronecker factors), the vec identity of
Sec. 3.1.1, the objective's invariance (X P)(P^-1 W) = X W, Alg. 1's shapes,
Table 1's counts, and special transforms whose result is known in closed form.
"""
import numpy as np
import pytest

from oracle import batq_oracle as o
import batq_inputs as bi

from conftest import golden_lines


def _factors(nb, seed=0, go=4, gi=8, eps=0.3):
    rng = np.random.default_rng(seed)
    G = np.eye(go) + eps * rng.standard_normal((go, go))
    P = np.eye(gi)[None] + eps * rng.standard_normal((nb, gi, gi))
    return G, P


def test_kron_blocks_is_numpy_kron():
    G, P = _factors(5, seed=1)
    T = o.kron_blocks(G, P)
    for k in range(5):
        assert np.array_equal(T[k], np.kron(G, P[k]))
    # the other split that Sec. 4.3 finds near-optimal (global 8x8 would be g_outer=8)
    G8, P4 = _factors(3, seed=2, go=8, gi=4)
    T = o.kron_blocks(G8, P4)
    for k in range(3):
        assert np.array_equal(T[k], np.kron(G8, P4[k]))


def test_vec_identity_two_step_route():
    # x kron(G, P) == vec(G^T V P) with V = reshape(x, 4, 8) row-major: the route a
    # register-level implementation takes, checked against the dense block
    G, P = _factors(1, seed=3)
    rng = np.random.default_rng(4)
    x = rng.standard_normal(32)
    dense = x @ o.kron_blocks(G, P)[0]
    V = x.reshape(4, 8)
    two_step = (G.T @ V @ P[0]).reshape(32)
    assert np.allclose(dense, two_step, rtol=0, atol=1e-13)
    # transposing either factor must break it (guards the index convention)
    assert not np.allclose(dense, (G @ V @ P[0]).reshape(32), atol=1e-6)
    assert not np.allclose(dense, (G.T @ V @ P[0].T).reshape(32), atol=1e-6)


def test_paper_order_identity_and_algorithm_1():
    # Sec. 3.1.1: vec(V)(B (x) A) = vec(B^T V A), V in R^{g2 x g1}
    rng = np.random.default_rng(6)
    g1, g2, nb = 8, 4, 3
    A = np.eye(g1) + 0.3 * rng.standard_normal((g1, g1))
    B = np.eye(g2)[None] + 0.3 * rng.standard_normal((nb, g2, g2))
    T = o.kron_blocks_private_outer(B, A)
    x = rng.standard_normal((5, nb * 32))
    y = o.apply_blocks(x, T)
    for k in range(nb):
        assert np.array_equal(T[k], np.kron(B[k], A))
        V = x[:, 32 * k:32 * k + 32].reshape(5, g2, g1)
        ident = np.einsum("ji,bjk,kl->bil", B[k], V, A).reshape(5, 32)      # B^T V A
        assert np.allclose(y[:, 32 * k:32 * k + 32], ident, atol=1e-12)
    # Alg. 1 (reshape to [-1, k, g2, g1], right-multiply by A, left-multiply by B_i) realises
    # B_i V A, i.e. the Kronecker product with B_i transposed
    Xr = x.reshape(5, nb, g2, g1)
    step1 = np.einsum("bgij,jk->bgik", Xr, A)
    step2 = np.einsum("gij,bgjk->bgik", B, step1).reshape(5, nb * 32)
    Tt = o.kron_blocks_private_outer(np.transpose(B, (0, 2, 1)), A)
    assert np.allclose(step2, o.apply_blocks(x, Tt), atol=1e-12)


def test_apply_blocks_is_block_diagonal_matmul():
    G, P = _factors(4, seed=8)
    T = o.kron_blocks(G, P)
    rng = np.random.default_rng(9)
    X = rng.standard_normal((6, 128))
    Pfull = np.zeros((128, 128))
    for k in range(4):
        Pfull[32 * k:32 * k + 32, 32 * k:32 * k + 32] = T[k]          # Eq. 1
    assert np.allclose(o.apply_blocks(X, T), X @ Pfull, atol=1e-12)
    # scalar loops on one row
    y = np.zeros(128)
    for k in range(4):
        for j2 in range(32):
            y[32 * k + j2] = sum(X[0, 32 * k + j] * T[k, j, j2] for j in range(32))
    assert np.allclose(o.apply_blocks(X, T)[0], y, atol=1e-12)


def test_invariance_before_quantisation():
    # (X P)(P^-1 W) = X W in fp64 (the objective of Sec. 3.1 with Q = identity)
    w = bi.make_workload(0)
    X = w.X.astype(np.float64)
    W = w.W.astype(np.float64)
    XT = o.apply_blocks(X, o.kron_blocks(w.G, w.P))
    Wt = o.inverse_transform_weight(W, w.G, w.P)
    ref = X @ W
    assert np.linalg.norm(XT @ Wt - ref) / np.linalg.norm(ref) < 1e-12


def test_invert_against_library_and_kron_of_inverses():
    G, P = _factors(3, seed=12)
    T = o.kron_blocks(G, P)
    for k in range(3):
        inv = o.invert(T[k])
        assert np.allclose(inv, np.linalg.inv(T[k]), rtol=1e-10, atol=1e-12)
        assert np.allclose(inv, np.kron(np.linalg.inv(G), np.linalg.inv(P[k])), rtol=1e-10, atol=1e-12)
        assert np.allclose(inv @ T[k], np.eye(32), atol=1e-12)
    # needs pivoting: zero on the diagonal
    Z = np.array([[0.0, 2.0], [1.0, 0.0]])
    assert np.allclose(o.invert(Z), np.array([[0.0, 1.0], [0.5, 0.0]]))
    with pytest.raises(np.linalg.LinAlgError):
        o.invert(np.ones((3, 3)))


def test_identity_transform_is_plain_rtn():
    w = bi.make_workload(0)
    I4, I8 = np.eye(4, dtype=np.float32), np.tile(np.eye(8, dtype=np.float32), (w.nb, 1, 1))
    a = o.quantize_act(w.X, I4, I8, w.clip)
    b = o.quantize_act(w.X, None, None, w.clip)
    c = o.mxfp4_quantize(w.X, w.clip)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1])


def test_permutation_transform_permutes_codes():
    w = bi.make_workload(0)
    rng = np.random.default_rng(17)
    pg = rng.permutation(4)
    G = np.eye(4)[pg]                                         # G[a, a2] = 1 iff a2 == pg[a]... row a has 1 at col pg[a]
    P = np.stack([np.eye(8)[rng.permutation(8)] for _ in range(w.nb)])
    codes0 = o.unpack_codes(o.quantize_act(w.X, None, None, None)[0]).reshape(w.M, w.nb, 32)
    pc, ps = o.quantize_act(w.X, G.astype(np.float32), P.astype(np.float32), None)
    codes1 = o.unpack_codes(pc).reshape(w.M, w.nb, 32)
    assert np.array_equal(ps, o.quantize_act(w.X, None, None, None)[1])
    for k in range(w.nb):
        T = np.kron(G, P[k])                                  # y[j2] = x[j] where T[j, j2] = 1
        src = np.argmax(T, axis=0)                            # for each output j2, the input j
        assert np.array_equal(codes1[:, k, :], codes0[:, k, src])


def test_power_of_two_transform_shifts_scale_only():
    w = bi.make_workload(0)
    base_c, base_s = o.quantize_act(w.X, None, None, w.clip)
    for p in (-3, 5):
        G = np.eye(4, dtype=np.float32) * np.float32(2.0 ** p)
        P = np.tile(np.eye(8, dtype=np.float32), (w.nb, 1, 1))
        c, s = o.quantize_act(w.X, G, P, w.clip)
        assert np.array_equal(c, base_c)
        assert np.array_equal(s.astype(np.int64), base_s.astype(np.int64) + p)


def test_block_hadamard_special_case():
    # block rotation: H32 = H4 (x) H8, orthogonal, inverse = transpose, norm preserved
    H2 = np.array([[1.0, 1.0], [1.0, -1.0]])
    H4 = np.kron(H2, H2) / 2.0
    H8 = np.kron(H2, np.kron(H2, H2)) / np.sqrt(8.0)
    nb = 4
    T = o.kron_blocks(H4, np.tile(H8, (nb, 1, 1)))
    for k in range(nb):
        assert np.allclose(T[k] @ T[k].T, np.eye(32), atol=1e-14)
        assert np.allclose(o.invert(T[k]), T[k].T, atol=1e-13)
    rng = np.random.default_rng(31)
    X = rng.standard_normal((9, 32 * nb))
    Y = o.apply_blocks(X, T)
    assert np.allclose(np.linalg.norm(Y.reshape(9, nb, 32), axis=2),
                       np.linalg.norm(X.reshape(9, nb, 32), axis=2), rtol=1e-13)
    # a one-hot block becomes a flat +-1/sqrt(32) block (the bimodal effect Sec. 2 describes)
    e = np.zeros((1, 32 * nb))
    e[0, 5] = 1.0
    assert np.allclose(np.abs(o.apply_blocks(e, T)[0, :32]), 1 / np.sqrt(32.0))


def test_prepare_weight_matches_definition_on_tiny_case():
    w = bi.make_small(4, 64, 5, seed=3, dtype="f32")
    wc, ws = o.prepare_weight(w.W, w.G, w.P, None)
    assert wc.shape == (5, 32) and ws.shape == (5, 2)
    # definition by hand: W~ = blockdiag(T_k)^-1 W, quantised along K per output column
    Pfull = np.zeros((64, 64))
    for k in range(2):
        Pfull[32 * k:32 * k + 32, 32 * k:32 * k + 32] = np.kron(w.G.astype(np.float64), w.P[k].astype(np.float64))
    Wt = np.linalg.solve(Pfull, w.W.astype(np.float64)).astype(np.float32)
    ec, es = o.mxfp4_quantize(np.ascontiguousarray(Wt.T), None)
    # solve and explicit inverse may differ in the last fp64 bit -> compare through values
    assert np.array_equal(ws, es)
    assert np.mean(wc != ec) < 0.01
    # weight clip ratios act per K-block
    cw = np.array([0.7, 1.0], np.float32)
    wc2, ws2 = o.prepare_weight(w.W, w.G, w.P, cw)
    assert np.array_equal(wc2[:, 16:], wc[:, 16:]) and np.array_equal(ws2[:, 1], ws[:, 1])
    assert np.all(ws2[:, 0] <= ws[:, 0])


def test_table1_parameter_counts():
    for line in golden_lines("table1_param_counts.txt"):
        method, count = line.split()
        assert o.param_count(4096, 32, 8, 4, method) == int(count)
    gpk = o.param_count(4096, 32, 8, 4, "gpk")
    assert 1 - gpk / o.param_count(4096, 32, 8, 4, "flatquant") > 0.74      # Sec. 3.1.1 claims
    assert 1 - gpk / o.param_count(4096, 32, 8, 4, "naive_kron") > 0.79
    # the split used by the benchmark workloads: global 4x4, private 8x8
    assert o.param_count(4096, 32, 4, 8, "gpk") == 16 + 128 * 64


def test_transform_rounds_once_to_fp32():
    w = bi.make_workload(0)
    Xt = o.transform(w.X, w.G, w.P)
    assert Xt.dtype == np.float32
    exact = o.apply_blocks(w.X, o.kron_blocks(w.G, w.P))
    assert np.array_equal(Xt, exact.astype(np.float32))
    assert np.max(np.abs(Xt - exact) / np.maximum(np.abs(exact), 1e-30)) <= 2.0 ** -24
