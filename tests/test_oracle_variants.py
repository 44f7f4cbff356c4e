"""Pins for the oracle's other transform forms and the two-ratio clipping of Eq. 3-4.

Each pin fixes the function to something other than itself: numpy.kron, the existing
Global-and-Private / private-outer builders, hand-computed blocks (tests/golden/), an exact
scalar re-derivation, and identities of the mathematics.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import batq_oracle as o
from conftest import golden_lines


def _rand_factor(rng, g, nb=None, eps=0.1):
    shape = (g, g) if nb is None else (nb, g, g)
    return np.eye(g) + eps * rng.standard_normal(shape)


@pytest.mark.parametrize("go,gi", [(4, 8), (8, 4), (2, 16)])
def test_general_kron_is_numpy_kron_per_block(go, gi):
    rng = np.random.default_rng(go)
    nb = 5
    O, I = _rand_factor(rng, go, nb), _rand_factor(rng, gi, nb)
    T = o.kron_blocks_general(O, I, nb)
    for k in range(nb):
        assert np.array_equal(T[k], np.kron(O[k], I[k]))
    Ts = o.kron_blocks_general(O[0], I, nb)
    for k in range(nb):
        assert np.array_equal(Ts[k], np.kron(O[0], I[k]))


def test_general_kron_reduces_to_the_two_named_forms():
    rng = np.random.default_rng(3)
    nb = 4
    G, P = _rand_factor(rng, 4), _rand_factor(rng, 8, nb)
    assert np.array_equal(o.kron_blocks_general(G, P, nb), o.kron_blocks(G, P))
    B, A = _rand_factor(rng, 4, nb), _rand_factor(rng, 8)
    assert np.array_equal(o.kron_blocks_general(B, A, nb), o.kron_blocks_private_outer(B, A))


def test_kron_forms_act_as_the_vec_identity():
    # x_k (O (x) I) = vec(O^T V I), V = reshape(x_k, go, gi) row-major (Sec. 3.1.1)
    rng = np.random.default_rng(4)
    nb = 3
    O, I = _rand_factor(rng, 8, nb), _rand_factor(rng, 4, nb)
    X = rng.standard_normal((6, 32 * nb))
    Y = o.apply_blocks(X, o.kron_blocks_general(O, I, nb))
    for k in range(nb):
        V = X[:, 32 * k:32 * k + 32].reshape(6, 8, 4)
        ref = np.einsum("ab,mac,cd->mbd", O[k], V, I[k]).reshape(6, 32)
        assert np.allclose(Y[:, 32 * k:32 * k + 32], ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("form", ["paper_order", "naive", "dense"])
def test_transform_then_inverse_leaves_the_layer_unchanged(form):
    # (X T)(T^-1 W) = X W for every form, before quantisation (Sec. 3.1 objective)
    rng = np.random.default_rng(5)
    nb, M, N = 4, 7, 9
    if form == "paper_order":
        T = o.kron_blocks_general(_rand_factor(rng, 4, nb), _rand_factor(rng, 8), nb)
    elif form == "naive":
        T = o.kron_blocks_general(_rand_factor(rng, 4, nb), _rand_factor(rng, 8, nb), nb)
    else:
        T = np.eye(32)[None] + 0.05 * rng.standard_normal((nb, 32, 32))
    X = rng.standard_normal((M, 32 * nb))
    W = rng.standard_normal((32 * nb, N))
    Xt = o.apply_blocks(X, T)
    Wt = np.concatenate([o.invert(T[k]) @ W[32 * k:32 * k + 32] for k in range(nb)])
    assert np.allclose(Xt @ Wt, X @ W, rtol=0, atol=1e-11)


def _block(vals):
    x = np.zeros(32, dtype=np.float32)
    x[:len(vals)] = np.asarray(vals, dtype=np.float32)
    return x[None, :]


@pytest.mark.parametrize("line", golden_lines("hand_blocks_minmax.txt"))
def test_hand_computed_minmax_blocks(line):
    name, rmin, rmax, vals, scale, codes = [f.strip() for f in line.split("|")]
    x = _block([float(v) for v in vals.split(",")])
    pc, ps = o.mxfp4_quantize_minmax(x, np.array([float(rmin)], np.float32), np.array([float(rmax)], np.float32))
    assert ps[0, 0] == int(scale), name
    got = "".join("%X" % c for c in o.unpack_codes(pc)[0])
    assert got == codes, name


def _exact_minmax_block(xs, rmin, rmax):
    """Scalar re-derivation with exact rationals: clamp, amax', exponent by comparison, nearest grid value."""
    lo = float(np.float32(rmin) * np.float32(min(float(v) for v in xs)))
    hi = float(np.float32(rmax) * np.float32(max(float(v) for v in xs)))
    cl = []
    for v in xs:
        v = float(v)
        cl.append(lo if v < lo else (hi if v > hi else v))
    amax = max(abs(v) for v in cl)
    if amax == 0.0:
        E = -127
    else:
        E = math.floor(math.log2(amax))
        while Fraction(2) ** (E + 1) <= Fraction(amax):
            E += 1
        while Fraction(2) ** E > Fraction(amax):
            E -= 1
        E = max(-127, min(127, E - 2))
    grid = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4), Fraction(6)]
    out = []
    for v in cl:
        mag = abs(Fraction(v)) / (Fraction(2) ** E)
        best = None
        for c, gval in enumerate(grid):
            d = abs(mag - gval)
            if best is None or d < best[0] or (d == best[0] and c % 2 == 0):
                best = (d, c)
        out.append(best[1] | (8 if math.copysign(1.0, v) < 0 else 0))
    return out, E + 127


def test_minmax_against_exact_scalar_reference():
    rng = np.random.default_rng(21)
    blocks = [rng.standard_normal(32) * s for s in (1e-3, 1.0, 41.0, 2.0 ** -120, 2.0 ** 90)]
    blocks.append(np.abs(rng.standard_normal(32)) + 0.5)             # all positive
    blocks.append(-np.abs(rng.standard_normal(32)) - 0.5)            # all negative
    blocks.append(np.array([6, -5, 3.5, -2.5, 1.75, -1.25, .75, -.25] * 4))
    x = np.stack(blocks).astype(np.float32)
    for rmin, rmax in ((1.0, 1.0), (0.9, 0.6), (0.5, 0.95), (0.3, 0.3)):
        pc, ps = o.mxfp4_quantize_minmax(x, np.array([rmin], np.float32), np.array([rmax], np.float32))
        got = o.unpack_codes(pc)
        for r in range(x.shape[0]):
            exp_codes, exp_scale = _exact_minmax_block(x[r], rmin, rmax)
            assert ps[r, 0] == exp_scale, (r, rmin, rmax)
            assert list(got[r]) == exp_codes, (r, rmin, rmax)


def test_minmax_with_unit_ratios_is_the_unclipped_quantiser():
    rng = np.random.default_rng(22)
    x = (rng.standard_normal((40, 96)) * np.exp(rng.standard_normal((40, 1)) * 3)).astype(np.float32)
    x[3, :32] = 0.0
    x[4, 5] = -0.0
    one = np.ones(3, np.float32)
    a = o.mxfp4_quantize_minmax(x, one, one)
    b = o.mxfp4_quantize(x, None)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_minmax_on_a_symmetric_block_is_the_symmetric_clip():
    # a block whose minimum is minus its maximum: [r*min, r*max] = [-r*amax, r*amax]
    rng = np.random.default_rng(23)
    h = rng.standard_normal((20, 16)).astype(np.float32)
    x = np.concatenate([h, -h], axis=1)
    r = np.array([0.7], np.float32)
    a = o.mxfp4_quantize_minmax(x, r, r)
    b = o.mxfp4_quantize(x, r)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_minmax_dequantised_range_and_monotonicity():
    rng = np.random.default_rng(24)
    x = (rng.standard_normal((64, 64)) * 3).astype(np.float32)
    rmin, rmax = np.array([0.6, 0.9], np.float32), np.array([0.8, 0.5], np.float32)
    pc, ps = o.mxfp4_quantize_minmax(x, rmin, rmax)
    dq = o.dequantize(pc, ps).reshape(64, 2, 32)
    xb = x.reshape(64, 2, 32)
    lo = (rmin[None] * xb.min(axis=2)).astype(np.float32)
    hi = (rmax[None] * xb.max(axis=2)).astype(np.float32)
    step = np.exp2(ps.astype(np.float64) - 127)                          # largest grid gap is 2 steps of 2^E
    assert np.all(dq >= lo[:, :, None] - step[:, :, None]) and np.all(dq <= hi[:, :, None] + step[:, :, None])
    order = np.argsort(xb, axis=2)
    assert np.all(np.diff(np.take_along_axis(dq, order, axis=2), axis=2) >= 0)


def test_blocks_paths_agree_with_the_named_paths():
    rng = np.random.default_rng(25)
    nb = 3
    G, P = _rand_factor(rng, 4, eps=0.05), _rand_factor(rng, 8, nb, eps=0.05)
    clip = rng.uniform(0.8, 1.0, nb).astype(np.float32)
    X = rng.standard_normal((10, 32 * nb)).astype(np.float32)
    W = (0.02 * rng.standard_normal((32 * nb, 12))).astype(np.float32)
    T = o.kron_blocks(G, P)
    a, b = o.quantize_act_blocks(X, T, clip), o.quantize_act(X, G, P, clip)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    a, b = o.prepare_weight_blocks(W, T, clip), o.prepare_weight(W, G, P, clip)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    a, b = o.quantize_act_blocks(X, None), o.quantize_act(X, None, None, None)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
