"""Pins for the oracle's MXFP8 (E4M3) activation quantiser and the mixed 8-bit x 4-bit product."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import batq_oracle as o
from conftest import golden_lines


def test_e4m3_values_from_the_bit_fields():
    # 1 sign, 4 exponent (bias 7), 3 mantissa bits; subnormals m/8 * 2^-6; largest finite 448
    vals = o.e4m3_value(np.arange(256))
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        if (c & 0x7F) == 0x7F:
            assert math.isnan(vals[c])
            continue
        mag = Fraction(m, 8) * Fraction(1, 64) if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)
        assert Fraction(float(vals[c])) == (-mag if s else mag)
    assert vals[0x7E] == 448.0 and vals[0x01] == 2.0 ** -9 and vals[0x08] == 2.0 ** -6
    finite = vals[:127]
    assert np.all(np.diff(finite) > 0)


def test_every_code_round_trips():
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    pad = (-codes.size) % 32
    x = o.e4m3_value(np.concatenate([codes, np.zeros(pad, np.uint8)])).astype(np.float32)
    x = x.reshape(-1, 32)
    x[:, 0] = np.where(np.abs(x).max(axis=1) < 256, 448.0, x[:, 0])      # pin every block's exponent to 0
    c, s = o.mxfp8_quantize(x)
    assert np.all(s == 127)
    assert np.array_equal(o.dequantize_fp8(c, s), x.astype(np.float64))
    assert np.array_equal(np.signbit(o.dequantize_fp8(c, s)), np.signbit(x))


def _block(vals):
    x = np.zeros(32, dtype=np.float32)
    x[:len(vals)] = np.asarray(vals, dtype=np.float32)
    return x[None, :]


@pytest.mark.parametrize("line", golden_lines("hand_blocks_fp8.txt"))
def test_hand_computed_fp8_blocks(line):
    name, clip, vals, scale, codes = [f.strip() for f in line.split("|")]
    vals = [float(v) for v in vals.split(",")]
    c, s = o.mxfp8_quantize(_block(vals), np.array([float(clip)], np.float32))
    assert s[0, 0] == int(scale), name
    exp = [int(h, 16) for h in codes.split()]
    assert list(c[0, :len(exp)]) == exp, (name, [hex(v) for v in c[0, :len(exp)]])
    assert np.all((c[0, len(exp):] & 0x7F) == 0), name


def _exact_block(xs, clip):
    amax = max(abs(float(v)) for v in xs)
    bound = float(np.float32(clip) * np.float32(amax))
    if bound == 0.0:
        E = -127
    else:
        E = math.floor(math.log2(bound))
        while Fraction(2) ** (E + 1) <= Fraction(bound):
            E += 1
        while Fraction(2) ** E > Fraction(bound):
            E -= 1
        E = max(-127, min(127, E - 8))
    grid = []
    for c in range(127):
        e, m = c >> 3, c & 7
        grid.append(Fraction(m, 8) * Fraction(1, 64) if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7))
    out = []
    for v in xs:
        neg = math.copysign(1.0, float(v)) < 0
        mag = min(abs(Fraction(float(v))), Fraction(bound)) / (Fraction(2) ** E)
        best = None
        for c, gval in enumerate(grid):
            d = abs(mag - gval)
            if best is None or d < best[0] or (d == best[0] and c % 2 == 0 and best[1] % 2 == 1):
                best = (d, c)
        out.append(best[1] | (0x80 if neg else 0))
    return out, E + 127


def test_against_exact_fraction_brute_force():
    rng = np.random.default_rng(31)
    blocks = [rng.standard_normal(32) * s for s in (1e-3, 1.0, 37.0, 2.0 ** -125, 2.0 ** 100)]
    blocks.append(np.array([448, 464, 240, 17, 1.0625, 2.0 ** -9, 3 * 2.0 ** -10, 2.0 ** -10] * 4))
    blocks.append(-np.array([500, 36, 34, 9.5, 0.3, 0.017, 2.0 ** -7, 2.0 ** -11] * 4) * 2.0 ** 5)
    x = np.stack(blocks).astype(np.float32)
    for clip in (1.0, 0.9, 0.5):
        c, s = o.mxfp8_quantize(x, np.array([clip], np.float32))
        for r in range(x.shape[0]):
            exp_codes, exp_scale = _exact_block(x[r], clip)
            assert s[r, 0] == exp_scale, (r, clip)
            assert list(c[r]) == exp_codes, (r, clip)


def test_invariants_on_random_blocks():
    rng = np.random.default_rng(32)
    x = (rng.standard_normal((200, 128)) * np.exp(rng.standard_normal((200, 1)) * 4)).astype(np.float32)
    c, s = o.mxfp8_quantize(x)
    dq = o.dequantize_fp8(c, s).reshape(200, 4, 32)
    xb = x.reshape(200, 4, 32).astype(np.float64)
    E = s.astype(np.float64) - 127
    amax = np.abs(xb).max(axis=2)
    # the block maximum lands in [256, 512) * 2^E, and never produces the NaN code
    assert np.all((amax >= 256 * np.exp2(E)) & (amax < 512 * np.exp2(E)))
    assert np.all((c & 0x7F) != 0x7F)
    # error: half a grid step (relative 2^-4 for normals) except where values above 448 * 2^E saturate
    sat = np.abs(xb) > 448 * np.exp2(E)[:, :, None]
    err = np.abs(dq - xb)
    step = np.maximum(np.abs(xb) * 2.0 ** -4, np.exp2(E)[:, :, None] * 2.0 ** -10)
    assert np.all(err[~sat] <= step[~sat])
    assert np.all(np.abs(dq[sat]) == np.broadcast_to((448 * np.exp2(E))[:, :, None], dq.shape)[sat])
    assert np.array_equal(np.signbit(dq), np.signbit(xb))
    # idempotent
    c2, s2 = o.mxfp8_quantize(dq.reshape(200, 128).astype(np.float32))
    assert np.array_equal(c2, c) and np.array_equal(s2, s)


def test_fp8_is_finer_than_fp4_on_the_same_blocks():
    rng = np.random.default_rng(33)
    x = rng.standard_normal((64, 256)).astype(np.float32)
    e8 = np.abs(o.dequantize_fp8(*o.mxfp8_quantize(x)) - x).mean()
    e4 = np.abs(o.dequantize(*o.mxfp4_quantize(x)) - x).mean()
    assert e8 < e4 / 4


def test_mixed_gemm_against_triple_loop():
    rng = np.random.default_rng(34)
    M, K, N = 3, 64, 4
    xc, xs = o.mxfp8_quantize(rng.standard_normal((M, K)).astype(np.float32))
    wc, ws = o.mxfp4_quantize(rng.standard_normal((N, K)).astype(np.float32))
    Y = o.gemm_a8w4(xc, xs, wc, ws)
    w4 = o.unpack_codes(wc)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                xv = Fraction(float(o.e4m3_value(xc[m, k]))) * Fraction(2) ** (int(xs[m, k // 32]) - 127)
                wv = Fraction(float(o.E2M1_GRID[w4[n, k] & 7])) * (-1 if w4[n, k] & 8 else 1) * Fraction(2) ** (int(ws[n, k // 32]) - 127)
                acc += xv * wv
            assert abs(float(acc) - Y[m, n]) <= 1e-12 * max(1.0, abs(float(acc)))


def test_quantize_act_fp8_uses_the_transform():
    rng = np.random.default_rng(35)
    nb = 2
    T = np.eye(32)[None] + 0.05 * rng.standard_normal((nb, 32, 32))
    X = rng.standard_normal((5, 64)).astype(np.float32)
    a = o.quantize_act_fp8(X, T)
    b = o.mxfp8_quantize(o.apply_blocks(X, T).astype(np.float32))
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    a = o.quantize_act_fp8(X, None)
    b = o.mxfp8_quantize(X)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
