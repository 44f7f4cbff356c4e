"""Pins for the oracle's MXFP4 quantiser (Sec. 2 MXFP definition; Eq. 3-4 clipping).

Each test checks the oracle against something other than itself: values the
paper prints, hand-computed blocks (tests/golden/), exact-arithmetic brute
force, and invariants of the format.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import batq_oracle as o

from conftest import golden_lines


def _block(vals):
    x = np.zeros(32, dtype=np.float32)
    x[:len(vals)] = np.asarray(vals, dtype=np.float32)
    return x[None, :]


def test_grid_is_the_papers():
    printed = [float(v) for v in golden_lines("e2m1_grid.txt")]
    assert list(o.E2M1_GRID[1:]) == printed
    assert o.E2M1_GRID[0] == 0.0 and len(o.E2M1_GRID) == 8


def test_bit_layout_sign_exponent_mantissa():
    # 1 sign, 2 exponent, 1 mantissa bit (Sec. 2): value = (-1)^S * 2^(e-1) * (1 + m/2), e>0;
    # e == 0 is subnormal: m * 0.5
    for code in range(16):
        s, e, m = code >> 3, (code >> 1) & 3, code & 1
        mag = m * 0.5 if e == 0 else 2.0 ** (e - 1) * (1 + m / 2)
        assert o.E2M1_GRID[code & 7] == mag
        packed = np.array([[code]], dtype=np.uint8)          # low nibble = element 0, high = 0
        dq = o.dequantize(np.repeat(packed, 16, axis=1), np.array([[127]], np.uint8))
        assert dq[0, 0] == (-mag if s else mag)
        assert math.copysign(1.0, dq[0, 0]) == (-1.0 if s else 1.0)


def test_all_sixteen_codes_round_trip():
    vals = np.concatenate([o.E2M1_GRID, -o.E2M1_GRID])
    x = np.concatenate([vals, vals]).astype(np.float32)[None]
    codes, scales = o.mxfp4_quantize(x)
    assert scales[0, 0] == 127                                # amax 6 -> E = 0
    got = o.unpack_codes(codes)[0]
    assert list(got) == list(range(16)) * 2
    assert np.array_equal(o.dequantize(codes, scales)[0], x[0].astype(np.float64))


@pytest.mark.parametrize("line", golden_lines("hand_blocks.txt"))
def test_hand_computed_blocks(line):
    name, clip, vals, scale, codes = [f.strip() for f in line.split("|")]
    x = _block([float(v) for v in vals.split(",")])
    pc, ps = o.mxfp4_quantize(x, np.array([float(clip)], dtype=np.float32))
    assert ps[0, 0] == int(scale), name
    got = "".join("%X" % c for c in o.unpack_codes(pc)[0])
    assert got == codes, name


def test_tie_table():
    # exact midpoints of neighbouring grid values go to the neighbour with the even code
    ties = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    for sgn in (1.0, -1.0):
        x = _block([6.0] + [sgn * t for t in ties])
        pc, ps = o.mxfp4_quantize(x)
        dq = o.dequantize(pc, ps)[0]
        assert list(dq[1:1 + len(ties)]) == [sgn * v for v in ties.values()]


def test_nibble_order_and_scale_layout():
    x = np.zeros((2, 64), dtype=np.float32)
    x[0, 0], x[0, 1] = 6.0, -1.0          # block 0: codes 7, 0xA
    x[1, 32 + 5] = 3.0                    # row 1, block 1, element 5 -> top code... amax 3 -> E=-1 -> 6.0 -> 7
    pc, ps = o.mxfp4_quantize(x)
    assert pc.shape == (2, 32) and ps.shape == (2, 2)
    assert pc[0, 0] == (0xA << 4) | 7
    assert pc[1, 16 + 2] == (7 << 4)      # element 37 is odd -> high nibble of byte 18
    assert list(ps[0]) == [127, 0] and list(ps[1]) == [0, 126]


def _exact_reference_block(xs, clip):
    """Exact-arithmetic (Fractions) scalar quantiser of one block, searching all 8 magnitudes."""
    amax = max(abs(float(v)) for v in xs)
    bound = float(np.float32(clip) * np.float32(amax))
    if bound == 0.0:
        E = -127
    else:
        E = math.floor(math.log2(bound))
        # guard the float log against boundary error with exact comparisons
        while Fraction(2) ** (E + 1) <= Fraction(bound):
            E += 1
        while Fraction(2) ** E > Fraction(bound):
            E -= 1
        E = max(-127, min(127, E - 2))
    grid = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4), Fraction(6)]
    out = []
    for v in xs:
        f = Fraction(float(v))
        neg = math.copysign(1.0, float(v)) < 0
        mag = min(abs(f), Fraction(bound)) / (Fraction(2) ** E)
        best = None
        for c, gval in enumerate(grid):
            d = abs(mag - gval)
            if best is None or d < best[0] or (d == best[0] and c % 2 == 0):
                best = (d, c)
        out.append(best[1] | (8 if neg else 0))
    return out, E + 127


def test_against_exact_fraction_brute_force():
    rng = np.random.default_rng(11)
    blocks = []
    for scale in (1e-3, 1.0, 37.0, 2.0 ** -130, 2.0 ** 100):
        blocks.append(rng.standard_normal(32) * scale)
    # values sitting exactly on ties and grid points at several scales
    blocks.append(np.array([6, 5, 3.5, 2.5, 1.75, 1.25, .75, .25] * 4) * 2.0 ** -7)
    blocks.append(np.array([7.5, -5, 3.5, -2.5, 1.75, -1.25, .75, -.25] * 4) * 2.0 ** 9)
    x = np.stack(blocks).astype(np.float32)
    for clip in (1.0, 0.9, 0.5):
        pc, ps = o.mxfp4_quantize(x, np.array([clip], np.float32))
        got = o.unpack_codes(pc)
        for r in range(x.shape[0]):
            exp_codes, exp_scale = _exact_reference_block(x[r], clip)
            assert ps[r, 0] == exp_scale
            assert list(got[r]) == exp_codes


def test_shared_exponent_against_math_log2():
    rng = np.random.default_rng(5)
    a = np.concatenate([2.0 ** rng.uniform(-120, 120, 2000), 2.0 ** np.arange(-126, 127.0)]).astype(np.float32)
    E = o.shared_exponent(a)
    for ai, Ei in zip(a, E):
        m, e = math.frexp(float(ai))
        assert Ei == max(-127, min(127, (e - 1) - 2))
        assert 2.0 ** (Ei + 2) <= float(ai) < 2.0 ** (Ei + 3) or Ei == -127
    assert o.shared_exponent(np.array([0.0]))[0] == -127
    # fp32 subnormal bound: true exponent below the E8M0 range -> clamped
    assert o.shared_exponent(np.array([1e-40], np.float32))[0] == -127
    # exponent field view: for normal fp32, floor(log2 a) = field - 127
    bits = a.view(np.uint32)
    field = ((bits >> 23) & 0xFF).astype(np.int64)
    assert np.array_equal(np.clip(field - 127 - 2, -127, 127), E)


def test_invariants_on_random_blocks():
    rng = np.random.default_rng(3)
    x = (rng.standard_t(3, size=(400, 256)) * 2.0 ** rng.integers(-20, 20, size=(400, 1))).astype(np.float32)
    clip = rng.uniform(0.5, 1.0, size=8).astype(np.float32)
    for c in (None, clip):
        pc, ps = o.mxfp4_quantize(x, c)
        codes = o.unpack_codes(pc).reshape(400, 8, 32)
        Xc, bound = o.clip_blocks(x, c)
        E = ps.astype(np.int64) - 127
        # the clipped bound lands in [4, 8) grid units; the top magnitude code is 6 or 7
        ratio = bound / np.exp2(E)
        assert np.all((ratio >= 4) & (ratio < 8))
        top = (codes & 7).max(axis=2)
        assert np.all((top == 6) | (top == 7))
        # error bound: half a grid step for in-range values, at most 2 units when saturated
        dq = o.dequantize(pc, ps).reshape(400, 8, 32)
        v = np.abs(Xc.astype(np.float64)) / np.exp2(E)[:, :, None]
        err = np.abs(np.abs(dq) / np.exp2(E)[:, :, None] - v)
        half_step = np.where(v < 2, 0.25, np.where(v < 4, 0.5, 1.0))
        assert np.all(err[v <= 6] <= half_step[v <= 6])
        assert np.all(err[v > 6] < 2.0)
        # signs preserved
        assert np.array_equal((codes >> 3).astype(bool), np.signbit(x.reshape(400, 8, 32)))
        # monotone: larger |x| never gets a smaller magnitude code within a block
        order = np.argsort(v, axis=2)
        sorted_codes = np.take_along_axis(codes & 7, order, axis=2)
        assert np.all(np.diff(sorted_codes.astype(np.int64), axis=2) >= 0)


def test_idempotent_on_dequantised_values():
    rng = np.random.default_rng(9)
    x = (rng.standard_normal((64, 128)) * 5).astype(np.float32)
    pc, ps = o.mxfp4_quantize(x)
    dq = o.dequantize(pc, ps).astype(np.float32)
    pc2, ps2 = o.mxfp4_quantize(dq)
    # quantised values are representable, so a second pass changes nothing unless the top
    # element rounded down a binade (top code 4.0 -> amax 4*2^E keeps E) -- it never moves
    assert np.array_equal(pc, pc2) and np.array_equal(ps, ps2)


def test_clip_properties():
    rng = np.random.default_rng(21)
    x = (rng.standard_normal((50, 96)) * 3).astype(np.float32)
    p1, s1 = o.mxfp4_quantize(x, None)
    p2, s2 = o.mxfp4_quantize(x, np.ones(3, np.float32))
    assert np.array_equal(p1, p2) and np.array_equal(s1, s2)          # ratio 1 == no clip
    prev = s1.astype(np.int64)
    for c in (0.95, 0.8, 0.6, 0.4):
        pc, ps = o.mxfp4_quantize(x, np.full(3, c, np.float32))
        assert np.all(ps.astype(np.int64) <= prev)                     # scale non-increasing in c
        prev = ps.astype(np.int64)
        Xc, bound = o.clip_blocks(x, np.full(3, c, np.float32))
        amax = np.abs(x.reshape(50, 3, 32)).max(axis=2)
        assert np.array_equal(bound, (np.float32(c) * amax).astype(np.float32))
        assert np.array_equal(np.abs(Xc).max(axis=2), bound)           # clipped amax = ratio * amax
        # every element beyond the bound carries the block's top code
        codes = o.unpack_codes(pc).reshape(50, 3, 32) & 7
        over = np.abs(x.reshape(50, 3, 32)) > bound[:, :, None]
        top = codes.max(axis=2, keepdims=True)
        assert np.all(np.where(over, codes == top, True))


def test_clamp_differs_from_saturation():
    # bound/2^E = 4.2 and an outlier at 5.5 units: clamping first gives 4, saturation alone gives 6
    x = _block([8.4, 5.5, 1.0])
    pc, ps = o.mxfp4_quantize(x, np.array([0.5], np.float32))          # bound 4.2 -> E = 0
    assert ps[0, 0] == 127
    assert list(o.unpack_codes(pc)[0][:3]) == [6, 6, 2]


def test_minmax_clip_as_printed():
    # Eq. 3-4: lower bound ratio*min, upper bound ratio*max, applied separately
    x = _block([4.0, -2.0, 1.0, -0.5])
    y = o.clip_blocks_minmax(x, np.array([0.5], np.float32), np.array([0.75], np.float32))[0, 0]
    assert list(y[:4]) == [3.0, -1.0, 1.0, -0.5]
    # with ratio 1 on both sides nothing changes
    z = o.clip_blocks_minmax(x, np.ones(1, np.float32), np.ones(1, np.float32))[0, 0]
    assert np.array_equal(z, x[0])
    # for a block symmetric about zero the two-ratio form with equal ratios equals the amax form
    xs = _block([3.0, -3.0, 2.9, -1.0, 0.3])
    a, _ = o.clip_blocks(xs, np.array([0.8], np.float32))
    b = o.clip_blocks_minmax(xs, np.array([0.8], np.float32), np.array([0.8], np.float32))
    assert np.array_equal(a, b)


def test_pack_unpack_inverse():
    rng = np.random.default_rng(0)
    codes = rng.integers(0, 16, size=(7, 3, 32)).astype(np.uint8)
    assert np.array_equal(o.unpack_codes(o.pack_codes(codes)), codes.reshape(7, 96))


def test_bf16_round_against_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.standard_normal(20000) * 2.0 ** rng.integers(-30, 30, 20000),
                        # exact ties between bf16 neighbours
                        (np.arange(1, 2001) * 2 + 1) * 2.0 ** -8 * 2.0 ** rng.integers(-10, 10, 2000)]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(o.bf16_round(x), ref)
    # from fp64: a value just above an fp32-representable bf16 tie must round up, not to even
    tie = 1.0 + 2.0 ** -8                        # midpoint of bf16 neighbours 1.0 and 1.0078125
    assert o.bf16_round(np.array([tie]))[0] == 1.0
    assert o.bf16_round(np.array([tie + 2.0 ** -40]))[0] == np.float32(1.0078125)
    assert o.bf16_round(np.array([-(tie + 2.0 ** -40)]))[0] == np.float32(-1.0078125)
