"""Pins for the oracle pieces behind the key/value-cache placement of the transforms (Sec. 3.2)."""
import numpy as np

from oracle import batq_oracle as o


def _softmax(a):
    a = a - a.max(axis=-1, keepdims=True)
    e = np.exp(a)
    return e / e.sum(axis=-1, keepdims=True)


def test_query_side_companion_keeps_the_scores():
    rng = np.random.default_rng(1)
    heads, hd, nq, nk = 3, 128, 5, 9                      # head_dim 128 = 4 blocks of 32 per head
    nb = heads * hd // 32
    T = np.eye(32)[None] + 0.1 * rng.standard_normal((nb, 32, 32))
    q = rng.standard_normal((nq, heads * hd))
    k = rng.standard_normal((nk, heads * hd))
    qt = o.apply_blocks(q, o.inverse_transpose_blocks(T))
    kt = o.apply_blocks(k, T)
    for h in range(heads):
        sl = slice(h * hd, (h + 1) * hd)
        assert np.allclose(qt[:, sl] @ kt[:, sl].T, q[:, sl] @ k[:, sl].T, rtol=0, atol=1e-11)
    # the plain inverse (not transposed) does not: a transposition mistake is caught
    bad = o.apply_blocks(q, o.inverse_blocks(T))
    assert not np.allclose(bad[:, :hd] @ kt[:, :hd].T, q[:, :hd] @ k[:, :hd].T, atol=1e-3)
    # block by block it is the textbook inverse transpose
    for kblk in (0, nb - 1):
        assert np.allclose(o.inverse_transpose_blocks(T)[kblk], np.linalg.inv(T[kblk]).T, rtol=0, atol=1e-12)
        assert np.allclose(o.inverse_blocks(T)[kblk] @ T[kblk], np.eye(32), rtol=0, atol=1e-12)


def test_value_transform_is_undone_on_the_attention_output():
    rng = np.random.default_rng(2)
    hd, nq, nk = 64, 4, 7
    nb = hd // 32
    Tk = np.eye(32)[None] + 0.1 * rng.standard_normal((nb, 32, 32))
    Tv = np.eye(32)[None] + 0.1 * rng.standard_normal((nb, 32, 32))
    q, k, v = (rng.standard_normal((n, hd)) for n in (nq, nk, nk))
    ref = _softmax(q @ k.T / np.sqrt(hd)) @ v
    qt = o.apply_blocks(q, o.inverse_transpose_blocks(Tk))
    kt = o.apply_blocks(k, Tk)
    vt = o.apply_blocks(v, Tv)
    out = o.apply_blocks(_softmax(qt @ kt.T / np.sqrt(hd)) @ vt, o.inverse_blocks(Tv))
    assert np.allclose(out, ref, rtol=0, atol=1e-11)


def test_quantised_cache_error_is_the_mx_rounding_error():
    # dequantise(quantise(k T)) differs from k T by at most half the largest grid step of the block, or, for the
    # values the shared exponent leaves above the largest code (amax / 2^E in [4, 8) against 6, [256, 512)
    # against 448), by the saturation: 2 grid units for E2M1, 64 for E4M3
    rng = np.random.default_rng(3)
    nb = 4
    T = np.eye(32)[None] + 0.1 * rng.standard_normal((nb, 32, 32))
    k = rng.standard_normal((11, 32 * nb))
    kt = o.apply_blocks(k, T).astype(np.float32)
    c4, s4 = o.mxfp4_quantize(kt, None)
    c8, s8 = o.mxfp8_quantize(kt, None)
    e4 = np.abs(o.dequantize(c4, s4) - kt).reshape(11, nb, 32)
    e8 = np.abs(o.dequantize_fp8(c8, s8) - kt).reshape(11, nb, 32)
    step4 = np.exp2(s4.astype(np.float64) - 127)[:, :, None] * 2
    step8 = np.exp2(s8.astype(np.float64) - 127)[:, :, None] * 64
    unsat4 = np.abs(kt).reshape(11, nb, 32) <= 6 * step4 / 2
    assert np.all(e4[unsat4] <= (step4 / 2 * np.ones_like(e4))[unsat4] * (1 + 1e-12))     # half of the largest step (2)
    assert np.all(e4 <= step4 * (1 + 1e-12)) and np.all(e8 <= step8 * (1 + 1e-12))
    # and the 8-bit cache is several times finer (3 mantissa bits against 1)
    assert np.mean(e8) < np.mean(e4) / 3
