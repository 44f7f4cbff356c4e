"""Pins for the oracle's dequantise + GEMM (the objective of Sec. 3.1) and the input generator."""
import numpy as np
import pytest

from oracle import batq_oracle as o
import batq_inputs as bi


def test_dequantize_known_bytes():
    codes = np.zeros((1, 16), dtype=np.uint8)
    codes[0, 0] = 0x7A            # element 0 = code A (-1.0), element 1 = code 7 (6.0)
    codes[0, 15] = 0x10           # element 31 = code 1 (0.5)
    for s, mul in ((127, 1.0), (130, 8.0), (120, 2.0 ** -7), (0, 2.0 ** -127), (254, 2.0 ** 127)):
        dq = o.dequantize(codes, np.array([[s]], np.uint8))[0]
        assert dq[0] == -1.0 * mul and dq[1] == 6.0 * mul and dq[31] == 0.5 * mul
        assert np.all(dq[2:31] == 0)


def test_gemm_is_dense_matmul_of_dequantised_operands():
    w = bi.make_small(24, 96, 40, seed=1, dtype="f32")
    xc, xs = o.quantize_act(w.X, w.G, w.P, w.clip)
    wc, ws = o.prepare_weight(w.W, w.G, w.P)
    Y = o.gemm(xc, xs, wc, ws)
    assert Y.shape == (24, 40) and Y.dtype == np.float64
    assert np.array_equal(Y, o.dequantize(xc, xs) @ o.dequantize(wc, ws).T)


def test_gemm_brute_force_triple_loop():
    w = bi.make_small(3, 64, 4, seed=2, dtype="f32")
    xc, xs = o.quantize_act(w.X, w.G, w.P, w.clip)
    wc, ws = o.prepare_weight(w.W, w.G, w.P)
    Y = o.gemm(xc, xs, wc, ws)
    grid = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]

    def val(packed, r, j):
        b = int(packed[r, j // 2])
        c = (b >> 4) if (j & 1) else (b & 0xF)
        return -grid[c & 7] if c & 8 else grid[c & 7]

    for m in range(3):
        for n in range(4):
            acc = 0.0
            for k in range(2):
                blk = 0.0
                for j in range(32):
                    blk += val(xc, m, 32 * k + j) * val(wc, n, 32 * k + j)
                acc += blk * 2.0 ** (int(xs[m, k]) - 127) * 2.0 ** (int(ws[n, k]) - 127)
            assert abs(acc - Y[m, n]) <= 1e-14 * max(1.0, abs(acc))


def test_single_block_products_are_exact_small_integers_over_four():
    # every E2M1 product is a multiple of 1/4, so a 32-term block dot is exact in fp32
    rng = np.random.default_rng(4)
    xc = rng.integers(0, 256, size=(8, 16)).astype(np.uint8)
    wc = rng.integers(0, 256, size=(8, 16)).astype(np.uint8)
    one = np.full((8, 1), 127, np.uint8)
    Y = o.gemm(xc, one, wc, one)
    assert np.array_equal(Y * 4, np.round(Y * 4))
    assert np.array_equal(Y.astype(np.float32).astype(np.float64), Y)
    assert np.abs(Y).max() <= 32 * 36


def test_linear_approximates_the_unquantised_layer():
    w = bi.make_workload(0)
    Y = o.linear(w.X, w.W, w.G, w.P, w.clip)
    ref = w.X.astype(np.float64) @ w.W.astype(np.float64)
    rel = np.linalg.norm(Y - ref) / np.linalg.norm(ref)
    assert 0.01 < rel < 0.5          # 4-bit error: far from exact, far from garbage
    # without outliers and clipping the 4-bit layer is within ~15%
    w2 = bi.make_small(64, 256, 64, seed=5, dtype="f32", outliers=False)
    Y2 = o.linear(w2.X, w2.W, w2.G, w2.P, None)
    ref2 = w2.X.astype(np.float64) @ w2.W.astype(np.float64)
    assert np.linalg.norm(Y2 - ref2) / np.linalg.norm(ref2) < 0.2


# ----------------------------------------------------------------------------- input generator
def test_generator_bf16_conversion_against_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(50000) * 2.0 ** rng.integers(-20, 20, 50000)).astype(np.float32)
    bits = bi.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    assert np.array_equal(bi.bf16_bits_to_f32(bits), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


@pytest.mark.parametrize("cfg", [0, 1])
def test_generator_shapes_and_determinism(cfg):
    a = bi.make_workload(cfg)
    b = bi.make_workload(cfg)
    name, M, K, N, dt, odt = bi.config_shape(cfg)
    assert a.X.shape == (M, K) and a.W.shape == (K, N)
    assert a.G.shape == (4, 4) and a.P.shape == (K // 32, 8, 8) and a.clip.shape == (K // 32,)
    assert a.X.dtype == (np.uint16 if dt == "bf16" else np.float32)
    assert np.array_equal(a.X, b.X) and np.array_equal(a.W, b.W) and np.array_equal(a.P, b.P)
    assert np.all((a.clip > 0.8) & (a.clip <= 1.0))
    X = a.X_f32()
    ch = a.meta["outlier_channels"]
    assert len(ch) == round({0: 0.02, 1: 0.01}[cfg] * K)
    rest = np.setdiff1d(np.arange(K), ch)
    assert X[:, ch].std() > 8 * X[:, rest].std()


def test_generator_large_config_slices():
    for cfg, rows in ((2, 8), (3, 8), (4, 8)):
        w = bi.make_workload(cfg, rows=rows, with_weight=False)
        name, M, K, N, dt, odt = bi.config_shape(cfg)
        assert w.X.shape == (rows, K) and w.W is None and w.X.dtype == np.uint16
        assert np.all(np.isfinite(w.X_f32()))
