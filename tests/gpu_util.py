"""Helpers shared by the GPU parity tests (marshalling between NumPy and device tensors)."""
import numpy as np
import pytest


def require_gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.fail("GPU test selected but no GPU is visible")
    return torch


def to_dev(a: np.ndarray, dtype: str):
    """NumPy storage array (fp32, or uint16 bf16 bits) -> device tensor."""
    import torch
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def y_to_f32(Y) -> np.ndarray:
    return Y.float().cpu().numpy()


def unpack(codes: np.ndarray) -> np.ndarray:
    """[R, K/2] packed bytes -> [R, K] nibbles (test-side unpack, independent of both paths)."""
    R, Kh = codes.shape
    out = np.empty((R, 2 * Kh), dtype=np.uint8)
    out[:, 0::2] = codes & 15
    out[:, 1::2] = codes >> 4
    return out


TIE_POINTS = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])


def code_value_mismatch(gc: np.ndarray, oc: np.ndarray) -> np.ndarray:
    """Boolean map of elements whose decoded value differs (+0 and -0 count as equal)."""
    g, o = unpack(gc), unpack(oc)
    gz, oz = (g & 7) == 0, (o & 7) == 0
    return (g != o) & ~(gz & oz)


def sample_rows(M: int, n: int, seed: int = 0) -> np.ndarray:
    """Sorted sample of row indices that always includes the first and last row."""
    if M <= n:
        return np.arange(M)
    rng = np.random.default_rng(seed)
    r = rng.choice(np.arange(1, M - 1), size=n - 2, replace=False)
    return np.sort(np.concatenate([[0, M - 1], r]))


def grouped_to_rowmajor(grouped: np.ndarray, rows: int, nb: int) -> np.ndarray:
    """De-interleave the library's grouped scale order, from the formula the header documents:
    index(row, k) = ((k // 8) * rows + row) * 8 + (k % 8) // 2 + 4 * (k % 2); pad bytes must be 127."""
    groups = (nb + 7) // 8
    assert grouped.size == groups * rows * 8
    k = np.arange(groups * 8)
    idx = ((k // 8)[None, :] * rows + np.arange(rows)[:, None]) * 8 + (k % 8)[None, :] // 2 + 4 * (k % 2)[None, :]
    full = grouped.reshape(-1)[idx]
    assert np.all(full[:, nb:] == 127), "padding scale bytes must be the neutral scale"
    return np.ascontiguousarray(full[:, :nb])


def rowmajor_to_grouped(rm: np.ndarray) -> np.ndarray:
    rows, nb = rm.shape
    groups = (nb + 7) // 8
    out = np.full(groups * rows * 8, 127, dtype=np.uint8)
    k = np.arange(nb)
    idx = ((k // 8)[None, :] * rows + np.arange(rows)[:, None]) * 8 + (k % 8)[None, :] // 2 + 4 * (k % 2)[None, :]
    out[idx] = rm
    return out
