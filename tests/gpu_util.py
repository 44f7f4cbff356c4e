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


def _chunk_offsets(rows: int, nb: int) -> np.ndarray:
    """Byte offset of the 16-byte chunk of block k of each row in the library's device code order
    (formula from the header): ((row//16)*S + k//4)*1024 + (row%16)*64 + (((k%4) ^ ((row%16)//4))*16)."""
    S = 2 * ((nb + 7) // 8)
    row = np.arange(rows)[:, None]
    k = np.arange(nb)[None, :]
    r = row % 16
    return ((row // 16) * S + k // 4) * 1024 + r * 64 + (((k % 4) ^ ((r // 4) % 4)) * 16)


def blocked_to_rowmajor(blocked: np.ndarray, rows: int, nb: int) -> np.ndarray:
    S = 2 * ((nb + 7) // 8)
    assert blocked.size == ((rows + 31) // 32) * 2 * S * 1024
    off = _chunk_offsets(rows, nb)
    idx = off[:, :, None] + np.arange(16)[None, None, :]
    out = blocked.reshape(-1)[idx].reshape(rows, nb * 16)
    # K padding up to a multiple of 8 blocks must hold zero codes
    nbp = ((nb + 7) // 8) * 8
    if nbp > nb:
        offp = _chunk_offsets_range(rows, nb, nbp)
        assert np.all(blocked.reshape(-1)[offp[:, :, None] + np.arange(16)[None, None, :]] == 0)
    return np.ascontiguousarray(out)


def _chunk_offsets_range(rows, k0, k1):
    S = 2 * ((k1 + 7) // 8)
    row = np.arange(rows)[:, None]
    k = np.arange(k0, k1)[None, :]
    r = row % 16
    return ((row // 16) * S + k // 4) * 1024 + r * 64 + (((k % 4) ^ ((r // 4) % 4)) * 16)


def rowmajor_to_blocked(rm: np.ndarray) -> np.ndarray:
    rows, kh = rm.shape
    nb = kh // 16
    S = 2 * ((nb + 7) // 8)
    out = np.zeros(((rows + 31) // 32) * 2 * S * 1024, dtype=np.uint8)
    off = _chunk_offsets(rows, nb)
    idx = off[:, :, None] + np.arange(16)[None, None, :]
    out[idx.reshape(-1)] = rm.reshape(-1)
    return out


# ---- 8-bit (MXFP8) activation codes: the documented device order, written out in NumPy
def _slot8_offsets(rows, k0, k1, nb_total):
    """byte offset of 16-byte slot h of block k of each row: [rows, k1-k0, 2]"""
    S8 = 4 * ((nb_total + 7) // 8)
    row = np.arange(rows)[:, None, None]
    k = np.arange(k0, k1)[None, :, None]
    h = np.arange(2)[None, None, :]
    r = row % 16
    return ((row // 16) * S8 + k // 2) * 1024 + r * 64 + ((((2 * (k % 2) + h)) ^ ((r // 4) % 4)) * 16)


def blocked8_to_rowmajor(blocked: np.ndarray, rows: int, nb: int) -> np.ndarray:
    S8 = 4 * ((nb + 7) // 8)
    assert blocked.size == ((rows + 31) // 32) * 2 * S8 * 1024
    off = _slot8_offsets(rows, 0, nb, nb)
    idx = off[..., None] + np.arange(16)
    out = blocked.reshape(-1)[idx].reshape(rows, nb * 32)
    nbp = ((nb + 7) // 8) * 8
    if nbp > nb:                                     # K padding must hold zero codes
        offp = _slot8_offsets(rows, nb, nbp, nb)
        assert np.all(blocked.reshape(-1)[offp[..., None] + np.arange(16)] == 0)
    return np.ascontiguousarray(out)


def rowmajor_to_blocked8(rm: np.ndarray) -> np.ndarray:
    rows, K = rm.shape
    nb = K // 32
    S8 = 4 * ((nb + 7) // 8)
    out = np.zeros(((rows + 31) // 32) * 2 * S8 * 1024, dtype=np.uint8)
    off = _slot8_offsets(rows, 0, nb, nb)
    idx = off[..., None] + np.arange(16)
    out[idx.reshape(-1)] = rm.reshape(-1)
    return out


def assert_same_quantisation(B, codes_a, scales_a, codes_b, scales_b, rows, K, bits, what=""):
    """Two quantisations of the same rows (device-order arrays laid out for `rows` rows) must agree in every code
    and scale byte: a row's codes do not depend on the batch it arrives in or on the kernel that serves it."""
    import torch
    to_rm = B.batq_codes8_to_rowmajor if bits == 8 else B.batq_codes_to_rowmajor
    ca, cb = to_rm(codes_a, rows, K), to_rm(codes_b, rows, K)
    sa, sb = B.batq_scales_to_rowmajor(scales_a, rows, K), B.batq_scales_to_rowmajor(scales_b, rows, K)
    assert torch.equal(sa, sb), what
    assert torch.equal(ca, cb), what
