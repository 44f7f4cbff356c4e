"""ctypes binding of libbatq's C ABI (include/batq.h, include/batq_debug.h).

Argument marshalling only: every step of the path runs inside the library's HIP
kernels.  PyTorch tensors are used as device memory; the current torch stream is
passed as the hipStream_t.  There is no CPU fallback: if the library has not
been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbatq.so")

F32, BF16 = 0, 1

STATUS_NAMES = {
    0: "BATQ_OK", 1: "BATQ_ERR_NULL", 2: "BATQ_ERR_SHAPE", 3: "BATQ_ERR_DTYPE", 4: "BATQ_ERR_UNSUPPORTED",
    5: "BATQ_ERR_SINGULAR", 6: "BATQ_ERR_CLIP_RANGE", 7: "BATQ_ERR_WORKSPACE", 8: "BATQ_ERR_ALLOC",
    9: "BATQ_ERR_DEVICE", 10: "BATQ_ERR_MISMATCH",
}

# every symbol the two headers declare: (restype, argtypes)
_vp, _i, _i64, _sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
_fp = C.POINTER(C.c_float)
SYMBOLS = {
    "batq_status_string": (C.c_char_p, [_i]),
    "batq_version": (C.c_char_p, []),
    "batq_transform_create": (_i, [C.POINTER(_vp), _i, _i, _i, _fp, _fp, _fp]),
    "batq_transform_create_ex": (_i, [C.POINTER(_vp), _vp]),
    "batq_transform_destroy": (_i, [_vp]),
    "batq_prepare_weight": (_i, [C.POINTER(_vp), _vp, _vp, _i, _i, _i, _i64, _i, _fp, _vp]),
    "batq_prepare_weight_minmax": (_i, [C.POINTER(_vp), _vp, _vp, _i, _i, _i, _i64, _i, _fp, _fp, _vp]),
    "batq_weight_export": (_i, [_vp, _vp, _vp, _vp]),
    "batq_weight_import": (_i, [C.POINTER(_vp), _vp, _vp, _i, _i, _vp]),
    "batq_weight_shape": (_i, [_vp, C.POINTER(_i), C.POINTER(_i)]),
    "batq_weight_destroy": (_i, [_vp]),
    "batq_quantize_act": (_i, [_vp, _vp, _i, _i, _i, _i64, _vp, _vp, _vp]),
    "batq_code_bytes": (_sz, [_i, _i]),
    "batq_code_chunk_offset": (_sz, [_i, _i, _i]),
    "batq_codes_to_rowmajor": (_i, [_vp, _vp, _i, _i, _vp]),
    "batq_codes_from_rowmajor": (_i, [_vp, _vp, _i, _i, _vp]),
    "batq_scale_bytes": (_sz, [_i, _i]),
    "batq_scale_index": (_sz, [_i, _i, _i]),
    "batq_scales_to_rowmajor": (_i, [_vp, _vp, _i, _i, _vp]),
    "batq_scales_from_rowmajor": (_i, [_vp, _vp, _i, _i, _vp]),
    "batq_gemm_mxfp4": (_i, [_vp, _vp, _vp, _i, _vp, _i, _i64, _vp]),
    "batq_gemm_workspace": (_sz, [_vp, _i, _i]),
    "batq_gemm_mxfp4_ws": (_i, [_vp, _vp, _vp, _i, _vp, _i, _i64, _vp, _sz, _vp]),
    "batq_gemm_a8w4_ws": (_i, [_vp, _vp, _vp, _i, _vp, _i, _i64, _vp, _sz, _vp]),
    "batq_gemm_mxfp4_noalloc": (_i, [_vp, _vp, _vp, _i, _vp, _i, _i64, _vp]),
    "batq_linear_workspace": (_sz, [_i, _i]),
    "batq_linear_workspace_for": (_sz, [_vp, _i, _i]),
    "batq_linear": (_i, [_vp, _vp, _vp, _i, _i, _i64, _vp, _i, _i64, _vp, _sz, _vp]),
    "batq_quantize_act_mxfp8": (_i, [_vp, _vp, _i, _i, _i, _i64, _vp, _vp, _vp]),
    "batq_code8_bytes": (_sz, [_i, _i]),
    "batq_code8_slot_offset": (_sz, [_i, _i, _i, _i]),
    "batq_codes8_to_rowmajor": (_i, [_vp, _vp, _i, _i, _vp]),
    "batq_codes8_from_rowmajor": (_i, [_vp, _vp, _i, _i, _vp]),
    "batq_gemm_a8w4": (_i, [_vp, _vp, _vp, _i, _vp, _i, _i64, _vp]),
    "batq_linear_a8w4_workspace": (_sz, [_i, _i]),
    "batq_linear_a8w4": (_i, [_vp, _vp, _vp, _i, _i, _i64, _vp, _i, _i64, _vp, _sz, _vp]),
    "batq_quantize_act_ex": (_i, [_vp, _vp, _i, _i, _i, _i64, _vp, _vp, _vp, _vp]),
    "batq_linear_ex": (_i, [_vp, _vp, _vp, _i, _i, _i64, _vp, _vp, _i, _i64, _vp, _sz, _vp]),
    "batq_row_rms_scale": (_i, [_vp, _i, _i, _i, _i64, C.c_float, _vp, _vp]),
    "batq_prepare_weight_gate_up": (_i, [C.POINTER(_vp), _vp, _vp, _vp, _i, _i, _i, _i64, _i, _fp, _vp]),
    "batq_gemm_glu": (_i, [_vp, _vp, _vp, _i, _i, _vp, _i, _i64, _vp]),
    "batq_linear_glu": (_i, [_vp, _vp, _vp, _i, _i, _i64, _vp, _vp, _i, _i64, _vp, _sz, _vp]),
    "batq_debug_tile_schedule": (_i, [_i, _i, _i, _i, _i, _i, _vp, _i]),
    "batq_dequantize": (_i, [_vp, _vp, _i, _i, _i, _vp, _i, _i64, _vp]),
    "batq_kv_append": (_i, [_vp, _vp, _i, _i, _i, _i64, _i, _vp, _vp, _i64, _i64, _vp]),
    "batq_kv_dequantize": (_i, [_vp, _vp, _i64, _i64, _i, _i, _i, _vp, _i, _i64, _vp]),
    "batq_transform_apply": (_i, [_vp, _vp, _i, _i, _i, _i64, _i, _vp, _i, _i64, _vp]),
}


FORM_IDENTITY, FORM_KRON, FORM_DENSE = 0, 1, 2


class TransformDesc(C.Structure):
    """batq_transform_desc of include/batq.h."""
    _fields_ = [("K", _i), ("form", _i), ("g_outer", _i), ("g_inner", _i),
                ("outer", _fp), ("outer_per_block", _i), ("inner", _fp), ("inner_per_block", _i),
                ("dense", _fp), ("clip", _fp), ("clip_min", _fp), ("clip_max", _fp)]


class BatqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.batq_status_string(status).decode() if lib is not None else "?"
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({msg})")


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2603_16590_amd.build` "
            "(there is no fallback path)")
    # The tensors this binding is handed live in torch's HIP runtime, and torch ships its own copy of it: that copy
    # has to be in the process before the library's dependency on the HIP runtime is resolved, or the library gets
    # a second runtime that knows none of torch's allocations (its first call then fails with BATQ_ERR_DEVICE).
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    l = C.CDLL(LIB_PATH)
    for name, (res, args) in SYMBOLS.items():
        fn = getattr(l, name)            # AttributeError if the library does not export it
        fn.restype = res
        fn.argtypes = args
    return l


lib: Optional[C.CDLL] = None
lib = _load()


def _check(status: int, where: str):
    if status != 0:
        raise BatqError(status, where)


def _fptr(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_fp)


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


class Transform:
    """Owns a batq_transform handle (shared factor G, private factors P, clip ratios)."""

    def __init__(self, K: int, G: Optional[np.ndarray], P: Optional[np.ndarray], clip: Optional[np.ndarray],
                 g_outer: int = 4, g_inner: int = 8):
        self.K, self.g_outer, self.g_inner = K, g_outer, g_inner
        self._h = _vp()
        G = None if G is None else np.ascontiguousarray(G, dtype=np.float32)
        P = None if P is None else np.ascontiguousarray(P, dtype=np.float32)
        clip = None if clip is None else np.ascontiguousarray(clip, dtype=np.float32)
        if G is not None:
            assert G.shape == (g_outer, g_outer) and P.shape == (K // 32, g_inner, g_inner)
        if clip is not None:
            assert clip.shape == (K // 32,)
        _check(lib.batq_transform_create(C.byref(self._h), K, g_outer, g_inner, _fptr(G), _fptr(P), _fptr(clip)),
               "batq_transform_create")

    @classmethod
    def general(cls, K: int, *, outer=None, inner=None, dense=None, clip=None, clip_min=None, clip_max=None):
        """batq_transform_create_ex: Kronecker form (``outer`` / ``inner`` 2-D = shared by all blocks,
        3-D = one per block), dense blocks [K/32, 32, 32], or identity (neither); symmetric ``clip`` or the
        two ratios ``clip_min`` / ``clip_max``."""
        self = cls.__new__(cls)
        self.K = K
        self._h = _vp()
        f32 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.float32)
        outer, inner, dense, clip, clip_min, clip_max = map(f32, (outer, inner, dense, clip, clip_min, clip_max))
        d = TransformDesc()
        d.K = K
        keep = [outer, inner, dense, clip, clip_min, clip_max]      # the arrays must outlive the call
        if dense is not None:
            assert dense.shape == (K // 32, 32, 32)
            d.form, d.dense = FORM_DENSE, _fptr(dense)
        elif outer is not None:
            d.form = FORM_KRON
            d.g_outer, d.g_inner = outer.shape[-1], inner.shape[-1]
            d.outer, d.outer_per_block = _fptr(outer), int(outer.ndim == 3)
            d.inner, d.inner_per_block = _fptr(inner), int(inner.ndim == 3)
        else:
            d.form = FORM_IDENTITY
        self.g_outer, self.g_inner = d.g_outer, d.g_inner
        d.clip, d.clip_min, d.clip_max = _fptr(clip), _fptr(clip_min), _fptr(clip_max)
        _check(lib.batq_transform_create_ex(C.byref(self._h), C.byref(d)), "batq_transform_create_ex")
        del keep
        return self

    @property
    def handle(self):
        return self._h

    def close(self):
        if self._h:
            lib.batq_transform_destroy(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Weight:
    """Owns a batq_weight handle (prepared MXFP4 weights on the device)."""

    def __init__(self, handle: _vp):
        self._h = handle
        k, n = _i(), _i()
        _check(lib.batq_weight_shape(self._h, C.byref(k), C.byref(n)), "batq_weight_shape")
        self.K, self.N = k.value, n.value

    @property
    def handle(self):
        return self._h

    def export(self):
        """Canonical (codes [N, K/2], scales [N, K/32]) as uint8 device tensors."""
        import torch
        codes = torch.empty((self.N, self.K // 2), dtype=torch.uint8, device="cuda")
        scales = torch.empty((self.N, self.K // 32), dtype=torch.uint8, device="cuda")
        _check(lib.batq_weight_export(self._h, codes.data_ptr(), scales.data_ptr(), _stream()), "batq_weight_export")
        return codes, scales

    def close(self):
        if self._h:
            lib.batq_weight_destroy(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def batq_prepare_weight(t: Transform, W, w_is_KxN: bool = True, clip_w: Optional[np.ndarray] = None) -> Weight:
    """W: 2-D device tensor (fp32 or bf16), K x N if ``w_is_KxN`` else N x K; rows may be strided."""
    assert W.is_cuda and W.dim() == 2 and W.stride(1) == 1
    K, N = (W.shape[0], W.shape[1]) if w_is_KxN else (W.shape[1], W.shape[0])
    clip_w = None if clip_w is None else np.ascontiguousarray(clip_w, dtype=np.float32)
    h = _vp()
    _check(lib.batq_prepare_weight(C.byref(h), t.handle, W.data_ptr(), _dtype_code(W), K, N, W.stride(0),
                                   1 if w_is_KxN else 0, _fptr(clip_w), _stream()), "batq_prepare_weight")
    return Weight(h)


def batq_prepare_weight_gate_up(t: Transform, W_gate, W_up, w_is_KxN: bool = True,
                                clip_w: Optional[np.ndarray] = None) -> Weight:
    """Gate and up projection (same shape, dtype and row stride) as one weight of 2 F interleaved columns."""
    assert W_gate.is_cuda and W_gate.dim() == 2 and W_gate.stride(1) == 1
    assert W_up.is_cuda and W_up.shape == W_gate.shape and W_up.dtype == W_gate.dtype and W_up.stride() == W_gate.stride()
    K, F = (W_gate.shape[0], W_gate.shape[1]) if w_is_KxN else (W_gate.shape[1], W_gate.shape[0])
    clip_w = None if clip_w is None else np.ascontiguousarray(clip_w, dtype=np.float32)
    h = _vp()
    _check(lib.batq_prepare_weight_gate_up(C.byref(h), t.handle, W_gate.data_ptr(), W_up.data_ptr(), _dtype_code(W_gate),
                                           K, F, W_gate.stride(0), 1 if w_is_KxN else 0, _fptr(clip_w), _stream()),
           "batq_prepare_weight_gate_up")
    return Weight(h)


def batq_prepare_weight_minmax(t: Transform, W, clip_w_min: np.ndarray, clip_w_max: np.ndarray,
                               w_is_KxN: bool = True) -> Weight:
    """As batq_prepare_weight with the two-ratio clipping (ratios on the block minimum and maximum)."""
    assert W.is_cuda and W.dim() == 2 and W.stride(1) == 1
    K, N = (W.shape[0], W.shape[1]) if w_is_KxN else (W.shape[1], W.shape[0])
    cmin = np.ascontiguousarray(clip_w_min, dtype=np.float32)
    cmax = np.ascontiguousarray(clip_w_max, dtype=np.float32)
    h = _vp()
    _check(lib.batq_prepare_weight_minmax(C.byref(h), t.handle, W.data_ptr(), _dtype_code(W), K, N, W.stride(0),
                                          1 if w_is_KxN else 0, _fptr(cmin), _fptr(cmax), _stream()),
           "batq_prepare_weight_minmax")
    return Weight(h)


def batq_weight_import(codes, scales, K: int, N: int) -> Weight:
    assert codes.is_cuda and scales.is_cuda and codes.is_contiguous() and scales.is_contiguous()
    h = _vp()
    _check(lib.batq_weight_import(C.byref(h), codes.data_ptr(), scales.data_ptr(), K, N, _stream()),
           "batq_weight_import")
    return Weight(h)


def batq_code_bytes(rows: int, K: int) -> int:
    return int(lib.batq_code_bytes(rows, K))


def batq_scale_bytes(rows: int, K: int) -> int:
    return int(lib.batq_scale_bytes(rows, K))


def batq_quantize_act(t: Transform, X, codes=None, scales=None):
    """X: M x K device tensor (fp32 or bf16, unit column stride).

    Returns (codes, scales): flat uint8 tensors in the library's device order."""
    import torch
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    if codes is None:
        codes = torch.empty((batq_code_bytes(M, K),), dtype=torch.uint8, device=X.device)
    if scales is None:
        scales = torch.empty((batq_scale_bytes(M, K),), dtype=torch.uint8, device=X.device)
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    _check(lib.batq_quantize_act(t.handle, X.data_ptr(), _dtype_code(X), M, K, ldx, codes.data_ptr(),
                                 scales.data_ptr(), _stream()), "batq_quantize_act")
    return codes, scales


def batq_codes_to_rowmajor(codes, rows: int, K: int):
    """Device-order codes -> [rows, K/2] uint8 tensor."""
    import torch
    out = torch.empty((rows, K // 2), dtype=torch.uint8, device=codes.device)
    _check(lib.batq_codes_to_rowmajor(codes.data_ptr(), out.data_ptr(), rows, K, _stream()), "batq_codes_to_rowmajor")
    return out


def batq_codes_from_rowmajor(rowmajor):
    """[rows, K/2] uint8 tensor -> flat device-order codes (K padding zeroed)."""
    import torch
    assert rowmajor.is_contiguous()
    rows, kh = rowmajor.shape
    out = torch.empty((batq_code_bytes(rows, kh * 2),), dtype=torch.uint8, device=rowmajor.device)
    _check(lib.batq_codes_from_rowmajor(rowmajor.data_ptr(), out.data_ptr(), rows, kh * 2, _stream()),
           "batq_codes_from_rowmajor")
    return out


def batq_scales_to_rowmajor(grouped, rows: int, K: int):
    """Grouped scale bytes -> [rows, K/32] uint8 tensor."""
    import torch
    out = torch.empty((rows, K // 32), dtype=torch.uint8, device=grouped.device)
    _check(lib.batq_scales_to_rowmajor(grouped.data_ptr(), out.data_ptr(), rows, K, _stream()),
           "batq_scales_to_rowmajor")
    return out


def batq_scales_from_rowmajor(rowmajor):
    """[rows, K/32] uint8 tensor -> flat grouped scale bytes."""
    import torch
    assert rowmajor.is_contiguous()
    rows, nb = rowmajor.shape
    out = torch.empty((batq_scale_bytes(rows, nb * 32),), dtype=torch.uint8, device=rowmajor.device)
    _check(lib.batq_scales_from_rowmajor(rowmajor.data_ptr(), out.data_ptr(), rows, nb * 32, _stream()),
           "batq_scales_from_rowmajor")
    return out


def batq_gemm_workspace(w: Weight, M: int, act_bits: int = 4) -> int:
    """Bytes of scratch with which the GEMM of M rows against w uses all the K parts it wants (0: none)."""
    return int(lib.batq_gemm_workspace(w.handle, M, act_bits))


def batq_gemm_mxfp4(xcodes, xscales, w: Weight, M: int, out_dtype=None, Y=None, workspace=None):
    """GEMM on device-order activation codes and scales of M rows. Returns Y (M x N).
    workspace: uint8 device tensor for the partial sums of K parts (batq_gemm_mxfp4_ws), or None (plain call)."""
    import torch
    if Y is None:
        Y = torch.empty((M, w.N), dtype=out_dtype or torch.float32, device=xcodes.device)
    ldy = Y.stride(0) if M > 1 else max(w.N, Y.stride(0))
    if workspace is None:
        _check(lib.batq_gemm_mxfp4(xcodes.data_ptr(), xscales.data_ptr(), w.handle, M, Y.data_ptr(), _dtype_code(Y),
                                   ldy, _stream()), "batq_gemm_mxfp4")
    else:
        _check(lib.batq_gemm_mxfp4_ws(xcodes.data_ptr(), xscales.data_ptr(), w.handle, M, Y.data_ptr(), _dtype_code(Y),
                                      ldy, workspace.data_ptr(), workspace.numel(), _stream()), "batq_gemm_mxfp4_ws")
    return Y


def batq_gemm_glu(xcodes, xscales, w: Weight, M: int, act_bits: int = 4, out_dtype=None, H=None):
    """silu(gate) * up of the gate/up GEMM on device-order activation codes. Returns H (M x N/2)."""
    import torch
    F = w.N // 2
    if H is None:
        H = torch.empty((M, F), dtype=out_dtype or torch.bfloat16, device=xcodes.device)
    _check(lib.batq_gemm_glu(xcodes.data_ptr(), xscales.data_ptr(), w.handle, M, act_bits, H.data_ptr(), _dtype_code(H),
                             H.stride(0) if M > 1 else max(F, H.stride(0)), _stream()), "batq_gemm_glu")
    return H


def batq_linear_workspace(M: int, K: int) -> int:
    return int(lib.batq_linear_workspace(M, K))


def batq_linear_workspace_for(w: Weight, M: int, act_bits: int = 4) -> int:
    """Workspace bytes with which the batq_linear family runs M rows against w as fast as it can."""
    return int(lib.batq_linear_workspace_for(w.handle, M, act_bits))


def batq_linear(t: Transform, w: Weight, X, out_dtype=None, Y=None, workspace=None):
    """Y = Q(X P) Q(P^-1 W): fused transform+quantise kernel, then the MXFP4 GEMM."""
    import torch
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    if Y is None:
        Y = torch.empty((M, w.N), dtype=out_dtype or torch.float32, device=X.device)
    if workspace is None:
        workspace = torch.empty((max(batq_linear_workspace_for(w, M, 4), 16),), dtype=torch.uint8, device=X.device)
    _check(lib.batq_linear(t.handle, w.handle, X.data_ptr(), _dtype_code(X), M,
                           X.stride(0) if M > 1 else max(K, X.stride(0)), Y.data_ptr(), _dtype_code(Y),
                           Y.stride(0) if M > 1 else max(w.N, Y.stride(0)), workspace.data_ptr(),
                           workspace.numel(), _stream()), "batq_linear")
    return Y


# ---- W4A8: MXFP8 (E4M3) activations against the same MXFP4 weights
def batq_code8_bytes(rows: int, K: int) -> int:
    return int(lib.batq_code8_bytes(rows, K))


def batq_quantize_act_mxfp8(t: Transform, X, codes8=None, scales=None):
    """X: M x K device tensor. Returns (codes8, scales): flat uint8 tensors in device order."""
    import torch
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    if codes8 is None:
        codes8 = torch.empty((batq_code8_bytes(M, K),), dtype=torch.uint8, device=X.device)
    if scales is None:
        scales = torch.empty((batq_scale_bytes(M, K),), dtype=torch.uint8, device=X.device)
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    _check(lib.batq_quantize_act_mxfp8(t.handle, X.data_ptr(), _dtype_code(X), M, K, ldx, codes8.data_ptr(),
                                       scales.data_ptr(), _stream()), "batq_quantize_act_mxfp8")
    return codes8, scales


def batq_codes8_to_rowmajor(codes8, rows: int, K: int):
    """Device-order 8-bit codes -> [rows, K] uint8 tensor."""
    import torch
    out = torch.empty((rows, K), dtype=torch.uint8, device=codes8.device)
    _check(lib.batq_codes8_to_rowmajor(codes8.data_ptr(), out.data_ptr(), rows, K, _stream()), "batq_codes8_to_rowmajor")
    return out


def batq_codes8_from_rowmajor(rowmajor):
    """[rows, K] uint8 tensor -> flat device-order 8-bit codes (K padding zeroed)."""
    import torch
    assert rowmajor.is_contiguous()
    rows, K = rowmajor.shape
    out = torch.empty((batq_code8_bytes(rows, K),), dtype=torch.uint8, device=rowmajor.device)
    _check(lib.batq_codes8_from_rowmajor(rowmajor.data_ptr(), out.data_ptr(), rows, K, _stream()),
           "batq_codes8_from_rowmajor")
    return out


def batq_gemm_a8w4(xcodes8, xscales, w: Weight, M: int, out_dtype=None, Y=None, workspace=None):
    import torch
    if Y is None:
        Y = torch.empty((M, w.N), dtype=out_dtype or torch.float32, device=xcodes8.device)
    ldy = Y.stride(0) if M > 1 else max(w.N, Y.stride(0))
    if workspace is None:
        _check(lib.batq_gemm_a8w4(xcodes8.data_ptr(), xscales.data_ptr(), w.handle, M, Y.data_ptr(), _dtype_code(Y),
                                  ldy, _stream()), "batq_gemm_a8w4")
    else:
        _check(lib.batq_gemm_a8w4_ws(xcodes8.data_ptr(), xscales.data_ptr(), w.handle, M, Y.data_ptr(), _dtype_code(Y),
                                     ldy, workspace.data_ptr(), workspace.numel(), _stream()), "batq_gemm_a8w4_ws")
    return Y


def batq_linear_a8w4_workspace(M: int, K: int) -> int:
    return int(lib.batq_linear_a8w4_workspace(M, K))


def batq_linear_a8w4(t: Transform, w: Weight, X, out_dtype=None, Y=None, workspace=None):
    """Y = Q8(X P) Q4(P^-1 W): MXFP8 activations, MXFP4 weights."""
    import torch
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    if Y is None:
        Y = torch.empty((M, w.N), dtype=out_dtype or torch.float32, device=X.device)
    if workspace is None:
        workspace = torch.empty((max(batq_linear_workspace_for(w, M, 8), 16),), dtype=torch.uint8, device=X.device)
    _check(lib.batq_linear_a8w4(t.handle, w.handle, X.data_ptr(), _dtype_code(X), M,
                                X.stride(0) if M > 1 else max(K, X.stride(0)), Y.data_ptr(), _dtype_code(Y),
                                Y.stride(0) if M > 1 else max(w.N, Y.stride(0)), workspace.data_ptr(),
                                workspace.numel(), _stream()), "batq_linear_a8w4")
    return Y


# ---- options form: fused row scaling (RMSNorm) and activation width
class ActOptions(C.Structure):
    """batq_act_options of include/batq.h."""
    _fields_ = [("act_bits", _i), ("row_scale", _vp), ("up", _vp), ("ld_up", C.c_int64)]


def _opts(act_bits: int, row_scale, up=None, X=None):
    o = ActOptions()
    o.act_bits = act_bits
    if row_scale is not None:
        import torch
        assert row_scale.is_cuda and row_scale.dtype == torch.float32 and row_scale.is_contiguous()
        o.row_scale = row_scale.data_ptr()
    if up is not None:
        assert up.is_cuda and up.shape == X.shape and up.dtype == X.dtype and up.stride(1) == 1
        o.up = up.data_ptr()
        o.ld_up = up.stride(0) if up.shape[0] > 1 else max(up.shape[1], up.stride(0))
    return o


def batq_row_rms_scale(X, eps: float = 1e-6):
    """1 / sqrt(mean(x^2) + eps) per row, fp32 device tensor [M]."""
    import torch
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    out = torch.empty((M,), dtype=torch.float32, device=X.device)
    _check(lib.batq_row_rms_scale(X.data_ptr(), _dtype_code(X), M, K, X.stride(0) if M > 1 else max(K, X.stride(0)),
                                  eps, out.data_ptr(), _stream()), "batq_row_rms_scale")
    return out


def batq_linear_glu(t: Transform, w: Weight, X, act_bits: int = 4, row_scale=None, out_dtype=None, H=None,
                    workspace=None, up=None):
    """Quantise X (options as batq_linear_ex), multiply with a gate/up weight, return silu(gate) * up."""
    import torch
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    F = w.N // 2
    if H is None:
        H = torch.empty((M, F), dtype=out_dtype or torch.bfloat16, device=X.device)
    if workspace is None:
        workspace = torch.empty((max(batq_linear_workspace_for(w, M, act_bits), 16),), dtype=torch.uint8, device=X.device)
    o = _opts(act_bits, row_scale, up, X)
    _check(lib.batq_linear_glu(t.handle, w.handle, X.data_ptr(), _dtype_code(X), M,
                               X.stride(0) if M > 1 else max(K, X.stride(0)), C.byref(o), H.data_ptr(),
                               _dtype_code(H), H.stride(0) if M > 1 else max(F, H.stride(0)),
                               workspace.data_ptr(), workspace.numel(), _stream()), "batq_linear_glu")
    return H


APPLY_FORWARD, APPLY_INVERSE, APPLY_INVERSE_T = 0, 1, 2


def batq_dequantize(codes, scales, M: int, K: int, bits: int = 4, out_dtype=None, out=None):
    """Device-order codes + grouped scales -> row-major [M, K] tensor (bf16 by default)."""
    import torch
    if out is None:
        out = torch.empty((M, K), dtype=out_dtype or torch.bfloat16, device=codes.device)
    _check(lib.batq_dequantize(codes.data_ptr(), scales.data_ptr(), M, K, bits, out.data_ptr(), _dtype_code(out),
                               out.stride(0) if M > 1 else max(K, out.stride(0)), _stream()), "batq_dequantize")
    return out


def batq_kv_append(t: Transform, X, codes, scales, row_offset: int, capacity_rows: int, bits: int = 4):
    """Quantise the rows of X into rows row_offset.. of a cache laid out for capacity_rows rows (codes, scales:
    flat uint8 device tensors of batq_code_bytes / batq_code8_bytes and batq_scale_bytes of capacity_rows)."""
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    _check(lib.batq_kv_append(t.handle, X.data_ptr(), _dtype_code(X), M, K,
                              X.stride(0) if M > 1 else max(K, X.stride(0)), bits, codes.data_ptr(), scales.data_ptr(),
                              row_offset, capacity_rows, _stream()), "batq_kv_append")


def batq_kv_dequantize(codes, scales, capacity_rows: int, row_offset: int, M: int, K: int, bits: int = 4,
                       out_dtype=None, out=None):
    """Rows row_offset .. row_offset + M - 1 of a cache laid out for capacity_rows rows -> [M, K] tensor."""
    import torch
    if out is None:
        out = torch.empty((M, K), dtype=out_dtype or torch.bfloat16, device=codes.device)
    _check(lib.batq_kv_dequantize(codes.data_ptr(), scales.data_ptr(), capacity_rows, row_offset, M, K, bits,
                                  out.data_ptr(), _dtype_code(out), out.stride(0) if M > 1 else max(K, out.stride(0)),
                                  _stream()), "batq_kv_dequantize")
    return out


def batq_transform_apply(t: Transform, X, mode: int = APPLY_FORWARD, out_dtype=None, out=None):
    """X T_k, X T_k^-1 or X T_k^-T block by block, without quantisation."""
    import torch
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    if out is None:
        out = torch.empty((M, K), dtype=out_dtype or X.dtype, device=X.device)
    _check(lib.batq_transform_apply(t.handle, X.data_ptr(), _dtype_code(X), M, K,
                                    X.stride(0) if M > 1 else max(K, X.stride(0)), mode, out.data_ptr(),
                                    _dtype_code(out), out.stride(0) if M > 1 else max(K, out.stride(0)), _stream()),
           "batq_transform_apply")
    return out


def batq_quantize_act_ex(t: Transform, X, act_bits: int = 4, row_scale=None, up=None):
    import torch
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    nbytes = batq_code8_bytes(M, K) if act_bits == 8 else batq_code_bytes(M, K)
    codes = torch.empty((nbytes,), dtype=torch.uint8, device=X.device)
    scales = torch.empty((batq_scale_bytes(M, K),), dtype=torch.uint8, device=X.device)
    o = _opts(act_bits, row_scale, up, X)
    _check(lib.batq_quantize_act_ex(t.handle, X.data_ptr(), _dtype_code(X), M, K,
                                    X.stride(0) if M > 1 else max(K, X.stride(0)), C.byref(o), codes.data_ptr(),
                                    scales.data_ptr(), _stream()), "batq_quantize_act_ex")
    return codes, scales


def batq_linear_ex(t: Transform, w: Weight, X, act_bits: int = 4, row_scale=None, out_dtype=None, Y=None,
                   workspace=None, up=None):
    import torch
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    if Y is None:
        Y = torch.empty((M, w.N), dtype=out_dtype or torch.float32, device=X.device)
    if workspace is None:
        workspace = torch.empty((max(batq_linear_workspace_for(w, M, act_bits), 16),), dtype=torch.uint8, device=X.device)
    o = _opts(act_bits, row_scale, up, X)
    _check(lib.batq_linear_ex(t.handle, w.handle, X.data_ptr(), _dtype_code(X), M,
                              X.stride(0) if M > 1 else max(K, X.stride(0)), C.byref(o), Y.data_ptr(),
                              _dtype_code(Y), Y.stride(0) if M > 1 else max(w.N, Y.stride(0)),
                              workspace.data_ptr(), workspace.numel(), _stream()), "batq_linear_ex")
    return Y
