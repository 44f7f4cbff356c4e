"""Seeded synthetic inputs for the W4A4 MXFP4 linear hot path.

This module only draws random tensors and casts them to their storage dtype.
It contains none of the method's arithmetic (no transform, clip, quantiser or
GEMM) and is the one module that the CPU oracle's tests, the GPU tests and the
benchmark all share.

The five workloads stand in for the activations and weights of the 8B-class
LLM / multimodal LLM whose projections the paper quantises (Sec. 4.1; the real
tensors need model weights and calibration data, which are not available).
Shapes follow the projection sizes; distributions mimic what the paper
describes qualitatively: a few outlier channels and heavy-tailed inputs to the
down projection (Sec. 2, "Observations and Motivation").

bf16 tensors are carried as ``uint16`` bit patterns because NumPy has no bf16
type; :func:`bf16_bits_to_f32` widens them exactly.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BLOCK = 32  # MXFP block size (Sec. 2, MXFP definition)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 storage (round-to-nearest-even), as uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


@dataclass
class Workload:
    """One synthetic W4A4 linear problem.

    ``X`` is M x K (tokens x in-features), ``W`` is K x N (in x out).  When
    ``dtype == "bf16"`` both hold uint16 bf16 bit patterns, otherwise fp32.
    ``G`` (g_outer x g_outer) is the global Kronecker factor, ``P``
    (K/32 x g_inner x g_inner) the private factors, ``clip`` (K/32) the
    activation clip ratios; all fp32.
    """

    cfg: int
    name: str
    M: int
    K: int
    N: int
    dtype: str            # "f32" | "bf16" storage of X and W
    out_dtype: str        # "f32" | "bf16" storage of Y
    X: np.ndarray
    W: Optional[np.ndarray]
    G: np.ndarray
    P: np.ndarray
    clip: np.ndarray
    meta: dict = field(default_factory=dict)

    @property
    def nb(self) -> int:
        return self.K // BLOCK

    def X_f32(self) -> np.ndarray:
        return bf16_bits_to_f32(self.X) if self.dtype == "bf16" else self.X

    def W_f32(self) -> np.ndarray:
        return bf16_bits_to_f32(self.W) if self.dtype == "bf16" else self.W


_SHAPES = {
    # cfg: (name, M, K, N, storage dtype, out dtype)
    0: ("tiny-linear", 64, 256, 256, "f32", "f32"),
    1: ("decode-qproj", 16, 4096, 4096, "bf16", "bf16"),
    2: ("prefill-mlp-upgate-8B", 2048, 4096, 14336, "bf16", "bf16"),
    3: ("prefill-mlp-down-8B", 4096, 14336, 4096, "bf16", "bf16"),
    4: ("mllm-mlp", 8192, 3584, 18944, "bf16", "bf16"),
}
_OUTLIER = {0: (0.02, 20.0), 1: (0.01, 30.0), 2: (0.01, 30.0), 3: (0.005, 50.0), 4: (0.01, 30.0)}
_CLIP_LO = {0: 0.85, 1: 0.85, 2: 0.85, 3: 0.8, 4: 0.85}


def config_shape(cfg: int):
    """(name, M, K, N, storage dtype, out dtype) of workload ``cfg``."""
    return _SHAPES[cfg]


def _streams(cfg: int, extra: int = 0):
    ss = np.random.SeedSequence([2603, 16590, cfg, extra])
    # fixed order: X, outlier channels, row scales, W, G, P, clip
    return [np.random.Generator(np.random.PCG64(s)) for s in ss.spawn(7)]


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    a32 = a.astype(np.float32)
    return f32_to_bf16_bits(a32) if dtype == "bf16" else a32


def make_factors(nb: int, rng_g, rng_p, rng_c, clip_lo: float, g_outer: int = 4, g_inner: int = 8,
                 eps: float = 0.05):
    """G = I + eps*N(0,1), P_k = I + eps*N(0,1), clip ~ U(clip_lo, 1); all fp32."""
    G = (np.eye(g_outer) + eps * rng_g.standard_normal((g_outer, g_outer))).astype(np.float32)
    P = (np.eye(g_inner)[None] + eps * rng_p.standard_normal((nb, g_inner, g_inner))).astype(np.float32)
    clip = rng_c.uniform(clip_lo, 1.0, size=nb).astype(np.float32)
    return G, P, clip


def make_workload(cfg: int, rows: Optional[int] = None, with_weight: bool = True,
                  g_outer: int = 4, g_inner: int = 8) -> Workload:
    """Build workload ``cfg`` (0..4).

    ``rows`` draws only ``rows`` token rows of X (a sample of the same
    distribution, not necessarily the head of the full tensor; cfg 4's
    vision/text split stays at row 6144).  ``with_weight=False`` skips W.
    """
    name, M, K, N, dtype, odt = _SHAPES[cfg]
    rx, rch, rrow, rw, rg, rp, rc = _streams(cfg)
    nb = K // BLOCK
    frac, mult = _OUTLIER[cfg]
    n_out = int(round(frac * K))
    chans = np.sort(rch.choice(K, size=n_out, replace=False))
    Mgen = M if rows is None else min(rows, M)

    if cfg == 3:
        X = rx.standard_t(3.0, size=(Mgen, K))
        X[:, chans] *= mult
    elif cfg == 4:
        n_vis = 6144
        mv = min(Mgen, n_vis)
        Xv = rx.standard_normal((mv, K)) * 2.0
        sign = np.where(rx.random((mv, K)) < 0.5, -1.5, 1.5)
        Xv += sign
        mt = Mgen - mv
        if mt > 0:
            Xt = rx.standard_normal((mt, K))
            Xt[:, chans] *= mult
            X = np.concatenate([Xv, Xt], axis=0)
        else:
            X = Xv
    else:
        X = rx.standard_normal((Mgen, K))
        X[:, chans] *= mult
        if cfg == 2:
            X *= rrow.lognormal(0.0, 0.5, size=(Mgen, 1))

    W = None
    if with_weight:
        # drawn in fp32 to keep the largest weight (68M elements) cheap to make
        W = rw.standard_normal((K, N), dtype=np.float32) * np.float32(0.02)
        W = _store(W, dtype)
    G, P, clip = make_factors(nb, rg, rp, rc, _CLIP_LO[cfg], g_outer, g_inner)
    return Workload(cfg=cfg, name=name, M=Mgen, K=K, N=N, dtype=dtype, out_dtype=odt,
                    X=_store(X, dtype), W=W, G=G, P=P, clip=clip,
                    meta={"outlier_channels": chans, "full_M": M})


def make_small(M: int, K: int, N: int, seed: int = 0, dtype: str = "bf16", outliers: bool = True,
               g_outer: int = 4, g_inner: int = 8, clip_lo: float = 0.85) -> Workload:
    """A small problem of arbitrary shape with config-0-style distributions."""
    rx, rch, rrow, rw, rg, rp, rc = _streams(1000 + seed, extra=M * 1315423911 % 65521 + K + N)
    nb = K // BLOCK
    X = rx.standard_normal((M, K))
    if outliers and K >= 64:
        chans = rch.choice(K, size=max(1, K // 64), replace=False)
        X[:, chans] *= 20.0
    W = rw.standard_normal((K, N)) * 0.02
    G, P, clip = make_factors(nb, rg, rp, rc, clip_lo, g_outer, g_inner)
    return Workload(cfg=-1, name=f"small-{M}x{K}x{N}-s{seed}", M=M, K=K, N=N, dtype=dtype,
                    out_dtype="f32", X=_store(X, dtype), W=_store(W, dtype), G=G, P=P, clip=clip)
