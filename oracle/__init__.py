"""GQSA CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Thin ctypes front-end of oracle/gqsa_oracle.c (plain C, float64 accumulation)
plus, in oracle/layout.py, an independent derivation of the device byte layout
from its written specification.  Only tests, the smoke check and the
benchmark's cpu_baseline leg import this package; the HIP library and its
Python binding never do.

Paper passages followed: Sec. 3.1 Eq. 1-3 (quantiser and dequantiser),
Sec. 3.2 with the Fig. 3 caption and the BSR listing (group pruning, storage),
Sec. 3.5 (the 1xNxK GEMV with activations addressed by real group index).
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB
    if not os.path.exists(path):
        _build.build()
    lib = C.CDLL(path)
    i32p = C.POINTER(C.c_int32)
    u8p = C.POINTER(C.c_uint8)
    u16p = C.POINTER(C.c_uint16)
    f32p = C.POINTER(C.c_float)
    f64p = C.POINTER(C.c_double)
    lib.gqsa_oracle_f16_to_f32.restype = C.c_float
    lib.gqsa_oracle_f16_to_f32.argtypes = [C.c_uint16]
    lib.gqsa_oracle_f32_to_f16.restype = C.c_uint16
    lib.gqsa_oracle_f32_to_f16.argtypes = [C.c_float]
    lib.gqsa_oracle_keep_count.restype = C.c_int32
    lib.gqsa_oracle_keep_count.argtypes = [C.c_int64, C.c_double]
    lib.gqsa_oracle_count.restype = C.c_int64
    lib.gqsa_oracle_count.argtypes = [i32p, C.c_int64]
    lib.gqsa_oracle_pack.restype = C.c_int
    lib.gqsa_oracle_pack.argtypes = [f32p, C.c_int64, C.c_int64, C.c_int, C.c_int, i32p, f32p,
                                     i32p, i32p, u8p, u16p, u16p]
    lib.gqsa_oracle_densify.restype = C.c_int
    lib.gqsa_oracle_densify.argtypes = [i32p, i32p, u8p, u16p, u16p, C.c_int64, C.c_int64,
                                        C.c_int, C.c_int, f64p]
    lib.gqsa_oracle_gemv.restype = C.c_int
    lib.gqsa_oracle_gemv.argtypes = [i32p, i32p, u8p, u16p, u16p, C.c_int64, C.c_int64,
                                     C.c_int, C.c_int, u16p, C.c_int, f64p, C.c_int]
    lib.gqsa_oracle_max_threads.restype = C.c_int
    lib.gqsa_oracle_max_threads.argtypes = []
    _lib = lib
    return lib


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


@dataclass
class Canonical:
    """The BSR arrays of Sec. 3.2's listing plus the per-group quantiser parameters."""
    N: int
    K: int
    G: int
    bits: int
    rowIndex: np.ndarray   # int32 [N+1]
    groups: np.ndarray     # int32 [nnzg]
    values: np.ndarray     # uint8 [nnzg*G*bits/8]
    scales: np.ndarray     # uint16 [nnzg], fp16 bit patterns
    zeros: np.ndarray      # uint16 [nnzg], fp16 bit patterns

    @property
    def nnzg(self) -> int:
        return int(self.rowIndex[-1])


def f32_to_f16_bits(v: float) -> int:
    return int(_load().gqsa_oracle_f32_to_f16(C.c_float(v)))


def f16_bits_to_f32(h: int) -> float:
    return float(_load().gqsa_oracle_f16_to_f32(C.c_uint16(h)))


def keep_counts(N: int, K: int, G: int, sparsity: float) -> np.ndarray:
    """Balanced per-row pruning: every row keeps K/G - floor(S*K/G + 0.5) groups."""
    k = _load().gqsa_oracle_keep_count(K // G, float(sparsity))
    return np.full(N, k, dtype=np.int32)


def pack(W: np.ndarray, G: int = 16, bits: int = 4, sparsity: float | None = None,
         keep_per_row: np.ndarray | None = None, hinv_diag: np.ndarray | None = None) -> Canonical:
    """Group-prune and quantise dense fp32 W[N,K] into the canonical BSR arrays.
    hinv_diag: diag(H^-1) of Eq. 4 (K positive numbers); None = magnitude saliency."""
    lib = _load()
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    if K % G != 0:
        raise ValueError("K must be a multiple of G")
    if keep_per_row is None:
        if sparsity is None:
            raise ValueError("give sparsity or keep_per_row")
        keep_per_row = keep_counts(N, K, G, sparsity)
    keep = np.ascontiguousarray(keep_per_row, dtype=np.int32)
    nnzg = int(lib.gqsa_oracle_count(_ptr(keep, C.c_int32), N))
    rowIndex = np.zeros(N + 1, dtype=np.int32)
    groups = np.zeros(max(nnzg, 1), dtype=np.int32)
    values = np.zeros(max(nnzg * G * bits // 8, 1), dtype=np.uint8)
    scales = np.zeros(max(nnzg, 1), dtype=np.uint16)
    zeros = np.zeros(max(nnzg, 1), dtype=np.uint16)
    dptr = None
    if hinv_diag is not None:
        hinv_diag = np.ascontiguousarray(hinv_diag, dtype=np.float32)
        if hinv_diag.shape != (K,):
            raise ValueError("hinv_diag must have K entries")
        dptr = _ptr(hinv_diag, C.c_float)
    rc = lib.gqsa_oracle_pack(_ptr(W, C.c_float), N, K, G, bits, _ptr(keep, C.c_int32), dptr,
                              _ptr(rowIndex, C.c_int32), _ptr(groups, C.c_int32),
                              _ptr(values, C.c_uint8), _ptr(scales, C.c_uint16),
                              _ptr(zeros, C.c_uint16))
    if rc != 0:
        raise ValueError(f"oracle pack rejected its arguments (code {rc})")
    return Canonical(N, K, G, bits, rowIndex, groups[:nnzg], values[:nnzg * G * bits // 8],
                     scales[:nnzg], zeros[:nnzg])


def _arrs(c: Canonical):
    def nz(a, dt):
        a = np.ascontiguousarray(a, dtype=dt)
        return a if a.size else np.zeros(1, dtype=dt)
    return (nz(c.rowIndex, np.int32), nz(c.groups, np.int32), nz(c.values, np.uint8),
            nz(c.scales, np.uint16), nz(c.zeros, np.uint16))


def densify(c: Canonical) -> np.ndarray:
    """Eq. 3 on every stored group, zeros elsewhere: float64 [N,K]."""
    ri, gr, va, sc, ze = _arrs(c)
    Wd = np.zeros((c.N, c.K), dtype=np.float64)
    rc = _load().gqsa_oracle_densify(_ptr(ri, C.c_int32), _ptr(gr, C.c_int32),
                                     _ptr(va, C.c_uint8), _ptr(sc, C.c_uint16),
                                     _ptr(ze, C.c_uint16), c.N, c.K, c.G, c.bits,
                                     _ptr(Wd, C.c_double))
    if rc != 0:
        raise ValueError(f"oracle densify failed (code {rc})")
    return Wd


def gemv(c: Canonical, x_f16: np.ndarray, threads: int = 0) -> np.ndarray:
    """y[b,n] = sum_k W^[n,k] x[b,k] in float64; x is fp16 [batch,K]."""
    x = np.ascontiguousarray(x_f16, dtype=np.float16)
    if x.ndim == 1:
        x = x[None, :]
    batch, K = x.shape
    if K != c.K:
        raise ValueError("x has the wrong length")
    ri, gr, va, sc, ze = _arrs(c)
    y = np.zeros((batch, c.N), dtype=np.float64)
    xb = x.view(np.uint16)
    rc = _load().gqsa_oracle_gemv(_ptr(ri, C.c_int32), _ptr(gr, C.c_int32),
                                  _ptr(va, C.c_uint8), _ptr(sc, C.c_uint16),
                                  _ptr(ze, C.c_uint16), c.N, c.K, c.G, c.bits,
                                  _ptr(xb, C.c_uint16), batch, _ptr(y, C.c_double),
                                  int(threads))
    if rc != 0:
        raise ValueError(f"oracle gemv failed (code {rc})")
    return y


def max_threads() -> int:
    return int(_load().gqsa_oracle_max_threads())


def algorithmic_bytes(N: int, K: int, G: int, bits: int, nnzg: int, batch: int) -> int:
    """Compressed bytes one GEMV call must move: per stored group its codes, an fp16
    scale, an fp16 zero and a 16-bit group-column; the row pointers; x and y."""
    return nnzg * (G * bits // 8 + 6) + (N + 1) * 4 + batch * (K + N) * 2


def rel_error(y: np.ndarray, y_ref: np.ndarray) -> float:
    """Max relative error with a floor on the denominator (1% of the rms of y_ref),
    so that outputs that cancel to ~0 are judged on the scale of the vector."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(y_ref * y_ref))) if y_ref.size else 0.0
    den = np.maximum(np.abs(y_ref), 1e-2 * rms)
    den = np.where(den == 0.0, 1.0, den)
    if y.size == 0:
        return 0.0
    return float(np.max(np.abs(y - y_ref) / den))


from .layout import device_blob, device_blob_for, panel_blob, row_positions  # noqa: E402,F401
