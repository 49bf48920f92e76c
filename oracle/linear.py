"""Oracle integer GEMM + dequantization epilogue -- test infrastructure.

Integer product: oracle/igemm.c (plain loops).  Epilogue: fp64, then ONE
rounding to fp16.  The layer is y = x W^T (+ bias) with x ~ xq*sx (per token)
and W ~ wq*sw (per output channel) or, for 4-bit weights, wq*sw[n,g] per group
of consecutive k; substituting gives

  W8A8:  y[m,n] = acc[m,n] * sx[m] * sw[n] + bias[n]
  W4A8:  y[m,n] = sx[m] * sum_g part[m,g,n] * sw[n,g] + bias[n]
"""
from __future__ import annotations

import ctypes

import numpy as np

from . import build as _build
from .quantizers import quant_act_per_token, unpack_int4

_lib = None


def _clib():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        i8p = ctypes.POINTER(ctypes.c_int8)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.oracle_igemm.restype = ctypes.c_int64
        lib.oracle_igemm.argtypes = [i8p, i8p, ctypes.c_int, ctypes.c_int, ctypes.c_int, i32p]
        lib.oracle_igemm_grouped.restype = ctypes.c_int64
        lib.oracle_igemm_grouped.argtypes = [i8p, i8p, f64p, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_int, ctypes.c_int, f64p, i32p, i32p]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the C loops use (OpenMP default: all cores of the affinity mask)."""
    return int(_clib().oracle_num_threads())


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _check_codes(xq, wq):
    if xq.dtype != np.int8 or wq.dtype != np.int8:
        raise TypeError("integer GEMM takes int8 codes")
    if xq.ndim != 2 or wq.ndim != 2 or xq.shape[1] != wq.shape[1]:
        raise ValueError("xq [M,K] and wq [N,K] must share K")
    return np.ascontiguousarray(xq), np.ascontiguousarray(wq)


def igemm(xq: np.ndarray, wq: np.ndarray) -> np.ndarray:
    """acc[m,n] = sum_k xq[m,k]*wq[n,k], exact, int32 [M,N]; raises on int32 overflow."""
    xq, wq = _check_codes(xq, wq)
    M, K = xq.shape
    N = wq.shape[0]
    acc = np.empty((M, N), dtype=np.int32)
    bad = _clib().oracle_igemm(_ptr(xq, ctypes.c_int8), _ptr(wq, ctypes.c_int8), M, N, K,
                               _ptr(acc, ctypes.c_int32))
    if bad:
        raise OverflowError(f"{bad} accumulators do not fit int32")
    return acc


def igemm_grouped(xq: np.ndarray, q: np.ndarray, sw: np.ndarray, group: int,
                  want_partials: bool = False):
    """Group-wise integer GEMM for 4-bit weights.

    q [N,K] sign-extended codes, sw [N,K/group] group scales (any float dtype;
    widened exactly to fp64).  Returns (accf float64 [M,N], total int32 [M,N],
    partials int32 [M,K/group,N] or None).
    """
    xq, q = _check_codes(xq, q)
    M, K = xq.shape
    N = q.shape[0]
    if group <= 0 or K % group:
        raise ValueError("group must divide K")
    G = K // group
    sw64 = np.ascontiguousarray(sw.astype(np.float64))
    if sw64.shape != (N, G):
        raise ValueError("sw must be [N, K/group]")
    accf = np.empty((M, N), dtype=np.float64)
    total = np.empty((M, N), dtype=np.int32)
    part = np.empty((M, G, N), dtype=np.int32) if want_partials else None
    pp = _ptr(part, ctypes.c_int32) if want_partials else ctypes.POINTER(ctypes.c_int32)()
    bad = _clib().oracle_igemm_grouped(_ptr(xq, ctypes.c_int8), _ptr(q, ctypes.c_int8),
                                       _ptr(sw64, ctypes.c_double), M, N, K, group,
                                       _ptr(accf, ctypes.c_double), _ptr(total, ctypes.c_int32), pp)
    if bad:
        raise OverflowError(f"{bad} accumulators do not fit int32")
    return accf, total, part


def _finish(y64: np.ndarray, bias16):
    if bias16 is not None:
        y64 = y64 + bias16.astype(np.float64)[None, :]
    return y64, y64.astype(np.float16)          # a single round-to-nearest-even to fp16


def linear_w8a8(x16, wq, sw, bias16=None, xq=None, sx=None):
    """W8A8 linear layer.  x16 fp16 [M,K]; wq int8 [N,K]; sw float32 [N].

    Pre-quantized activations (xq, sx) may be given instead of x16.
    Returns dict(xq, sx, acc, y64, y16).
    """
    if xq is None:
        xq, sx = quant_act_per_token(x16)
    acc = igemm(xq, wq)
    y64 = acc.astype(np.float64) * sx.astype(np.float64)[:, None] * sw.astype(np.float64)[None, :]
    y64, y16 = _finish(y64, bias16)
    return dict(xq=xq, sx=sx, acc=acc, y64=y64, y16=y16)


def linear_w4a8(x16, packed, sw16, group=128, bias16=None, xq=None, sx=None,
                want_partials=False):
    """W4A8 linear layer.  packed uint8 [N,K/2]; sw16 float16 [N,K/group].

    Returns dict(xq, sx, acc (sum over groups), partials, y64, y16).
    """
    if xq is None:
        xq, sx = quant_act_per_token(x16)
    q = unpack_int4(packed)
    accf, total, part = igemm_grouped(xq, q, sw16, group, want_partials)
    y64 = accf * sx.astype(np.float64)[:, None]
    y64, y16 = _finish(y64, bias16)
    return dict(xq=xq, sx=sx, acc=total, partials=part, y64=y64, y16=y16)
