"""Oracle quantizers (numpy, one IEEE fp32 operation per line) -- test infrastructure.

The paper's quantizer (Eq. 1-2) maps X to round(X/s), clamped to the signed
n-bit range, with s taken from max|X|.  The reading used here and in the HIP
path (symmetric setting of the paper's Experimental Setup):

  * s = max|X| / (2^(n-1) - 1), codes clamped to +-(2^(n-1) - 1): +-127 / +-7
  * round = round-half-to-even (np.rint)
  * all scale arithmetic in fp32; the decision "which integer" is taken in
    fp32 on both sides
  * activations (hot path): inv = 127/amax once per token, code = rint(x*inv)
  * weights (offline): code = rint(w / stored_scale), the literal Eq. 1 form
  * an all-zero token / channel / group stores scale 1 and codes 0

Each numpy ufunc call below on float32 arrays is a single correctly rounded
IEEE-754 binary32 operation per element (no fused multiply-add, no reordering).
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


def _as_f32(x16: np.ndarray) -> np.ndarray:
    # fp16 = the layer's own operands; fp32 = operands after one of the paper's transforms (Eq. 3-4)
    if x16.dtype not in (np.float16, np.float32):
        raise TypeError("oracle quantizers take fp16 (or already transformed fp32) input")
    x = x16.astype(F32)                       # exact widening
    if not np.isfinite(x).all():
        raise ValueError("non-finite input: behaviour is unspecified")
    return x


def quant_act_per_token(x16: np.ndarray):
    """Per-token dynamic int8 quantization of activations x[M,K] (fp16).

    Granularity: one scale per token over its whole feature dimension
    (Preliminary, granularity paragraph); quantizer: Eq. 1-2 with n = 8.
    Returns (xq int8 [M,K], sx float32 [M]).
    """
    x = _as_f32(x16)
    amax = np.abs(x).max(axis=1)                          # exact
    zero = amax == 0
    safe = np.where(zero, F32(1), amax)
    sx = np.where(zero, F32(1), safe / F32(127))          # one fp32 division per token
    inv = np.where(zero, F32(0), F32(127) / safe)         # one fp32 division per token
    t = x * inv[:, None]                                  # one fp32 multiply per element
    r = np.rint(t)                                        # round half to even
    r = np.minimum(np.maximum(r, F32(-127)), F32(127))
    return r.astype(np.int8), sx.astype(F32)


def quant_weight_int8(w16: np.ndarray):
    """Per-output-channel symmetric int8 quantization of w[N,K] (fp16), offline.

    One scale per output channel (row n of w[N,K] = column n of W in Y = XW).
    Returns (wq int8 [N,K], sw float32 [N]).
    """
    w = _as_f32(w16)
    amax = np.abs(w).max(axis=1)
    s = amax / F32(127)                                   # fp32 division
    s = np.where(s == 0, F32(1), s).astype(F32)
    t = w / s[:, None]                                    # fp32 division by the stored scale
    r = np.rint(t)
    r = np.minimum(np.maximum(r, F32(-127)), F32(127))
    return r.astype(np.int8), s


def quant_weight_int4(w16: np.ndarray, group: int = 128):
    """Group-wise symmetric int4 quantization of w[N,K] (fp16), offline.

    Fixed-size groups along K, each with its own fp16 scale (group-wise
    granularity).  The code is computed against the *stored* fp16 scale, so
    dequantization uses exactly the scale that produced the code.
    Returns (packed uint8 [N,K/2], q int8 [N,K] in [-7,7], sw float16 [N,K/group]).
    """
    w = _as_f32(w16)
    N, K = w.shape
    if group <= 0 or K % group or group % 2:
        raise ValueError("group must be even and divide K")
    wg = w.reshape(N, K // group, group)
    amax = np.abs(wg).max(axis=2)
    s32 = amax / F32(7)                                   # fp32 division
    s16 = s32.astype(np.float16)                          # round to nearest even
    s16 = np.where(s16 == 0, np.float16(1), s16).astype(np.float16)
    t = wg / s16.astype(F32)[:, :, None]                  # fp32 division by the stored scale
    r = np.rint(t)
    r = np.minimum(np.maximum(r, F32(-7)), F32(7))
    q = r.astype(np.int8).reshape(N, K)
    return pack_int4(q), q, s16


def pack_int4(q: np.ndarray) -> np.ndarray:
    """Two's-complement nibbles, two per byte along K: even k in bits 3:0, odd k in bits 7:4."""
    if q.dtype != np.int8 or q.shape[-1] % 2:
        raise ValueError("pack_int4 takes int8 with an even last dimension")
    if q.min(initial=0) < -8 or q.max(initial=0) > 7:
        raise ValueError("value does not fit a signed nibble")
    u = q.astype(np.uint8) & np.uint8(0xF)
    return (u[..., 0::2] | (u[..., 1::2] << np.uint8(4))).astype(np.uint8)


def unpack_int4(packed: np.ndarray) -> np.ndarray:
    """Inverse of pack_int4: sign-extended int8, last dimension doubled."""
    if packed.dtype != np.uint8:
        raise TypeError("unpack_int4 takes uint8")
    lo = (packed & np.uint8(0xF)).astype(np.int16)
    hi = (packed >> np.uint8(4)).astype(np.int16)
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.int8)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out


def quant_eq2_literal(x16: np.ndarray, n_bits: int):
    """Eq. 2 exactly as printed, one scale per row: s = 2*max|X|/(2^n - 1),
    codes clamped to [-2^(n-1), 2^(n-1) - 1].  Test-only: quantifies how the
    printed formula differs from the symmetric reading used on the hot path.
    Returns (codes int8, s float32).
    """
    x = _as_f32(x16)
    amax = np.abs(x).max(axis=1)
    s = (F32(2) * amax) / F32(2 ** n_bits - 1)
    s = np.where(s == 0, F32(1), s).astype(F32)
    r = np.rint(x / s[:, None])
    lo, hi = F32(-(2 ** (n_bits - 1))), F32(2 ** (n_bits - 1) - 1)
    r = np.minimum(np.maximum(r, lo), hi)
    return r.astype(np.int8), s


# ---------------------------------------------------------------------------------------------
# The other quantizer forms of the paper's Preliminary section: Eq. 2 as printed, per-tensor
# granularity, and a calibrated (static) activation scale (Experimental Setup: scales derived from
# calibration data).  All of them use the literal Eq. 1 form  code = round(X / s)  with the stored
# fp32 scale s (one IEEE fp32 division per element), then the clamp of Eq. 2.

RANGE_SYMMETRIC = 0      # s = amax / (2^(n-1) - 1), codes in +-(2^(n-1) - 1)
RANGE_EQ2 = 1            # s = 2 amax / (2^n - 1),   codes in [-2^(n-1), 2^(n-1) - 1]   (Eq. 2 as printed)
SCOPE_FINE = 0           # per token (activations), per output channel / per group (weights)
SCOPE_TENSOR = 1         # one scale for the whole tensor, from its own abs-max
SCOPE_STATIC = 2         # activations only: one calibrated scale supplied by the caller


def scale_from_amax(amax, n_bits: int, rng: int):
    """fp32 scale(s) of Eq. 2 from abs-max value(s); 0 stays 0 (callers replace it by 1 on use)."""
    amax = np.asarray(amax, dtype=F32)
    if rng == RANGE_SYMMETRIC:
        return (amax / F32(2 ** (n_bits - 1) - 1)).astype(F32)        # one fp32 division
    if rng == RANGE_EQ2:
        return ((F32(2) * amax) / F32(2 ** n_bits - 1)).astype(F32)   # exact doubling, one fp32 division
    raise ValueError("unknown range")


def _limits(n_bits: int, rng: int):
    hi = 2 ** (n_bits - 1) - 1
    return (F32(-hi), F32(hi)) if rng == RANGE_SYMMETRIC else (F32(-hi - 1), F32(hi))


def _codes(x: np.ndarray, s: np.ndarray, n_bits: int, rng: int) -> np.ndarray:
    lo, hi = _limits(n_bits, rng)
    r = np.rint(x / s)                                                # Eq. 1: fp32 division, half to even
    return np.minimum(np.maximum(r, lo), hi).astype(np.int8)          # clamp of Eq. 2


def act_scale_calibrate(batches, rng: int = RANGE_SYMMETRIC) -> np.float32:
    """Calibrated per-tensor activation scale: Eq. 2's s from the largest |x| seen over the batches."""
    amax = F32(0)
    for b in batches:
        amax = max(amax, np.abs(_as_f32(b)).max(initial=F32(0)))
    return F32(scale_from_amax(amax, 8, rng))


def quant_act_opt(x16: np.ndarray, rng: int = RANGE_SYMMETRIC, scope: int = SCOPE_FINE, static_scale=None):
    """int8 activation quantization with the given range / granularity.  Returns (xq int8 [M,K],
    sx float32 [M]): one entry per token whatever the granularity, so the GEMM epilogue is unchanged."""
    x = _as_f32(x16)
    M = x.shape[0]
    if scope == SCOPE_FINE:
        s = scale_from_amax(np.abs(x).max(axis=1), 8, rng)
    elif scope == SCOPE_TENSOR:
        s = np.full(M, scale_from_amax(np.abs(x).max(initial=F32(0)), 8, rng), dtype=F32)
    elif scope == SCOPE_STATIC:
        if static_scale is None or not np.isfinite(static_scale) or static_scale < 0:
            raise ValueError("static scope takes a finite non-negative scale")
        s = np.full(M, F32(static_scale), dtype=F32)
    else:
        raise ValueError("unknown scope")
    s = np.where(s == 0, F32(1), s).astype(F32)
    return _codes(x, s[:, None], 8, rng), s


def quant_weight_opt(w16: np.ndarray, n_bits: int, group: int = 0, rng: int = RANGE_SYMMETRIC,
                     scope: int = SCOPE_FINE):
    """Weight quantization with the given range / granularity.
    n_bits 8: returns (wq int8 [N,K], sw float32 [N]);
    n_bits 4: returns (packed uint8 [N,K/2], q int8 [N,K], sw float16 [N,K/group]) -- the scale is
    rounded to fp16 before the codes are computed, as in quant_weight_int4."""
    w = _as_f32(w16)
    N, K = w.shape
    if scope not in (SCOPE_FINE, SCOPE_TENSOR):
        raise ValueError("weights take fine or per-tensor scope")
    if n_bits == 8:
        amax = np.abs(w).max(axis=1) if scope == SCOPE_FINE else np.full(N, np.abs(w).max(initial=F32(0)), dtype=F32)
        s = scale_from_amax(amax, 8, rng)
        s = np.where(s == 0, F32(1), s).astype(F32)
        return _codes(w, s[:, None], 8, rng), s
    if n_bits != 4 or group <= 0 or K % group or group % 2:
        raise ValueError("4-bit weights take an even group length that divides K")
    wg = w.reshape(N, K // group, group)
    amax = np.abs(wg).max(axis=2) if scope == SCOPE_FINE else \
        np.full((N, K // group), np.abs(w).max(initial=F32(0)), dtype=F32)
    s16 = scale_from_amax(amax, 4, rng).astype(np.float16)            # round to nearest even
    s16 = np.where(s16 == 0, np.float16(1), s16).astype(np.float16)
    q = _codes(wg, s16.astype(F32)[:, :, None], 4, rng).reshape(N, K)
    return pack_int4(q), q, s16
