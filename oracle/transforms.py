"""Oracle for the two outlier-mitigation transforms of the paper's W4A8 variants -- test infrastructure.

SmoothQuant variant (Eq. 3):  Y = (X S^-1)(S W),  S = diag(s),
    s_j = max|X_j|^alpha / max|W_j|^(1 - alpha)   (alpha = 0.5 in the paper's experiments)
Hadamard variant (Eq. 4):     Y = (X H)(H^T W),   H a normalized Hadamard matrix.

Both leave Y unchanged in exact arithmetic; what changes is what the quantizers (Eq. 1-2) see.  The
transformed operands are fp32 arrays here and go to the same quantizers as the plain ones.

Readings (the paper gives the formulas only):
  * X_j is input channel j of a calibration batch (column j of X[M,K]), W_j the weights that multiply it
    (row j of W in Y = XW, i.e. column j of the stored w[N,K]); a channel whose activation or weight
    maximum is 0 keeps s_j = 1.
  * s is an offline parameter vector in fp32; activations are multiplied by the fp32 reciprocal 1/s_j (one
    IEEE division, done once), weights by s_j -- one fp32 multiply per element, no rounding back to fp16.
  * H is the Sylvester (natural-order) Hadamard matrix.  The paper does not say what happens when K is not a
    power of two; here H is block diagonal, I (x) H_B / sqrt(B), with B the largest power of two that divides
    K, capped at 4096 -- still orthogonal, so Eq. 4 holds.  It is applied as the textbook in-place butterfly
    in fp32, stages h = 1, 2, 4, ..., B/2 in that order ((a, b) -> (a + b, a - b), one addition each), then
    one multiply by fp32(1/sqrt(B)).  With the stage order fixed every result is a fixed sequence of single
    fp32 operations, so an implementation that keeps the order is bit-identical however it assigns the work.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32
MAX_BLOCK = 4096


def channel_absmax(x16: np.ndarray) -> np.ndarray:
    """max|X_j| per input channel of a calibration batch x[M,K] (fp16) -> float32 [K] (exact)."""
    if x16.dtype != np.float16:
        raise TypeError("calibration activations are fp16")
    return np.abs(x16.astype(F32)).max(axis=0) if x16.shape[0] else np.zeros(x16.shape[1], F32)


def smooth_scales(x_absmax: np.ndarray, w16: np.ndarray, alpha: float = 0.5):
    """Eq. 3: s_j = max|X_j|^alpha / max|W_j|^(1-alpha) for w[N,K] (fp16) -> (s, 1/s) float32 [K]."""
    if w16.dtype != np.float16:
        raise TypeError("weights are fp16")
    wmax = np.abs(w16.astype(np.float64)).max(axis=0)
    xmax = x_absmax.astype(np.float64)
    live = (xmax > 0) & (wmax > 0)
    s = np.ones_like(xmax)
    s[live] = xmax[live] ** alpha / wmax[live] ** (1.0 - alpha)
    s = s.astype(F32)
    inv = (F32(1) / s).astype(F32)                        # one fp32 division per channel
    return s, inv


def smooth_act(x16: np.ndarray, inv_s: np.ndarray) -> np.ndarray:
    """X S^-1: one fp32 multiply per element."""
    return (x16.astype(F32) * inv_s.astype(F32)[None, :]).astype(F32)


def smooth_weight(w16: np.ndarray, s: np.ndarray) -> np.ndarray:
    """S W for the stored w[N,K]: column j times s_j, one fp32 multiply per element."""
    return (w16.astype(F32) * s.astype(F32)[None, :]).astype(F32)


def hadamard_block(K: int) -> int:
    """Largest power of two that divides K, capped at MAX_BLOCK."""
    if K <= 0:
        raise ValueError("K must be positive")
    b = K & -K
    return min(b, MAX_BLOCK)


def fwht_blocks(v: np.ndarray, block: int) -> np.ndarray:
    """v[..., K] (fp16 or fp32) times the block-diagonal normalized Hadamard matrix, along the last axis.

    Stages h = 1, 2, ..., block/2 in order, every output one fp32 addition or subtraction of two inputs;
    then one fp32 multiply by fp32(1/sqrt(block)).
    """
    if block < 1 or block & (block - 1):
        raise ValueError("block must be a power of two")
    K = v.shape[-1]
    if K % block:
        raise ValueError("block must divide K")
    a = v.astype(F32).reshape(-1, K // block, block).copy()
    h = 1
    while h < block:
        a = a.reshape(a.shape[0], K // block, block // (2 * h), 2, h)
        lo = a[:, :, :, 0, :] + a[:, :, :, 1, :]          # one fp32 addition
        hi = a[:, :, :, 0, :] - a[:, :, :, 1, :]          # one fp32 subtraction
        a = np.stack([lo, hi], axis=3).reshape(a.shape[0], K // block, block)
        h *= 2
    norm = F32(1.0 / np.sqrt(float(block)))
    return (a * norm).astype(F32).reshape(v.shape)


def rmsnorm_act(x16: np.ndarray, gamma16: np.ndarray, eps: float) -> np.ndarray:
    """RMSNorm in front of the activation quantizer (the pre-normalisation of the decoder layers the quantized
    linears sit in; the paper does not spell it out -- this is the textbook definition, Zhang & Sennrich 2019):
        h_k = x_k / sqrt(mean_k(x^2) + eps) * gamma_k
    Reading, one correctly rounded fp32 operation per step, so that a fused kernel can be bit-identical:
        ss   = fp32(fp64(sum_k x_k^2))    the exact sum (every square of an fp16 value is exact) rounded to fp64
                                          (math.fsum), then to fp32: two roundings, which differ from a single one
                                          only if the fp64 value lands exactly on an fp32 tie
        mean = ss / K                     K as fp32 (exact up to 2^24)
        r    = 1 / sqrt(mean + eps)       one addition, one square root, one division
        h_k  = (x_k * r) * gamma_k        two multiplications, gamma widened from fp16
    The result is an fp32 array that goes to the per-token quantizer like the other transformed activations.
    """
    if x16.dtype != np.float16 or gamma16.dtype != np.float16:
        raise TypeError("activations and gamma are fp16")
    M, K = x16.shape
    if gamma16.shape != (K,):
        raise ValueError("gamma has one entry per feature")
    if not (eps >= 0 and np.isfinite(eps)):
        raise ValueError("eps must be finite and non-negative")
    import math
    x64 = x16.astype(np.float64)
    # exact: squares of fp16 values are exact in fp64 and math.fsum returns the correctly rounded sum of exact terms
    ss = np.array([math.fsum((row * row).tolist()) for row in x64], dtype=np.float64).astype(F32)
    mean = (ss / F32(K)).astype(F32)
    t = (mean + F32(eps)).astype(F32)
    r = (F32(1) / np.sqrt(t).astype(F32)).astype(F32)     # mean + eps == 0: r = inf, the caller must not ask for it
    x = x16.astype(F32)
    h = ((x * r[:, None]).astype(F32) * gamma16.astype(F32)[None, :]).astype(F32)
    return h


# ---- SwiGLU in front of the activation quantizer --------------------------------------------------------------
# The gated MLP of a decoder layer multiplies the two halves of the fused gate+up projection before the down
# projection:  h_j = silu(gate_j) * up_j,  silu(g) = g * sigmoid(g) = g / (1 + exp(-g))   (textbook definition,
# Shazeer 2020; the paper names no activation function).  Reading: fp32 throughout, no rounding of h back to fp16,
# every step ONE correctly rounded fp32 operation so that a fused kernel can be bit-identical -- which needs exp
# itself to be a stated sequence of such operations (library exponentials differ in their last bit):
#     t = clamp(-g, -80, 80)
#     n = rint(t * log2(e))                                  (round half to even)
#     r = (t - n * LN2_HI) - n * LN2_LO                      (two-constant range reduction: |r| <= 0.347)
#     p = 1 + r (1 + r (1/2 + r (1/6 + r (1/24 + r (1/120 + r (1/720 + r / 5040))))))    (Horner, mul then add)
#     exp(t) ~ p * 2^n                                       (exact scaling)
#     h = (g * (1 / (1 + exp(t)))) * u                       (add, divide, two multiplies)
LOG2E = F32(1.4426950408889634)
LN2_HI = F32(0.693359375)                  # 355/512: n * LN2_HI is exact for |n| < 2^15
LN2_LO = F32(-2.12194440e-4)               # ln 2 - LN2_HI
EXP_COEFFS = [F32(1.0 / 5040), F32(1.0 / 720), F32(1.0 / 120), F32(1.0 / 24), F32(1.0 / 6), F32(0.5), F32(1.0), F32(1.0)]


def exp_f32_steps(t: np.ndarray) -> np.ndarray:
    """exp(t) for fp32 t in [-80, 80] by the sequence above (each line one fp32 operation per element)."""
    t = t.astype(F32)
    n = np.rint((t * LOG2E).astype(F32)).astype(F32)
    r = (t - (n * LN2_HI).astype(F32)).astype(F32)
    r = (r - (n * LN2_LO).astype(F32)).astype(F32)
    p = np.full_like(r, EXP_COEFFS[0])
    for c in EXP_COEFFS[1:]:
        p = ((p * r).astype(F32) + c).astype(F32)
    return np.ldexp(p, n.astype(np.int32)).astype(F32)      # times 2^n: exact (results stay normal)


def swiglu_act(gate_up16: np.ndarray) -> np.ndarray:
    """h[M,F] = silu(gate) * up for the fused projection output gate_up[M, 2F] (fp16: gate = columns 0..F-1,
    up = columns F..2F-1), as an fp32 array that goes to the per-token quantizer unrounded."""
    if gate_up16.dtype != np.float16 or gate_up16.ndim != 2 or gate_up16.shape[1] % 2:
        raise TypeError("gate_up is fp16 [M, 2F]")
    F = gate_up16.shape[1] // 2
    g = gate_up16[:, :F].astype(F32)
    u = gate_up16[:, F:].astype(F32)
    t = np.minimum(np.maximum(-g, F32(-80)), F32(80)).astype(F32)
    e = exp_f32_steps(t)
    d = (F32(1) + e).astype(F32)
    sg = (F32(1) / d).astype(F32)
    return ((g * sg).astype(F32) * u).astype(F32)
