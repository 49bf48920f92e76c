"""Pins for the oracle's RMSNorm-in-front-of-the-quantizer (textbook definition, fp32 step by step)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle

F32 = np.float32


def test_hand_example():
    # x = (3, 4, 0, 0): sum of squares 25, mean 6.25, sqrt 2.5, r = 0.4 (fp32), gamma = (1, 0.5, 2, 1)
    x = np.array([[3, 4, 0, 0]], dtype=np.float16)
    g = np.array([1, 0.5, 2, 1], dtype=np.float16)
    h = oracle.rmsnorm_act(x, g, 0.0)
    r = F32(1) / F32(2.5)
    assert h.dtype == np.float32
    assert h[0, 0] == F32(3) * r and h[0, 1] == (F32(4) * r) * F32(0.5) and h[0, 2] == 0 and h[0, 3] == 0
    # quantized: amax = |h0| = 1.2, codes 127 and round(0.8 / 1.2 * 127) = 85
    q, s = oracle.quant_act_per_token(h)
    assert q.tolist() == [[127, 85, 0, 0]] and s[0] == h[0, 0] / F32(127)


def test_unit_gamma_gives_unit_mean_square():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((7, 512)) * rng.uniform(0.01, 30, (7, 1))).astype(np.float16)
    h = oracle.rmsnorm_act(x, np.ones(512, np.float16), 0.0).astype(np.float64)
    assert np.allclose((h * h).mean(axis=1), 1.0, rtol=2e-6)


def test_scale_invariance_and_sign():
    """RMSNorm forgets the scale of a token (eps = 0): a power-of-two multiple of x gives bit-identical h."""
    rng = np.random.default_rng(4)
    x = rng.standard_normal((5, 256)).astype(np.float16)
    g = rng.uniform(0.5, 1.5, 256).astype(np.float16)
    h1 = oracle.rmsnorm_act(x, g, 0.0)
    h4 = oracle.rmsnorm_act((x.astype(np.float32) * 4).astype(np.float16), g, 0.0)
    assert (h1.view(np.uint32) == h4.view(np.uint32)).all()
    hn = oracle.rmsnorm_act(-x, g, 0.0)
    assert (hn == -h1).all()


def test_sum_of_squares_is_the_exactly_rounded_one():
    """One large square and many small ones: a float32 running sum loses the small ones, the oracle must not."""
    x = np.zeros((1, 4096), dtype=np.float16)
    x[0, 0] = 64.0
    x[0, 1:] = 2.0 ** -7                   # 4095 squares of 2^-14 (each below half an ulp of 4096) against 4096
    exact = Fraction(64) ** 2 + 4095 * Fraction(1, 2 ** 14)
    ss = F32(float(exact))                  # float(Fraction) is correctly rounded to fp64, then to fp32: no double-rounding issue here
    mean = ss / F32(4096)
    r = F32(1) / np.sqrt(mean + F32(0))
    h = oracle.rmsnorm_act(x, np.ones(4096, np.float16), 0.0)
    assert h[0, 0] == F32(64) * r
    naive = np.float32(0)
    for v in x[0].astype(np.float32):
        naive = np.float32(naive + v * v)
    assert naive != ss                      # the pin bites: a sequential fp32 sum differs


def test_eps_dominates_tiny_tokens():
    x = np.full((1, 64), 2.0 ** -14, dtype=np.float16)
    h = oracle.rmsnorm_act(x, np.ones(64, np.float16), 1.0)
    # mean = 2^-28, mean + 1 rounds to 1 in fp32, r = 1: h = x
    assert (h == x.astype(np.float32)).all()


def test_against_float64_formula():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((16, 1536)) * 3).astype(np.float16)
    g = rng.uniform(-2, 2, 1536).astype(np.float16)
    eps = 1e-5
    h = oracle.rmsnorm_act(x, g, eps)
    x64 = x.astype(np.float64)
    ref = x64 / np.sqrt((x64 * x64).mean(axis=1, keepdims=True) + eps) * g.astype(np.float64)
    assert np.abs(h - ref).max() <= 4e-7 * np.abs(ref).max()


def test_argument_checks():
    with pytest.raises(TypeError):
        oracle.rmsnorm_act(np.zeros((1, 4), np.float32), np.ones(4, np.float16), 0.0)
    with pytest.raises(ValueError):
        oracle.rmsnorm_act(np.zeros((1, 4), np.float16), np.ones(5, np.float16), 0.0)
    with pytest.raises(ValueError):
        oracle.rmsnorm_act(np.zeros((1, 4), np.float16), np.ones(4, np.float16), -1.0)
