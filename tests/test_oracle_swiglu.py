"""Pins for the oracle's SwiGLU-in-front-of-the-quantizer (textbook definition h = silu(gate) * up, fp32 step by
step with the exponential as a stated sequence of fp32 operations)."""
import math

import numpy as np
import pytest

import oracle

F32 = np.float32


def test_exponential_sequence_against_the_library_exponential():
    """The step sequence is an exponential: within 2 fp32 ulps of the correctly rounded one over its whole range."""
    t = np.concatenate([np.linspace(-80, 80, 200001), np.array([0.0, -0.0, 1.0, -1.0, 0.5 * math.log(2), 80.0, -80.0])])
    t = t.astype(F32)
    e = oracle.exp_f32_steps(t).astype(np.float64)
    ref = np.exp(t.astype(np.float64))
    assert np.abs(e / ref - 1).max() <= 2.5e-7
    assert oracle.exp_f32_steps(np.zeros(1, F32))[0] == 1.0
    # exact powers of two at multiples of ln 2 up to the rounding of the argument
    assert abs(float(oracle.exp_f32_steps(np.array([math.log(2) * 10], F32))[0]) / 1024 - 1) < 3e-7


def test_hand_values():
    # gate 0 -> sigmoid 1/2, silu 0, whatever up is; and the sign of a zero gate is kept by the product
    gu = np.array([[0.0, 3.0]], dtype=np.float16)
    assert oracle.swiglu_act(gu)[0, 0] == 0.0
    # gate large and positive: exp(-g) vanishes against 1, sigmoid == 1 exactly, h = g * u in one rounding
    gu = np.array([[30.0, 0.3330078125]], dtype=np.float16)
    assert oracle.swiglu_act(gu)[0, 0] == F32(30) * F32(np.float16(0.3330078125))
    # gate large and negative: h = g * u / (1 + e^|g|), tiny and of the sign of -u
    gu = np.array([[-30.0, 2.0]], dtype=np.float16)
    h = float(oracle.swiglu_act(gu)[0, 0])
    assert h < 0 and abs(h / (-60.0 / (1 + math.exp(30.0))) - 1) < 1e-6
    # beyond the clamp nothing overflows
    gu = np.array([[-60000.0, 60000.0, 60000.0, 60000.0]], dtype=np.float16)   # F = 2: gates (-6e4, 6e4), ups (6e4, 6e4)
    h = oracle.swiglu_act(gu)
    assert np.isfinite(h).all() and h[0, 1] == F32(60000) * F32(60000) and abs(h[0, 0]) < 1e-20


def test_against_the_closed_form_in_float64():
    rng = np.random.default_rng(11)
    gu = (rng.standard_normal((64, 2 * 384)) * rng.uniform(0.1, 6, (64, 1))).astype(np.float16)
    h = oracle.swiglu_act(gu).astype(np.float64)
    g, u = gu[:, :384].astype(np.float64), gu[:, 384:].astype(np.float64)
    ref = g / (1 + np.exp(-g)) * u
    assert np.abs(h - ref).max() <= 4e-7 * np.abs(ref).max()
    rel = np.abs(h - ref) / np.maximum(np.abs(ref), 1e-30)
    assert rel[np.abs(ref) > 1e-6].max() <= 6e-7
    assert h.shape == (64, 384)


def test_identities_of_the_sigmoid():
    """silu(g) - silu(-g) = g and silu(g) + silu(-g) = g tanh(g/2): the halves of the tensor are not swapped, the
    sign of the exponent is right, and the gate (not the up half) goes through the sigmoid."""
    g = np.linspace(-12, 12, 97).astype(np.float16)
    one = np.ones_like(g)
    pos = oracle.swiglu_act(np.concatenate([g, one])[None, :]).astype(np.float64)[0]
    neg = oracle.swiglu_act(np.concatenate([-g, one])[None, :]).astype(np.float64)[0]
    g64 = g.astype(np.float64)
    assert np.abs((pos - neg) - g64).max() <= 2e-6
    assert np.abs((pos + neg) - g64 * np.tanh(g64 / 2)).max() <= 2e-6
    # linear in the up half, not in the gate half
    two = oracle.swiglu_act(np.concatenate([g, 2 * one])[None, :])[0]
    assert (two == 2 * oracle.swiglu_act(np.concatenate([g, one])[None, :])[0]).all()
    sw = oracle.swiglu_act(np.concatenate([one, g])[None, :]).astype(np.float64)[0]
    assert np.abs(sw - g64 / (1 + math.exp(-1.0))).max() <= 1e-5


def test_quantized_codes_of_a_hand_example():
    # gates (0, 40), ups (5, 0.25): h = (0, 10) -> amax 10, codes (0, 127), scale 10/127
    gu = np.array([[0.0, 40.0, 5.0, 0.25]], dtype=np.float16)
    q, s = oracle.quant_act_per_token(oracle.swiglu_act(gu))
    assert q.tolist() == [[0, 127]] and s[0] == F32(10) / F32(127)


def test_rejects_wrong_inputs():
    with pytest.raises(TypeError):
        oracle.swiglu_act(np.zeros((2, 4), np.float32))
    with pytest.raises(TypeError):
        oracle.swiglu_act(np.zeros((2, 3), np.float16))
