"""Pins for the oracle's SmoothQuant (paper Eq. 3) and Hadamard (Eq. 4) transforms: library Hadamard matrices,
exact integer cases, closed forms, the equivalence the paper states, and the effect its Figure 1 shows."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.linalg

import oracle
from paper_2512_23367_amd import synth


# ------------------------------------------------------------------ Hadamard (Eq. 4)
@pytest.mark.parametrize("B", [1, 2, 4, 64, 256])
def test_fwht_is_the_sylvester_hadamard_matrix_exactly_on_integers(B):
    rng = np.random.default_rng(B)
    x = rng.integers(-8, 9, (5, B)).astype(np.float32)
    H = scipy.linalg.hadamard(B).astype(np.float64) if B > 1 else np.ones((1, 1))
    got = oracle.fwht_blocks(x, B).astype(np.float64)
    if int(np.log2(B)) % 2 == 0:          # 1/sqrt(B) is a power of two: every step is exact
        assert (got == x.astype(np.float64) @ H / np.sqrt(B)).all()
    else:
        np.testing.assert_allclose(got, x.astype(np.float64) @ H / np.sqrt(B), rtol=2e-7, atol=0)


def test_fwht_hand_example():
    # H_4 / 2 applied to (1, 2, 3, 4): sums (10, -2, -4, 0) / 2
    got = oracle.fwht_blocks(np.array([[1, 2, 3, 4]], np.float32), 4)
    assert got.tolist() == [[5.0, -1.0, -2.0, 0.0]]
    # a unit vector picks a row of H: e_1 -> (+, -, +, -) / 2
    got = oracle.fwht_blocks(np.array([[0, 1, 0, 0]], np.float32), 4)
    assert got.tolist() == [[0.5, -0.5, 0.5, -0.5]]


def test_fwht_is_block_diagonal_and_orthogonal():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((4, 192)).astype(np.float32)
    B = oracle.hadamard_block(192)
    assert B == 64
    y = oracle.fwht_blocks(x, B)
    for b in range(3):                    # each block only sees its own 64 inputs
        blk = oracle.fwht_blocks(x[:, 64 * b:64 * (b + 1)], 64)
        assert (y[:, 64 * b:64 * (b + 1)] == blk).all()
    # H is symmetric and orthogonal: applying it twice gives the input back (to fp32 rounding), norms are kept
    np.testing.assert_allclose(oracle.fwht_blocks(y, B), x, atol=4e-6)
    np.testing.assert_allclose(np.linalg.norm(y.astype(np.float64), axis=1),
                               np.linalg.norm(x.astype(np.float64), axis=1), rtol=1e-6)
    # involution is exact on small integers when 1/sqrt(B) is a power of two
    xi = rng.integers(-4, 5, (3, 256)).astype(np.float32)
    assert (oracle.fwht_blocks(oracle.fwht_blocks(xi, 256), 256) == xi).all()


def test_fwht_matches_float64_matrix_product_on_real_inputs():
    x = synth.activations(16, 4096, 1, "qkv")
    H = scipy.linalg.hadamard(4096).astype(np.float64) / 64.0
    ref = x.astype(np.float64) @ H
    got = oracle.fwht_blocks(x, 4096).astype(np.float64)
    # 12 stages of fp32 additions on values up to ~1e3
    assert np.abs(got - ref).max() <= 12 * 2.0 ** -24 * np.abs(ref).max() * 4


@pytest.mark.parametrize("K,B", [(4096, 4096), (11008, 256), (1536, 512), (6144, 2048), (512, 512), (192, 64),
                                 (131072, 4096), (8192, 4096), (64, 64)])
def test_hadamard_block(K, B):
    assert oracle.hadamard_block(K) == B
    assert K % B == 0 and (B == 4096 or (K // B) % 2 == 1)


def test_eq4_equivalence_in_full_precision():
    x = synth.activations(24, 1536, 1, "qkv")
    w = synth.weights(40, 1536, 1, "qkv")
    B = oracle.hadamard_block(1536)
    xh = oracle.fwht_blocks(x, B).astype(np.float64)
    wh = oracle.fwht_blocks(w, B).astype(np.float64)         # rows of w[N,K] = columns of W: H^T W
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    np.testing.assert_allclose(xh @ wh.T, ref, atol=2e-5 * np.abs(ref).max())


# ------------------------------------------------------------------ SmoothQuant (Eq. 3)
def test_smooth_scales_hand_example_and_zero_channels():
    xmax = np.array([4.0, 16.0, 0.0, 9.0], np.float32)
    w = np.array([[0.25, -1.0, 0.5, 0.0], [-0.125, 0.25, 0.5, 0.0]], np.float16)   # column maxima .25, 1, .5, 0
    s, inv = oracle.smooth_scales(xmax, w, 0.5)
    assert s.tolist() == [4.0, 4.0, 1.0, 1.0]             # sqrt(4)/sqrt(.25), sqrt(16)/sqrt(1), dead channels 1
    assert inv.tolist() == [0.25, 0.25, 1.0, 1.0]
    s, _ = oracle.smooth_scales(xmax, w, 1.0)             # alpha = 1: all of the activation range moves over
    assert s.tolist() == [4.0, 16.0, 1.0, 1.0]
    s, _ = oracle.smooth_scales(xmax, w, 0.0)
    assert s.tolist() == [4.0, 1.0, 1.0, 1.0]             # 1 / max|W_j|


def test_smooth_scales_against_exact_rationals():
    rng = np.random.default_rng(11)
    xmax = (rng.integers(1, 50, 16) ** 2).astype(np.float32)                # perfect squares
    wcol = (1.0 / rng.integers(1, 9, 16) ** 2).astype(np.float16)           # 1 / perfect squares (exact or not)
    w = np.zeros((3, 16), np.float16)
    w[1] = wcol
    s, _ = oracle.smooth_scales(xmax, w, 0.5)
    for j in range(16):
        exact = np.sqrt(float(xmax[j])) / np.sqrt(float(wcol[j]))
        assert abs(float(s[j]) - exact) <= 2.0 ** -23 * exact
    assert Fraction(float(s[0])) > 0


def test_channel_absmax_and_balanced_ranges():
    x = synth.activations(64, 512, 1, "qkv")
    w = synth.weights(48, 512, 1, "qkv")
    xmax = oracle.channel_absmax(x)
    assert xmax.dtype == np.float32 and (xmax == np.abs(x.astype(np.float64)).max(axis=0)).all()
    s, inv = oracle.smooth_scales(xmax, w, 0.5)
    xs, ws = oracle.smooth_act(x, inv), oracle.smooth_weight(w, s)
    # alpha = 0.5 balances the two sides: after the transform both channel maxima equal sqrt(xmax * wmax)
    wmax = np.abs(w.astype(np.float64)).max(axis=0)
    target = np.sqrt(xmax.astype(np.float64) * wmax)
    np.testing.assert_allclose(np.abs(xs).max(axis=0), target, rtol=1e-6)
    np.testing.assert_allclose(np.abs(ws).max(axis=0), target, rtol=1e-6)


def test_eq3_equivalence_in_full_precision():
    x = synth.activations(24, 512, 1, "qkv")
    w = synth.weights(40, 512, 1, "qkv")
    s, inv = oracle.smooth_scales(oracle.channel_absmax(x), w, 0.5)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    got = oracle.smooth_act(x, inv).astype(np.float64) @ oracle.smooth_weight(w, s).astype(np.float64).T
    np.testing.assert_allclose(got, ref, atol=1e-6 * np.abs(ref).max())


# ------------------------------------------------------------------ what the transforms are for (Figure 1, Table 2)
def _rel(y, ref):
    return np.linalg.norm(y - ref) / np.linalg.norm(ref)


def _errors(x_t, w_t, ref):
    xq, sx = oracle.quant_act_per_token(x_t)
    act_only = _rel((xq.astype(np.float64) * sx[:, None]) @ w_t.astype(np.float64).T, ref)
    q8, s8 = oracle.quant_weight_int8(w_t)
    packed, _, s16 = oracle.quant_weight_int4(w_t, 128)
    return (act_only, _rel(oracle.linear_w8a8(x_t, q8, s8)["y64"], ref),
            _rel(oracle.linear_w4a8(x_t, packed, s16, 128)["y64"], ref))


def test_transforms_flatten_outlier_channels_and_cut_the_quantization_error():
    x = synth.activations(128, 1024, 3, "qkv")            # 1 % of the channels scaled x20
    w = synth.weights(96, 1024, 3, "qkv")
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    base = _errors(x, w, ref)
    peak = lambda a: np.abs(a).max(axis=0).max() / np.median(np.abs(a).max(axis=0))
    # Hadamard: activation channel maxima become uniform
    B = oracle.hadamard_block(1024)
    xh, wh = oracle.fwht_blocks(x, B), oracle.fwht_blocks(w, B)
    assert peak(x.astype(np.float32)) > 10 and peak(xh) < 2.5
    had = _errors(xh, wh, ref)
    # SmoothQuant: the outlier range is shared with the weights
    s, inv = oracle.smooth_scales(oracle.channel_absmax(x), w, 0.5)
    xs, ws = oracle.smooth_act(x, inv), oracle.smooth_weight(w, s)
    assert peak(xs) < peak(x.astype(np.float32)) / 3
    smo = _errors(xs, ws, ref)
    # the outliers hurt the per-token activation quantizer: that error falls by 4-5x, the W8A8 error with it;
    # the W4A8 error is dominated by the int4 weights of these outlier-free Gaussian weights and falls a little
    for t in (had, smo):
        assert t[0] < base[0] / 3 and t[1] < base[1] / 2 and t[2] < base[2]
