"""Pins for the oracle's quantizers (CPU only).

The oracle is checked against things other than itself: hand-derived vectors
(tests/golden/hand_vectors.json), exact rational arithmetic, closed forms and
the round-trip error bound |x - q*s| <= s/2.
"""
import json
import os
import struct
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2512_23367_amd import synth

GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_vectors.json")))


# |x - q*s| <= s/2 holds for exact arithmetic.  In fp32 the quotient/product that is rounded to
# an integer carries a relative error of at most 2 ulp (2^-23) at magnitude <= 127, and the stored
# scale another 2^-24, so the bound is s/2 * (1 + 127*2^-21) at worst; 2^-14 covers it.
SLACK = 2.0 ** -14


def f16(a):
    return np.asarray(a, dtype=np.float64).astype(np.float16)


# ---------------------------------------------------------------- hand vectors
@pytest.mark.parametrize("case", GOLDEN["act_int8"])
def test_act_hand_vectors(case):
    x = f16([case["x"]])
    assert (x.astype(np.float64) == np.asarray([case["x"]])).all(), "inputs must be exact in fp16"
    q, s = oracle.quant_act_per_token(x)
    assert q.dtype == np.int8 and s.dtype == np.float32
    assert q[0].tolist() == case["q"]
    assert s[0] == np.float32(case["scale_num"]) / np.float32(case["scale_den"])
    # the scale is the correctly rounded quotient: nearest fp32 to the exact rational
    exact = Fraction(case["scale_num"]) / Fraction(case["scale_den"])
    ulp = Fraction(np.spacing(s[0]).item())
    assert abs(Fraction(s[0].item()) - exact) <= ulp / 2


def test_act_hand_vectors_in_a_batch_rows_are_independent():
    rows = [c["x"] + [0.0] * (8 - len(c["x"])) for c in GOLDEN["act_int8"]]
    q, _ = oracle.quant_act_per_token(f16(rows))
    for r, c in zip(q, GOLDEN["act_int8"]):
        assert r[: len(c["q"])].tolist() == c["q"]
        assert (r[len(c["q"]):] == 0).all()


@pytest.mark.parametrize("case", GOLDEN["weight_int8"])
def test_weight_int8_hand_vector(case):
    w = f16([np.asarray(case["w_times_64"]) / 64.0])
    q, s = oracle.quant_weight_int8(w)
    assert q[0].tolist() == case["q"]
    assert s[0] == np.float32(case["scale"])


@pytest.mark.parametrize("case", GOLDEN["weight_int4"])
def test_weight_int4_hand_vector(case):
    w = np.zeros((2, 256), dtype=np.float16)
    v = f16(np.asarray(case["w_times_64"]) / 64.0)
    w[0, : len(v)] = v                   # group (0,0)
    w[1, 128 + 3: 128 + 3 + len(v)] = v  # group (1,1), other groups all zero
    packed, q, s = oracle.quant_weight_int4(w, 128)
    assert s.dtype == np.float16 and s.shape == (2, 2)
    assert q[0, : len(v)].tolist() == case["q"]
    assert q[1, 131: 131 + len(v)].tolist() == case["q"]
    assert s[0, 0] == np.float16(case["scale"]) and s[1, 1] == np.float16(case["scale"])
    # all-zero groups: scale 1, codes 0
    assert s[0, 1] == 1 and s[1, 0] == 1
    assert (q[0, 128:] == 0).all() and (q[1, :128] == 0).all()
    assert (oracle.unpack_int4(packed) == q).all()


# -------------------------------------------------------------- nibble packing
def test_nibble_hand_bytes():
    for c in GOLDEN["nibble_pairs"]:
        b = oracle.pack_int4(np.array([[c["lo"], c["hi"]]], dtype=np.int8))
        assert b.shape == (1, 1) and int(b[0, 0]) == int(c["byte"], 16)


def test_nibble_all_bytes_sign_extend():
    allb = np.arange(256, dtype=np.uint8).reshape(256, 1)
    u = oracle.unpack_int4(allb)
    for b in range(256):
        lo, hi = b & 15, b >> 4
        lo = lo - 16 if lo > 7 else lo
        hi = hi - 16 if hi > 7 else hi
        assert u[b].tolist() == [lo, hi]


def test_nibble_pack_unpack_identity_and_order():
    vals = np.arange(-7, 8, dtype=np.int8)
    pairs = np.array([[a, b] for a in vals for b in vals], dtype=np.int8)     # 225 pairs
    assert (oracle.unpack_int4(oracle.pack_int4(pairs)) == pairs).all()
    q = np.array([[1, 2, 3, 4, 5, 6]], dtype=np.int8)                         # even k -> low nibble
    assert oracle.pack_int4(q).tolist() == [[0x21, 0x43, 0x65]]
    with pytest.raises(ValueError):
        oracle.pack_int4(np.array([[8, 0]], dtype=np.int8))


# ------------------------------------------------- exact-arithmetic brute force
def _f32(v: float) -> float:
    return struct.unpack("f", struct.pack("f", v))[0]


def _round_half_even(fr: Fraction) -> int:
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def test_act_codes_against_exact_rationals():
    """q must be the nearest integer (ties to even) of the fp32 product x*inv, where inv
    is the correctly rounded fp32 quotient 127/amax; all of it redone with Fractions."""
    rng = np.random.default_rng(7)
    x = (rng.standard_normal((6, 40)) * 3).astype(np.float16)
    x[2] *= np.float16(0.001)
    x[3, 5] = 60000.0
    q, s = oracle.quant_act_per_token(x)
    for m in range(x.shape[0]):
        amax = max(abs(Fraction(float(v))) for v in x[m])
        inv = Fraction(_f32(float(Fraction(127) / amax)))          # double -> fp32: innocuous double rounding
        assert Fraction(s[m].item()) == Fraction(_f32(float(amax / 127)))
        for k in range(x.shape[1]):
            t = Fraction(_f32(float(Fraction(float(x[m, k])) * inv)))
            want = max(-127, min(127, _round_half_even(t)))
            assert int(q[m, k]) == want, (m, k)


def test_act_codes_near_exact_quotient():
    """Independent of the fp32 op order: every code is within 1/2 + 127*2^-22 of 127*x/amax."""
    x = synth.activations(32, 512, 0, "single")
    q, s = oracle.quant_act_per_token(x)
    x64 = x.astype(np.float64)
    t = 127.0 * x64 / np.abs(x64).max(axis=1, keepdims=True)
    assert np.abs(q - t).max() <= 0.5 + 127 * 2.0 ** -22
    # and the two plausible fp32 forms (x*inv vs x/s) may only differ where t is near a tie
    assert (q == np.rint(t)).mean() > 0.999


# ------------------------------------------------------------ round-trip bound
@pytest.mark.parametrize("shape", [(64, 512), (16, 1536), (4, 11008)])
def test_act_round_trip_bound(shape):
    x = synth.activations(shape[0], shape[1], 0, "single")
    q, s = oracle.quant_act_per_token(x)
    err = np.abs(x.astype(np.float64) - q.astype(np.float64) * s.astype(np.float64)[:, None])
    assert (err <= 0.5 * s.astype(np.float64)[:, None] * (1 + SLACK)).all()
    assert np.abs(q).max(axis=1).min() == 127        # the row maximum always lands on +-127
    assert q.min() >= -127


def test_weight_round_trip_bounds():
    w = synth.weights(48, 512, 0, "single")
    q, s = oracle.quant_weight_int8(w)
    err = np.abs(w.astype(np.float64) - q.astype(np.float64) * s.astype(np.float64)[:, None])
    assert (err <= 0.5 * s.astype(np.float64)[:, None] * (1 + SLACK)).all()
    assert (np.abs(q).max(axis=1) == 127).all()

    packed, q4, s16 = oracle.quant_weight_int4(w, 128)
    assert packed.shape == (48, 256) and s16.shape == (48, 4) and s16.dtype == np.float16
    assert q4.min() >= -7 and q4.max() <= 7
    sfull = np.repeat(s16.astype(np.float64), 128, axis=1)
    err = np.abs(w.astype(np.float64) - q4.astype(np.float64) * sfull)
    assert (err <= 0.5 * sfull * (1 + SLACK)).all()          # no clamping error: |w|/s16 < 7.5
    assert (np.abs(q4.reshape(48, 4, 128)).max(axis=2) == 7).all()


# ---------------------------------------------------------------- closed forms
def test_constant_rows_and_power_of_two_scaling():
    x = f16([[0.37] * 16, [-5.5] * 16])
    x[0, 3] = -x[0, 3]
    q, s = oracle.quant_act_per_token(x)
    assert q[0].tolist() == [127, 127, 127, -127] + [127] * 12
    assert (q[1] == -127).all()

    a = synth.activations(8, 256, 0, "single")
    q1, s1 = oracle.quant_act_per_token(a)
    q2, s2 = oracle.quant_act_per_token((a.astype(np.float32) * np.float32(0.125)).astype(np.float16))
    assert (q1 == q2).all() and (s2 == s1 * np.float32(0.125)).all()


def test_zero_rows_store_scale_one():
    x = np.zeros((3, 32), dtype=np.float16)
    x[1, 4] = 2.0
    q, s = oracle.quant_act_per_token(x)
    assert s[0] == 1 and s[2] == 1 and (q[0] == 0).all() and (q[2] == 0).all()
    assert q[1, 4] == 127 and s[1] == np.float32(2) / np.float32(127)
    qw, sw = oracle.quant_weight_int8(x)
    assert sw[0] == 1 and (qw[0] == 0).all() and qw[1, 4] == 127


def test_int4_scale_underflow_stores_one():
    w = np.zeros((1, 128), dtype=np.float16)
    w[0, 0] = np.float16(6e-8)                  # smallest subnormal: amax/7 rounds to 0 in fp16
    packed, q, s = oracle.quant_weight_int4(w, 128)
    assert s[0, 0] == 1 and (q == 0).all() and (packed == 0).all()


def test_identity_weight():
    w = np.eye(16, dtype=np.float16)
    q, s = oracle.quant_weight_int8(w)
    assert (q == 127 * np.eye(16, dtype=np.int8)).all()
    assert (s == np.float32(1) / np.float32(127)).all()


def test_granularity_axes():
    """Scales are per token (row of x) and per output channel (row of w[N,K]); per group along K."""
    x = np.ones((2, 256), dtype=np.float16)
    x[1] *= 4
    _, s = oracle.quant_act_per_token(x)
    assert s.shape == (2,) and s[1] == 4 * s[0]
    w = np.ones((3, 256), dtype=np.float16)
    w[:, 128:] *= 2
    w[2] *= 8
    _, sw = oracle.quant_weight_int8(w)
    assert sw.shape == (3,) and sw[0] == sw[1] and sw[2] == 8 * sw[0]
    _, _, s4 = oracle.quant_weight_int4(w, 128)
    assert s4.shape == (3, 2) and (s4[:, 1] == 2 * s4[:, 0]).all() and s4[2, 0] == 8 * s4[0, 0]


def test_eq2_literal_mode():
    """The formula as printed: s = 2*amax/(2^n-1); the positive maximum maps to 127.5 -> 128 -> clamp 127,
    the negative maximum to -127.5 -> -128 (tie to even), which the printed range allows."""
    x = f16([[127.5, -127.5, 63.5, 0.0]])             # s = 2*127.5/255 = 1 exactly
    q, s = oracle.quant_eq2_literal(x, 8)
    assert s[0] == 1
    assert q[0].tolist() == [127, -128, 64, 0]
    x4 = f16([[7.5, -7.5, 3.5, 0.0]])                 # s = 2*7.5/15 = 1 exactly
    q4, s4 = oracle.quant_eq2_literal(x4, 4)
    assert s4[0] == 1
    assert q4[0].tolist() == [7, -8, 4, 0]
    _, s1 = oracle.quant_eq2_literal(f16([[1.0, -0.25]]), 8)
    assert s1[0] == np.float32(2) / np.float32(255)
    # against the symmetric reading: same codes except where the wider range bites
    a = synth.activations(16, 512, 0, "single")
    ql, _ = oracle.quant_eq2_literal(a, 8)
    qs, _ = oracle.quant_act_per_token(a)
    assert np.abs(ql.astype(int) - qs.astype(int)).max() <= 1


def test_rejects_non_finite_and_wrong_dtype():
    with pytest.raises(ValueError):
        oracle.quant_act_per_token(f16([[1.0, np.inf]]))
    with pytest.raises(TypeError):
        oracle.quant_act_per_token(np.ones((1, 4), dtype=np.float64))
    # fp32 = operands after the SmoothQuant / Hadamard transforms: same quantizer, same result as the fp16 values
    x = f16([[0.5, -2.0, 1.25, 0.0]])
    a, b = oracle.quant_act_per_token(x), oracle.quant_act_per_token(x.astype(np.float32))
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()
