"""Pins for the oracle's other quantizer forms (paper Preliminary section: Eq. 2 as printed, per-tensor
granularity; Experimental Setup: calibrated scales) -- hand-derived vectors, exact rational arithmetic,
invariants and reductions to the already pinned per-token / per-channel / per-group quantizers."""
import json
import os
import struct
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2512_23367_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))
with open(os.path.join(HERE, "golden", "hand_vectors.json")) as f:
    CASES = json.load(f)["quantizer_options"]["cases"]
RANGE = {"symmetric": oracle.RANGE_SYMMETRIC, "eq2": oracle.RANGE_EQ2}
SCOPE = {"fine": oracle.SCOPE_FINE, "tensor": oracle.SCOPE_TENSOR, "static": oracle.SCOPE_STATIC}


def f16(a):
    return np.array(a, dtype=np.float16)


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_hand_vectors(case):
    rng, scope = RANGE[case["range"]], SCOPE[case["scope"]]
    if case["kind"] == "act":
        x = f16(case["x"])
        assert (x.astype(np.float64) == np.array(case["x"])).all()        # inputs exact in fp16
        q, s = oracle.quant_act_opt(x, rng, scope, case.get("static_scale"))
    elif case["kind"] == "weight8":
        q, s = oracle.quant_weight_opt(f16(case["w"]), 8, 0, rng, scope)
    else:
        packed, q, s = oracle.quant_weight_opt(f16(case["w"]), 4, case["group"], rng, scope)
        assert (oracle.unpack_int4(packed) == q).all()
    assert q.tolist() == case["codes"]
    assert s.astype(np.float64).tolist() == case["scales"]


# ------------------------------------------------------------------ exact rationals
def _f32(v: float) -> float:
    return struct.unpack("f", struct.pack("f", v))[0]


def _round_half_even(fr: Fraction) -> int:
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    return fl + 1 if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1) else fl


def _fdiv32(a: Fraction, b: Fraction) -> Fraction:
    """Correctly rounded fp32 quotient of two fp32 values (the double quotient of two 24-bit significands
    is never close enough to an fp32 rounding boundary for the second rounding to matter)."""
    return Fraction(_f32(float(a / b)))


@pytest.mark.parametrize("rng_name,den,lo,hi", [("symmetric", 127, -127, 127), ("eq2", 255, -128, 127)])
def test_act_codes_against_exact_rationals(rng_name, den, lo, hi):
    g = np.random.default_rng(11)
    x = (g.standard_normal((5, 48)) * 2.5).astype(np.float16)
    x[1] *= np.float16(0.002)
    x[2, 7] = -60000.0
    for scope in ("fine", "tensor"):
        q, s = oracle.quant_act_opt(x, RANGE[rng_name], SCOPE[scope])
        for m in range(x.shape[0]):
            rows = x[m] if scope == "fine" else x
            amax = max(abs(Fraction(float(v))) for v in rows.ravel())
            num = amax * 2 if rng_name == "eq2" else amax
            want_s = _fdiv32(num, Fraction(den))
            assert Fraction(s[m].item()) == want_s
            for k in range(x.shape[1]):
                t = _fdiv32(Fraction(float(x[m, k])), want_s)
                assert int(q[m, k]) == max(lo, min(hi, _round_half_even(t))), (scope, m, k)


@pytest.mark.parametrize("rng_name,den,lo,hi", [("symmetric", 7, -7, 7), ("eq2", 15, -8, 7)])
def test_int4_codes_against_exact_rationals(rng_name, den, lo, hi):
    g = np.random.default_rng(12)
    w = (g.standard_normal((3, 32)) * 0.05).astype(np.float16)
    _, q, s = oracle.quant_weight_opt(w, 4, 16, RANGE[rng_name], oracle.SCOPE_FINE)
    for n in range(3):
        for grp in range(2):
            seg = w[n, grp * 16:(grp + 1) * 16]
            amax = max(abs(Fraction(float(v))) for v in seg)
            s32 = _fdiv32(amax * 2 if rng_name == "eq2" else amax, Fraction(den))
            s16 = Fraction(float(np.float32(float(s32)).astype(np.float16)))   # round to nearest even fp16
            assert Fraction(float(s[n, grp])) == s16
            for k in range(16):
                t = _fdiv32(Fraction(float(seg[k])), s16)
                assert int(q[n, grp * 16 + k]) == max(lo, min(hi, _round_half_even(t)))


# ------------------------------------------------------------------ reductions and invariants
def test_fine_symmetric_weights_reduce_to_the_pinned_quantizers():
    w = synth.weights(24, 256, 0, "single")
    q8, s8 = oracle.quant_weight_opt(w, 8)
    r8, t8 = oracle.quant_weight_int8(w)
    assert (q8 == r8).all() and (s8 == t8).all()
    p4, q4, s4 = oracle.quant_weight_opt(w, 4, 128)
    rp, rq, rs = oracle.quant_weight_int4(w, 128)
    assert (p4 == rp).all() and (q4 == rq).all() and (s4 == rs).all()


def test_fine_symmetric_activations_differ_from_the_hot_path_only_near_ties():
    """The hot path multiplies by the rounded reciprocal, Eq. 1 as printed divides by the scale: the same
    scales, and codes that differ only where the quotient sits within fp32 rounding of a tie."""
    x = synth.activations(64, 512, 0, "single")
    qd, sd = oracle.quant_act_opt(x)
    qm, sm = oracle.quant_act_per_token(x)
    assert (sd == sm).all()
    assert np.abs(qd.astype(int) - qm.astype(int)).max() <= 1
    assert (qd == qm).mean() > 0.999


def test_eq2_fine_reduces_to_the_printed_formula_row_by_row():
    x = synth.activations(16, 256, 0, "single")
    q, s = oracle.quant_act_opt(x, oracle.RANGE_EQ2)
    for m in range(16):
        amax = np.float32(np.abs(x[m].astype(np.float32)).max())
        sm = np.float32(np.float32(2) * amax) / np.float32(255)
        assert s[m] == sm
        want = np.clip(np.rint(x[m].astype(np.float32) / sm), -128, 127)
        assert (q[m] == want).all()


def test_tensor_scope_is_the_fine_scope_of_the_flattened_tensor():
    x = synth.activations(8, 128, 1, "single")
    for rng in (oracle.RANGE_SYMMETRIC, oracle.RANGE_EQ2):
        qt, st = oracle.quant_act_opt(x, rng, oracle.SCOPE_TENSOR)
        qf, sf = oracle.quant_act_opt(x.reshape(1, -1), rng, oracle.SCOPE_FINE)
        assert (st == sf[0]).all() and (qt.reshape(1, -1) == qf).all()
        qw, sw = oracle.quant_weight_opt(x, 8, 0, rng, oracle.SCOPE_TENSOR)
        assert (qw == qt).all() and (sw == st).all()


def test_static_scale_equal_to_the_dynamic_one_reproduces_it_and_calibration_is_the_running_max():
    a = synth.activations(8, 128, 2, "single")
    b = (a.astype(np.float32) * 0.5).astype(np.float16)
    for rng in (oracle.RANGE_SYMMETRIC, oracle.RANGE_EQ2):
        s = oracle.act_scale_calibrate([b, a, b], rng)
        _, st = oracle.quant_act_opt(a, rng, oracle.SCOPE_TENSOR)
        assert s == st[0]
        qs, ss = oracle.quant_act_opt(a, rng, oracle.SCOPE_STATIC, s)
        qt, _ = oracle.quant_act_opt(a, rng, oracle.SCOPE_TENSOR)
        assert (qs == qt).all() and (ss == s).all()
        assert oracle.act_scale_calibrate([a], rng) == oracle.act_scale_calibrate([a, a], rng)


def test_round_trip_error_bounds():
    x = synth.activations(32, 512, 3, "single")
    x32 = x.astype(np.float64)
    for rng, lo_extra in ((oracle.RANGE_SYMMETRIC, 0.0), (oracle.RANGE_EQ2, 0.0)):
        for scope in (oracle.SCOPE_FINE, oracle.SCOPE_TENSOR):
            q, s = oracle.quant_act_opt(x, rng, scope)
            err = np.abs(q * s[:, None].astype(np.float64) - x32)
            # unclamped codes are within half a step (+ fp32 rounding); Eq. 2 as printed clamps +127.5 to 127:
            # its positive extreme is off by exactly half a step as well
            assert (err <= s[:, None] * (0.5 + 1e-4)).all()
    # a static scale four times too small clamps: the error of the clamped elements is what is left over
    q, s = oracle.quant_act_opt(x, oracle.RANGE_SYMMETRIC, oracle.SCOPE_STATIC,
                                oracle.act_scale_calibrate([x]) / np.float32(4))
    big = np.abs(x32) > 127 * float(s[0])
    assert big.any() and (np.abs(q[big]) == 127).all()
    assert (np.abs(q * float(s[0]) - x32)[~big] <= float(s[0]) * (0.5 + 1e-4)).all()


def test_eq2_uses_the_extra_negative_code_and_a_finer_step():
    x = f16([[-255.0, 255.0, 0.5, -0.5]])                   # s = 2 exactly: the extremes sit on +-127.5
    q, s = oracle.quant_act_opt(x, oracle.RANGE_EQ2)
    assert q[0, 0] == -128 and q[0, 1] == 127
    # (with a scale that is not exact the extreme lands within fp32 rounding of -127.5: -128 or -127)
    q1, _ = oracle.quant_act_opt(f16([[-1.0, 1.0]]), oracle.RANGE_EQ2)
    assert q1[0, 0] in (-128, -127) and q1[0, 1] == 127
    _, ss = oracle.quant_act_opt(x, oracle.RANGE_SYMMETRIC)
    assert s[0] < ss[0] and np.isclose(s[0] / ss[0], 254 / 255, rtol=1e-6)


def test_zero_tensors_and_zero_static_scale_store_one():
    z = np.zeros((3, 32), dtype=np.float16)
    for rng in (oracle.RANGE_SYMMETRIC, oracle.RANGE_EQ2):
        for scope in (oracle.SCOPE_FINE, oracle.SCOPE_TENSOR):
            q, s = oracle.quant_act_opt(z, rng, scope)
            assert (q == 0).all() and (s == 1).all()
        q, s = oracle.quant_act_opt(f16([[3.0, -200.0]]), rng, oracle.SCOPE_STATIC, 0.0)
        assert s[0] == 1 and q[0].tolist() == [3, -127 if rng == oracle.RANGE_SYMMETRIC else -128]
        _, q4, s4 = oracle.quant_weight_opt(z, 4, 16, rng, oracle.SCOPE_TENSOR)
        assert (q4 == 0).all() and (s4 == 1).all()


def test_argument_errors():
    x = f16([[1.0, 2.0]])
    with pytest.raises(ValueError):
        oracle.quant_act_opt(x, 7)
    with pytest.raises(ValueError):
        oracle.quant_act_opt(x, oracle.RANGE_EQ2, oracle.SCOPE_STATIC)          # no scale given
    with pytest.raises(ValueError):
        oracle.quant_act_opt(x, oracle.RANGE_EQ2, oracle.SCOPE_STATIC, -1.0)
    with pytest.raises(ValueError):
        oracle.quant_weight_opt(x, 8, 0, oracle.RANGE_EQ2, oracle.SCOPE_STATIC)
    with pytest.raises(ValueError):
        oracle.quant_weight_opt(x, 4, 3)
