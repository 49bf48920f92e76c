"""Pins for the oracle's integer GEMM and dequantization epilogue (CPU only)."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2512_23367_amd import synth

GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_vectors.json")))


def _codes(rng, shape, lim):
    return rng.integers(-lim, lim + 1, size=shape, dtype=np.int8)


def test_igemm_hand_example():
    g = GOLDEN["igemm"]
    acc = oracle.igemm(np.array(g["A"], dtype=np.int8), np.array(g["W"], dtype=np.int8))
    assert acc.dtype == np.int32 and acc.tolist() == g["acc"]


@pytest.mark.parametrize("M,N,K", [(1, 1, 2), (2, 3, 4), (3, 2, 128), (4, 4, 256), (1, 5, 6)])
def test_igemm_brute_force_python_ints(M, N, K):
    rng = np.random.default_rng(M * 1000 + N * 100 + K)
    a, w = _codes(rng, (M, K), 127), _codes(rng, (N, K), 127)
    want = [[sum(int(a[m, k]) * int(w[n, k]) for k in range(K)) for n in range(N)] for m in range(M)]
    assert oracle.igemm(a, w).tolist() == want


def test_igemm_equals_int64_and_exact_float64_products():
    rng = np.random.default_rng(11)
    a, w = _codes(rng, (37, 640), 127), _codes(rng, (53, 640), 127)
    acc = oracle.igemm(a, w)
    assert (acc == a.astype(np.int64) @ w.astype(np.int64).T).all()
    # float64 BLAS is exact here: every partial sum is an integer below 2^53
    assert (acc == a.astype(np.float64) @ w.astype(np.float64).T).all()


def test_igemm_extremes_and_overflow():
    K = 11008
    a = np.full((1, K), 127, dtype=np.int8)
    w = np.stack([np.full(K, 127, dtype=np.int8), np.full(K, -127, dtype=np.int8)])
    v = GOLDEN["extreme_K11008"]["value"]
    assert oracle.igemm(a, w).tolist() == [[v, -v]]
    K = 133145                                    # 133145*127*127 > 2^31 - 1
    with pytest.raises(OverflowError):
        oracle.igemm(np.full((1, K), 127, dtype=np.int8), np.full((1, K), 127, dtype=np.int8))
    K = 133144                                    # largest K that cannot overflow
    assert oracle.igemm(np.full((1, K), 127, dtype=np.int8),
                        np.full((1, K), 127, dtype=np.int8))[0, 0] == K * 127 * 127


def test_igemm_k_permutation_invariance_and_orientation():
    rng = np.random.default_rng(5)
    a, w = _codes(rng, (9, 96), 127), _codes(rng, (7, 96), 127)
    p = rng.permutation(96)
    assert (oracle.igemm(a, w) == oracle.igemm(a[:, p], w[:, p])).all()
    # row n of w is output channel n: a one-hot weight row picks one activation column
    w1 = np.zeros((7, 96), dtype=np.int8)
    for n in range(7):
        w1[n, 10 * n + 1] = 1
    assert (oracle.igemm(a, w1) == a[:, [10 * n + 1 for n in range(7)]]).all()


def test_grouped_partials_sum_and_match_plain():
    rng = np.random.default_rng(3)
    a, q = _codes(rng, (5, 384), 127), _codes(rng, (6, 384), 7)
    sw = (rng.random((6, 3)) + 0.5).astype(np.float16)
    accf, total, part = oracle.igemm_grouped(a, q, sw, 128, want_partials=True)
    assert part.shape == (5, 3, 6)
    assert (total == oracle.igemm(a, q)).all()
    assert (part.sum(axis=1) == total).all()
    for g in range(3):
        assert (part[:, g, :] == oracle.igemm(a[:, 128 * g:128 * (g + 1)], q[:, 128 * g:128 * (g + 1)])).all()
    # accf against exact rationals
    for m in range(5):
        for n in range(6):
            ex = sum(Fraction(int(part[m, g, n])) * Fraction(float(sw[n, g])) for g in range(3))
            assert abs(Fraction(accf[m, n]) - ex) <= abs(ex) * Fraction(1, 2 ** 50) + Fraction(1, 2 ** 60)


def test_epilogue_hand_example():
    g, e = GOLDEN["igemm"], GOLDEN["epilogue_w8a8"]
    r = oracle.linear_w8a8(None, np.array(g["W"], dtype=np.int8), np.array(e["sw"], dtype=np.float32),
                           np.array(e["bias"], dtype=np.float16),
                           xq=np.array(g["A"], dtype=np.int8), sx=np.array(e["sx"], dtype=np.float32))
    assert r["y64"].tolist() == e["y64"]
    assert (r["y16"] == np.array(e["y64"]).astype(np.float16)).all()
    assert r["y16"].dtype == np.float16


def test_identity_weight_reduces_layer_to_dequantized_activations():
    x = synth.activations(8, 64, 0, "single")
    wq, sw = oracle.quant_weight_int8(np.eye(64, dtype=np.float16))
    r = oracle.linear_w8a8(x, wq, sw)
    deq = r["xq"].astype(np.float64) * r["sx"].astype(np.float64)[:, None]
    np.testing.assert_allclose(r["y64"], deq, rtol=2e-7, atol=0)       # 127 * fl(1/127) = 1 - O(2^-24)
    assert np.abs(r["y64"] - x.astype(np.float64)).max() <= 0.5 * r["sx"].max() * 1.001


def test_w4a8_equal_group_scales_reduce_to_single_scale():
    rng = np.random.default_rng(8)
    a, q = _codes(rng, (4, 256), 127), _codes(rng, (3, 256), 7)
    sx = np.array([0.5, 0.25, 2.0, 1.0], dtype=np.float32)
    sw = np.full((3, 2), 0.125, dtype=np.float16)
    r = oracle.linear_w4a8(None, oracle.pack_int4(q), sw, 128, xq=a, sx=sx)
    want = oracle.igemm(a, q).astype(np.float64) * 0.125 * sx.astype(np.float64)[:, None]
    assert (r["y64"] == want).all() and (r["acc"] == oracle.igemm(a, q)).all()


def test_w4a8_group_scales_enter_per_group():
    a = np.ones((1, 256), dtype=np.int8)
    q = np.ones((1, 256), dtype=np.int8)
    sw = np.array([[2.0, 0.5]], dtype=np.float16)
    r = oracle.linear_w4a8(None, oracle.pack_int4(q), sw, 128, bias16=np.array([1.0], dtype=np.float16),
                           xq=a, sx=np.array([0.25], dtype=np.float32))
    assert r["y64"][0, 0] == (128 * 2.0 + 128 * 0.5) * 0.25 + 1.0


@pytest.mark.parametrize("bits", [8, 4])
def test_layer_close_to_fp64_linear(bits):
    """Sanity, not parity: the quantized layer approximates x @ w^T (the paper states no error bound)."""
    sh = synth.workload(0)[0]
    x, w, _ = synth.tensors(sh)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    if bits == 8:
        wq, sw = oracle.quant_weight_int8(w)
        y = oracle.linear_w8a8(x, wq, sw)["y64"]
        lim = 0.05
    else:
        packed, _, s16 = oracle.quant_weight_int4(w, 128)
        y = oracle.linear_w4a8(x, packed, s16, 128)["y64"]
        lim = 0.25
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    assert rel < lim, rel


def test_bias_is_added_per_output_channel_before_rounding():
    a = np.array([[1, 0], [0, 1]], dtype=np.int8)
    w = np.array([[1, 0], [0, 1], [1, 1]], dtype=np.int8)
    r = oracle.linear_w8a8(None, w, np.ones(3, dtype=np.float32), np.array([10, 20, 30], dtype=np.float16),
                           xq=a, sx=np.ones(2, dtype=np.float32))
    assert r["y64"].tolist() == [[11, 20, 31], [10, 21, 31]]
