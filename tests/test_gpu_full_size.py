"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The GPU computes the whole layer; the oracle recomputes a stratified sample of token rows (rows are
independent under per-token quantization): the first and last row of every 256-row tile plus seeded
random rows, all N columns.  Weights quantized on the GPU are compared bit-for-bit in full.
"""
import numpy as np
import pytest

import oracle
from paper_2512_23367_amd import synth

pytestmark = pytest.mark.gpu
TOL = 1e-3


def _sample_rows(M, seed, extra=24):
    rows = set()
    for t in range(0, M, 256):
        rows.add(t)
        rows.add(min(t + 255, M - 1))
    rng = np.random.default_rng(seed)
    rows.update(int(r) for r in rng.integers(0, M, size=extra))
    rows = sorted(rows)
    if len(rows) > 72:
        keep = rng.choice(len(rows), size=72, replace=False)
        rows = sorted(rows[i] for i in keep)
    return np.array(rows)


def _check_shape(G, sh):
    x, w, b = synth.tensors(sh)
    g = G.gpu_quant_weight(w, sh.bits, sh.group)
    if sh.bits == 8:
        wq_o, sw_o = oracle.quant_weight_int8(w)
        assert (g["canon"] == wq_o).all() and (g["scales"] == sw_o).all()
    else:
        p_o, _, s_o = oracle.quant_weight_int4(w, sh.group)
        assert (g["canon"] == p_o).all() and (g["scales"].view(np.uint16) == s_o.view(np.uint16)).all()
    y = G.gpu_linear(x, g, b)
    rows = _sample_rows(sh.M, sh.K + sh.N)
    if sh.bits == 8:
        ref = oracle.linear_w8a8(x[rows], g["canon"], g["scales"], b)
    else:
        ref = oracle.linear_w4a8(x[rows], g["canon"], g["scales"], sh.group, b)
    assert np.isfinite(y).all()
    # normalise by the largest magnitude of the sampled reference rows
    assert G.norm_err(y[rows], ref["y64"]) <= TOL, sh.name
    # activation codes of the sampled rows, bit-exact
    xq_g, sx_g, _ = G.gpu_quant_act(x[rows])
    assert (xq_g == ref["xq"]).all() and (sx_g == ref["sx"]).all()


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


@pytest.mark.parametrize("sh", synth.workload(1), ids=lambda s: s.name)
def test_config1_1b_prefill_w8a8(G, sh):
    _check_shape(G, sh)


@pytest.mark.parametrize("sh", synth.workload(2), ids=lambda s: s.name)
def test_config2_7b_prefill_w8a8_bias(G, sh):
    _check_shape(G, sh)


@pytest.mark.parametrize("sh", synth.workload(3), ids=lambda s: s.name)
def test_config3_7b_prefill_w4a8(G, sh):
    _check_shape(G, sh)


@pytest.mark.parametrize("sh", [s for s in synth.workload(4) if s.M <= 32], ids=lambda s: s.name)
def test_config4_decode(G, sh):
    _check_shape(G, sh)


def _few_token_shapes():
    out = []
    for s in synth.workload(4):
        if s.M == 1:
            for M in (64, 256):
                out.append(synth.Shape(s.config, s.layer, M, s.K, s.N, s.bits, s.group, s.bias))
    return out


@pytest.mark.parametrize("sh", _few_token_shapes(), ids=lambda s: s.name)
def test_config4_few_tokens(G, sh):
    """64 and 256 tokens on the 7B shapes (the benchmark's few-token detail rows): the automatic choice between
    the decode kernels on token blocks and the tile kernels, every sampled row against the oracle."""
    _check_shape(G, sh)


def test_config4_long_prefill_accumulators(G):
    """M=16384 down projection: integer accumulators of sampled rows, bit-exact, plus the fp16 layer."""
    sh = [s for s in synth.workload(4) if s.M > 32][0]
    _check_shape(G, sh)
