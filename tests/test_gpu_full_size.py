"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The GPU computes the whole layer; the oracle recomputes a stratified sample of token rows (rows are
independent under per-token quantization): the first and last row of every 256-row tile plus seeded
random rows, all N columns.  Checked per shape:
  * weights quantized on the GPU against the oracle's own quantization of the same fp16 weights, in full, bit
    for bit (codes and scales);
  * activation codes and scales of the sampled rows, bit for bit;
  * the raw int32 accumulators of the full-size GEMM (the accumulator hook runs the same main loop, tile order
    and kernel choice as the fp16 call) on the sampled rows, bit for bit -- for int4 weights the sums over the
    groups and, for a window of rows that straddles a token-tile edge, every group partial;
  * the fp16 output of the sampled rows within 1e-3 (max-abs error normalised by the largest reference value).
The oracle works from its own quantized weights throughout; nothing it consumes comes from the GPU.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_23367_amd import binding as ql
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


def _scratch_bytes(sh):
    """The split-K scratch a ql_*_linear call of this shape hands to its GEMM: what ql_workspace_bytes reports
    beyond the quantized activations and their scales."""
    up = lambda n: (n + 255) // 256 * 256
    return ql.ql_workspace_bytes(sh.M, sh.N, sh.K, sh.bits) - up(ql.ql_act_kernel_bytes(sh.M, sh.K)) - up(4 * sh.M)


def _check_shape(G, sh):
    x, w, b = synth.tensors(sh)
    g = G.gpu_quant_weight(w, sh.bits, sh.group, check=False)     # compared in full right below
    if sh.bits == 8:
        wq_o, sw_o = oracle.quant_weight_int8(w)
        assert (g["canon"] == wq_o).all() and (g["scales"].view(np.uint32) == sw_o.view(np.uint32)).all()
    else:
        wq_o, _, sw_o = oracle.quant_weight_int4(w, sh.group)
        assert (g["canon"] == wq_o).all() and (g["scales"].view(np.uint16) == sw_o.view(np.uint16)).all()
    y = G.gpu_linear(x, g, b)
    rows = _sample_rows(sh.M, sh.K + sh.N)
    if sh.bits == 8:
        ref = oracle.linear_w8a8(x[rows], wq_o, sw_o, b)
    else:
        ref = oracle.linear_w4a8(x[rows], wq_o, sw_o, sh.group, b)
    assert np.isfinite(y).all()
    # normalise by the largest magnitude of the sampled reference rows
    assert G.norm_err(y[rows], ref["y64"]) <= TOL, sh.name
    # activation codes of the sampled rows, bit-exact
    xq_g, sx_g, _ = G.gpu_quant_act(x[rows])
    assert (xq_g == ref["xq"]).all() and (sx_g.view(np.uint32) == ref["sx"].view(np.uint32)).all()

    # integer accumulators of the full problem: the GPU quantizes all tokens (bit-checked on the sampled rows
    # above), the accumulator hook multiplies them with the same kernel choice as the fp16 call
    xd = G.dev(x)
    xk = G.empty_bytes(ql.ql_act_kernel_bytes(sh.M, sh.K))
    sx = torch.empty(sh.M, dtype=torch.float32, device=G.DEV)
    ql.ql_quant_act_per_token(xd, None, xk, sx)
    acc = torch.full((sh.M, sh.N), -12345, dtype=torch.int32, device=G.DEV)
    scratch = _scratch_bytes(sh)
    ws = G.empty_bytes(scratch) if scratch > 0 else None
    rows_d = torch.from_numpy(rows).to(G.DEV)
    if sh.bits == 8:
        ql.ql_w8a8_gemm_acc_i32(xk, sh.M, sh.K, g["kernel"], sh.N, acc, ws)
        torch.cuda.synchronize()
        assert (acc[rows_d].cpu().numpy() == ref["acc"]).all(), sh.name
    else:
        # totals first (split-K allowed, as in the fp16 call), then the group partials of a row window across the
        # first 128-token tile edge (the partials dump takes the unsplit kernel)
        ql.ql_w4a8_gemm_acc_i32(xk, sh.M, sh.K, g["kernel"], sh.group, sh.N, acc, None, 0, 0, ws)
        torch.cuda.synchronize()
        assert (acc[rows_d].cpu().numpy() == ref["acc"]).all(), sh.name
        row0 = max(0, min(sh.M - 8, 124))
        nrows = min(8, sh.M)
        G_ = sh.K // sh.group
        part = torch.full((nrows, G_, sh.N), -12345, dtype=torch.int32, device=G.DEV)
        acc.fill_(-12345)
        ql.ql_w4a8_gemm_acc_i32(xk, sh.M, sh.K, g["kernel"], sh.group, sh.N, acc, part, row0, nrows, None)
        torch.cuda.synchronize()
        xq_w, _ = oracle.quant_act_per_token(x[row0:row0 + nrows])
        _, total, part_o = oracle.igemm_grouped(xq_w, oracle.unpack_int4(wq_o), sw_o, sh.group, want_partials=True)
        assert (part.cpu().numpy() == part_o).all(), sh.name
        assert (acc[row0:row0 + nrows].cpu().numpy() == total).all(), sh.name
        assert (acc[rows_d].cpu().numpy() == ref["acc"]).all(), sh.name


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
    """64 and 256 tokens on the 7B shapes: the automatic choice between the decode kernels on token blocks and
    the tile kernels (split-K included), every sampled row against the oracle."""
    _check_shape(G, sh)


def test_config4_long_prefill(G):
    """M=16384 down projection (64 token tiles, several passes over the CUs, every XCD's share of the tile order):
    accumulators of the sampled rows bit-exact, fp16 layer within tolerance."""
    sh = [s for s in synth.workload(4) if s.M > 32][0]
    _check_shape(G, sh)


def test_7b_down_projection_input_through_swiglu(G):
    """SwiGLU + quantizer at the size of the 7B layer's down-projection input (4096 tokens x 11008 features from a
    4096 x 22016 gate+up output): codes and scales of sampled tokens bit-exact against the oracle (tokens are
    independent), the whole tile-order copy consistent with the row-major one."""
    from test_gpu_swiglu import _gate_up
    M, F = 4096, 11008
    gu = _gate_up(M, F, 5)
    rows = _sample_rows(M, F)
    xq_o, sx_o = oracle.quant_act_per_token(oracle.swiglu_act(gu[rows]))
    d = G.dev(gu)
    xq = torch.empty((M, F), dtype=torch.int8, device=G.DEV)
    sx = torch.empty((M,), dtype=torch.float32, device=G.DEV)
    xk = G.empty_bytes(ql.ql_act_kernel_bytes(M, F))
    ql.ql_quant_act_swiglu(d, xq, xk, sx)
    xk2 = G.empty_bytes(ql.ql_act_kernel_bytes(M, F))
    ql.ql_act_repack(xq, xk2)
    torch.cuda.synchronize()
    assert (xq.cpu().numpy()[rows] == xq_o).all()
    assert (sx.cpu().numpy()[rows].view(np.uint32) == sx_o.view(np.uint32)).all()
    assert torch.equal(xk, xk2)
