"""GPU: a W8A8 GEMM that the automatic choice runs as two launches on disjoint channel ranges (whole passes over the
CUs first, the remaining channels with the configuration that suits them) gives the results of one launch bit for bit,
and both match the oracle: int32 accumulators exactly, fp16 outputs within 1e-3 (max-abs error normalised by the
largest reference value), with a ragged channel count, a padded output row stride and bias."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_23367_amd import binding as ql
from paper_2512_23367_amd import synth

pytestmark = pytest.mark.gpu
TOL = 1e-3


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _inputs(M, N, K, layer):
    return synth.activations(M, K, 0, layer), synth.weights(N, K, 0, layer), synth.bias(N, 0, layer)


@pytest.mark.parametrize("M,N,K,layer", [(1100, 21767, 2048, "qkv"), (2048, 12289, 2048, "o"), (1500, 18820, 2048, "gate_up")])
def test_two_launches_equal_one_and_the_oracle(G, M, N, K, layer):
    plan = ql.ql_plan_gemm(M, N, K, 8, 0, 0)
    assert plan.rest_channels > 0 and plan.family == ql.QL_FAMILY_TILE, "shape chosen so that the plan splits the channels"
    x, w, b = _inputs(M, N, K, layer)
    g = G.gpu_quant_weight(w, 8, 0, check=False)
    wq_o, sw_o = oracle.quant_weight_int8(w)
    assert (g["canon"] == wq_o).all() and (g["scales"].view(np.uint32) == sw_o.view(np.uint32)).all()
    xd = G.dev(x)
    xk = G.empty_bytes(ql.ql_act_kernel_bytes(M, K))
    sx = torch.empty(M, dtype=torch.float32, device=G.DEV)
    ql.ql_quant_act_per_token(xd, None, xk, sx)
    sw = g["scales_dev"].view(torch.float32)
    bd = G.dev(b)
    ld = (N + 7) // 8 * 8 + 8
    ys, accs = [], []
    try:
        for variant in (0, 2):      # 0: automatic (two launches here), 2: automatic, always one launch
            ql.ql_set_kernel_variant(variant)
            ybuf = torch.full((M, ld), float("nan"), dtype=torch.float16, device=G.DEV)
            ql.ql_w8a8_gemm(xk, sx, M, K, g["kernel"], sw, bd, N, ybuf[:, :N])
            acc = torch.full((M, N), -12345, dtype=torch.int32, device=G.DEV)
            ql.ql_w8a8_gemm_acc_i32(xk, M, K, g["kernel"], N, acc)
            torch.cuda.synchronize()
            assert torch.isnan(ybuf[:, N:]).all(), "nothing written beyond the N channels of a row"
            ys.append(ybuf[:, :N].cpu().numpy())
            accs.append(acc.cpu().numpy())
    finally:
        ql.ql_set_kernel_variant(0)
    assert (ys[0].view(np.uint16) == ys[1].view(np.uint16)).all()
    assert (accs[0] == accs[1]).all()
    rows = np.unique(np.concatenate([[0, 255, 256, M - 1], np.random.default_rng(N).integers(0, M, 20)]))
    ref = oracle.linear_w8a8(x[rows], wq_o, sw_o, b)
    assert (accs[0][rows] == ref["acc"]).all()
    assert G.norm_err(ys[0][rows], ref["y64"]) <= TOL
