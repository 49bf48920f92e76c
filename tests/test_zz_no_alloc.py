"""ql_w8a8_linear_static (the entry point that allocates nothing: its workspace is a static device array of the
library) against ql_w8a8_linear with a caller-allocated workspace: same kernels, so the fp16 outputs must agree bit
for bit (and lie within the 1e-3 bar of the oracle), on calls in a row that share the array -- each smaller than the
one before, so stale contents of the larger call lie behind the smaller one's data."""
import ctypes

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


def _both(G, M, K, N, bias):
    x = synth.activations(M, K, 0, "single")
    w = synth.weights(N, K, 0, "single")
    b = synth.bias(N, 0, "single") if bias else None
    g = G.gpu_quant_weight(w, 8, 0)
    y_ref = G.gpu_linear(x, g, b)                      # ql_w8a8_linear, workspace from ql_workspace_bytes
    xd, bd = G.dev(x), (G.dev(b) if bias else None)
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device=G.DEV)
    ql.ql_w8a8_linear_static(xd, g["kernel"], g["scales_dev"].view(torch.float32), bd, N, y)
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    assert (y.view(np.uint16) == y_ref.view(np.uint16)).all(), (M, K, N)
    wq_o, sw_o = oracle.quant_weight_int8(w)
    assert G.norm_err(y, oracle.linear_w8a8(x, wq_o, sw_o, b)["y64"]) <= TOL


def test_static_workspace_matches_caller_workspace_on_consecutive_calls(G):
    # split-K candidates (few tiles, long K), tile kernels, blocked decode kernels, decode with and without the
    # quantizer fused in: every family that touches the workspace, largest first
    for M, K, N, bias in [(300, 4096, 520, True), (200, 11008, 136, False), (100, 1536, 264, True),
                          (40, 512, 72, False), (8, 4096, 200, True), (1, 4096, 520, False)]:
        _both(G, M, K, N, bias)


def test_static_workspace_rejects_what_does_not_fit(G):
    vp = ctypes.c_void_p
    lib = ql.lib()
    # 16384 x 11008 int8 activations are 172 MiB: beyond the static array; nothing is launched
    assert lib.ql_w8a8_linear_static(vp(0x1000), 11008, 16384, 11008, vp(0x2000), vp(0x3000), None, 4096,
                                     vp(0x4000), 4096, None) == 5
    assert "ql_w8a8_linear_static" in ql.ql_last_error()
    # M == 0 stays a no-op
    assert lib.ql_w8a8_linear_static(None, 128, 0, 128, None, None, None, 64, None, 64, None) == 0
