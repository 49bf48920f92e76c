"""The library only enqueues kernels on the caller's stream (no allocation, no synchronization, no memset nodes),
so its calls can be captured into a HIP graph.  Each case is captured once after an eager warm-up call (the first
launch of a kernel configuration sets a function attribute, which is not a stream operation) and replayed several
times with eager work and synchronizations in between; every replay must reproduce the eager result bit for bit."""
import numpy as np
import pytest

from paper_2512_23367_amd import binding as ql, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    from tests import gpu_util
    return gpu_util


def _replay_and_compare(torch, enqueue, outputs):
    """enqueue(): the library calls; outputs: tensors they write."""
    enqueue()                                             # eager warm-up + reference
    torch.cuda.synchronize()
    want = [o.clone() for o in outputs]
    side = torch.cuda.Stream()                            # default priority
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for o in outputs:
            o.zero_()
        with torch.cuda.graph(graph, stream=side):
            enqueue()
    torch.cuda.synchronize()
    for rep in range(3):
        for o in outputs:
            o.fill_(-1 if o.dtype == torch.int8 else 7)   # eager work between replays: poison the outputs
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, w in zip(outputs, want):
            assert torch.equal(o.view(torch.uint8), w.view(torch.uint8)), f"replay {rep} differs from the eager run"


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,K,N", [(300, 1536, 520),      # prefill tile kernels
                                   (128, 11008, 512),     # split-K: two kernels, partial sums in the workspace
                                   (2, 4096, 520),        # decode with the quantizer fused into the GEMM
                                   (8, 4096, 520),        # decode behind the separate quantizer
                                   (24, 1536, 4608),      # decode, 17..32 tokens
                                   (64, 4096, 520),       # decode kernels on token blocks (33 tokens and more)
                                   (200, 2048, 1000)])    # the same, several blocks
def test_linear_layer_in_a_graph(G, bits, M, K, N):
    import torch
    x = G.dev(synth.activations(M, K, 0, "single"))
    g = G.gpu_quant_weight(synth.weights(N, K, 0, "single"), bits, 0 if bits == 8 else 128)
    b = G.dev(synth.bias(N, 0, "single"))
    y = torch.zeros((M, N), dtype=torch.float16, device="cuda:0")
    ws = G.empty_bytes(ql.ql_workspace_bytes(M, N, K, bits))

    def enqueue():
        if bits == 8:
            ql.ql_w8a8_linear(x, g["kernel"], g["scales_dev"].view(torch.float32), b, N, y, ws)
        else:
            ql.ql_w4a8_linear(x, g["kernel"], 128, b, N, y, ws)
    _replay_and_compare(torch, enqueue, [y])


def test_quantizers_in_a_graph(G):
    """The per-tensor quantizer clears its 4-byte scratch with a one-thread kernel, not a memset node."""
    import torch
    M, K = 100, 1536
    x = G.dev(synth.activations(M, K, 1, "single"))
    xq = torch.zeros((M, K), dtype=torch.int8, device="cuda:0")
    xk = G.empty_bytes(ql.ql_act_kernel_bytes(M, K))
    xk.zero_()
    sx = torch.zeros(M, dtype=torch.float32, device="cuda:0")
    xq2 = torch.zeros((M, K), dtype=torch.int8, device="cuda:0")
    sx2 = torch.zeros(M, dtype=torch.float32, device="cuda:0")
    xq3 = torch.zeros((M, K), dtype=torch.int8, device="cuda:0")
    sx3 = torch.zeros(M, dtype=torch.float32, device="cuda:0")
    scratch = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    B = ql.ql_hadamard_block(K)
    xq4 = torch.zeros((M, K), dtype=torch.int8, device="cuda:0")
    sx4 = torch.zeros(M, dtype=torch.float32, device="cuda:0")
    gamma = torch.full((K,), 0.75, dtype=torch.float16, device="cuda:0")

    def enqueue():
        ql.ql_quant_act_per_token(x, xq, xk, sx)
        ql.ql_quant_act_opt(x, ql.QL_RANGE_EQ2, ql.QL_SCOPE_TENSOR, None, xq2, None, sx2, scratch)
        ql.ql_quant_act_per_token_transformed(x, None, B, xq3, None, sx3)
        ql.ql_quant_act_rmsnorm(x, gamma, 1e-6, xq4, None, sx4)
    _replay_and_compare(torch, enqueue, [xq, sx, xq2, sx2, xq3, sx3, xq4, sx4])


def test_static_workspace_linear_and_swiglu_in_a_graph(G):
    """The entry point for callers that cannot allocate is the one a graph-capturing caller would use: captured after
    one eager call (which looks up the static workspace's device address), every replay reproduces the eager result.
    The SwiGLU quantizer in front of a GEMM goes through the same check."""
    import torch
    M, K, N, F = 300, 1536, 520, 512
    x = G.dev(synth.activations(M, K, 0, "single"))
    g = G.gpu_quant_weight(synth.weights(N, K, 0, "single"), 8, 0)
    b = G.dev(synth.bias(N, 0, "single"))
    y = torch.zeros((M, N), dtype=torch.float16, device="cuda:0")
    gu = G.dev(synth.activations(M, 2 * F, 1, "single"))
    gd = G.gpu_quant_weight(synth.weights(N, F, 1, "single"), 8, 0)
    xk = G.empty_bytes(ql.ql_act_kernel_bytes(M, F))
    sx = torch.zeros(M, dtype=torch.float32, device="cuda:0")
    y2 = torch.zeros((M, N), dtype=torch.float16, device="cuda:0")

    def enqueue():
        ql.ql_w8a8_linear_static(x, g["kernel"], g["scales_dev"].view(torch.float32), b, N, y)
        ql.ql_quant_act_swiglu(gu, None, xk, sx)
        ql.ql_w8a8_gemm(xk, sx, M, F, gd["kernel"], gd["scales_dev"].view(torch.float32), None, N, y2)
    _replay_and_compare(torch, enqueue, [y, sx, y2])
