"""GPU parity of the SwiGLU fused in front of the activation quantizer: codes and scales bit-exact against
oracle.quant_act_per_token(oracle.swiglu_act(.)) (both sides follow the same stated sequence of fp32 operations),
and the down projection fed by it within the fp16 tolerance."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_23367_amd import binding as ql, synth

pytestmark = pytest.mark.gpu
TOL = 1e-3


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _gate_up(M, F, seed):
    """Stand-in for a fused gate+up projection output: N(0, 2) values with a few large ones (both signs) and a row
    of zeros, as fp16."""
    rng = np.random.default_rng(seed)
    gu = (rng.standard_normal((M, 2 * F)) * 2).astype(np.float32)
    gu[:, rng.integers(0, 2 * F, 8)] *= 12
    if M > 2:
        gu[1] = 0
        gu[2, :F] = -gu[2, :F].__abs__() - 20          # all gates far negative: h tiny
    return gu.astype(np.float16)


def gpu_swiglu(G, gu, ld=None):
    M, F2 = gu.shape
    F = F2 // 2
    if ld is None:
        d = G.dev(gu)
    else:
        buf = torch.full((M, ld), float("nan"), dtype=torch.float16, device=G.DEV)
        buf[:, :F2] = G.dev(gu)
        d = buf[:, :F2]
    xq = torch.empty((M, F), dtype=torch.int8, device=G.DEV)
    sx = torch.empty((M,), dtype=torch.float32, device=G.DEV)
    xk = G.empty_bytes(ql.ql_act_kernel_bytes(M, F))
    ql.ql_quant_act_swiglu(d, xq, xk, sx)
    torch.cuda.synchronize()
    return xq.cpu().numpy(), sx.cpu().numpy(), xk, sx


@pytest.mark.parametrize("M,F,ld", [(33, 512, None), (5, 1536, 3080), (64, 4096, None), (3, 11008, None), (2, 64, None),
                                    (7, 6144, None), (1, 16384, None), (40, 192, 392),
                                    (515, 4096, None), (600, 1536, None), (517, 11008, None), (2048, 6144, None)])
def test_swiglu_quantization_bit_exact(G, M, F, ld):
    gu = _gate_up(M, F, M + F)
    xq_o, sx_o = oracle.quant_act_per_token(oracle.swiglu_act(gu))
    xq, sx, xk, _ = gpu_swiglu(G, gu, ld)
    assert (sx.view(np.uint32) == sx_o.view(np.uint32)).all()
    assert (xq == xq_o).all()
    # the tile-order copy holds the same codes (bytes of rows >= M are never written)
    Mp = (M + 31) // 32 * 32
    idx = np.arange(Mp * F)
    valid = (idx // 1024 // (F // 32)) * 32 + (idx % 1024 // 16) % 32 < M
    assert (G.repack_act(xq_o).cpu().numpy()[valid] == xk.cpu().numpy()[valid]).all()


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M", [8, 300])
def test_down_projection_behind_swiglu(G, bits, M):
    """gate_up -> SwiGLU + quantizer -> GEMM of the down projection, against the oracle's chain."""
    F, N = 1536, 520
    gu = _gate_up(M, F, 7 * M + bits)
    w = synth.weights(N, F, 0, "single")
    b = synth.bias(N, 0, "single")
    g = G.gpu_quant_weight(w, bits, 0 if bits == 8 else 128)
    h = oracle.swiglu_act(gu)
    xq_o, sx_o = oracle.quant_act_per_token(h)
    if bits == 8:
        wq_o, sw_o = oracle.quant_weight_int8(w)
        acc = oracle.igemm(xq_o, wq_o)
        ref = acc.astype(np.float64) * sx_o.astype(np.float64)[:, None] * sw_o.astype(np.float64)[None, :] + b.astype(np.float64)
    else:
        p_o, _, s_o = oracle.quant_weight_int4(w, 128)
        accf, _, _ = oracle.igemm_grouped(xq_o, oracle.unpack_int4(p_o), s_o, 128)
        ref = accf * sx_o.astype(np.float64)[:, None] + b.astype(np.float64)
    _, _, xk, sx = gpu_swiglu(G, gu)
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device=G.DEV)
    if bits == 8:
        ql.ql_w8a8_gemm(xk, sx, M, F, g["kernel"], g["scales_dev"].view(torch.float32), G.dev(b), N, y)
    else:
        ql.ql_w4a8_gemm(xk, sx, M, F, g["kernel"], 128, G.dev(b), N, y)
    torch.cuda.synchronize()
    assert G.norm_err(y.cpu().numpy(), ref) <= TOL
    # and the quantized SwiGLU output is what the transform is for: close to the unquantized product
    exact = h.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)
    assert np.linalg.norm(ref - exact) / np.linalg.norm(exact) < (0.05 if bits == 8 else 0.25)


def test_argument_errors(G):
    gu = G.dev(_gate_up(4, 64, 1))
    sx = torch.empty(4, dtype=torch.float32, device=G.DEV)
    xq = torch.empty((4, 64), dtype=torch.int8, device=G.DEV)
    with pytest.raises(ql.QlError) as e:
        ql.ql_quant_act_swiglu(gu[:, :96], xq, None, sx)          # F = 48: not a multiple of 64
    assert e.value.status == 2
    with pytest.raises(ql.QlError) as e:
        ql.ql_quant_act_swiglu(gu, None, None, sx)                 # no output
    assert e.value.status == 1
