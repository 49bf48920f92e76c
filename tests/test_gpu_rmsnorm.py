"""GPU parity of the RMSNorm fused in front of the activation quantizer: codes and scales bit for bit against the
oracle (textbook RMSNorm, fp32 step by step, exact sum of squares), then through the GEMM."""
import numpy as np
import pytest

import oracle
from paper_2512_23367_amd import binding as ql
from paper_2512_23367_amd import synth

pytestmark = pytest.mark.gpu
TOL = 1e-3


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _run(G, x, gamma, eps, ldx=None):
    import torch
    M, K = x.shape
    if ldx is None:
        xd = G.dev(x)
    else:
        buf = torch.full((M, ldx), float("nan"), dtype=torch.float16, device=G.DEV)
        buf[:, :K] = G.dev(x)
        xd = buf[:, :K]
    xq = torch.full((M, K), 99, dtype=torch.int8, device=G.DEV)
    sx = torch.full((M,), -1.0, dtype=torch.float32, device=G.DEV)
    xk = G.empty_bytes(ql.ql_act_kernel_bytes(M, K))
    ql.ql_quant_act_rmsnorm(xd, G.dev(gamma), eps, xq, xk, sx)
    torch.cuda.synchronize()
    return xq.cpu().numpy(), sx.cpu().numpy(), xk


@pytest.mark.parametrize("M,K,ldx", [(1, 64, None), (5, 1536, None), (33, 4096, 4104), (300, 11008, None), (2, 16384, None),
                                     (3, 22016, None), (2, 131072, None), (64, 128, 136)])
@pytest.mark.parametrize("eps", [1e-6, 0.0])
def test_codes_and_scales_bit_exact(G, M, K, ldx, eps):
    x = synth.activations(M, K, M + K, "single")
    if M >= 3:
        x[2] *= np.float16(1 / 64)           # a quiet token
    rng = np.random.default_rng(K)
    gamma = rng.uniform(0.25, 2.0, K).astype(np.float16)
    gamma[::7] *= -1
    h = oracle.rmsnorm_act(x, gamma, eps)
    q_o, s_o = oracle.quant_act_per_token(h)
    q_g, s_g, xk = _run(G, x, gamma, eps, ldx)
    assert (s_g.view(np.uint32) == s_o.view(np.uint32)).all()
    assert (q_g == q_o).all()
    # the tile-order copy holds the same codes on the rows that exist
    from test_gpu_parity import _kernel_layout_mask
    a = xk.cpu().numpy().view(np.int8)
    b = G.repack_act(q_o).cpu().numpy().view(np.int8)
    valid = _kernel_layout_mask(M, K)
    assert (a[valid] == b[valid]).all()


def test_extreme_magnitudes(G):
    """Largest fp16 values (sum of squares ~ 2^32 * K) and subnormals with eps carrying the denominator."""
    K = 4096
    x = np.zeros((3, K), dtype=np.float16)
    x[0] = 65504.0
    x[0, ::2] = -65504.0
    x[1] = np.float16(6e-8)                  # fp16 subnormals
    x[2, 5] = 1.0                            # one non-zero element
    gamma = np.ones(K, dtype=np.float16)
    for eps in (1e-5, 1.0):
        h = oracle.rmsnorm_act(x, gamma, eps)
        q_o, s_o = oracle.quant_act_per_token(h)
        q_g, s_g, _ = _run(G, x, gamma, eps)
        assert (s_g.view(np.uint32) == s_o.view(np.uint32)).all() and (q_g == q_o).all()


@pytest.mark.parametrize("bits", [8, 4])
def test_layer_with_fused_rmsnorm_within_tolerance(G, bits):
    """RMSNorm + quantizer + GEMM against the oracle chain (fp64 reference of the dequantized product)."""
    import torch
    M, K, N = 200, 1536, 520
    x = synth.activations(M, K, 1, "single")
    gamma = np.random.default_rng(2).uniform(0.5, 1.5, K).astype(np.float16)
    w = synth.weights(N, K, 0, "single")
    b = synth.bias(N, 0, "single")
    g = G.gpu_quant_weight(w, bits, 0 if bits == 8 else 128)
    h = oracle.rmsnorm_act(x, gamma, 1e-6)
    ref = (oracle.linear_w8a8(h, g["canon"], g["scales"], b) if bits == 8
           else oracle.linear_w4a8(h, g["canon"], g["scales"], 128, b))
    sx = torch.empty((M,), dtype=torch.float32, device=G.DEV)
    xk = G.empty_bytes(ql.ql_act_kernel_bytes(M, K))
    ql.ql_quant_act_rmsnorm(G.dev(x), G.dev(gamma), 1e-6, None, xk, sx)
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device=G.DEV)
    if bits == 8:
        ql.ql_w8a8_gemm(xk, sx, M, K, g["kernel"], g["scales_dev"].view(torch.float32), G.dev(b), N, y, None)
    else:
        ql.ql_w4a8_gemm(xk, sx, M, K, g["kernel"], 128, G.dev(b), N, y, None)
    torch.cuda.synchronize()
    assert G.norm_err(y.cpu().numpy(), ref["y64"]) <= TOL


def test_argument_errors(G):
    import torch
    x = G.dev(np.zeros((4, 128), np.float16))
    gam = G.dev(np.ones(128, np.float16))
    sx = torch.empty(4, dtype=torch.float32, device=G.DEV)
    xq = torch.empty((4, 128), dtype=torch.int8, device=G.DEV)
    with pytest.raises(ql.QlError) as e:
        ql.ql_quant_act_rmsnorm(x, gam, -1.0, xq, None, sx)
    assert e.value.status == 2
    with pytest.raises(ql.QlError) as e:
        ql.ql_quant_act_rmsnorm(x, gam, float("nan"), xq, None, sx)
    assert e.value.status == 2
    # gamma == NULL, straight through the C ABI
    import ctypes
    vp = ctypes.c_void_p
    assert ql.lib().ql_quant_act_rmsnorm(vp(x.data_ptr()), 128, 4, 128, None, 1e-6, vp(xq.data_ptr()), None,
                                         vp(sx.data_ptr()), None) == 1
