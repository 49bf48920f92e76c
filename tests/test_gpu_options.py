"""GPU parity of the other quantizer forms of the paper's Preliminary section (Eq. 2 as printed, per-tensor
granularity, calibrated static activation scale) against the oracle: codes and scales bit-exact, both output
layouts, calibration as a running maximum, and the layer through the ordinary GEMM entry points (which must cope
with codes of -128 / -8)."""
import numpy as np
import pytest

import oracle
from paper_2512_23367_amd import binding as ql, synth

pytestmark = pytest.mark.gpu
TOL = 1e-3
RANGES = [oracle.RANGE_SYMMETRIC, oracle.RANGE_EQ2]


@pytest.fixture(scope="module")
def G():
    from tests import gpu_util
    return gpu_util


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def test_enums_match_the_oracle():
    assert (ql.QL_RANGE_SYMMETRIC, ql.QL_RANGE_EQ2) == (oracle.RANGE_SYMMETRIC, oracle.RANGE_EQ2)
    assert (ql.QL_SCOPE_FINE, ql.QL_SCOPE_TENSOR, ql.QL_SCOPE_STATIC) == \
        (oracle.SCOPE_FINE, oracle.SCOPE_TENSOR, oracle.SCOPE_STATIC)


def gpu_act(G, x, rng, scope, static=None, ldx=None):
    import torch
    M, K = x.shape
    if ldx is None:
        xd = _dev(x)
    else:
        buf = torch.full((M, ldx), float("nan"), dtype=torch.float16, device="cuda:0")
        buf[:, :K] = _dev(x)
        xd = buf[:, :K]
    xq = torch.full((M, K), 99, dtype=torch.int8, device="cuda:0")
    sx = torch.full((M,), float("nan"), dtype=torch.float32, device="cuda:0")
    xk = G.empty_bytes(ql.ql_act_kernel_bytes(M, K))
    scratch = torch.full((1,), 12345, dtype=torch.int32, device="cuda:0")       # stale contents must not matter
    st = None if static is None else torch.tensor([static], dtype=torch.float32, device="cuda:0")
    ql.ql_quant_act_opt(xd, rng, scope, st, xq, xk, sx, scratch)
    torch.cuda.synchronize()
    return xq.cpu().numpy(), sx.cpu().numpy(), xk, sx


def gpu_weight(G, w, bits, rng, scope):
    import torch
    N, K = w.shape
    group = 0 if bits == 8 else 128
    cb, sb, kb = ql.ql_weight_bytes(N, K, bits, group)
    canon, scales, kern = G.empty_bytes(cb), G.empty_bytes(sb), G.empty_bytes(kb)
    scratch = torch.full((1,), 0x7F000000, dtype=torch.int32, device="cuda:0")
    ql.ql_quant_weight_opt(_dev(w), bits, group, rng, scope, canon, scales, kern, scratch)
    torch.cuda.synchronize()
    if bits == 8:
        c = canon.cpu().numpy().view(np.int8).reshape(N, K)
        s = scales.cpu().numpy().view(np.float32).reshape(N)
    else:
        c = canon.cpu().numpy().reshape(N, K // 2)
        s = scales.cpu().numpy().view(np.float16).reshape(N, K // 128)
    return dict(canon=c, scales=s, scales_dev=scales, kernel=kern, N=N, K=K, bits=bits, group=group)


@pytest.mark.parametrize("rng", RANGES)
@pytest.mark.parametrize("scope", [oracle.SCOPE_FINE, oracle.SCOPE_TENSOR, oracle.SCOPE_STATIC])
@pytest.mark.parametrize("M,K,ldx", [(1, 64, None), (37, 1536, None), (300, 4096, 4104), (5, 11008, None), (1100, 512, None)])
def test_activation_codes_and_scales_bit_exact(G, rng, scope, M, K, ldx):
    x = synth.activations(M, K, 5, "qkv")
    if M > 2:
        x[1] = 0                                          # a zero token
    static = None
    if scope == oracle.SCOPE_STATIC:                      # a scale that clamps part of the outlier channels
        static = float(oracle.act_scale_calibrate([x], rng)) / 3.0
    if rng == oracle.RANGE_SYMMETRIC and scope == oracle.SCOPE_FINE:
        q_o, s_o = oracle.quant_act_per_token(x)          # documented: this combination is the hot-path quantizer
    else:
        q_o, s_o = oracle.quant_act_opt(x, rng, scope, None if static is None else np.float32(static))
    q_g, s_g, xk, _ = gpu_act(G, x, rng, scope, static, ldx)
    assert (s_g == s_o).all()
    assert (q_g == q_o).all()
    if scope == oracle.SCOPE_STATIC and M > 2:
        assert (np.abs(q_o.astype(int)) >= 127).sum() > M // 2   # the clamp really is exercised
    tiles = xk.cpu().numpy().view(np.int8)
    want = G.repack_act(q_o).cpu().numpy().view(np.int8)
    rows = (np.arange(tiles.size) // 16) % 32 + 32 * (np.arange(tiles.size) // (1024 * (K // 32)))
    assert (tiles[rows < M] == want[rows < M]).all()


def test_symmetric_fine_is_the_per_token_quantizer_itself(G):
    x = synth.activations(64, 1536, 6, "qkv")
    q_g, s_g, _, _ = gpu_act(G, x, oracle.RANGE_SYMMETRIC, oracle.SCOPE_FINE)
    q_o, s_o = oracle.quant_act_per_token(x)
    assert (q_g == q_o).all() and (s_g == s_o).all()


@pytest.mark.parametrize("rng", RANGES)
def test_calibration_is_the_running_maximum(G, rng):
    import torch
    batches = [synth.activations(50, 1536, s, "qkv") for s in (1, 2, 3)]
    batches[1] = (batches[1].astype(np.float32) * 3).astype(np.float16)       # the largest values sit in the middle batch
    scale = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    seen = []
    for b in batches:
        ql.ql_act_scale_calibrate(_dev(b), rng, scale)
        torch.cuda.synchronize()
        seen.append(np.float32(scale.item()))
    assert seen[0] == oracle.act_scale_calibrate(batches[:1], rng)
    assert seen[1] == oracle.act_scale_calibrate(batches[:2], rng)
    assert seen[2] == oracle.act_scale_calibrate(batches, rng) == seen[1]
    ql.ql_act_scale_calibrate(_dev(np.zeros((4, 64), dtype=np.float16)), rng, scale)   # zeros change nothing
    assert np.float32(scale.item()) == seen[2]


@pytest.mark.parametrize("rng", RANGES)
@pytest.mark.parametrize("scope", [oracle.SCOPE_FINE, oracle.SCOPE_TENSOR])
@pytest.mark.parametrize("bits,N,K", [(8, 200, 1536), (8, 33, 4096), (4, 136, 1024), (4, 264, 1536), (4, 40, 11008)])
def test_weight_codes_and_scales_bit_exact(G, rng, scope, bits, N, K):
    w = synth.weights(N, K, 7, "qkv")
    w[3] = 0                                              # a zero channel
    g = gpu_weight(G, w, bits, rng, scope)
    if bits == 8:
        q_o, s_o = oracle.quant_weight_opt(w, 8, 0, rng, scope)
        assert (g["scales"] == s_o).all() and (g["canon"] == q_o).all()
    else:
        p_o, q_o, s_o = oracle.quant_weight_opt(w, 4, 128, rng, scope)
        assert (g["scales"] == s_o).all() and (g["canon"] == p_o).all()
    if rng == oracle.RANGE_EQ2 and scope == oracle.SCOPE_FINE:
        assert (q_o == (-128 if bits == 8 else -8)).any()  # the extra negative code really occurs
    c2, s2 = G.gpu_export(g["kernel"], N, K, bits, g["group"])            # the kernel layout holds the same codes
    assert (c2 == g["canon"]).all()
    if bits == 4:
        assert (s2 == g["scales"]).all()


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("rng,scope_x,scope_w", [(oracle.RANGE_EQ2, oracle.SCOPE_FINE, oracle.SCOPE_FINE),
                                                   (oracle.RANGE_EQ2, oracle.SCOPE_TENSOR, oracle.SCOPE_TENSOR),
                                                   (oracle.RANGE_SYMMETRIC, oracle.SCOPE_STATIC, oracle.SCOPE_TENSOR),
                                                   (oracle.RANGE_EQ2, oracle.SCOPE_STATIC, oracle.SCOPE_FINE)])
@pytest.mark.parametrize("M,K,N", [(1, 1024, 136), (24, 4096, 200), (300, 1536, 264)])
def test_layer_end_to_end_through_the_gemm_entry_points(G, bits, rng, scope_x, scope_w, M, K, N):
    """Integer sums bit-exact (prefill and decode kernels multiply codes of -128 / -8 correctly) and the fp16
    output within tolerance of the oracle layer on the oracle's codes."""
    import torch
    x = synth.activations(M, K, 8, "qkv")
    w = synth.weights(N, K, 8, "qkv")
    b = synth.bias(N, 8, "qkv")
    static = np.float32(oracle.act_scale_calibrate([x], rng)) if scope_x == oracle.SCOPE_STATIC else None
    xq_o, sx_o = oracle.quant_act_opt(x, rng, scope_x, static)
    g = gpu_weight(G, w, bits, rng, scope_w)
    _, _, xk, sx = gpu_act(G, x, rng, scope_x, None if static is None else float(static))
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda:0")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda:0")
    if bits == 8:
        ql.ql_w8a8_gemm(xk, sx, M, K, g["kernel"], g["scales_dev"].view(torch.float32), _dev(b), N, y)
        ql.ql_w8a8_gemm_acc_i32(xk, M, K, g["kernel"], N, acc)
        ref = oracle.linear_w8a8(None, g["canon"], g["scales"], b, xq=xq_o, sx=sx_o)
    else:
        ql.ql_w4a8_gemm(xk, sx, M, K, g["kernel"], 128, _dev(b), N, y)
        ql.ql_w4a8_gemm_acc_i32(xk, M, K, g["kernel"], 128, N, acc, None, 0, 0)
        ref = oracle.linear_w4a8(None, g["canon"], g["scales"], 128, b, xq=xq_o, sx=sx_o)
    torch.cuda.synchronize()
    assert (acc.cpu().numpy() == ref["acc"]).all()
    assert G.norm_err(y.cpu().numpy(), ref["y64"]) <= TOL


@pytest.mark.parametrize("M", [2, 20, 40, 300])
def test_extreme_codes_everywhere(G, M):
    """Every activation -128 and every weight -128 / -8: the largest products the GEMMs (decode and prefill
    kernels) can meet."""
    import torch
    K, N = 2048, 72
    x = np.full((M, K), -255.0, dtype=np.float16)         # s = 2*255/255 = 2 exactly: -255/2 = -127.5 -> -128
    xq_o, sx_o = oracle.quant_act_opt(x, oracle.RANGE_EQ2)
    assert (xq_o == -128).all()
    _, _, xk, sx = gpu_act(G, x, oracle.RANGE_EQ2, oracle.SCOPE_FINE)
    for bits in (8, 4):
        w = np.full((N, K), -255.0 if bits == 8 else -7.5, dtype=np.float16)   # scales 2 and 1: -127.5 -> -128, -7.5 -> -8
        g = gpu_weight(G, w, bits, oracle.RANGE_EQ2, oracle.SCOPE_FINE)
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda:0")
        if bits == 8:
            q_o, _ = oracle.quant_weight_opt(w, 8, 0, oracle.RANGE_EQ2)
            ql.ql_w8a8_gemm_acc_i32(xk, M, K, g["kernel"], N, acc)
        else:
            _, q_o, _ = oracle.quant_weight_opt(w, 4, 128, oracle.RANGE_EQ2)
            ql.ql_w4a8_gemm_acc_i32(xk, M, K, g["kernel"], 128, N, acc, None, 0, 0)
        assert (q_o == (-128 if bits == 8 else -8)).all()
        torch.cuda.synchronize()
        assert (acc.cpu().numpy() == oracle.igemm(xq_o, q_o)).all()


def test_argument_errors(G):
    import torch
    x = torch.zeros((4, 512), dtype=torch.float16, device="cuda:0")
    xq = torch.empty((4, 512), dtype=torch.int8, device="cuda:0")
    sx = torch.empty(4, dtype=torch.float32, device="cuda:0")
    scratch = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    with pytest.raises(ql.QlError):
        ql.ql_quant_act_opt(x, 2, 0, None, xq, None, sx, scratch)                       # unknown range
    with pytest.raises(ql.QlError):
        ql.ql_quant_act_opt(x, 0, 3, None, xq, None, sx, scratch)                       # unknown scope
    with pytest.raises(ql.QlError):
        ql.ql_quant_act_opt(x, 1, ql.QL_SCOPE_STATIC, None, xq, None, sx, scratch)      # no static scale
    with pytest.raises(ql.QlError):
        ql.ql_quant_act_opt(x, 1, ql.QL_SCOPE_TENSOR, None, xq, None, sx, None)         # no scratch
    w = torch.zeros((32, 512), dtype=torch.float16, device="cuda:0")
    cb, sb, kb = ql.ql_weight_bytes(32, 512, 8, 0)
    canon, scales = G.empty_bytes(cb), G.empty_bytes(sb)
    with pytest.raises(ql.QlError):
        ql.ql_quant_weight_opt(w, 8, 0, 0, ql.QL_SCOPE_STATIC, canon, scales, None, scratch)   # static: activations only
    with pytest.raises(ql.QlError):
        ql.ql_quant_weight_opt(w, 8, 0, 0, ql.QL_SCOPE_TENSOR, canon, scales, None, None)
    big = torch.zeros((1, 131072), dtype=torch.float16, device="cuda:0")
    with pytest.raises(ql.QlError):                                                     # Eq. 2 range: K limit
        ql.ql_quant_act_opt(big, 1, 0, None, torch.empty((1, 131072), dtype=torch.int8, device="cuda:0"), None,
                            sx[:1], scratch)
