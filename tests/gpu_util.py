"""Helpers for the GPU parity tests: host arrays in, host arrays out, everything through the C ABI."""
from __future__ import annotations

import numpy as np
import torch

from paper_2512_23367_amd import binding as ql

DEV = "cuda:0"


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def empty_bytes(n: int) -> torch.Tensor:
    return torch.empty(max(int(n), 1), dtype=torch.uint8, device=DEV)


def gpu_quant_act(x16: np.ndarray, ldx: int | None = None):
    """Returns (xq int8 [M,K] row-major, sx float32 [M], xq_kernel device tensor)."""
    M, K = x16.shape
    if ldx is None:
        xd = dev(x16)
    else:
        buf = torch.zeros((M, ldx), dtype=torch.float16, device=DEV)
        buf[:, :K] = dev(x16)
        xd = buf[:, :K]
    xq = torch.empty((M, K), dtype=torch.int8, device=DEV)
    sx = torch.empty((M,), dtype=torch.float32, device=DEV)
    xk = empty_bytes(ql.ql_act_kernel_bytes(M, K))
    ql.ql_quant_act_per_token(xd, xq, xk, sx)
    torch.cuda.synchronize()
    return xq.cpu().numpy(), sx.cpu().numpy(), xk


def gpu_quant_weight(w16: np.ndarray, bits: int, group: int, check: bool = True):
    """Quantizes w16 on the GPU and returns dict(canon, scales, kernel (device), N, K, ...).

    With `check` (default) the oracle quantizes the same weights itself, the GPU's codes and scales are compared with
    its bit for bit, and the host arrays returned as `canon` / `scales` are the ORACLE's: every reference a test then
    computes from them comes from the oracle alone, nothing the oracle consumes was produced by the GPU."""
    N, K = w16.shape
    cb, sb, kb = ql.ql_weight_bytes(N, K, bits, group)
    canon = empty_bytes(cb)
    scales = empty_bytes(sb)
    kern = empty_bytes(kb)
    ql.ql_quant_weight(dev(w16), bits, group, canon, scales, kern)
    torch.cuda.synchronize()
    if bits == 8:
        c = canon.cpu().numpy().view(np.int8).reshape(N, K)
        s = scales.cpu().numpy().view(np.float32).reshape(N)
    else:
        c = canon.cpu().numpy().reshape(N, K // 2)
        s = scales.cpu().numpy().view(np.float16).reshape(N, K // group)
    if check:
        import oracle
        if bits == 8:
            c_o, s_o = oracle.quant_weight_int8(w16)
            assert (c == c_o).all() and (s.view(np.uint32) == s_o.view(np.uint32)).all(), "GPU weight quantization differs from the oracle's"
        else:
            c_o, _, s_o = oracle.quant_weight_int4(w16, group)
            assert (c == c_o).all() and (s.view(np.uint16) == s_o.view(np.uint16)).all(), "GPU weight quantization differs from the oracle's"
        c, s = c_o, s_o
    return dict(canon=c, scales=s, scales_dev=scales, kernel=kern, N=N, K=K, bits=bits, group=group)


def gpu_export(wk, N, K, bits, group):
    cb, sb, _ = ql.ql_weight_bytes(N, K, bits, group)
    canon = empty_bytes(cb)
    scales = empty_bytes(sb)
    ql.ql_export_canonical(wk, N, K, bits, group, canon, scales if bits == 4 else None)
    torch.cuda.synchronize()
    if bits == 8:
        return canon.cpu().numpy().view(np.int8).reshape(N, K), None
    return canon.cpu().numpy().reshape(N, K // 2), scales.cpu().numpy().view(np.float16).reshape(N, K // group)


def repack_act(xq: np.ndarray) -> torch.Tensor:
    M, K = xq.shape
    xk = empty_bytes(ql.ql_act_kernel_bytes(M, K))
    ql.ql_act_repack(dev(xq), xk)
    return xk


def gpu_acc(xq: np.ndarray, wq, want_partials=False, ws=None, row0=0, nrows=None):
    """Raw integer accumulators of the GEMM main loop for host codes xq and a gpu_quant_weight dict
    (int4 with want_partials: also the group partials of tokens row0 .. row0 + nrows - 1, default all)."""
    M, K = xq.shape
    N = wq["N"]
    xk = repack_act(xq)
    acc = torch.full((M, N), -12345, dtype=torch.int32, device=DEV)
    part = None
    if wq["bits"] == 8:
        ql.ql_w8a8_gemm_acc_i32(xk, M, K, wq["kernel"], N, acc, ws)
    else:
        G = K // wq["group"]
        nrows = M if nrows is None else nrows
        part = torch.full((nrows, G, N), -12345, dtype=torch.int32, device=DEV) if want_partials else None
        ql.ql_w4a8_gemm_acc_i32(xk, M, K, wq["kernel"], wq["group"], N, acc, part, row0, nrows if want_partials else 0)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), (part.cpu().numpy() if part is not None else None)


def gpu_linear(x16: np.ndarray, wq, bias16=None, ldy=None, ldx=None, extra_ws=0) -> np.ndarray:
    M, K = x16.shape
    N = wq["N"]
    if ldx is None:
        xd = dev(x16)
    else:
        xbuf = torch.full((M, ldx), float("nan"), dtype=torch.float16, device=DEV)
        xbuf[:, :K] = dev(x16)
        xd = xbuf[:, :K]
    ld = ldy or ((N + 7) // 8 * 8)
    ybuf = torch.full((M, ld), float("nan"), dtype=torch.float16, device=DEV)
    y = ybuf[:, :N]
    ws = empty_bytes(ql.ql_workspace_bytes(M, N, K, wq["bits"]) + extra_ws)
    b = dev(bias16) if bias16 is not None else None
    if wq["bits"] == 8:
        ql.ql_w8a8_linear(xd, wq["kernel"], wq["scales_dev"].view(torch.float32), b, N, y, ws)
    else:
        ql.ql_w4a8_linear(xd, wq["kernel"], wq["group"], b, N, y, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def norm_err(y: np.ndarray, ref64: np.ndarray) -> float:
    """max|y - ref| / max|ref| (the tolerance the parity bar is stated in)."""
    return float(np.abs(y.astype(np.float64) - ref64).max() / max(np.abs(ref64).max(), 1e-30))
