"""ctypes binding of libqlinear.so: same names as include/qlinear.h, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used as plain device buffers; every call is enqueued on
torch's current stream.  There is no fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqlinear.so")

QL_OK = 0
STATUS_NAMES = {0: "QL_OK", 1: "QL_ERR_NULL", 2: "QL_ERR_SHAPE", 3: "QL_ERR_ALIGN",
                4: "QL_ERR_UNSUPPORTED", 5: "QL_ERR_WORKSPACE", 6: "QL_ERR_HIP"}

EXPORTS = [
    "ql_version", "ql_last_error", "ql_weight_bytes", "ql_act_kernel_bytes", "ql_workspace_bytes",
    "ql_quant_act_per_token", "ql_quant_act_rmsnorm", "ql_quant_act_swiglu", "ql_act_repack", "ql_quant_weight", "ql_export_canonical",
    "ql_w8a8_linear", "ql_w8a8_linear_static", "ql_w4a8_linear", "ql_w8a8_gemm", "ql_w4a8_gemm",
    "ql_w8a8_gemm_acc_i32", "ql_w4a8_gemm_acc_i32", "ql_set_kernel_variant", "ql_plan_gemm",
    "ql_hadamard_block", "ql_smooth_calibrate", "ql_smooth_scales",
    "ql_quant_act_per_token_transformed", "ql_quant_weight_transformed",
    "ql_act_scale_calibrate", "ql_quant_act_opt", "ql_quant_weight_opt",
]

QL_RANGE_SYMMETRIC, QL_RANGE_EQ2 = 0, 1
QL_FAMILY_DECODE, QL_FAMILY_TILE = 1, 2


class QlPlan(ctypes.Structure):
    """Mirror of the C struct ql_plan."""
    _fields_ = [("family", ctypes.c_int), ("variant", ctypes.c_int), ("tile_tokens", ctypes.c_int),
                ("tile_channels", ctypes.c_int), ("splits", ctypes.c_int), ("est_us", ctypes.c_double),
                ("rest_channels", ctypes.c_int), ("rest_variant", ctypes.c_int)]


QL_SCOPE_FINE, QL_SCOPE_TENSOR, QL_SCOPE_STATIC = 0, 1, 2


class QlError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (python -m paper_2512_23367_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2512_23367_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        l = ctypes.CDLL(LIB_PATH)
        c = ctypes
        vp, i, i64, sz = c.c_void_p, c.c_int, c.c_int64, c.c_size_t
        szp = c.POINTER(c.c_size_t)
        l.ql_version.restype = i
        l.ql_version.argtypes = []
        l.ql_last_error.restype = c.c_char_p
        l.ql_last_error.argtypes = []
        sigs = {
            "ql_set_kernel_variant": [i],
            "ql_plan_gemm": [i, i, i, i, i, sz, c.POINTER(QlPlan)],
            "ql_weight_bytes": [i, i, i, i, szp, szp, szp],
            "ql_act_kernel_bytes": [i, i, szp],
            "ql_workspace_bytes": [i, i, i, i, szp],
            "ql_quant_act_per_token": [vp, i64, i, i, vp, vp, vp, vp],
            "ql_quant_act_rmsnorm": [vp, i64, i, i, vp, c.c_float, vp, vp, vp, vp],
            "ql_quant_act_swiglu": [vp, i64, i, i, vp, vp, vp, vp],
            "ql_act_repack": [vp, i, i, vp, vp],
            "ql_quant_weight": [vp, i, i, i, i, vp, vp, vp, vp],
            "ql_export_canonical": [vp, i, i, i, i, vp, vp, vp],
            "ql_w8a8_linear": [vp, i64, i, i, vp, vp, vp, i, vp, i64, vp, sz, vp],
            "ql_w4a8_linear": [vp, i64, i, i, vp, i, vp, i, vp, i64, vp, sz, vp],
            "ql_w8a8_linear_static": [vp, i64, i, i, vp, vp, vp, i, vp, i64, vp],
            "ql_w8a8_gemm": [vp, vp, i, i, vp, vp, vp, i, vp, i64, vp, sz, vp],
            "ql_w4a8_gemm": [vp, vp, i, i, vp, i, vp, i, vp, i64, vp, sz, vp],
            "ql_w8a8_gemm_acc_i32": [vp, i, i, vp, i, vp, vp, sz, vp],
            "ql_w4a8_gemm_acc_i32": [vp, i, i, vp, i, i, vp, vp, i, i, vp, sz, vp],
            "ql_hadamard_block": [i, c.POINTER(c.c_int)],
            "ql_smooth_calibrate": [vp, i64, i, i, vp, vp],
            "ql_smooth_scales": [vp, vp, i, i, c.c_float, vp, vp, vp],
            "ql_quant_act_per_token_transformed": [vp, i64, i, i, vp, i, vp, vp, vp, vp],
            "ql_quant_weight_transformed": [vp, i, i, i, i, vp, i, vp, vp, vp, vp, vp],
            "ql_act_scale_calibrate": [vp, i64, i, i, i, vp, vp],
            "ql_quant_act_opt": [vp, i64, i, i, i, i, vp, vp, vp, vp, vp, vp],
            "ql_quant_weight_opt": [vp, i, i, i, i, i, i, vp, vp, vp, vp, vp],
        }
        for name, args in sigs.items():
            fn = getattr(l, name)
            fn.restype = i
            fn.argtypes = args
        _lib = l
    return _lib


def _check(status: int):
    if status != QL_OK:
        raise QlError(status, lib().ql_last_error().decode())


def _p(t):
    """Device pointer of a tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _want(t, dtype, name):
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    return t


def ql_version() -> int:
    return lib().ql_version()


def ql_last_error() -> str:
    return lib().ql_last_error().decode()


def ql_set_kernel_variant(variant: int):
    _check(lib().ql_set_kernel_variant(variant))


def ql_plan_gemm(M: int, N: int, K: int, bits: int, group: int, scratch_bytes: int = 0) -> QlPlan:
    """What the automatic choice launches for this GEMM shape and the estimate it goes by (host only)."""
    plan = QlPlan()
    _check(lib().ql_plan_gemm(M, N, K, bits, group, scratch_bytes, ctypes.byref(plan)))
    return plan


def ql_hadamard_block(K: int) -> int:
    b = ctypes.c_int()
    _check(lib().ql_hadamard_block(K, ctypes.byref(b)))
    return b.value


def ql_smooth_calibrate(x, xmax):
    _want(x, torch.float16, "x"), _want(xmax, torch.float32, "xmax")
    M, K = x.shape
    _check(lib().ql_smooth_calibrate(_p(x), _ld(x) if M else K, M, K, _p(xmax), _stream()))


def ql_smooth_scales(xmax, w, alpha, smooth, inv_smooth):
    _want(w, torch.float16, "w"), _want(xmax, torch.float32, "xmax")
    N, K = w.shape
    _check(lib().ql_smooth_scales(_p(xmax), _p(w), N, K, float(alpha), _p(smooth), _p(inv_smooth), _stream()))


def ql_quant_act_per_token_transformed(x, inv_smooth, hadamard_block, xq_rowmajor, xq_kernel, sx):
    _want(x, torch.float16, "x")
    M, K = x.shape
    _check(lib().ql_quant_act_per_token_transformed(_p(x), _ld(x) if M else K, M, K, _p(inv_smooth), hadamard_block,
                                                    _p(xq_rowmajor), _p(xq_kernel), _p(sx), _stream()))


def ql_quant_weight_transformed(w, bits, group, smooth, hadamard_block, w32, wq_canonical, scales, wq_kernel):
    _want(w, torch.float16, "w"), _want(w32, torch.float32, "w32")
    N, K = w.shape
    _check(lib().ql_quant_weight_transformed(_p(w), N, K, bits, group, _p(smooth), hadamard_block, _p(w32),
                                             _p(wq_canonical), _p(scales), _p(wq_kernel), _stream()))


def ql_act_scale_calibrate(x, rng, scale):
    _want(x, torch.float16, "x"), _want(scale, torch.float32, "scale")
    M, K = x.shape
    _check(lib().ql_act_scale_calibrate(_p(x), _ld(x) if M else K, M, K, rng, _p(scale), _stream()))


def ql_quant_act_opt(x, rng, scope, static_scale, xq_rowmajor, xq_kernel, sx, scratch):
    _want(x, torch.float16, "x")
    M, K = x.shape
    _check(lib().ql_quant_act_opt(_p(x), _ld(x) if M else K, M, K, rng, scope, _p(static_scale), _p(xq_rowmajor),
                                  _p(xq_kernel), _p(sx), _p(scratch), _stream()))


def ql_quant_weight_opt(w, bits, group, rng, scope, wq_canonical, scales, wq_kernel, scratch):
    _want(w, torch.float16, "w")
    N, K = w.shape
    _check(lib().ql_quant_weight_opt(_p(w), N, K, bits, group, rng, scope, _p(wq_canonical), _p(scales),
                                     _p(wq_kernel), _p(scratch), _stream()))


def ql_weight_bytes(N, K, bits, group):
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().ql_weight_bytes(N, K, bits, group, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def ql_act_kernel_bytes(M, K) -> int:
    a = ctypes.c_size_t()
    _check(lib().ql_act_kernel_bytes(M, K, ctypes.byref(a)))
    return a.value


def ql_workspace_bytes(M, N, K, bits) -> int:
    a = ctypes.c_size_t()
    _check(lib().ql_workspace_bytes(M, N, K, bits, ctypes.byref(a)))
    return a.value


def _ld(t):
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("2-D tensor with unit inner stride expected")
    return t.stride(0)


def ql_quant_act_per_token(x, xq_rowmajor=None, xq_kernel=None, sx=None):
    _want(x, torch.float16, "x")
    M, K = x.shape
    _check(lib().ql_quant_act_per_token(_p(x), _ld(x) if M else K, M, K, _p(xq_rowmajor), _p(xq_kernel), _p(sx),
                                        _stream()))


def ql_quant_act_rmsnorm(x, gamma, eps, xq_rowmajor=None, xq_kernel=None, sx=None):
    _want(x, torch.float16, "x"), _want(gamma, torch.float16, "gamma")
    M, K = x.shape
    _check(lib().ql_quant_act_rmsnorm(_p(x), _ld(x) if M else K, M, K, _p(gamma), float(eps), _p(xq_rowmajor),
                                      _p(xq_kernel), _p(sx), _stream()))


def ql_quant_act_swiglu(gate_up, xq_rowmajor=None, xq_kernel=None, sx=None):
    """gate_up: fp16 [M, 2F] (gate half, then up half); quantizes silu(gate) * up per token (K = F)."""
    _want(gate_up, torch.float16, "gate_up")
    M, F2 = gate_up.shape
    if F2 % 2:
        raise ValueError("gate_up has an even number of columns")
    _check(lib().ql_quant_act_swiglu(_p(gate_up), _ld(gate_up) if M else F2, M, F2 // 2, _p(xq_rowmajor), _p(xq_kernel),
                                     _p(sx), _stream()))


def ql_act_repack(xq_rowmajor, xq_kernel):
    _want(xq_rowmajor, torch.int8, "xq_rowmajor")
    M, K = xq_rowmajor.shape
    _check(lib().ql_act_repack(_p(xq_rowmajor), M, K, _p(xq_kernel), _stream()))


def ql_quant_weight(w, bits, group, wq_canonical=None, scales=None, wq_kernel=None):
    _want(w, torch.float16, "w")
    N, K = w.shape
    if not w.is_contiguous():
        raise ValueError("w must be contiguous")
    _check(lib().ql_quant_weight(_p(w), N, K, bits, group, _p(wq_canonical), _p(scales), _p(wq_kernel), _stream()))


def ql_export_canonical(wq_kernel, N, K, bits, group, wq_canonical=None, scales=None):
    _check(lib().ql_export_canonical(_p(wq_kernel), N, K, bits, group, _p(wq_canonical), _p(scales), _stream()))


def _ws(ws):
    return (_p(ws), ws.numel() * ws.element_size()) if ws is not None else (None, 0)


def _nbytes(t):
    return t.numel() * t.element_size()


def _check_gemm_buffers(M, K, N, bits, group, w_kernel, sw, bias, y, xq_kernel=None, sx=None):
    """Host-side size checks the C side cannot make (it sees pointers only): a buffer that is too small or of the
    wrong layout would be read or written out of bounds by the kernels."""
    if w_kernel is None or _nbytes(w_kernel) < ql_weight_bytes(N, K, bits, group)[2]:
        raise ValueError("w_kernel is smaller than the kernel-layout blob of ql_weight_bytes (canonical codes passed?)")
    if y.dim() != 2 or tuple(y.shape) != (M, N) or (M and y.stride(1) != 1):
        raise ValueError(f"y must be [M,N] = [{M},{N}] with unit inner stride")
    if bits == 8 and (sw is None or sw.numel() < N):
        raise ValueError("sw needs N fp32 entries")
    if bias is not None and (bias.dtype != torch.float16 or bias.numel() < N):
        raise ValueError("bias must be fp16 with N entries")
    if xq_kernel is not None and _nbytes(xq_kernel) < ql_act_kernel_bytes(M, K):
        raise ValueError("xq_kernel is smaller than ql_act_kernel_bytes")
    if sx is not None and (sx.dtype != torch.float32 or sx.numel() < M):
        raise ValueError("sx needs M fp32 entries")


def ql_w8a8_linear(x, wq_kernel, sw, bias, N, y, ws):
    _want(x, torch.float16, "x"), _want(y, torch.float16, "y"), _want(sw, torch.float32, "sw")
    M, K = x.shape
    _check_gemm_buffers(M, K, N, 8, 0, wq_kernel, sw, bias, y)
    wsp, wsb = _ws(ws)
    _check(lib().ql_w8a8_linear(_p(x), _ld(x) if M else K, M, K, _p(wq_kernel), _p(sw), _p(bias), N, _p(y),
                                _ld(y) if M else N, wsp, wsb, _stream()))


def ql_w8a8_linear_static(x, wq_kernel, sw, bias, N, y):
    """ql_w8a8_linear on the library's own static workspace (allocates nothing)."""
    _want(x, torch.float16, "x"), _want(y, torch.float16, "y"), _want(sw, torch.float32, "sw")
    M, K = x.shape
    _check_gemm_buffers(M, K, N, 8, 0, wq_kernel, sw, bias, y)
    _check(lib().ql_w8a8_linear_static(_p(x), _ld(x) if M else K, M, K, _p(wq_kernel), _p(sw), _p(bias), N, _p(y),
                                       _ld(y) if M else N, _stream()))


def ql_w4a8_linear(x, w4_kernel, group, bias, N, y, ws):
    _want(x, torch.float16, "x"), _want(y, torch.float16, "y")
    M, K = x.shape
    _check_gemm_buffers(M, K, N, 4, group, w4_kernel, None, bias, y)
    wsp, wsb = _ws(ws)
    _check(lib().ql_w4a8_linear(_p(x), _ld(x) if M else K, M, K, _p(w4_kernel), group, _p(bias), N, _p(y),
                                _ld(y) if M else N, wsp, wsb, _stream()))


def ql_w8a8_gemm(xq_kernel, sx, M, K, wq_kernel, sw, bias, N, y, ws=None):
    _want(y, torch.float16, "y")
    _check_gemm_buffers(M, K, N, 8, 0, wq_kernel, sw, bias, y, xq_kernel, sx)
    wsp, wsb = _ws(ws)
    _check(lib().ql_w8a8_gemm(_p(xq_kernel), _p(sx), M, K, _p(wq_kernel), _p(sw), _p(bias), N, _p(y),
                              _ld(y) if M else N, wsp, wsb, _stream()))


def ql_w4a8_gemm(xq_kernel, sx, M, K, w4_kernel, group, bias, N, y, ws=None):
    _want(y, torch.float16, "y")
    _check_gemm_buffers(M, K, N, 4, group, w4_kernel, None, bias, y, xq_kernel, sx)
    wsp, wsb = _ws(ws)
    _check(lib().ql_w4a8_gemm(_p(xq_kernel), _p(sx), M, K, _p(w4_kernel), group, _p(bias), N, _p(y),
                              _ld(y) if M else N, wsp, wsb, _stream()))


def ql_w8a8_gemm_acc_i32(xq_kernel, M, K, wq_kernel, N, acc, ws=None):
    _want(acc, torch.int32, "acc")
    if acc.numel() < M * N or not acc.is_contiguous():
        raise ValueError("acc must be a contiguous int32 [M,N]")
    if _nbytes(wq_kernel) < ql_weight_bytes(N, K, 8, 0)[2] or _nbytes(xq_kernel) < ql_act_kernel_bytes(M, K):
        raise ValueError("wq_kernel / xq_kernel smaller than their size queries report")
    wsp, wsb = _ws(ws)
    _check(lib().ql_w8a8_gemm_acc_i32(_p(xq_kernel), M, K, _p(wq_kernel), N, _p(acc), wsp, wsb, _stream()))


def ql_w4a8_gemm_acc_i32(xq_kernel, M, K, w4_kernel, group, N, acc, partials=None, row0=0, nrows=0, ws=None):
    _want(acc, torch.int32, "acc")
    if acc.numel() < M * N or not acc.is_contiguous():
        raise ValueError("acc must be a contiguous int32 [M,N]")
    if _nbytes(w4_kernel) < ql_weight_bytes(N, K, 4, group)[2] or _nbytes(xq_kernel) < ql_act_kernel_bytes(M, K):
        raise ValueError("w4_kernel / xq_kernel smaller than their size queries report")
    if partials is not None and (partials.dtype != torch.int32 or partials.numel() < nrows * (K // group) * N):
        raise ValueError("partials must be int32 [nrows, K/group, N]")
    wsp, wsb = _ws(ws)
    _check(lib().ql_w4a8_gemm_acc_i32(_p(xq_kernel), M, K, _p(w4_kernel), group, N, _p(acc), _p(partials), row0,
                                      nrows, wsp, wsb, _stream()))
