"""ctypes binding of libqlprobe.so, the benchmark's ceiling probes (bench_probe/qlprobe.h).

Not part of the quantized linear layer: bench.py uses it to report what the GPU sustains on the int8 matrix
pipe and on HBM reads next to the kernels' own numbers.
"""
from __future__ import annotations

import ctypes
import os

import torch

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libqlprobe.so")
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_23367_amd.build`")
        l = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        l.qlprobe_mfma_int8.restype = ctypes.c_int
        l.qlprobe_mfma_int8.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_int64), vp]
        l.qlprobe_hbm_read.restype = ctypes.c_int
        l.qlprobe_hbm_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        l.qlprobe_l2_to_lds.restype = ctypes.c_int
        l.qlprobe_l2_to_lds.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_int64), vp]
        _lib = l
    return _lib


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def mfma_int8(workgroups: int, iters: int, random_operands: int, sink) -> int:
    """Enqueues the matrix-pipe probe on torch's current stream; returns the number of int8 operations."""
    ops = ctypes.c_int64()
    rc = lib().qlprobe_mfma_int8(workgroups, iters, int(random_operands), ctypes.c_void_p(sink.data_ptr()),
                                 ctypes.byref(ops), _stream())
    if rc:
        raise RuntimeError(f"qlprobe_mfma_int8 failed ({rc})")
    return ops.value


def hbm_read(buf, sink):
    """Enqueues one pass of the read-stream probe over the whole of `buf`."""
    rc = lib().qlprobe_hbm_read(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                ctypes.c_void_p(sink.data_ptr()), _stream())
    if rc:
        raise RuntimeError(f"qlprobe_hbm_read failed ({rc})")


def l2_to_lds(buf, iters: int, sink) -> int:
    """Enqueues the global->LDS load probe over `buf` (64 KiB per workgroup); returns the bytes it moves."""
    moved = ctypes.c_int64()
    rc = lib().qlprobe_l2_to_lds(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(), int(iters),
                                 ctypes.c_void_p(sink.data_ptr()), ctypes.byref(moved), _stream())
    if rc:
        raise RuntimeError(f"qlprobe_l2_to_lds failed ({rc})")
    return moved.value
