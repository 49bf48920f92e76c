"""Seeded synthetic inputs for the quantized linear layer.

This module only *draws* tensors: it holds none of the method's arithmetic (no
quantizer, no GEMM, no dequantization), so both the CPU oracle's tests and the
HIP path's tests/bench may use it without sharing any code of the method.

Recipe (stands in for the decoder-layer activations and weights of the paper's
models, whose heavy-tailed outlier channels are shown in its Figure 1):
  * activations  fp32 N(0,1) [M,K]; round(0.01*K) channels, chosen by a seeded
    permutation, are multiplied by 20; then rounded to fp16
  * weights      fp32 N(0,0.02) [N,K] -> fp16   (row n = output channel n)
  * bias         fp32 N(0,0.01) [N]   -> fp16   (only where the workload has one)
Every tensor has its own stream: seed sequence (BASE_SEED, config, layer, role).
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20251223
OUTLIER_FRACTION = 0.01
OUTLIER_GAIN = 20.0
ACT_STD = 1.0
WEIGHT_STD = 0.02
BIAS_STD = 0.01

_ROLE_X, _ROLE_W, _ROLE_B, _ROLE_COLS = 0, 1, 2, 3


@dataclass(frozen=True)
class Shape:
    """One linear layer of a workload: y[M,N] = x[M,K] @ w[N,K]^T (+ bias)."""
    config: int        # index into the benchmark's configuration list
    layer: str         # "single", "qkv", "o", "gate_up", "down"
    M: int
    K: int
    N: int
    bits: int          # weight bits: 8 (per-channel scales) or 4 (group scales)
    group: int         # 0 = per output channel; else group length along K
    bias: bool

    @property
    def name(self) -> str:
        return f"c{self.config}.{self.layer}.M{self.M}.K{self.K}.N{self.N}.w{self.bits}"

    @property
    def ops(self) -> int:
        return 2 * self.M * self.N * self.K


_LAYER_ID = {"single": 0, "qkv": 1, "o": 2, "gate_up": 3, "down": 4}


def _layer_shapes_1b():
    d = 1536
    return [("qkv", d, 3 * d), ("o", d, d), ("gate_up", d, 12288), ("down", 6144, d)]


def _layer_shapes_7b():
    d = 4096
    return [("qkv", d, 3 * d), ("o", d, d), ("gate_up", d, 22016), ("down", 11008, d)]


def workload(config: int) -> list[Shape]:
    """The layer shapes of benchmark configuration `config` (0..4)."""
    if config == 0:
        return [Shape(0, "single", 64, 512, 512, 8, 0, False)]
    if config == 1:
        return [Shape(1, l, 2048, k, n, 8, 0, False) for l, k, n in _layer_shapes_1b()]
    if config == 2:
        return [Shape(2, l, 4096, k, n, 8, 0, True) for l, k, n in _layer_shapes_7b()]
    if config == 3:
        return [Shape(3, l, 4096, k, n, 4, 128, False) for l, k, n in _layer_shapes_7b()]
    if config == 4:
        out = []
        for m in (1, 8, 32):
            out += [Shape(4, l, m, k, n, 8, 0, False) for l, k, n in _layer_shapes_7b()]
            out += [Shape(4, l, m, k, n, 4, 128, False) for l, k, n in _layer_shapes_7b()]
        out.append(Shape(4, "down", 16384, 11008, 4096, 8, 0, False))
        return out
    raise ValueError(f"no such configuration: {config}")


def _rng(config: int, layer: str, role: int, extra: int = 0) -> np.random.Generator:
    return np.random.default_rng([BASE_SEED, config, _LAYER_ID[layer], role, extra])


def outlier_channels(K: int, config: int, layer: str) -> np.ndarray:
    """Sorted indices of the round(0.01*K) amplified activation channels."""
    n = int(round(OUTLIER_FRACTION * K))
    perm = _rng(config, layer, _ROLE_COLS).permutation(K)
    return np.sort(perm[:n])


def activations(M: int, K: int, config: int = 0, layer: str = "single",
                rows: slice | None = None) -> np.ndarray:
    """fp16 [M,K] activations; `rows` returns a row slice of the same tensor."""
    g = _rng(config, layer, _ROLE_X)
    x = g.standard_normal((M, K), dtype=np.float32) * np.float32(ACT_STD)
    x[:, outlier_channels(K, config, layer)] *= np.float32(OUTLIER_GAIN)
    if rows is not None:
        x = x[rows]
    return x.astype(np.float16)


def weights(N: int, K: int, config: int = 0, layer: str = "single") -> np.ndarray:
    """fp16 [N,K] weights, row n = output channel n (K contiguous)."""
    g = _rng(config, layer, _ROLE_W)
    w = g.standard_normal((N, K), dtype=np.float32) * np.float32(WEIGHT_STD)
    return w.astype(np.float16)


def bias(N: int, config: int = 0, layer: str = "single") -> np.ndarray:
    g = _rng(config, layer, _ROLE_B)
    return (g.standard_normal(N, dtype=np.float32) * np.float32(BIAS_STD)).astype(np.float16)


def tensors(shape: Shape):
    """(x, w, bias_or_None) of one Shape."""
    x = activations(shape.M, shape.K, shape.config, shape.layer)
    w = weights(shape.N, shape.K, shape.config, shape.layer)
    b = bias(shape.N, shape.config, shape.layer) if shape.bias else None
    return x, w, b


def sha256(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()
