"""The four quantized linears of a decoder layer, chained on the device (buffer management and call order only:
every step runs in the library's kernels).

    x [M,d] --qkv--> [M,3d] --(first d columns stand in for the attention output)--> o --> [M,d]
      --gate_up--> [M,2F] --SwiGLU + per-token quantizer (ql_quant_act_swiglu)--> int8 [M,F] --down--> [M,d]

This is the prefill workload whose latency and weight memory the paper tabulates by batch size (Efficiency
Evaluation, Table 3: INT8 against FP16); attention itself, the normalisations and the residual adds are not part of
the quantized-linear path and are left out (the slice of the QKV output only makes the four GEMMs depend on each
other the way a layer's do).
"""
from __future__ import annotations

import torch

from . import binding as ql


class DecoderLayerLinears:
    def __init__(self, w_qkv, w_o, w_gate_up, w_down, bits: int, max_tokens: int, biases=None):
        """w_*: fp16 device tensors [N,K] (qkv [3d,d], o [d,d], gate_up [2F,d], down [d,F]); bits 8 (per-channel
        int8) or 4 (int4, groups of 128); biases: optional dict name -> fp16 [N]."""
        self.bits, self.group = bits, (0 if bits == 8 else 128)
        self.d = w_o.shape[0]
        self.F = w_down.shape[1]
        assert w_qkv.shape == (3 * self.d, self.d) and w_gate_up.shape == (2 * self.F, self.d) and w_down.shape == (self.d, self.F)
        dev = w_o.device
        self.w = {}
        self.weight_bytes = 0
        for name, w in (("qkv", w_qkv), ("o", w_o), ("gate_up", w_gate_up), ("down", w_down)):
            N, K = w.shape
            _, sb, kb = ql.ql_weight_bytes(N, K, bits, self.group)
            scales = torch.empty(sb, dtype=torch.uint8, device=dev)
            kern = torch.empty(kb, dtype=torch.uint8, device=dev)
            ql.ql_quant_weight(w.contiguous(), bits, self.group, None, scales, kern)
            self.w[name] = (kern, scales.view(torch.float32) if bits == 8 else None, (biases or {}).get(name), N, K)
            self.weight_bytes += kb + (sb if bits == 8 else 0)
        M = max_tokens
        self.max_tokens = M
        self.y_qkv = torch.empty((M, 3 * self.d), dtype=torch.float16, device=dev)
        self.y_o = torch.empty((M, self.d), dtype=torch.float16, device=dev)
        self.y_gu = torch.empty((M, 2 * self.F), dtype=torch.float16, device=dev)
        self.y = torch.empty((M, self.d), dtype=torch.float16, device=dev)
        self.xq = torch.empty(ql.ql_act_kernel_bytes(M, self.F), dtype=torch.uint8, device=dev)
        self.sx = torch.empty(M, dtype=torch.float32, device=dev)
        ws = max(ql.ql_workspace_bytes(M, N, K, bits) for (_, _, _, N, K) in self.w.values())
        self.ws = torch.empty(ws, dtype=torch.uint8, device=dev)

    def _linear(self, x, name, y):
        kern, sw, bias, N, _ = self.w[name]
        if self.bits == 8:
            ql.ql_w8a8_linear(x, kern, sw, bias, N, y, self.ws)
        else:
            ql.ql_w4a8_linear(x, kern, self.group, bias, N, y, self.ws)

    def forward(self, x):
        """x fp16 [M,d], M <= max_tokens; returns the fp16 [M,d] output of the down projection (a view of an
        internal buffer, overwritten by the next call).  Everything is enqueued on torch's current stream."""
        M = x.shape[0]
        assert M <= self.max_tokens and x.shape[1] == self.d
        y_qkv, y_o, y_gu, y = self.y_qkv[:M], self.y_o[:M], self.y_gu[:M], self.y[:M]
        self._linear(x, "qkv", y_qkv)
        self._linear(y_qkv[:, :self.d], "o", y_o)
        self._linear(y_o, "gate_up", y_gu)
        ql.ql_quant_act_swiglu(y_gu, None, self.xq, self.sx)
        kern, sw, bias, N, K = self.w["down"]
        if self.bits == 8:
            ql.ql_w8a8_gemm(self.xq, self.sx, M, K, kern, sw, bias, N, y, self.ws)
        else:
            ql.ql_w4a8_gemm(self.xq, self.sx, M, K, kern, self.group, bias, N, y, self.ws)
        return y
