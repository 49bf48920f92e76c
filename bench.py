#!/usr/bin/env python3
"""Benchmark of the quantized linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config1] [--no-detail] [--no-cpu]

One "step" is one pass of the whole hot path over one batch: for every linear of the workload's
decoder layer, per-token activation quantization + int8 (or int4xint8) GEMM + dequantization
epilogue (`ql_w8a8_linear` / `ql_w4a8_linear`), inputs and quantized weights already resident in
HBM.  Prints ONE JSON line (see the keys below); per-shape detail for the other configurations
goes into its "detail" list.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

METRIC = "int8 TOPS (% of MFMA peak) prefill GEMM; HBM GB/s (% peak) decode GEMM"
PEAK_INT8_TOPS = 5000.0     # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published
MALL_BYTES = 256 << 20      # Infinity Cache: decode weights are rotated over > 2x this


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Layer:
    """Device-resident state of one linear: input, quantized weights, output, workspace."""

    def __init__(self, sh, torch, ql, synth, copies=1):
        self.sh = sh
        dev = "cuda:0"
        x, w, b = synth.tensors(sh)
        self.x = torch.from_numpy(x).to(dev)
        wd = torch.from_numpy(w).to(dev)
        self.bias = torch.from_numpy(b).to(dev) if b is not None else None
        cb, sb, kb = ql.ql_weight_bytes(sh.N, sh.K, sh.bits, sh.group)
        self.scales = torch.empty(sb, dtype=torch.uint8, device=dev)
        kern = torch.empty(kb, dtype=torch.uint8, device=dev)
        ql.ql_quant_weight(wd, sh.bits, sh.group, None, self.scales, kern)
        self.kernels = [kern] + [kern.clone() for _ in range(copies - 1)]
        self.sw = self.scales.view(torch.float32) if sh.bits == 8 else None
        self.ys = [torch.empty((sh.M, sh.N), dtype=torch.float16, device=dev) for _ in range(min(copies, 4))]
        self.ws = torch.empty(ql.ql_workspace_bytes(sh.M, sh.N, sh.K, sh.bits), dtype=torch.uint8, device=dev)
        self.xq = torch.empty(ql.ql_act_kernel_bytes(sh.M, sh.K), dtype=torch.uint8, device=dev)
        self.sx = torch.empty(sh.M, dtype=torch.float32, device=dev)
        self.weight_bytes = kb
        self.ql = ql
        del wd

    def linear(self, i=0):
        sh, ql = self.sh, self.ql
        k, y = self.kernels[i % len(self.kernels)], self.ys[i % len(self.ys)]
        if sh.bits == 8:
            ql.ql_w8a8_linear(self.x, k, self.sw, self.bias, sh.N, y, self.ws)
        else:
            ql.ql_w4a8_linear(self.x, k, sh.group, self.bias, sh.N, y, self.ws)

    def quant(self):
        self.ql.ql_quant_act_per_token(self.x, None, self.xq, self.sx)

    def gemm(self, i=0):
        sh, ql = self.sh, self.ql
        k, y = self.kernels[i % len(self.kernels)], self.ys[i % len(self.ys)]
        if sh.bits == 8:
            ql.ql_w8a8_gemm(self.xq, self.sx, sh.M, sh.K, k, self.sw, self.bias, sh.N, y)
        else:
            ql.ql_w4a8_gemm(self.xq, self.sx, sh.M, sh.K, k, sh.group, self.bias, sh.N, y)

    # algorithmic bytes of one GEMM launch: int8 activations + their scales, weights (+ scales), fp16 output (+ bias)
    def gemm_bytes(self):
        sh = self.sh
        wbytes = sh.N * sh.K if sh.bits == 8 else sh.N * sh.K // 2 + sh.N * (sh.K // sh.group) * 2
        sbytes = sh.N * 4 if sh.bits == 8 else 0
        return sh.M * sh.K + sh.M * 4 + wbytes + sbytes + sh.M * sh.N * 2 + (sh.N * 2 if sh.bias else 0)

    def quant_bytes(self):
        return self.sh.M * self.sh.K * 3 + self.sh.M * 4


def event_time_ms(torch, fn, reps, per_launch):
    """Average GPU time of fn() in ms over `reps` launches on torch's current stream (the stream the
    library launches on), from HIP events: one pair per launch, or one pair around all launches."""
    if per_launch:
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i, (a, b) in enumerate(ev):
            a.record()
            fn(i)
            b.record()
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in ev) / reps
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for i in range(reps):
        fn(i)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def best_time_ms(torch, fn, reps, per_launch=False, warm=30, rounds=5):
    """Warm up, then the best of `rounds` event-timed averages (the first tens of launches on fresh buffers
    run 10-15 % slower)."""
    for i in range(warm):
        fn(i)
    return min(event_time_ms(torch, fn, reps, per_launch) for _ in range(rounds))


def profiled_traffic(cfg):
    """HBM bytes per GEMM launch (average over the workload's linears) from the committed rocprofv3
    FETCH_SIZE + WRITE_SIZE summary of this workload, copy-kernel calibrated; None if not profiled."""
    path = os.path.join(ROOT, "profiles", f"prefill_gemm_config{cfg}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch="):
                return float(line.split("=", 1)[1])
    except OSError:
        pass
    return None


def cpu_baseline(shapes, synth):
    """The oracle as it stands, timed on the host cores on the same workload (all rows)."""
    import oracle
    from oracle import linear as olin
    t_total, ops = 0.0, 0
    for sh in shapes:
        x, w, b = synth.tensors(sh)
        if sh.bits == 8:
            wq, sw = oracle.quant_weight_int8(w)        # offline, not timed
            t0 = time.perf_counter()
            oracle.linear_w8a8(x, wq, sw, b)
        else:
            p, _, s = oracle.quant_weight_int4(w, sh.group)
            t0 = time.perf_counter()
            oracle.linear_w4a8(x, p, s, sh.group, b)
        t_total += time.perf_counter() - t0
        ops += sh.ops
    return dict(value=ops / t_total / 1e12, unit="TOPS", cores=olin.num_threads(), kind="oracle",
                sample=f"all {len(shapes)} linears of the workload in full (every token row), "
                       f"{ops / 1e9:.1f} GOP in {t_total:.1f} s; weight quantization not timed")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="config1", help="config1 (default), config2, config3")
    ap.add_argument("--variant", type=int, default=0, help="kernel variant (0 = automatic)")
    ap.add_argument("--no-detail", action="store_true", help="skip the per-shape table of the other configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--only-step", action="store_true", help="only the timed steps (for profiling)")
    ap.add_argument("--copy-only", action="store_true",
                    help="run a plain 1 GiB device-to-device copy 5 times and exit (calibrates the profiler's "
                         "FETCH_SIZE / WRITE_SIZE counters against a known size)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py measures one GPU: every box of this build has one MI355X and the path uses no "
            "collectives; --gpus must be 1")
        sys.exit(2)

    import torch
    from paper_2512_23367_amd import binding as ql
    from paper_2512_23367_amd import synth

    if not torch.cuda.is_available():
        log("no GPU visible")
        sys.exit(1)
    if args.copy_only:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_per_launch": src.numel() * 4, "launches": 5}), flush=True)
        return
    ql.lib()
    ql.ql_set_kernel_variant(args.variant)
    cfg = int(args.workload.replace("config", ""))
    shapes = [s for s in synth.workload(cfg) if s.M > 32]
    descr = {1: "config1: W8A8 linears of a 1B-class decoder layer, prefill M=2048, d=1536 (qkv, o, gate_up, down)",
             2: "config2: W8A8 linears (+bias) of a 7B-class decoder layer, prefill M=4096, d=4096",
             3: "config3: W4A8 (group 128) linears of a 7B-class decoder layer, prefill M=4096, d=4096",
             4: "config4: long-reasoning prefill of the down projection, M=16384, W8A8"}[cfg]

    layers = [Layer(s, torch, ql, synth) for s in shapes]
    total_ops = sum(s.ops for s in shapes)

    def step(i=0):
        for l in layers:
            l.linear(i)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = total_ops / (dt / args.steps) / 1e12
    log(f"[step] {descr}: {ms_per_step:.4f} ms/step, {value:.1f} TOPS whole layer (quant + GEMM + epilogue)")

    out = {
        "metric": METRIC, "value": round(value, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": descr, "layers": [s.name for s in shapes],
                   "weights": "int8 per-channel" if shapes[0].bits == 8 else "int4 group-128",
                   "activations": "int8 per-token dynamic", "output": "fp16"},
    }
    if args.only_step:
        print(json.dumps(out), flush=True)
        return

    # ---- roofline of the dominant kernel (the prefill GEMM), timed with HIP events on the launch stream
    for l in layers:
        l.quant()
    reps = max(20, min(args.steps, 100))
    gemm_ms, gemm_ms_b2b, quant_ms = [], [], []
    for l in layers:
        # one event pair around `reps` back-to-back launches: per-launch pairs add ~2-7 us of event
        # overhead to kernels this short and would not agree with the profiler's kernel durations
        gemm_ms.append(best_time_ms(torch, l.gemm, reps))
        gemm_ms_b2b.append(best_time_ms(torch, l.gemm, reps, per_launch=True, warm=0, rounds=1))
        quant_ms.append(best_time_ms(torch, lambda i, l=l: l.quant(), reps))
    achieved = total_ops / (sum(gemm_ms) * 1e-3) / 1e12
    out["roofline"] = {
        "bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
        "frac": round(achieved / PEAK_INT8_TOPS, 4), "traffic": profiled_traffic(cfg),
        "kernel": "gemm_prefill_kernel (int8 MFMA GEMM + fused dequant epilogue), one launch per linear",
        "launch_us": {l.sh.layer: round(t * 1e3, 2) for l, t in zip(layers, gemm_ms)},
        "launch_us_event_pair_each": {l.sh.layer: round(t * 1e3, 2) for l, t in zip(layers, gemm_ms_b2b)},
        "per_layer_tops": {l.sh.layer: round(l.sh.ops / (t * 1e-3) / 1e12, 1) for l, t in zip(layers, gemm_ms)},
        "act_quant_us": {l.sh.layer: round(t * 1e3, 2) for l, t in zip(layers, quant_ms)},
        "act_quant_gbs": {l.sh.layer: round(l.quant_bytes() / (t * 1e-3) / 1e9, 1) for l, t in zip(layers, quant_ms)},
    }
    log("[roofline]", json.dumps(out["roofline"]))

    # ---- detail: GEMM-only throughput of the other configurations (parity-test cases, not the headline)
    if not args.no_detail:
        detail = []
        del layers
        torch.cuda.empty_cache()
        for c in (2, 3, 4):
            shapes_c = [s for s in synth.workload(c) if not (c == cfg and s.M > 32)]
            # decode shapes differ only in M: quantize each weight matrix once and rotate over enough
            # copies that the stream comes from HBM, not from the Infinity Cache
            groups = {}
            for sh in shapes_c:
                groups.setdefault((sh.layer, sh.K, sh.N, sh.bits, sh.M <= 32), []).append(sh)
            for (layer, K, N, bits, _), shs in groups.items():
                wbytes = N * K // (1 if bits == 8 else 2)
                decode = shs[0].M <= 32
                copies = -(-3 * MALL_BYTES // wbytes) if decode else 1
                base = Layer(shs[0], torch, ql, synth, copies)
                for sh in shs:
                    l = base if sh is shs[0] else Layer(sh, torch, ql, synth, 1)
                    if l is not base:
                        l.kernels, l.scales, l.sw = base.kernels, base.scales, base.sw
                    l.quant()
                    r = 20 if not decode else max(50, 2 * copies)
                    t_bb = best_time_ms(torch, l.gemm, r)
                    t_lin = best_time_ms(torch, l.linear, r, warm=3, rounds=2)
                    row = {"shape": sh.name, "gemm_us": round(t_bb * 1e3, 2), "linear_us": round(t_lin * 1e3, 2)}
                    if not decode:
                        row["tops"] = round(sh.ops / (t_bb * 1e-3) / 1e12, 1)
                        row["frac_mfma_peak"] = round(row["tops"] / PEAK_INT8_TOPS, 4)
                    else:
                        row["gbs"] = round(l.gemm_bytes() / (t_bb * 1e-3) / 1e9, 1)
                        row["frac_hbm_peak"] = round(row["gbs"] / PEAK_HBM_GBS, 4)
                        row["weight_copies_rotated"] = copies
                    detail.append(row)
                    log("[detail]", json.dumps(row))
                del base, l
                torch.cuda.empty_cache()
        out["detail"] = detail

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(shapes, synth)
        log("[cpu]", json.dumps(out["cpu_baseline"]))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
