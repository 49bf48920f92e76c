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
            ql.ql_w8a8_gemm(self.xq, self.sx, sh.M, sh.K, k, self.sw, self.bias, sh.N, y, self.ws)
        else:
            ql.ql_w4a8_gemm(self.xq, self.sx, sh.M, sh.K, k, sh.group, self.bias, sh.N, y, self.ws)

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


def graph_time_ms(torch, fn, reps, warm=10, rounds=5):
    """Average GPU time of fn(i) with `reps` launches captured into one HIP graph and replayed: for kernels
    of a few microseconds the Python/ctypes/hipLaunchKernel path (~7 us per call) would otherwise be what is
    measured.  Best of `rounds` replays, each bracketed by HIP events on the replay stream."""
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(reps):
            fn(i)
    g.replay()
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(rounds):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        g.replay()
        b.record()
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b) / reps)
    return best


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


def measured_ceilings(torch, ql):
    """What this GPU sustains on the matrix pipe and on HBM reads, measured here and now (context for
    `roofline.frac`, which stays against the published peaks): register-resident int8 MFMA loop on every CU
    with constant and with hashed operands, and a read stream over 2 GiB."""
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    out = {}
    for name, rnd in (("mfma_int8_constant_operands_tops", False), ("mfma_int8_random_operands_tops", True)):
        ops = [0]

        def f(i, rnd=rnd):
            ops[0] = ql.ql_probe_mfma_int8(2048, 2000, rnd, sink)
        ms = best_time_ms(torch, f, 3, warm=2, rounds=3)
        out[name] = round(ops[0] / (ms * 1e-3) / 1e12, 1)
    buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda:0")
    buf.zero_()
    ms = best_time_ms(torch, lambda i: ql.ql_probe_hbm_read(buf, sink), 5, warm=2, rounds=3)
    out["hbm_read_stream_gbs"] = round(buf.numel() / (ms * 1e-3) / 1e9, 1)
    del buf
    torch.cuda.empty_cache()
    return out


def cpu_baseline(shapes, synth):
    """The oracle as it stands, timed on the host cores on the same workload (all rows)."""
    import oracle
    from oracle import linear as olin
    t_total, ops, passes = 0.0, 0, 0
    prepared = []
    for sh in shapes:
        x, w, b = synth.tensors(sh)
        if sh.bits == 8:
            wq, sw = oracle.quant_weight_int8(w)        # offline, not timed
            prepared.append((sh, lambda x=x, wq=wq, sw=sw, b=b: oracle.linear_w8a8(x, wq, sw, b)))
        else:
            p, _, s = oracle.quant_weight_int4(w, sh.group)
            prepared.append((sh, lambda x=x, p=p, s=s, g=sh.group, b=b: oracle.linear_w4a8(x, p, s, g, b)))
    while t_total < 10.0 and passes < 20:               # bounded: about 10 s of CPU work
        for sh, run in prepared:
            t0 = time.perf_counter()
            run()
            t_total += time.perf_counter() - t0
            ops += sh.ops
        passes += 1
    return dict(value=ops / t_total / 1e12, unit="TOPS", cores=olin.num_threads(), kind="oracle",
                sample=f"all {len(shapes)} linears of the workload in full (every token row), {passes} passes, "
                       f"{ops / 1e9:.1f} GOP in {t_total:.1f} s; weight quantization not timed")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="config1",
                    help="config1 (default), config2, config3, config4 (long prefill), decode8, decode4 "
                         "(the 7B-class decode GEMMs of config 4, int8 / int4 weights)")
    ap.add_argument("--decode-m", type=int, default=1, help="tokens of the decode workloads: 1 .. 1024 (automatic kernel choice: beyond 32 tokens the tile kernels where they are estimated faster)")
    ap.add_argument("--variant", type=int, default=0, help="kernel variant (0 = automatic)")
    ap.add_argument("--weight-copies", type=int, default=0,
                    help="copies of every weight matrix the launches rotate through (0 = enough that the copies of "
                         "a matrix exceed three times the 256 MB Infinity Cache, i.e. weights come from HBM as in a model)")
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
    decode = args.workload.startswith("decode")
    if decode:
        bits = int(args.workload.replace("decode", ""))
        cfg = 4
        if not 1 <= args.decode_m <= 1024:
            sys.exit("bench.py: --decode-m must be between 1 and 1024 (the decode kernels' range)")
        shapes = [synth.Shape(s.config, s.layer, args.decode_m, s.K, s.N, s.bits, s.group, s.bias)
                  for s in synth.workload(4) if s.M == 1 and s.bits == bits]
    else:
        cfg = int(args.workload.replace("config", ""))
        shapes = [s for s in synth.workload(cfg) if s.M > 32]
    descr = {1: "config1: W8A8 linears of a 1B-class decoder layer, prefill M=2048, d=1536 (qkv, o, gate_up, down)",
             2: "config2: W8A8 linears (+bias) of a 7B-class decoder layer, prefill M=4096, d=4096",
             3: "config3: W4A8 (group 128) linears of a 7B-class decoder layer, prefill M=4096, d=4096",
             4: "config4: long-reasoning prefill of the down projection, M=16384, W8A8"}[cfg]
    if decode:
        descr = (f"config4 decode: {'W8A8' if bits == 8 else 'W4A8 (group 128)'} linears of a 7B-class decoder "
                 f"layer, M={args.decode_m} (qkv, o, gate_up, down), weights rotated over >768 MB of copies")

    def copies_for(s):   # enough copies that the weights cannot come from the Infinity Cache, per matrix:
        if args.weight_copies:   # the per-layer GEMM timings below rotate one matrix at a time
            return args.weight_copies
        return -(-3 * MALL_BYTES // (s.N * s.K // (1 if s.bits == 8 else 2)))

    layers = [Layer(s, torch, ql, synth, copies_for(s)) for s in shapes]
    total_ops = sum(s.ops for s in shapes)

    def step(i=0):
        for l in layers:
            l.linear(i)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    graph = None
    if decode:
        # a decode step is 8 launches of 4-16 us: replay them from a HIP graph so that the GPU, not the
        # launch path, is timed (the warm-up above ran every kernel once outside the capture)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(args.steps):
                step(i)
        graph.replay()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graph is not None:
        graph.replay()
    else:
        for i in range(args.steps):
            step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = total_ops / (dt / args.steps) / 1e12
    unit = "TOPS"
    if decode:   # memory-bound: report the algorithmic bytes of the GEMMs per second
        value = sum(l.gemm_bytes() for l in layers) / (dt / args.steps) / 1e9
        unit = "GB/s"
    log(f"[step] {descr}: {ms_per_step:.4f} ms/step, {value:.1f} {unit} whole layer (quant + GEMM + epilogue)")

    out = {
        "metric": METRIC, "value": round(value, 2), "unit": unit, "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8",
        "data": "synthetic; every launch takes the next of enough copies of its weight matrix that the weights come "
                "from HBM, not from the 256 MB Infinity Cache" if not args.weight_copies else
                f"synthetic; {args.weight_copies} cop{'y' if args.weight_copies == 1 else 'ies'} of every weight matrix",
        "launch": "hip graph replay" if decode else "stream launches",
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
        timer = graph_time_ms if decode else best_time_ms
        reps_l = max(reps, len(l.kernels))   # at least one cycle through the weight copies
        gemm_ms.append(timer(torch, l.gemm, reps_l))
        gemm_ms_b2b.append(best_time_ms(torch, l.gemm, reps_l, per_launch=True, warm=0, rounds=1))
        # the quantizer runs 2-10 us: replay it from a HIP graph, or the launch path is what gets timed
        quant_ms.append(graph_time_ms(torch, lambda i, l=l: l.quant(), reps))
    achieved = total_ops / (sum(gemm_ms) * 1e-3) / 1e12
    roof = {"bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
            "frac": round(achieved / PEAK_INT8_TOPS, 4), "traffic": profiled_traffic(cfg),
            "kernel": "gemm_prefill_kernel (int8 MFMA GEMM + fused dequant epilogue), one launch per linear"}
    if decode:
        achieved = sum(l.gemm_bytes() for l in layers) / (sum(gemm_ms) * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": None,
                "kernel": "gemm_decode_kernel (weight-streaming int8 MFMA GEMM + fused epilogue), one launch per linear",
                "per_layer_gbs": {l.sh.layer: round(l.gemm_bytes() / (t * 1e-3) / 1e9, 1) for l, t in zip(layers, gemm_ms)}}
    out["roofline"] = {
        **roof,
        "launch_us": {l.sh.layer: round(t * 1e3, 2) for l, t in zip(layers, gemm_ms)},
        "launch_us_event_pair_each": {l.sh.layer: round(t * 1e3, 2) for l, t in zip(layers, gemm_ms_b2b)},
        "per_layer_tops": {l.sh.layer: round(l.sh.ops / (t * 1e-3) / 1e12, 1) for l, t in zip(layers, gemm_ms)},
        "act_quant_us": {l.sh.layer: round(t * 1e3, 2) for l, t in zip(layers, quant_ms)},
        "act_quant_gbs": {l.sh.layer: round(l.quant_bytes() / (t * 1e-3) / 1e9, 1) for l, t in zip(layers, quant_ms)},
    }
    ceil = measured_ceilings(torch, ql)
    ref = ceil["hbm_read_stream_gbs"] if decode else ceil["mfma_int8_random_operands_tops"]
    out["roofline"]["measured_ceilings"] = {**ceil, "achieved_over_measured": round(out["roofline"]["achieved"] / ref, 4),
                                            "note": "context only; frac is against the published peak. The matrix-pipe probe "
                                                    "keeps its operands in registers; hashed operands lower the shader clock"}
    log("[roofline]", json.dumps(out["roofline"]))

    # ---- detail: GEMM-only throughput of the other configurations (parity-test cases, not the headline)
    if not args.no_detail and not decode:
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
                copies = -(-3 * MALL_BYTES // wbytes)
                base = Layer(shs[0], torch, ql, synth, copies)
                for sh in shs:
                    l = base if sh is shs[0] else Layer(sh, torch, ql, synth, 1)
                    if l is not base:
                        l.kernels, l.scales, l.sw = base.kernels, base.scales, base.sw
                    l.quant()
                    r = max(20, copies) if not decode else max(50, 2 * copies)   # at least one cycle through the copies
                    timer = graph_time_ms if decode else best_time_ms
                    t_bb = timer(torch, l.gemm, r)
                    t_lin = timer(torch, l.linear, r, warm=3, rounds=2)
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
        # between decode and prefill: 64 and 256 tokens on the 7B-class shapes (weights rotated as for decode);
        # these are weight-stream-bound, so the rate is weight bytes per second
        for base_sh in [s_ for s_ in synth.workload(4) if s_.M == 1]:
            wbytes = base_sh.N * base_sh.K * base_sh.bits // 8
            copies = -(-3 * MALL_BYTES // wbytes)
            base = None
            for M in (64, 256):
                sh = synth.Shape(base_sh.config, base_sh.layer, M, base_sh.K, base_sh.N, base_sh.bits, base_sh.group, base_sh.bias)
                l = Layer(sh, torch, ql, synth, copies if base is None else 1)
                if base is None:
                    base = l
                else:
                    l.kernels, l.scales, l.sw = base.kernels, base.scales, base.sw
                l.quant()
                r = max(50, 2 * copies)
                t_bb = graph_time_ms(torch, l.gemm, r)
                t_lin = graph_time_ms(torch, l.linear, r)
                row = {"shape": sh.name, "gemm_us": round(t_bb * 1e3, 2), "linear_us": round(t_lin * 1e3, 2),
                       "weight_gbs": round(wbytes / (t_bb * 1e-3) / 1e9, 1),
                       "frac_hbm_peak": round(wbytes / (t_bb * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                       "weight_copies_rotated": copies}
                detail.append(row)
                log("[detail]", json.dumps(row))
            del base, l
            torch.cuda.empty_cache()
        # context for the paper's Table 3 (INT8 against FP16 prefill latency, weight memory): the same linears
        # as FP16 GEMMs of the vendor library (torch.matmul -> hipBLASLt/rocBLAS), a comparison system, not
        # part of this library; W8A8 / W4A8 = quantize + GEMM + epilogue through ql_*_linear
        for c, bits_list in ((1, (8,)), (2, (8, 4))):
            tot = {"fp16": 0.0, "w8a8": 0.0, "w4a8": 0.0}
            mem = {"fp16": 0, "w8a8": 0, "w4a8": 0}
            for sh in [s_ for s_ in synth.workload(c) if s_.M > 32]:
                xh = torch.randn((sh.M, sh.K), dtype=torch.float16, device="cuda:0")
                wh = torch.randn((sh.N, sh.K), dtype=torch.float16, device="cuda:0") * 0.02
                tot["fp16"] += best_time_ms(torch, lambda i: torch.matmul(xh, wh.t()), 20, warm=5, rounds=3)
                mem["fp16"] += sh.N * sh.K * 2
                del xh, wh
                for b in bits_list + ((4,) if c == 1 else ()):
                    l = Layer(synth.Shape(sh.config, sh.layer, sh.M, sh.K, sh.N, b, 0 if b == 8 else 128, sh.bias),
                              torch, ql, synth)
                    key = "w8a8" if b == 8 else "w4a8"
                    tot[key] += best_time_ms(torch, l.linear, 20, warm=5, rounds=3)
                    mem[key] += l.weight_bytes + (sh.N * 4 if b == 8 else 0)
                    del l
                torch.cuda.empty_cache()
            row = {"shape": f"layer.c{c}.prefill", "fp16_library_gemm_us": round(tot["fp16"] * 1e3, 1),
                   "w8a8_linear_us": round(tot["w8a8"] * 1e3, 1), "w4a8_linear_us": round(tot["w4a8"] * 1e3, 1),
                   "w8a8_speedup_over_fp16": round(tot["fp16"] / tot["w8a8"], 2),
                   "w4a8_speedup_over_fp16": round(tot["fp16"] / tot["w4a8"], 2),
                   "weight_mb": {k: round(v / 1e6, 1) for k, v in mem.items()}}
            log("[detail]", json.dumps(row))
            detail.append(row)
        # the activation quantizer alone and with the paper's two operand transforms fused in front of it
        # (SmoothQuant per-channel multiply, block Hadamard rotation), graph-replayed; 3 B per element
        for M, K in ((2048, 1536), (4096, 4096), (4096, 11008)):
            x = torch.randn((M, K), dtype=torch.float16, device="cuda:0")
            kl = torch.empty(ql.ql_act_kernel_bytes(M, K), dtype=torch.uint8, device="cuda:0")
            sxv = torch.empty(M, dtype=torch.float32, device="cuda:0")
            inv = torch.rand(K, dtype=torch.float32, device="cuda:0") + 0.5
            B = ql.ql_hadamard_block(K)
            scratch = torch.zeros(1, dtype=torch.int32, device="cuda:0")
            static = torch.full((1,), 0.05, dtype=torch.float32, device="cuda:0")
            gam = (torch.rand(K, dtype=torch.float32, device="cuda:0") + 0.5).to(torch.float16)
            row = {"shape": f"act_quant.M{M}.K{K}", "hadamard_block": B}
            for name, fn in (("plain", lambda i: ql.ql_quant_act_per_token(x, None, kl, sxv)),
                             ("smoothquant", lambda i: ql.ql_quant_act_per_token_transformed(x, inv, 0, None, kl, sxv)),
                             ("hadamard", lambda i: ql.ql_quant_act_per_token_transformed(x, None, B, None, kl, sxv)),
                             # RMSNorm (textbook definition) fused in front of the quantizer
                             ("rmsnorm", lambda i: ql.ql_quant_act_rmsnorm(x, gam, 1e-6, None, kl, sxv)),
                             # the other quantizer forms: Eq. 2 as printed, per-tensor dynamic, calibrated static scale
                             ("eq2_per_token", lambda i: ql.ql_quant_act_opt(x, ql.QL_RANGE_EQ2, ql.QL_SCOPE_FINE, None,
                                                                             None, kl, sxv, None)),
                             ("per_tensor", lambda i: ql.ql_quant_act_opt(x, ql.QL_RANGE_SYMMETRIC, ql.QL_SCOPE_TENSOR,
                                                                          None, None, kl, sxv, scratch)),
                             ("static_scale", lambda i: ql.ql_quant_act_opt(x, ql.QL_RANGE_SYMMETRIC, ql.QL_SCOPE_STATIC,
                                                                            static, None, kl, sxv, None))):
                t = graph_time_ms(torch, fn, 50)
                row[name + "_us"] = round(t * 1e3, 2)
                row[name + "_gbs"] = round(3 * M * K / (t * 1e-3) / 1e9, 1)
            log("[detail]", json.dumps(row))
            detail.append(row)
            del x, kl
        out["detail"] = detail

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(shapes, synth)
        log("[cpu]", json.dumps(out["cpu_baseline"]))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
