#!/usr/bin/env python3
"""Benchmark of the quantized linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config2] [--no-detail] [--no-decode] [--no-cpu]

One "step" is one pass of the whole hot path over one batch: for every linear of the workload's
decoder layer, per-token activation quantization + int8 (or int4xint8) GEMM + dequantization
epilogue (`ql_w8a8_linear` / `ql_w4a8_linear`), inputs and quantized weights already resident in
HBM.  Prints ONE JSON line: the headline (whole-layer throughput of the timed steps), `roofline`
(the GEMM kernel alone: median of at least 5 repeats of at least 50 back-to-back launches per linear,
HIP events on the launch stream; plus the decode GEMMs of the 7B-class shapes against HBM
bandwidth), `cpu_baseline` (the CPU oracle timed on the host cores) and a compact `detail` list
for the other configurations.  Progress and per-shape rows go to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

METRIC = "int8 TOPS (% of MFMA peak) prefill GEMM; HBM GB/s (% peak) decode GEMM"
PEAK_INT8_TOPS = 5000.0     # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published
MALL_BYTES = 256 << 20      # Infinity Cache: weights are rotated over 3x this so that they come from HBM
MIN_LAUNCHES, MIN_REPEATS = 50, 5   # timing protocol of the roofline figures
WARM_PASSES = 60                    # untimed passes over the workload's GEMMs before the first timing


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Layer:
    """Device-resident state of one linear: input, quantized weights, output, workspace."""

    def __init__(self, sh, torch, ql, synth, copies=1, share=None, hashes=None):
        self.sh = sh
        dev = "cuda:0"
        x = synth.activations(sh.M, sh.K, sh.config, sh.layer)
        self.x = torch.from_numpy(x).to(dev)
        b = synth.bias(sh.N, sh.config, sh.layer) if sh.bias else None
        self.bias = torch.from_numpy(b).to(dev) if b is not None else None
        if hashes is not None:
            hashes[sh.name + ".x"] = synth.sha256(x)[:16]
        if share is not None:     # same weight matrix as another Layer (the decode shapes differ only in M)
            self.scales, self.kernels, self.sw, self.weight_bytes = share.scales, share.kernels, share.sw, share.weight_bytes
        else:
            w = synth.weights(sh.N, sh.K, sh.config, sh.layer)
            if hashes is not None:
                hashes[sh.name + ".w"] = synth.sha256(w)[:16]
            wd = torch.from_numpy(w).to(dev)
            cb, sb, kb = ql.ql_weight_bytes(sh.N, sh.K, sh.bits, sh.group)
            self.scales = torch.empty(sb, dtype=torch.uint8, device=dev)
            kern = torch.empty(kb, dtype=torch.uint8, device=dev)
            ql.ql_quant_weight(wd, sh.bits, sh.group, None, self.scales, kern)
            self.kernels = [kern] + [kern.clone() for _ in range(copies - 1)]
            self.sw = self.scales.view(torch.float32) if sh.bits == 8 else None
            self.weight_bytes = kb
            del wd
        self.ys = [torch.empty((sh.M, sh.N), dtype=torch.float16, device=dev) for _ in range(min(len(self.kernels), 4))]
        self.ws = torch.empty(ql.ql_workspace_bytes(sh.M, sh.N, sh.K, sh.bits), dtype=torch.uint8, device=dev)
        self.xq = torch.empty(ql.ql_act_kernel_bytes(sh.M, sh.K), dtype=torch.uint8, device=dev)
        self.sx = torch.empty(sh.M, dtype=torch.float32, device=dev)
        self.ql = ql

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


def copies_for(sh, forced=0):
    """Copies of a weight matrix the launches rotate through: enough that consecutive launches never find it in
    the Infinity Cache (in a model a layer's weights always come from HBM)."""
    if forced:
        return forced
    return -(-3 * MALL_BYTES // (sh.N * sh.K // (1 if sh.bits == 8 else 2)))


def event_times_ms(torch, fn, launches, repeats, warm):
    """`repeats` averages (ms per launch), each from one HIP-event pair on torch's current stream (the stream the
    library launches on) around `launches` back-to-back launches; `warm` untimed launches first."""
    for i in range(warm):
        fn(i)
    out = []
    for _ in range(repeats):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(launches):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        out.append(a.elapsed_time(b) / launches)
    return out


def graph_times_ms(torch, fn, launches, repeats, warm=10):
    """The same with the launches captured into one HIP graph and replayed: for kernels of a few microseconds the
    Python/ctypes/hipLaunchKernel path (~7 us per call) would otherwise be what is measured."""
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(launches):
            fn(i)
    g.replay()
    torch.cuda.synchronize()
    out = []
    for _ in range(repeats):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        g.replay()
        b.record()
        torch.cuda.synchronize()
        out.append(a.elapsed_time(b) / launches)
    return out


def median_ms(torch, fn, launches=MIN_LAUNCHES, repeats=MIN_REPEATS, graph=False, warm=30):
    ts = graph_times_ms(torch, fn, launches, repeats) if graph else event_times_ms(torch, fn, launches, repeats, warm)
    return statistics.median(ts)


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


def gpu_state_under_load(torch, enqueue_pass, passes):
    """Clocks and power as rocm-smi reports them while `passes` passes over the workload's GEMMs are running
    (a child process; None where the tool or its counters are not accessible)."""
    import shutil
    import subprocess
    exe = shutil.which("rocm-smi") or "/opt/rocm/bin/rocm-smi"
    if not os.path.exists(exe):
        return None
    for i in range(passes):
        enqueue_pass(i)
    state = None
    try:
        r = subprocess.run([exe, "--showclocks", "--showpower", "--json"], capture_output=True, text=True, timeout=20)
        cards = json.loads(r.stdout) if r.returncode == 0 and r.stdout.strip().startswith("{") else {}
        card = cards.get("card0") or (next(iter(cards.values())) if cards else None)
        if isinstance(card, dict):
            state = {k: v for k, v in card.items() if any(t in k.lower() for t in ("sclk", "mclk", "fclk", "power"))}
    except Exception as e:     # the tool is optional context
        log("[gpu_state] rocm-smi not usable:", repr(e))
    torch.cuda.synchronize()
    return state or None


def measured_ceilings(torch):
    """What this GPU sustains on the matrix pipe and on HBM reads, measured here and now (context for
    `roofline.frac`, which stays against the published peaks): register-resident int8 MFMA loop on every CU
    with constant and with hashed operands, a read stream over 2 GiB, and the global->LDS loads of an L2-resident
    buffer (helper library libqlprobe.so)."""
    from paper_2512_23367_amd import probe
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    out = {}
    for name, rnd in (("mfma_int8_constant_operands_tops", 0), ("mfma_int8_random_operands_tops", 1),
                      ("mfma_int8_layer_like_operands_tops", 2), ("mfma_int8_16x16x64_random_operands_tops", 3)):
        ops = [0]

        def f(i, rnd=rnd):
            ops[0] = probe.mfma_int8(2048, 2000, rnd, sink)
        ms = min(event_times_ms(torch, f, 3, 3, 2))
        out[name] = round(ops[0] / (ms * 1e-3) / 1e12, 1)
    buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda:0")
    buf.zero_()
    ms = min(event_times_ms(torch, lambda i: probe.hbm_read(buf, sink), 5, 3, 2))
    out["hbm_read_stream_gbs"] = round(buf.numel() / (ms * 1e-3) / 1e9, 1)
    del buf
    # the path the GEMM tiles travel by: 16-byte-per-lane global->LDS loads on an L2-resident buffer, all 256 CUs
    l2buf = torch.zeros(256 * 65536, dtype=torch.uint8, device="cuda:0")
    moved = [0]

    def g(i):
        moved[0] = probe.l2_to_lds(l2buf, 2000, sink)
    ms = min(event_times_ms(torch, g, 2, 3, 1))
    out["l2_to_lds_loads_gbs"] = round(moved[0] / (ms * 1e-3) / 1e9, 1)
    del l2buf
    torch.cuda.empty_cache()
    return out


def cpu_baseline(shapes, synth, slice_rows):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload: the first
    `slice_rows` token rows of every linear (rows are independent under per-token quantization), all host
    threads, repeated until about 10 s of CPU work; then one pass of a quarter of those rows on one thread."""
    import ctypes
    import oracle
    from oracle import linear as olin
    prepared = []
    for sh in shapes:
        rows = min(slice_rows, sh.M)
        x = synth.activations(sh.M, sh.K, sh.config, sh.layer, rows=slice(0, rows))
        w = synth.weights(sh.N, sh.K, sh.config, sh.layer)
        b = synth.bias(sh.N, sh.config, sh.layer) if sh.bias else None
        if sh.bits == 8:
            wq, sw = oracle.quant_weight_int8(w)        # offline, not timed
            run = lambda x, wq=wq, sw=sw, b=b: oracle.linear_w8a8(x, wq, sw, b)
        else:
            p, _, s = oracle.quant_weight_int4(w, sh.group)
            run = lambda x, p=p, s=s, g=sh.group, b=b: oracle.linear_w4a8(x, p, s, g, b)
        prepared.append((sh, x, run))
        del w
    threads = olin.num_threads()
    t_total, ops, passes = 0.0, 0, 0
    while t_total < 10.0 and passes < 20:
        for sh, x, run in prepared:
            t0 = time.perf_counter()
            run(x)
            t_total += time.perf_counter() - t0
            ops += 2 * x.shape[0] * sh.N * sh.K
        passes += 1
    out = dict(value=ops / t_total / 1e12, unit="TOPS", cores=threads, kind="oracle")
    # one thread: OpenMP's own switch, the oracle is untouched
    one = None
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_set_num_threads(1)
        t1, ops1 = 0.0, 0
        for sh, x, run in prepared:
            xs = x[:max(1, x.shape[0] // 4)]
            t0 = time.perf_counter()
            run(xs)
            t1 += time.perf_counter() - t0
            ops1 += 2 * xs.shape[0] * sh.N * sh.K
        gomp.omp_set_num_threads(threads)
        one = ops1 / t1 / 1e12
    except OSError:
        pass
    out["value_one_thread"] = one
    out["sample"] = (f"first {slice_rows} token rows of each of the workload's {len(shapes)} linears (quantize + integer GEMM + "
                     f"epilogue), {passes} passes on {threads} threads: {ops / 1e9:.1f} GOP in {t_total:.1f} s; one thread: "
                     f"a quarter of those rows once; weight quantization not timed")
    return out


def decode_table(torch, ql, synth, forced_copies, hashes):
    """GEMM-only time of every decode shape of config 4 (7B-class layer, M in {1, 8, 32}, int8 and int4 weights)
    against HBM bandwidth: algorithmic bytes / median launch time, launches replayed from a HIP graph, the weight
    matrix rotated through enough copies that it comes from HBM."""
    rows = []
    groups = {}
    for sh in synth.workload(4):
        if sh.M <= 32:
            groups.setdefault((sh.layer, sh.bits), []).append(sh)
    for (layer, bits), shs in groups.items():
        copies = copies_for(shs[0], forced_copies)
        base = None
        for sh in shs:
            l = Layer(sh, torch, ql, synth, copies, share=base, hashes=hashes if sh.M == 1 and bits == 8 else None)
            base = base or l
            l.quant()
            launches = max(MIN_LAUNCHES, 2 * copies)
            t = median_ms(torch, l.gemm, launches, MIN_REPEATS, graph=True)
            t_lin = median_ms(torch, l.linear, launches, 3, graph=True)
            gbs = l.gemm_bytes() / (t * 1e-3) / 1e9
            row = {"shape": sh.name, "gemm_us": round(t * 1e3, 2), "linear_us": round(t_lin * 1e3, 2),
                   "gbs": round(gbs, 1), "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4), "weight_copies_rotated": copies}
            rows.append(row)
            log("[decode]", json.dumps(row))
        del base, l
        torch.cuda.empty_cache()
    return rows


def decode_summary(rows):
    """Compact forms of the decode table for the JSON line: a string 'w8 M1 qkv/o/gate_up/down 0.61/0.41/...' and
    the extremes."""
    def frac(bits, M, layer):
        for r in rows:
            if r["shape"].startswith(f"c4.{layer}.M{M}.") and r["shape"].endswith(f".w{bits}"):
                return r["frac_hbm_peak"]
        return None
    parts = []
    for bits in (8, 4):
        for M in (1, 8, 32):
            fr = [frac(bits, M, l) for l in ("qkv", "o", "gate_up", "down")]
            parts.append(f"w{bits} M{M} " + "/".join("-" if f is None else f"{f:.2f}" for f in fr))
    w8 = [r["frac_hbm_peak"] for r in rows if r["shape"].endswith(".w8")]
    w4 = [r["frac_hbm_peak"] for r in rows if r["shape"].endswith(".w4")]
    return "frac of 8 TB/s, qkv/o/gate_up/down: " + "; ".join(parts), w8, w4


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="config2",
                    help="config2 (default: the 7B-class W8A8 prefill layer, the largest single-GPU decoder-layer "
                         "workload), config1, config3, config4 (long prefill), decode8, decode4 (the 7B-class decode "
                         "GEMMs of config 4, int8 / int4 weights)")
    ap.add_argument("--decode-m", type=int, default=1, help="tokens of the decode workloads: 1 .. 1024")
    ap.add_argument("--variant", type=int, default=0, help="kernel variant (0 = automatic)")
    ap.add_argument("--weight-copies", type=int, default=0,
                    help="copies of every weight matrix the launches rotate through (0 = enough that the copies of "
                         "a matrix exceed three times the 256 MB Infinity Cache, i.e. weights come from HBM as in a model)")
    ap.add_argument("--no-detail", action="store_true", help="skip the rows of the other configurations")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode table (roofline.decode)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--only-step", action="store_true", help="only the timed steps (for profiling)")
    ap.add_argument("--only-gemm", action="store_true",
                    help="quantize once, then only GEMM launches of the workload (for profiling the GEMM kernels)")
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
             2: "config2: W8A8 linears (+bias) of a 7B-class decoder layer, prefill M=4096, d=4096 (qkv, o, gate_up, down)",
             3: "config3: W4A8 (group 128) linears of a 7B-class decoder layer, prefill M=4096, d=4096",
             4: "config4: long-reasoning prefill of the down projection, M=16384, W8A8"}[cfg]
    if decode:
        descr = (f"config4 decode: {'W8A8' if bits == 8 else 'W4A8 (group 128)'} linears of a 7B-class decoder "
                 f"layer, M={args.decode_m} (qkv, o, gate_up, down), weights rotated over >768 MB of copies")

    hashes = {}
    layers = [Layer(s, torch, ql, synth, copies_for(s, args.weight_copies), hashes=hashes) for s in shapes]
    total_ops = sum(s.ops for s in shapes)
    log("[inputs] sha256[:16] of the host tensors:", json.dumps(hashes))

    if args.only_gemm:
        for l in layers:
            l.quant()
        for i in range(args.warmup + args.steps):
            for l in layers:
                l.gemm(i)
        torch.cuda.synchronize()
        print(json.dumps({"only_gemm": True, "launches_per_linear": args.warmup + args.steps,
                          "layers": [s.name for s in shapes]}), flush=True)
        return

    def step(i=0):
        for l in layers:
            l.linear(i)

    # The roofline timing runs first: right after a process starts loading the GPU its power management lets the clock
    # overshoot, clamps it (kernels up to 35 % slower around the fifth pass) and settles after some 40 passes -- the timed
    # steps below then measure the steady state a serving process lives in, like the roofline passes (which warm up longer).
    roof = None
    if not args.only_step:
        # ---- roofline of the dominant kernel (the GEMM + fused epilogue), timed with HIP events on the launch stream:
        # median of MIN_REPEATS repeats of >= MIN_LAUNCHES back-to-back launches per linear, whatever --steps says
        for l in layers:
            l.quant()
        for i in range(WARM_PASSES):       # through the start-of-run transient before anything is timed
            for l in layers:
                l.gemm(i)
        gemm_ms, quant_ms = [], []
        for l in layers:
            launches = max(MIN_LAUNCHES, len(l.kernels))   # at least one cycle through the weight copies
            gemm_ms.append(median_ms(torch, l.gemm, launches, MIN_REPEATS, graph=decode, warm=max(30, 2 * len(l.kernels))))
            # the quantizer runs 2-30 us: replay it from a HIP graph, or the launch path is what gets timed
            quant_ms.append(median_ms(torch, lambda i, l=l: l.quant(), MIN_LAUNCHES, MIN_REPEATS, graph=True))

        # the figure of record: the workload's GEMMs in the order of the step (qkv, o, gate_up, down, qkv, ...), as in the
        # timed region and as `--only-gemm` launches them under the profiler; one HIP-event pair around >= MIN_LAUNCHES passes
        def gemm_pass(i):
            for l in layers:
                l.gemm(i)
        passes = max(MIN_LAUNCHES, max(len(l.kernels) for l in layers))
        pass_ms = median_ms(torch, gemm_pass, passes, MIN_REPEATS, graph=decode, warm=passes)
        timing = (f"median of {MIN_REPEATS} repeats of {passes} passes over the workload's GEMM launches in step order, one HIP-event "
                  f"pair per repeat; per_layer: the same with each linear's launches back to back")
        if not decode:
            achieved = total_ops / (pass_ms * 1e-3) / 1e12
            roof = {"bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                    "frac": round(achieved / PEAK_INT8_TOPS, 4), "traffic": profiled_traffic(cfg),
                    "kernel": "gemm_prefill_kernel (int8 MFMA GEMM + fused dequant epilogue), one launch per linear (two on disjoint channel ranges where the plan says so: gate_up)",
                    "timing": timing, "us_per_pass": round(pass_ms * 1e3, 1),
                    "per_layer": "; ".join(f"{l.sh.layer} {t * 1e3:.1f} us {l.sh.ops / (t * 1e-3) / 1e12:.0f} TOPS "
                                           f"{l.sh.ops / (t * 1e-3) / 1e12 / PEAK_INT8_TOPS:.3f}" for l, t in zip(layers, gemm_ms))}
        else:
            achieved = sum(l.gemm_bytes() for l in layers) / (pass_ms * 1e-3) / 1e9
            roof = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": None,
                    "kernel": "gemm_decode_kernel (weight-streaming int8 MFMA GEMM + fused epilogue), one launch per linear",
                    "timing": timing + " (launches replayed from a HIP graph)",
                    "per_layer": "; ".join(f"{l.sh.layer} {t * 1e3:.2f} us {l.gemm_bytes() / (t * 1e-3) / 1e9:.0f} GB/s"
                                           for l, t in zip(layers, gemm_ms))}
        roof["act_quant"] = "; ".join(f"{l.sh.layer} {t * 1e3:.1f} us {l.quant_bytes() / (t * 1e-3) / 1e9:.0f} GB/s"
                                      for l, t in zip(layers, quant_ms))
        if not decode:
            # ~0.25 s of GEMM work in flight while the tool samples
            roof["gpu_state_under_load"] = gpu_state_under_load(torch, gemm_pass, 400)
            log("[gpu_state]", json.dumps(roof["gpu_state_under_load"]))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    graph = None
    if decode:
        # a decode step is 4-8 launches of 4-16 us: replay them from a HIP graph so that the GPU, not the
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
        "inputs_sha256_16": hashes,
        "config": {"workload": descr, "layers": [s.name for s in shapes],
                   "weights": "int8 per-channel" if shapes[0].bits == 8 else "int4 group-128",
                   "activations": "int8 per-token dynamic", "output": "fp16"},
    }
    if args.only_step:
        print(json.dumps(out), flush=True)
        return

    out["roofline"] = roof
    log("[roofline]", json.dumps(roof))
    del layers
    torch.cuda.empty_cache()

    # ---- the decode GEMMs of config 4 against HBM bandwidth (the second half of the metric)
    if not args.no_decode and not decode:
        rows = decode_table(torch, ql, synth, args.weight_copies, hashes)
        text, w8, w4 = decode_summary(rows)
        roof["decode"] = text
        roof["decode_w8a8_frac_min"], roof["decode_w8a8_frac_max"] = min(w8), max(w8)
        roof["decode_w4a8_frac_min"], roof["decode_w4a8_frac_max"] = min(w4), max(w4)
        roof["decode_rows"] = {r["shape"]: [r["gemm_us"], r["linear_us"], r["gbs"]] for r in rows}
        roof["decode_rows_columns"] = "gemm_us, linear_us (quantize + GEMM), GB/s of algorithmic bytes"

    # ---- detail: the other prefill configurations (parity-test cases, not the headline), GEMM-only
    if not args.no_detail and not decode:
        detail = []
        for c in (1, 2, 3, 4):
            if c == cfg:
                continue
            for sh in [s for s in synth.workload(c) if s.M > 32]:
                l = Layer(sh, torch, ql, synth, copies_for(sh, args.weight_copies))
                l.quant()
                launches = max(MIN_LAUNCHES if sh.ops < 5e11 else 20, len(l.kernels))
                # warm-up: two cycles through the weight copies (the first launches on fresh buffers run ~10 % slower)
                t = median_ms(torch, l.gemm, launches, MIN_REPEATS, warm=max(30, 2 * len(l.kernels)))
                t_lin = median_ms(torch, l.linear, launches, 3, warm=5)
                tops = sh.ops / (t * 1e-3) / 1e12
                row = {"shape": sh.name, "gemm_us": round(t * 1e3, 1), "linear_us": round(t_lin * 1e3, 1),
                       "tops": round(tops, 1), "frac_mfma_peak": round(tops / PEAK_INT8_TOPS, 4)}
                detail.append(row)
                log("[detail]", json.dumps(row))
                del l
                torch.cuda.empty_cache()
        detail += layer_table(torch, ql, synth)
        detail += act_quant_rows(torch, ql)
        out["detail"] = detail

    # ---- what the GPU sustains on the two resources (context; last, so that the probes' heat does not touch the rows above)
    ceil = measured_ceilings(torch)
    # the prefill kernels run on the 16x16x64 instruction: that probe is their ceiling
    ref = ceil["hbm_read_stream_gbs"] if decode else ceil["mfma_int8_16x16x64_random_operands_tops"]
    roof["measured_ceilings"] = {**ceil, "achieved_over_measured": round(roof["achieved"] / ref, 4)}
    roof["measured_ceilings_note"] = ("context only; frac is against the published peak. The matrix-pipe probe keeps its "
                                      "operands in registers; hashed operands lower the shader clock")
    log("[ceilings]", json.dumps(roof["measured_ceilings"]))

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(shapes, synth, 256 if shapes[0].K >= 4096 else shapes[0].M)
        log("[cpu]", json.dumps(out["cpu_baseline"]))
    print(json.dumps(out), flush=True)


def layer_table(torch, ql, synth):
    """Context for the paper's Table 3 (INT8 against FP16 prefill latency and memory by batch size): the four
    chained linears of the 7B-class layer (qkv -> o -> gate_up -> SwiGLU -> down; paper_2512_23367_amd.layer) over a
    sweep of token counts, as W8A8 and W4A8 (quantize + GEMM + epilogue, SwiGLU fused into the down projection's
    quantizer) and as FP16 GEMMs of the vendor library (torch.matmul + torch's SiLU: a comparison system that is not
    part of this library); weight bytes per precision."""
    from paper_2512_23367_amd.layer import DecoderLayerLinears
    import torch.nn.functional as tf
    rows = []
    d, F, max_m = 4096, 11008, 16384
    shapes = {s.layer: s for s in synth.workload(2)}
    wh = {k: torch.from_numpy(synth.weights(shapes[k].N, shapes[k].K, 2, k)).to("cuda:0") for k in ("qkv", "o", "gate_up", "down")}
    layers = {b: DecoderLayerLinears(wh["qkv"], wh["o"], wh["gate_up"], wh["down"], b, max_m) for b in (8, 4)}
    mem = {"fp16": sum(w.numel() * 2 for w in wh.values()), "w8a8": layers[8].weight_bytes, "w4a8": layers[4].weight_bytes}

    def fp16_chain(x):
        q = torch.matmul(x, wh["qkv"].t())
        o = torch.matmul(q[:, :d], wh["o"].t())
        gu = torch.matmul(o, wh["gate_up"].t())
        return torch.matmul(tf.silu(gu[:, :F]) * gu[:, F:], wh["down"].t())

    for M in (512, 1024, 2048, 4096, 8192, 16384):
        x = torch.from_numpy(synth.activations(M, d, 2, "qkv")).to("cuda:0")
        reps = 5 if M >= 8192 else 10
        t = {"fp16": statistics.median(event_times_ms(torch, lambda i: fp16_chain(x), reps, 3, 2))}
        for b in (8, 4):
            t["w8a8" if b == 8 else "w4a8"] = statistics.median(event_times_ms(torch, lambda i, b=b: layers[b].forward(x), reps, 3, 2))
        row = {"shape": f"layer7b.prefill.M{M}", "fp16_library_us": round(t["fp16"] * 1e3, 1),
               "w8a8_us": round(t["w8a8"] * 1e3, 1), "w4a8_us": round(t["w4a8"] * 1e3, 1),
               "w8a8_speedup_over_fp16": round(t["fp16"] / t["w8a8"], 2),
               "w4a8_speedup_over_fp16": round(t["fp16"] / t["w4a8"], 2)}
        log("[detail]", json.dumps(row))
        rows.append(row)
        del x
    rows.append({"shape": "layer7b.weight_mb", **{k: round(v / 1e6, 1) for k, v in mem.items()}})
    log("[detail]", json.dumps(rows[-1]))
    del layers, wh
    torch.cuda.empty_cache()
    return rows


def act_quant_rows(torch, ql):
    """The activation quantizer alone and with the operand transforms fused in front of it (SmoothQuant per-channel
    multiply, block Hadamard rotation, RMSNorm, SwiGLU), graph-replayed; 3 B per element (SwiGLU: 5)."""
    rows = []
    for M, K in ((2048, 1536), (4096, 4096), (4096, 11008)):
        x = torch.randn((M, K), dtype=torch.float16, device="cuda:0")
        kl = torch.empty(ql.ql_act_kernel_bytes(M, K), dtype=torch.uint8, device="cuda:0")
        sxv = torch.empty(M, dtype=torch.float32, device="cuda:0")
        inv = torch.rand(K, dtype=torch.float32, device="cuda:0") + 0.5
        B = ql.ql_hadamard_block(K)
        gam = (torch.rand(K, dtype=torch.float32, device="cuda:0") + 0.5).to(torch.float16)
        row = {"shape": f"act_quant.M{M}.K{K}"}
        for name, fn in (("plain", lambda i: ql.ql_quant_act_per_token(x, None, kl, sxv)),
                         ("smoothquant", lambda i: ql.ql_quant_act_per_token_transformed(x, inv, 0, None, kl, sxv)),
                         ("hadamard", lambda i: ql.ql_quant_act_per_token_transformed(x, None, B, None, kl, sxv)),
                         ("rmsnorm", lambda i: ql.ql_quant_act_rmsnorm(x, gam, 1e-6, None, kl, sxv))):
            t = median_ms(torch, fn, MIN_LAUNCHES, 3, graph=True)
            row[name + "_us"] = round(t * 1e3, 2)
            row[name + "_gbs"] = round(3 * M * K / (t * 1e-3) / 1e9, 1)
        # SwiGLU of a fused gate+up output [M, 2K] in front of the quantizer: 4 B read + 1 B written per element
        gu = torch.randn((M, 2 * K), dtype=torch.float16, device="cuda:0")
        t = median_ms(torch, lambda i: ql.ql_quant_act_swiglu(gu, None, kl, sxv), MIN_LAUNCHES, 3, graph=True)
        row["swiglu_us"], row["swiglu_gbs"] = round(t * 1e3, 2), round(5 * M * K / (t * 1e-3) / 1e9, 1)
        del gu
        log("[detail]", json.dumps(row))
        rows.append(row)
        del x, kl
    return rows


if __name__ == "__main__":
    main()
