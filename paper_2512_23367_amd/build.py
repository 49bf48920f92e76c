"""Builds libqlinear.so (HIP, gfx950 only) next to this file with hipcc.

    python -m paper_2512_23367_amd.build

Every .hip under csrc/ is compiled to an object file in parallel and linked into
one shared library whose exported symbols are the C ABI of include/qlinear.h.
The benchmark's ceiling probes (bench_probe/) become a library of their own,
libqlprobe.so, which the quantized linear layer does not depend on.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libqlinear.so")
PROBE_LIB = os.path.join(HERE, "libqlprobe.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
PROBE_DIR = os.path.join(HERE, "bench_probe")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                                   # quantizer arithmetic: one rounding per operation
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fvisibility=hidden", "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", PROBE_DIR,
]


def sources() -> list[str]:
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
    subprocess.run([HIPCC, *FLAGS, "-c", src, "-o", obj], check=True)
    return obj


def _link(objs: list[str], lib: str) -> None:
    tmp = lib + f".tmp{os.getpid()}"
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp], check=True)
    os.replace(tmp, lib)


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    probe_src = os.path.join(PROBE_DIR, "probe.hip")
    with ThreadPoolExecutor(max_workers=min(8, len(sources()) + 1)) as ex:
        objs = list(ex.map(_compile, sources() + [probe_src]))
    _link(objs[:-1], LIB)
    _link(objs[-1:], PROBE_LIB)
    if verbose:
        print("built", LIB, "and", PROBE_LIB, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build()
