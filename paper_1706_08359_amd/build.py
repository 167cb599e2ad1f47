"""Compile csrc/gbdt_hist.hip into libgbdt_hist.so (in-tree, next to this file).

hipcc cross-compiles for gfx950 without a GPU.  Run as
    python -m paper_1706_08359_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "csrc", "gbdt_hist.hip")
LIB = os.path.join(_HERE, "libgbdt_hist.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    "-ffp-contract=off",          # the fp64 gain scan must not be fused into FMAs
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = False) -> str:
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC] + FLAGS + ["-o", tmp, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    return LIB


# The stand-alone micro-benchmark of the two secondary ceilings (local-memory atomic rate,
# streaming-read rate): repo root, next to bench.py.
CEIL_SRC = os.path.join(os.path.dirname(_HERE), "bench_ceilings.hip")
CEIL_BIN = os.path.join(os.path.dirname(_HERE), "bench_ceilings")


def build_ceilings(verbose: bool = False) -> str:
    tmp = CEIL_BIN + ".tmp%d" % os.getpid()
    # -munsafe-fp-atomics: the float add is measured as the single LDS instruction, not as a
    # compare-and-swap loop (the library itself issues no float atomics)
    cmd = [HIPCC] + COMMON + ["-munsafe-fp-atomics", "-o", tmp, CEIL_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, CEIL_BIN)
    return CEIL_BIN


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_ceilings(verbose=True))
    sys.exit(0)
