"""Builds libagentsam.so (host automaton builder + HIP kernels for gfx950) in-tree with hipcc, and the
benchmark's small helper library libagentsam_bench.so (a streaming-read probe; not part of the product)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libagentsam.so")
BENCH_LIB = os.path.join(HERE, "libagentsam_bench.so")
SOURCES = ["sam_host.cpp", "sam_builder.cpp", "controllers.cpp", "sam_draft.hip", "spec_accept.hip", "spec_verify_attn.hip"]
BENCH_SOURCES = ["bench/stream_probe.hip"]


def _hipcc(sources, out, verbose):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    for s in sources:
        cmd += ["-x", "hip", os.path.join(CSRC, s)]
    cmd += ["-pthread", "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)


def build(verbose: bool = False) -> str:
    _hipcc(SOURCES, LIB, verbose)
    _hipcc(BENCH_SOURCES, BENCH_LIB, verbose)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
