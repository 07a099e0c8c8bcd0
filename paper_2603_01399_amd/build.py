"""Compile the HIP sources into the in-tree shared library (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libquasar.so")
SOURCES = ["quasar_api.hip"]
HEADERS = ["quasar_device.hpp", "stream_gemm.hpp", "stream_sequence.hpp", "stream_w8a8.hpp", "stream_w4.hpp", "drafter.hpp", "attention.hpp", "sample.hpp", "pack.hpp", "probe.hpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 vector instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the whole-step kernel keeps rarely executed phase-entry code inside a fully unrolled round;
    # without this the compiler silently refuses "#pragma unroll" once that body grows
    "-mllvm", "-pragma-unroll-threshold=1000000",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = False, extra_flags=()) -> str:
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip()]
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose and lines:
        print("\n".join(lines))
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True, extra_flags=sys.argv[1:]))
