"""Builds liboppo_attn.so (gfx950 code object + host ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liboppo_attn.so")
# stand-alone measurement of the chip's power-limited MFMA rate (not part of the library)
CEILING_BENCH = os.path.join(HERE, "ceiling_bench")

SOURCES = ["kernels.hip", "rope.hip", "api.cpp", "pool.cpp", "sched.cpp"]
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # no NaN ever enters a max/min here (masked scores are -inf): lets the
    # compiler use three-input maxima without canonicalising their operands
    "-fno-honor-nans",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def build(verbose: bool = True, extra_flags=()) -> str:
    cmd = [hipcc(), "-shared", "-o", LIB] + HIP_FLAGS + list(extra_flags)
    cmd += ["-x", "hip"] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    cmd = [hipcc(), "-o", CEILING_BENCH] + [f for f in HIP_FLAGS if f != "-fPIC"] + [os.path.join(CSRC, "ceiling_bench.hip")]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    return LIB


if __name__ == "__main__":
    build()
    print(LIB)
