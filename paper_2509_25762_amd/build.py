"""Builds liboppo_attn.so (gfx950 code object + host ABI) in-tree with hipcc.

`build()` makes the library.  `build_host_checked()` makes a CPU-only test program
from the host sources alone (argument checks, planner, slot pool, scheduler) with
the kernel launchers replaced by stand-ins, compiled by the host compiler under
AddressSanitizer and UndefinedBehaviorSanitizer; the CPU test suite runs it.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liboppo_attn.so")
HOST_CHECKED_EXE = os.path.join(HERE, "oppo_host_checked")

DEVICE_SOURCES = ["kernels.hip", "rope.hip", "gemm.hip"]
HOST_SOURCES = ["api.cpp", "pool.cpp", "sched.cpp"]
COMMON_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]
# Kernel files only: no NaN ever enters a max/min there (masked scores are -inf), which
# lets the compiler use three-input maxima without canonicalising their operands.  The
# host files reject NaN arguments with ordinary comparisons and are built without it.
DEVICE_ONLY_FLAGS = ["-fno-honor-nans"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"{cmd[0]} failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = True, extra_flags=(), out: str = LIB) -> str:
    """Compiles every source to an object of its own (kernel files and host files take
    different flags) and links them into the shared library."""
    with tempfile.TemporaryDirectory(prefix="oppo_build_") as tmp:
        objs = []
        procs = []
        for src in DEVICE_SOURCES + HOST_SOURCES:
            if not os.path.exists(os.path.join(CSRC, src)):
                continue
            obj = os.path.join(tmp, src + ".o")
            flags = COMMON_FLAGS + (DEVICE_ONLY_FLAGS if src in DEVICE_SOURCES else []) + list(extra_flags)
            cmd = [hipcc(), "-c", "-o", obj] + flags + ["-x", "hip", os.path.join(CSRC, src)]
            if verbose:
                print(" ".join(cmd), flush=True)
            procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
            objs.append(obj)
        for cmd, p in procs:
            text = p.communicate()[0]
            text = "\n".join(l for l in text.splitlines() if "not a recognized feature" not in l)
            if p.returncode != 0:
                raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + text)
            if verbose and text.strip():
                print(text)
        _run([hipcc(), "-shared", "-o", out, "--offload-arch=gfx950", "-fPIC"] + objs, verbose)
    return out


def build_host_checked(verbose: bool = False) -> str:
    """The host sources + launcher stand-ins + tests/host_checked_main.cpp as one program under
    -fsanitize=address,undefined (host compiler, no GPU code, no HIP).  Returns its path."""
    cxx = shutil.which("g++") or shutil.which("c++")
    if not cxx:
        raise RuntimeError("no host C++ compiler found")
    main = os.path.join(os.path.dirname(HERE), "tests", "host_checked_main.cpp")
    cmd = [cxx, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-fno-omit-frame-pointer", "-o", HOST_CHECKED_EXE, main]
    cmd += [os.path.join(CSRC, s) for s in HOST_SOURCES + ["launch_stubs.cpp"]]
    _run(cmd, verbose)
    return HOST_CHECKED_EXE


if __name__ == "__main__":
    build()
    print(LIB)
    if "--host-checked" in sys.argv:
        print(build_host_checked(verbose=True))
