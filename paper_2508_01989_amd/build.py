"""Build libtc_mi355x.so (hipcc, gfx950 only) next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtc_mi355x.so")
SCHED_LIB = os.path.join(HERE, "libtc_sched.so")  # host-only scheduling core, built with the host compiler
SOURCES = ["tc_plan.cpp", "tc_api.cpp", "tc_kernels.hip", "tc_probe.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


TRACE_LIB = os.path.join(HERE, "libtc_mi355x_trace.so")  # the same library with per-workgroup time stamps in the attention kernel


def build(verbose: bool = False, extra=(), trace: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if trace:
        extra = [*extra, "-DTC_WG_TRACE"]
    cmd = [hipcc, *FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        cmd += (["-x", "hip", path] if s.endswith(".cpp") else ["-x", "hip", path])
    cmd += ["-o", TRACE_LIB if trace else LIB]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return TRACE_LIB if trace else LIB


def build_sched(verbose: bool = False) -> str:
    """The scheduling core has no GPU code: plain g++, so it also loads where no ROCm runtime is."""
    cmd = [os.environ.get("CXX", "g++"), "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra", "-ffp-contract=off",
           "-I", os.path.join(ROOT, "include"), os.path.join(CSRC, "tc_sched.cpp"), "-o", SCHED_LIB]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("g++ failed:\n" + r.stderr)
    if verbose and r.stderr.strip():
        print(r.stderr)
    return SCHED_LIB


if __name__ == "__main__":
    print(build_sched(verbose=True))
    if "--trace" in sys.argv[1:]:
        print(build(verbose=True, trace=True))
    else:
        print(build(verbose=True, extra=[a for a in sys.argv[1:] if a.startswith("-")]))
