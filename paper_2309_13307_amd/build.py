"""Build step of the HIP library: one hipcc invocation, gfx950 only, output kept in-tree."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libcore_hip.so")
PROBE_PATH = os.path.join(_HERE, "issue_probe")   # standalone VALU issue-cost microbenchmark

SOURCES = ["core_api.hip"]
HEADERS = ["core_rng.hpp", "core_kernels.hpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # scalar fp32 code must not be auto-vectorised into packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unknown-warning-option",
]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    deps.append(os.path.join(os.path.dirname(_HERE), "include", "core.h"))
    return any(os.path.getmtime(p) > t for p in deps)


def build_library(verbose: bool = False) -> str:
    """Compile csrc/*.hip into libcore_hip.so (always compiles when called)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB_PATH] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return LIB_PATH


def build_issue_probe(verbose: bool = False) -> str:
    """Compile csrc/issue_probe.hip into the standalone executable `issue_probe`."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc] + flags + ["-o", PROBE_PATH, os.path.join(CSRC, "issue_probe.hip")]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return PROBE_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_issue_probe(verbose=True))
