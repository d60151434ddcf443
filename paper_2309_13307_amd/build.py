"""Build step of the HIP library: one hipcc invocation, gfx950 only, output kept in-tree.

The library carries an identifier of the sources and flags it was built from (`core_build_id`);
`built_id()` reads it out of the file without loading it, so that a loader can tell a stale
binary from a current one whatever the file times say.
"""
from __future__ import annotations

import hashlib
import os
import re
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libcore_hip.so")

SOURCES = ["core_api.hip"]
HEADERS = ["core_rng.hpp", "core_common.hpp", "core_kernels.hpp", "core_project.hpp", "core_project_few.hpp",
           "core_reduce.hpp", "core_reconstruct.hpp", "core_steps.hpp", "core_debug.hpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # scalar fp32 code must not be auto-vectorised into packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unknown-warning-option",
]

_ID_MARKER = re.compile(rb"CORE_BUILD_ID=([0-9a-f]{16})")


def _dependencies():
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    deps.append(os.path.join(os.path.dirname(_HERE), "include", "core.h"))
    return deps


def source_id() -> str:
    """Hash of the sources and compiler flags the library is built from."""
    h = hashlib.sha256()
    h.update(" ".join(HIPCC_FLAGS).encode())
    for path in _dependencies():
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def built_id(path: str = LIB_PATH) -> str | None:
    """The identifier stored in a built library (None: no library, or one without an id)."""
    if not os.path.exists(path):
        return None
    with open(path, "rb") as f:
        m = _ID_MARKER.search(f.read())
    return m.group(1).decode() if m else None


def is_stale() -> bool:
    return built_id() != source_id()


def hipcc_path() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build_library(verbose: bool = False) -> str:
    """Compile csrc/*.hip into libcore_hip.so (always compiles when called)."""
    cmd = ([hipcc_path()] + HIPCC_FLAGS + [f'-DCORE_BUILD_ID="{source_id()}"', "-o", LIB_PATH]
           + [os.path.join(CSRC, s) for s in SOURCES])
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
