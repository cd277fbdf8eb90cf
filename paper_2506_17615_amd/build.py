"""Builds libequarx.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
CSRC = os.path.join(_PKG, "csrc")
INCLUDE = os.path.join(_ROOT, "include")
LIB_PATH = os.path.join(_PKG, "libequarx.so")
SOURCES = [os.path.join(CSRC, "equarx_api.hip")]
HEADERS = [os.path.join(CSRC, "equarx_device.hpp"), os.path.join(CSRC, "equarx_strided.hpp"),
           os.path.join(INCLUDE, "equarx.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    # every rounding is written out in the kernels: no implicit multiply-add fusion
    "-ffp-contract=off",
    # packed-fp32 instructions stay out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-shared", "-fPIC",
    "-I", INCLUDE, "-I", CSRC,
]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > built for p in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library; returns its path.  Raises if hipcc fails."""
    if not force and not is_stale():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *SOURCES, "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    return LIB_PATH


def ensure_built() -> str:
    """Build only if no library is there at all (tests, smoke and bench call this; they never rebuild)."""
    if not os.path.exists(LIB_PATH):
        build(force=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
