"""Builds tests/abi_client (the plain C99 client of libequarx the GPU tests run) with gcc, in-tree."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
SOURCE = os.path.join(_HERE, "abi_client.c")
BINARY = os.path.join(_HERE, "abi_client")
_PKG = os.path.join(_ROOT, "paper_2506_17615_amd")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build(force: bool = True) -> str:
    """Compile and link against the built libequarx.so and the HIP runtime; returns the binary's path."""
    if not force and os.path.exists(BINARY) and os.path.getmtime(BINARY) >= os.path.getmtime(SOURCE):
        return BINARY
    cmd = ["gcc", "-std=c99", "-Wall", "-O1", "-D__HIP_PLATFORM_AMD__", "-isystem", os.path.join(ROCM, "include"),
           "-I", os.path.join(_ROOT, "include"), SOURCE, "-o", BINARY,
           "-L", _PKG, "-lequarx", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
           "-Wl,-rpath," + os.path.join(ROCM, "lib"), "-Wl,-rpath,$ORIGIN/../paper_2506_17615_amd"]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("gcc failed:\n" + proc.stdout + proc.stderr)
    return BINARY


def ensure_built() -> str:
    return build(force=False) if not os.path.exists(BINARY) else BINARY


if __name__ == "__main__":
    print(build())
