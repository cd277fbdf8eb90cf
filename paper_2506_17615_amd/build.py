"""Builds libequarx.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
CSRC = os.path.join(_PKG, "csrc")
INCLUDE = os.path.join(_ROOT, "include")
LIB_PATH = os.path.join(_PKG, "libequarx.so")
SOURCES = [os.path.join(CSRC, "equarx_api.hip"), os.path.join(CSRC, "equarx_devtools.hip")]
HEADERS = [os.path.join(CSRC, name) for name in ("equarx_device.hpp", "equarx_strided.hpp", "equarx_launch.hpp", "equarx_passes.hpp",
                                                  "equarx_devtools_kernels.hpp")]
HEADERS += [os.path.join(INCLUDE, "equarx.h"), os.path.join(INCLUDE, "equarx_devtools.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    # every rounding is written out in the kernels: no implicit multiply-add fusion
    "-ffp-contract=off",
    # packed-fp32 instructions stay out of the generated code.  The feature belongs to the gfx950 pass, which
    # honours it (tests/test_build_flags.py looks at the device assembly); hipcc hands -Xclang options to its
    # x86 host pass as well, which answers each with a harmless "not a recognized feature for this target".
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-shared", "-fPIC",
    "-I", INCLUDE, "-I", CSRC,
]


STAMP_PATH = LIB_PATH + ".stamp"


def source_digest() -> str:
    """SHA-256 over the build flags and the text of every source and header the library is built from."""
    import hashlib
    h = hashlib.sha256(" ".join(HIPCC_FLAGS[:-4]).encode())      # flags without the -I paths (machine-specific)
    for path in SOURCES + HEADERS:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_stale() -> bool:
    """True if there is no library, or the one there was not built from the sources as they are now.  Decided
    by content (a digest written next to the library at build time), not by file times, which a copy of the tree
    to another machine does not keep."""
    if not os.path.exists(LIB_PATH) or not os.path.exists(STAMP_PATH):
        return True
    with open(STAMP_PATH) as f:
        return f.read().strip() != source_digest()


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library; returns its path.  Raises if hipcc fails."""
    if not force and not is_stale():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *SOURCES, "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    digest = source_digest()
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    with open(STAMP_PATH, "w") as f:
        f.write(digest + "\n")
    return LIB_PATH


def ensure_built() -> str:
    """What tests, smoke and bench call before loading the library: build it if it is missing, and never run a
    library that is older than the sources beside it -- rebuild where hipcc exists, refuse where it does not."""
    if not is_stale():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if os.path.exists(LIB_PATH) and not os.path.exists(hipcc):
        raise RuntimeError(f"{LIB_PATH} is older than its sources and {hipcc} is not there to rebuild it")
    build(force=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
