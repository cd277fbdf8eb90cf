"""Host-side sanitizer runs (CPU only): the C oracle under the whole pin suite, and the host code of the HIP
library under the argument-validation tests, each built with AddressSanitizer + UndefinedBehaviorSanitizer and run
in a child interpreter that preloads the matching sanitizer runtime.  Device code is not instrumented (the
sanitizer flags go to the host pass only).  Skipped where a compiler or its runtime is missing."""
import glob
import os
import subprocess
import sys

import pytest

from oracle import equarx_oracle as o
from paper_2506_17615_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLEAN = "SANITIZED RUN CLEAN"


def _child(code, runtime, timeout=900):
    env = dict(os.environ)
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # leaks are the interpreter's own; link order: the runtime is preloaded, not linked first into python
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    env["PYTHONPATH"] = os.pathsep.join([ROOT, os.path.join(ROOT, "tests"), env.get("PYTHONPATH", "")])
    return subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=timeout,
                          cwd=ROOT)


def test_oracle_under_asan_and_ubsan(tmp_path):
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    lib = o.build(force=True, lib=str(tmp_path / "liboracle_san.so"),
                  extra_flags=("-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"))
    code = f"""
import oracle_pins
from oracle import equarx_oracle as o
lib = o.load({lib!r})
for pin in oracle_pins.ALL_PINS:
    pin(lib)
print({CLEAN!r}, len(oracle_pins.ALL_PINS))
"""
    run = _child(code, runtime)
    assert run.returncode == 0 and CLEAN in run.stdout, run.stdout[-2000:] + run.stderr[-4000:]
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error:" not in run.stderr, run.stderr[-4000:]


def test_sanitized_oracle_run_would_notice_an_overrun(tmp_path):
    """The harness above is not blind: a copy of the oracle whose quantizer reads one element past its block (a
    planted mistake, CPU only) is reported by AddressSanitizer in the same kind of child run."""
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    with open(os.path.join(os.path.dirname(o.__file__), "equarx_oracle.c")) as f:
        src = f.read()
    old = "    for (int64_t j = 0; j < len; ++j) {\n        float m = fabsf(v[j]);"
    assert src.count(old) == 1
    bad = tmp_path / "overrun.c"
    bad.write_text(src.replace(old, "    for (int64_t j = 0; j <= len; ++j) {\n        float m = fabsf(v[j]);"))
    lib = o.build(force=True, src=str(bad), lib=str(tmp_path / "liboverrun.so"),
                  extra_flags=("-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"))
    code = f"""
import numpy as np
from oracle import equarx_oracle as o
lib = o.load({lib!r})
o.quantize_f32(np.ones(64, np.float32), 64, lib=lib)
print({CLEAN!r})
"""
    run = _child(code, runtime)
    assert run.returncode != 0 and "AddressSanitizer" in run.stderr and CLEAN not in run.stdout


def test_library_host_code_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    runtimes = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not os.path.exists(hipcc) or not runtimes:
        pytest.skip("hipcc or clang's AddressSanitizer runtime is not installed")
    lib = str(tmp_path / "libequarx_san.so")
    flags = list(build.HIPCC_FLAGS) + ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                                       "-Xarch_host", "-fno-sanitize-recover=undefined", "-shared-libsan"]
    made = subprocess.run([hipcc, *flags, *build.SOURCES, "-o", lib], capture_output=True, text=True)
    if made.returncode != 0 and "sanitize" in made.stderr:
        pytest.skip("this hipcc cannot build host code with sanitizers: " + made.stderr[-300:])
    assert made.returncode == 0, made.stderr[-3000:]
    code = f"""
from paper_2506_17615_amd import binding, build
build.LIB_PATH = {lib!r}
lib = binding.load()
import test_abi
test_abi.test_status_strings(lib)
test_abi.test_size_queries(lib)
test_abi.test_validation_rejects_before_launch(lib)
test_abi.test_overlapping_buffers_are_rejected_before_launch(lib)
test_abi.test_timing_hooks_do_not_outlive_the_next_call(lib)
import test_zz_no_alloc
test_zz_no_alloc.test_static_workspace_limit_is_enforced()
print({CLEAN!r})
"""
    run = _child(code, runtimes[0])
    assert run.returncode == 0 and CLEAN in run.stdout, run.stdout[-2000:] + run.stderr[-4000:]
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error:" not in run.stderr, run.stderr[-4000:]
