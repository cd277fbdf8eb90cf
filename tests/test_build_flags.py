"""What the build flags promise, checked on the generated gfx950 assembly of this library's own kernels (CPU only:
hipcc cross-compiles): no packed-fp32 arithmetic instruction in any kernel, and no fused multiply-add beyond the
ones the sources write out (-ffp-contract=off)."""
import os
import re
import subprocess

import pytest

from paper_2506_17615_amd import build

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def device_asm(tmp_path_factory):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc is not installed here")
    out = tmp_path_factory.mktemp("asm")
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    text = {}
    for src in build.SOURCES:
        dst = out / (os.path.basename(src) + ".s")
        subprocess.run([HIPCC, *flags, "--cuda-device-only", "-S", src, "-o", str(dst)], check=True, capture_output=True)
        text[os.path.basename(src)] = dst.read_text()
    return text


def test_no_packed_fp32_arithmetic(device_asm):
    for name, asm in device_asm.items():
        assert ".amdgcn_target" in asm and "gfx950" in asm, name
        packed = re.findall(r"^\s*(v_pk_(?:add|mul|fma)_f32)\b", asm, flags=re.M)
        assert not packed, f"{name}: {len(packed)} packed fp32 instructions"


def test_kernels_are_there_and_use_what_the_sources_say(device_asm):
    asm = device_asm["equarx_api.hip"]
    # the hop kernel of the benchmark's block size exists, widens int8 with byte-select converts, exchanges lanes
    # with DPP and the row swaps, and converts to bf16 in hardware where it writes bf16
    assert re.search(r"^_ZN6equarx10hop_kernelILi256ELi\d+ELb[01]EEEv", asm, flags=re.M)
    assert "v_permlane32_swap" in asm and "v_permlane16_swap" in asm and "row_mirror" in asm
    assert "v_cvt_pk_bf16_f32" in asm
    assert "v_perm_b32" in asm
