"""The C-ABI library loads without a GPU, exports what include/equarx.h declares, and rejects bad arguments
on the host (no kernel is launched by any call here)."""
import ctypes
import os
import re

import pytest

from paper_2506_17615_amd import binding, build

HEADER = os.path.join(os.path.dirname(build.INCLUDE), "include", "equarx.h")


@pytest.fixture(scope="module")
def lib():
    if build.is_stale():
        build.build()
    return binding.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(equarx_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree(lib):
    names = declared_functions()
    assert "equarx_quantize" in names and "equarx_reduce_quantized" in names
    assert set(names) == set(binding.SIGNATURES), "binding.SIGNATURES must list exactly the header's functions"
    for name in names:
        assert hasattr(lib, name), f"{name} declared in equarx.h but not exported"


def test_status_strings(lib):
    seen = {binding.status_string(s) for s in range(0, 7)}
    assert len(seen) == 7 and "unknown status" not in seen
    assert binding.status_string(99) == "unknown status"


def test_size_queries(lib):
    assert binding.num_blocks(4096, 256) == 16
    assert binding.num_blocks(4097, 256) == 17
    assert binding.num_blocks(0, 32) == 0
    assert binding.num_blocks(100, 100) == 0            # unsupported block
    assert binding.num_blocks(-1, 32) == 0
    assert binding.wire_row_codes(4097) == 4112 and binding.wire_row_scales(4097, 256) == 20
    n, B = 22_020_096, 256
    assert binding.workspace_bytes(8, n, B) == 2 * (n + 4 * n // B)
    assert binding.workspace_bytes(8, 1000, 32) == 2 * (1024 + 256)
    assert binding.workspace_bytes(0, n, B) == 0 and binding.workspace_bytes(65, n, B) == 0
    assert binding.workspace_bytes(8, n, 48) == 0


A = 0x7F0000001000          # a 16-byte aligned, never dereferenced address
ODD = A + 8


def test_validation_rejects_before_launch(lib):
    q, d, st, rq = lib.equarx_quantize, lib.equarx_dequantize, lib.equarx_reduce_stage, lib.equarx_reduce_quantized
    B = binding
    # block sizes
    for bad in (0, 1, 16, 48, 100, 1024, -256):
        assert q(A, 4096, bad, A, A, None) == B.STATUS_BAD_BLOCK
        assert d(A, A, 4096, bad, A, None) == B.STATUS_BAD_BLOCK
        assert st(A, A, A, 4096, bad, A, A, None) == B.STATUS_BAD_BLOCK
    # shapes
    assert q(A, -1, 256, A, A, None) == B.STATUS_BAD_SHAPE
    assert q(A, (1 << 40) + 1, 256, A, A, None) == B.STATUS_BAD_SHAPE
    assert d(A, A, -5, 256, A, None) == B.STATUS_BAD_SHAPE
    # n == 0 is a valid no-op, even with NULL buffers
    assert q(None, 0, 256, None, None, None) == B.STATUS_OK
    assert d(None, None, 0, 32, None, None) == B.STATUS_OK
    assert st(None, None, None, 0, 64, None, None, None) == B.STATUS_OK
    # NULL pointers
    assert q(None, 4096, 256, A, A, None) == B.STATUS_NULL_POINTER
    assert q(A, 4096, 256, None, A, None) == B.STATUS_NULL_POINTER
    assert q(A, 4096, 256, A, None, None) == B.STATUS_NULL_POINTER
    assert d(A, None, 4096, 256, A, None) == B.STATUS_NULL_POINTER
    assert st(A, A, None, 4096, 256, A, A, None) == B.STATUS_NULL_POINTER
    # alignment
    assert q(ODD, 4096, 256, A, A, None) == B.STATUS_MISALIGNED
    assert q(A, 4096, 256, ODD, A, None) == B.STATUS_MISALIGNED
    assert q(A, 4096, 256, A, A + 4, None) == B.STATUS_MISALIGNED
    assert d(A, A, 4096, 256, A + 2, None) == B.STATUS_MISALIGNED
    assert st(A, A, ODD, 4096, 256, A, A, None) == B.STATUS_MISALIGNED

    def table(*ptrs):
        return (ctypes.c_void_p * len(ptrs))(*ptrs)

    n, blk = 4096, 256
    need = B.workspace_bytes(4, n, blk)
    ok4 = table(A, A + 0x10000, A + 0x20000, A + 0x30000)
    OUT, WS = A + 0x100000, A + 0x200000
    assert rq(ok4, 0, n, blk, OUT, WS, need, None, None, None) == B.STATUS_BAD_SHAPE
    assert rq(ok4, 65, n, blk, OUT, WS, need, None, None, None) == B.STATUS_BAD_SHAPE
    assert rq(None, 4, n, blk, OUT, WS, need, None, None, None) == B.STATUS_NULL_POINTER
    assert rq(ok4, 4, n, blk, None, WS, need, None, None, None) == B.STATUS_NULL_POINTER
    assert rq(ok4, 4, n, blk, OUT, None, need, None, None, None) == B.STATUS_NULL_POINTER
    assert rq(ok4, 4, n, blk, OUT, WS, need - 1, None, None, None) == B.STATUS_WORKSPACE_TOO_SMALL
    assert rq(ok4, 4, n, blk, OUT, WS + 16, need, None, None, None) == B.STATUS_MISALIGNED
    assert rq(table(A, 0, A, A), 4, n, blk, OUT, WS, need, None, None, None) == B.STATUS_NULL_POINTER
    assert rq(table(A, A, ODD, A), 4, n, blk, OUT, WS, need, None, None, None) == B.STATUS_MISALIGNED
    assert rq(table(A, OUT + 64, A, A), 4, n, blk, OUT, WS, need, None, None, None) == B.STATUS_BAD_SHAPE   # out overlaps a partial without being it
    assert rq(ok4, 4, n, blk, OUT, WS, need, A, None, None) == B.STATUS_NULL_POINTER                   # wire arrays come in pairs
    assert rq(ok4, 4, n, blk, OUT, None, 0, ODD, A, None) == B.STATUS_MISALIGNED
    assert rq(ok4, 4, n, 100, OUT, WS, need, None, None, None) == B.STATUS_BAD_BLOCK
    assert rq(ok4, 4, 0, blk, None, None, 0, None, None, None) == B.STATUS_OK
    rf = lib.equarx_reduce_fused
    assert rf(ok4, 0, n, blk, OUT, None, None, None) == B.STATUS_BAD_SHAPE
    assert rf(ok4, 65, n, blk, OUT, None, None, None) == B.STATUS_BAD_SHAPE
    assert rf(None, 4, n, blk, OUT, None, None, None) == B.STATUS_NULL_POINTER
    assert rf(ok4, 4, n, blk, None, None, None, None) == B.STATUS_NULL_POINTER
    assert rf(ok4, 4, n, blk, OUT, A, None, None) == B.STATUS_NULL_POINTER
    assert rf(ok4, 4, n, blk, OUT + 2, None, None, None) == B.STATUS_MISALIGNED
    assert rf(ok4, 4, n, blk, OUT, ODD, A, None) == B.STATUS_MISALIGNED
    assert rf(table(A, A, 0, A), 4, n, blk, OUT, None, None, None) == B.STATUS_NULL_POINTER
    assert rf(table(A, A, A, ODD), 4, n, blk, OUT, None, None, None) == B.STATUS_MISALIGNED
    assert rf(table(OUT - 2 * n + 16, A, A, A), 4, n, blk, OUT, None, None, None) == B.STATUS_BAD_SHAPE     # overlap
    assert rf(ok4, 4, n, 7, OUT, None, None, None) == B.STATUS_BAD_BLOCK
    assert rf(ok4, 4, -3, blk, OUT, None, None, None) == B.STATUS_BAD_SHAPE
    assert rf(ok4, 4, 0, blk, None, None, None, None) == B.STATUS_OK
    rv = lib.equarx_reduce_variant
    assert rv(ok4, 4, n, blk, 2 | 4, OUT, None) == B.STATUS_BAD_SHAPE
    assert rv(ok4, 4, n, blk, 1 | 2, OUT, None) == B.STATUS_BAD_SHAPE
    assert rv(ok4, 4, n, blk, 16, OUT, None) == B.STATUS_BAD_SHAPE
    assert rv(ok4, 0, n, blk, 0, OUT, None) == B.STATUS_BAD_SHAPE
    assert rv(None, 4, n, blk, 1, OUT, None) == B.STATUS_NULL_POINTER
    assert rv(ok4, 4, n, blk, 8, None, None) == B.STATUS_NULL_POINTER
    assert rv(ok4, 4, n, blk, 1, OUT + 4, None) == B.STATUS_MISALIGNED
    assert rv(table(A, A, A, ODD), 4, n, blk, 4, OUT, None) == B.STATUS_MISALIGNED
    assert rv(table(A, OUT + 16, A, A), 4, n, blk, 9, OUT, None) == B.STATUS_BAD_SHAPE
    assert rv(ok4, 4, n, 96, 0, OUT, None) == B.STATUS_BAD_BLOCK
    assert rv(ok4, 4, 0, blk, 1, None, None) == B.STATUS_OK
    qs_, ds_, ss_, rs_ = (lib.equarx_quantize_strided, lib.equarx_dequantize_strided, lib.equarx_reduce_stage_strided,
                          lib.equarx_reduce_quantized_strided)
    ns = 1024 * 64
    assert qs_(A, ns, 48, A, A, None) == B.STATUS_BAD_BLOCK and qs_(A, ns, 256, A, A, None) == B.STATUS_BAD_BLOCK
    assert qs_(A, ns + 1024, 64, A, A, None) == B.STATUS_BAD_SHAPE and qs_(A, -ns, 64, A, A, None) == B.STATUS_BAD_SHAPE
    assert qs_(None, ns, 64, A, A, None) == B.STATUS_NULL_POINTER and qs_(A, ns, 64, ODD, A, None) == B.STATUS_MISALIGNED
    assert qs_(None, 0, 64, None, None, None) == B.STATUS_OK
    assert ds_(A, None, ns, 64, A, None) == B.STATUS_NULL_POINTER and ds_(A, A, ns, 64, A + 2, None) == B.STATUS_MISALIGNED
    assert ds_(A, A, ns // 2, 64, A, None) == B.STATUS_BAD_SHAPE
    assert ss_(A, A, None, ns, 64, A, A, None) == B.STATUS_NULL_POINTER and ss_(A, A, A, ns, 7, A, A, None) == B.STATUS_BAD_BLOCK
    assert rs_(ok4, 4, ns, 64, OUT, WS, 0, None) == B.STATUS_WORKSPACE_TOO_SMALL
    assert rs_(ok4, 4, ns, 64, OUT, None, 1 << 30, None) == B.STATUS_NULL_POINTER
    assert rs_(ok4, 0, ns, 64, OUT, WS, 1 << 30, None) == B.STATUS_BAD_SHAPE
    assert rs_(table(A, OUT + 16, A, A), 4, ns, 64, OUT, WS, 1 << 30, None) == B.STATUS_BAD_SHAPE
    assert rs_(ok4, 4, ns, 64, OUT, WS + 8, 1 << 30, None) == B.STATUS_MISALIGNED
    vh, vw = lib.equarx_reduce_variant_hops, lib.equarx_variant_workspace_bytes
    assert vw(0, 4, n, blk) == need and vw(B.SEMI_LOOP, 4, n, blk) == need // 2 * 3 and vw(0, 4, n, 100) == 0
    need3 = vw(B.SEMI_LOOP, 4, n, blk)
    for bad_flags in (B.RS_UNQUANTIZED, B.RING_ORDER | B.RS_UNQUANTIZED, 16, B.SEMI_LOOP | B.RING_ORDER):
        assert vh(ok4, 4, n, blk, bad_flags, OUT, WS, need3, None) == B.STATUS_BAD_SHAPE
    assert vh(ok4, 0, n, blk, 0, OUT, WS, need3, None) == B.STATUS_BAD_SHAPE
    assert vh(None, 4, n, blk, 0, OUT, WS, need3, None) == B.STATUS_NULL_POINTER
    assert vh(ok4, 4, n, blk, 0, OUT, None, need3, None) == B.STATUS_NULL_POINTER
    assert vh(ok4, 4, n, blk, 0, OUT, WS + 16, need3, None) == B.STATUS_MISALIGNED
    assert vh(ok4, 4, n, blk, 0, OUT, WS, need - 1, None) == B.STATUS_WORKSPACE_TOO_SMALL
    assert vh(ok4, 4, n, blk, B.SEMI_LOOP, OUT, WS, need, None) == B.STATUS_WORKSPACE_TOO_SMALL      # needs three buffers
    assert vh(table(A, OUT + 16, A, A), 4, n, blk, B.SEMI_LOOP, OUT, WS, need3, None) == B.STATUS_BAD_SHAPE
    assert vh(ok4, 4, n, 100, 0, OUT, WS, need3, None) == B.STATUS_BAD_BLOCK and vh(ok4, 4, 0, blk, 0, None, None, 0, None) == B.STATUS_OK
    sr = lib.equarx_selftest_rounding
    assert sr(0, 16, None, None) == B.STATUS_NULL_POINTER and sr(0, 16, A + 4, None) == B.STATUS_MISALIGNED
    assert sr(0x42FFFFFF, 2, A, None) == B.STATUS_BAD_SHAPE and sr(0, 0, None, None) == B.STATUS_OK
    ht = lib.equarx_calib_hop_traffic
    C0, C1 = A + 0x300000, A + 0x400000
    assert ht(None, 4, n, blk, C0, C0 + 0x1000, C1, C1 + 0x1000, None) == B.STATUS_NULL_POINTER
    assert ht(ok4, 4, n, blk, None, C0 + 0x1000, C1, C1 + 0x1000, None) == B.STATUS_NULL_POINTER
    assert ht(ok4, 4, n + 8, blk, C0, C0 + 0x1000, C1, C1 + 0x1000, None) == B.STATUS_BAD_SHAPE
    assert ht(ok4, 4, n, 100, C0, C0 + 0x1000, C1, C1 + 0x1000, None) == B.STATUS_BAD_BLOCK
    assert ht(ok4, 65, n, blk, C0, C0 + 0x1000, C1, C1 + 0x1000, None) == B.STATUS_BAD_SHAPE
    assert ht(ok4, 4, n, blk, ODD, C0 + 0x1000, C1, C1 + 0x1000, None) == B.STATUS_MISALIGNED
    assert ht(ok4, 4, n, blk, C0, C0 + 0x1000, C0, C1 + 0x1000, None) == B.STATUS_BAD_SHAPE
    assert ht(table(A, 0, A, A), 4, n, blk, C0, C0 + 0x1000, C1, C1 + 0x1000, None) == B.STATUS_NULL_POINTER
    assert ht(ok4, 4, 0, blk, None, None, None, None, None) == B.STATUS_OK
    fe = lib.equarx_reduce_quantized_fused_ends
    assert fe(ok4, 0, n, blk, OUT, WS, need, None) == B.STATUS_BAD_SHAPE and fe(ok4, 65, n, blk, OUT, WS, need, None) == B.STATUS_BAD_SHAPE
    assert fe(None, 4, n, blk, OUT, WS, need, None) == B.STATUS_NULL_POINTER and fe(ok4, 4, n, blk, None, WS, need, None) == B.STATUS_NULL_POINTER
    assert fe(ok4, 4, n, blk, OUT, None, need, None) == B.STATUS_NULL_POINTER
    assert fe(ok4, 4, n, blk, OUT, WS, need - 1, None) == B.STATUS_WORKSPACE_TOO_SMALL
    assert fe(ok4, 4, n, blk, OUT, WS + 16, need, None) == B.STATUS_MISALIGNED
    assert fe(table(A, 0, A, A), 4, n, blk, OUT, WS, need, None) == B.STATUS_NULL_POINTER
    assert fe(table(A, A, ODD, A), 4, n, blk, OUT, WS, need, None) == B.STATUS_MISALIGNED
    assert fe(table(A, OUT + 16, A, A), 4, n, blk, OUT, WS, need, None) == B.STATUS_BAD_SHAPE
    assert fe(ok4, 4, n, 100, OUT, WS, need, None) == B.STATUS_BAD_BLOCK and fe(ok4, 4, 0, blk, None, None, 0, None) == B.STATUS_OK
    fs_ = lib.equarx_reduce_fused_strided
    assert fs_(ok4, 4, ns, 64, None, None) == B.STATUS_NULL_POINTER and fs_(ok4, 4, ns, 96, OUT, None) == B.STATUS_BAD_BLOCK
    assert fs_(ok4, 4, ns + 8, 64, OUT, None) == B.STATUS_BAD_SHAPE and fs_(ok4, 65, ns, 64, OUT, None) == B.STATUS_BAD_SHAPE
    assert fs_(table(A, A, ODD, A), 4, ns, 64, OUT, None) == B.STATUS_MISALIGNED
    assert fs_(table(A, A, OUT + 16, A), 4, ns, 64, OUT, None) == B.STATUS_BAD_SHAPE
    assert fs_(None, 4, 0, 64, None, None) == B.STATUS_NULL_POINTER and fs_(ok4, 4, 0, 64, None, None) == B.STATUS_OK
    qb = lib.equarx_quantize_batch
    xs, cs, ss = table(A, A + 0x1000), table(A + 0x2000, A + 0x3000), table(A + 0x4000, A + 0x5000)
    assert qb(xs, cs, ss, 65, n, blk, None) == B.STATUS_BAD_SHAPE
    assert qb(xs, cs, ss, -1, n, blk, None) == B.STATUS_BAD_SHAPE
    assert qb(None, cs, ss, 2, n, blk, None) == B.STATUS_NULL_POINTER
    assert qb(table(A, 0), cs, ss, 2, n, blk, None) == B.STATUS_NULL_POINTER
    assert qb(xs, table(A + 0x2000, ODD), ss, 2, n, blk, None) == B.STATUS_MISALIGNED
    assert qb(xs, table(A + 0x2000, A + 0x2000), ss, 2, n, blk, None) == B.STATUS_BAD_SHAPE
    assert qb(xs, cs, ss, 2, n, 5, None) == B.STATUS_BAD_BLOCK
    assert qb(None, None, None, 0, n, blk, None) == B.STATUS_OK
    fl = lib.equarx_reduce_flat
    ctab, stab = table(A, A + 0x10000), table(A + 0x20000, A + 0x30000)
    assert fl(A + 0x40000, ctab, stab, 2, n, blk, None, None, None, None) == B.STATUS_NULL_POINTER
    assert fl(None, ctab, stab, 2, n, blk, OUT, None, None, None) == B.STATUS_NULL_POINTER
    assert fl(A + 0x40000, None, stab, 2, n, blk, OUT, None, None, None) == B.STATUS_NULL_POINTER
    assert fl(A + 0x40000, ctab, stab, 2, n, blk, OUT, A + 0x50000, None, None) == B.STATUS_NULL_POINTER
    assert fl(A + 0x40000, ctab, stab, 64, n, blk, OUT, None, None, None) == B.STATUS_BAD_SHAPE
    assert fl(A + 0x40000, ctab, stab, -1, n, blk, OUT, None, None, None) == B.STATUS_BAD_SHAPE
    assert fl(A + 0x40000, table(A, ODD), stab, 2, n, blk, OUT, None, None, None) == B.STATUS_MISALIGNED
    assert fl(A + 0x40000, table(A, 0), stab, 2, n, blk, OUT, None, None, None) == B.STATUS_NULL_POINTER
    assert fl(A + 0x40000, ctab, stab, 2, n, blk, A + 0x40000, None, None, None) == B.STATUS_BAD_SHAPE
    assert fl(A + 0x40000, ctab, stab, 2, n, blk, OUT + 8, None, None, None) == B.STATUS_MISALIGNED
    assert fl(A + 0x40000, ctab, stab, 2, n, 33, OUT, None, None, None) == B.STATUS_BAD_BLOCK
    assert fl(None, None, None, 0, 0, blk, None, None, None, None) == B.STATUS_OK
    # calibration copy
    cp = lib.equarx_calib_copy
    assert cp(A, A + 0x1000, 0, None) == B.STATUS_OK
    assert cp(None, A, 64, None) == B.STATUS_NULL_POINTER
    assert cp(A, A + 0x1000, 40, None) == B.STATUS_BAD_SHAPE
    assert cp(A, ODD, 64, None) == B.STATUS_MISALIGNED


def test_missing_library_is_an_error(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(build, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load()


def test_header_is_plain_c(tmp_path):
    """include/equarx.h is a C header: a C99 translation unit that includes it and takes the address of every
    declared function compiles with gcc (no C++, no HIP, no torch types in the signatures)."""
    import subprocess
    names = declared_functions()
    src = tmp_path / "use_header.c"
    body = "\n".join(f"    p[{i}] = (void (*)(void))&{n};" for i, n in enumerate(names))
    src.write_text(f'#include "equarx.h"\nvoid (*p[{len(names)}])(void);\nvoid take(void) {{\n{body}\n}}\n')
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-c", str(src), "-I", os.path.dirname(HEADER),
                    "-o", str(tmp_path / "use_header.o")], check=True)


def test_plain_c_client_builds_and_links():
    """A C99 program that uses nothing but include/equarx.h and the HIP runtime's C API compiles and links against
    the library (it runs in the GPU tests)."""
    from tests import build_abi_client
    binding.load()      # the library must be there to link against
    path = build_abi_client.build(force=True)
    assert os.path.exists(path) and os.access(path, os.X_OK)
