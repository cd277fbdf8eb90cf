"""The C-ABI library loads without a GPU, exports what include/equarx.h declares, and rejects bad arguments
on the host (no kernel is launched by any call here)."""
import ctypes
import os
import re

import pytest

from paper_2506_17615_amd import binding, build

HEADER = os.path.join(build.INCLUDE, "equarx.h")
DEVTOOLS_HEADER = os.path.join(build.INCLUDE, "equarx_devtools.h")


@pytest.fixture(scope="module")
def lib():
    if build.is_stale():
        build.build()
    return binding.load()


def declared_functions(header=HEADER):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(equarx_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree(lib):
    names = declared_functions()
    assert "equarx_quantize" in names and "equarx_reduce_quantized" in names
    assert set(names) == set(binding.SIGNATURES), "binding.SIGNATURES must list exactly the header's functions"
    dev = declared_functions(DEVTOOLS_HEADER)
    assert set(dev) == set(binding.DEVTOOLS_SIGNATURES), "binding.DEVTOOLS_SIGNATURES must list exactly equarx_devtools.h"
    assert not set(dev) & set(names)
    for name in names + dev:
        assert hasattr(lib, name), f"{name} declared in a header but not exported"
    # the product header declares the method's calls and size queries only: no calibration, self-test or timing aid
    assert not [n for n in names if re.search(r"calib|selftest|time_|eval_", n)]


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
    for bad_flags in (B.RS_UNQUANTIZED, B.RING_ORDER | B.RS_UNQUANTIZED, 16, B.SEMI_LOOP | B.RS_UNQUANTIZED):
        assert vh(ok4, 4, n, blk, bad_flags, OUT, WS, need3, None) == B.STATUS_BAD_SHAPE
    assert vw(B.SEMI_LOOP | B.RING_ORDER, 4, n, blk) == 2 * need       # both chains advance per launch: four wire buffers
    assert vh(ok4, 4, n, blk, B.SEMI_LOOP | B.RING_ORDER, OUT, WS, need3, None) == B.STATUS_WORKSPACE_TOO_SMALL
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
    vs_ = lib.equarx_reduce_variant_strided
    assert vs_(ok4, 4, ns, 64, 0, None, None) == B.STATUS_NULL_POINTER and vs_(ok4, 4, ns, 96, 0, OUT, None) == B.STATUS_BAD_BLOCK
    assert vs_(ok4, 4, ns + 8, 64, 0, OUT, None) == B.STATUS_BAD_SHAPE and vs_(ok4, 65, ns, 64, 0, OUT, None) == B.STATUS_BAD_SHAPE
    for bad_flags in (B.RS_UNQUANTIZED | B.AG_UNQUANTIZED, B.SEMI_LOOP | B.RS_UNQUANTIZED, B.RING_ORDER | B.RS_UNQUANTIZED | B.AG_UNQUANTIZED, 16):
        assert vs_(ok4, 4, ns, 64, bad_flags, OUT, None) == B.STATUS_BAD_SHAPE
    assert vs_(table(A, A, ODD, A), 4, ns, 64, B.SEMI_LOOP, OUT, None) == B.STATUS_MISALIGNED
    assert vs_(table(A, A, OUT + 16, A), 4, ns, 64, B.SEMI_LOOP, OUT, None) == B.STATUS_BAD_SHAPE
    assert vs_(None, 4, 0, 64, 0, None, None) == B.STATUS_NULL_POINTER and vs_(ok4, 4, 0, 64, B.SEMI_LOOP, None, None) == B.STATUS_OK
    hs_ = lib.equarx_reduce_variant_hops_strided
    need_s = lib.equarx_variant_workspace_bytes(B.SEMI_LOOP, 4, ns, 64)
    assert hs_(ok4, 4, ns, 64, 0, None, WS, need_s, None) == B.STATUS_NULL_POINTER
    assert hs_(ok4, 4, ns, 64, 0, OUT, None, need_s, None) == B.STATUS_NULL_POINTER
    assert hs_(ok4, 4, ns, 96, 0, OUT, WS, need_s, None) == B.STATUS_BAD_BLOCK
    assert hs_(ok4, 4, ns + 8, 64, 0, OUT, WS, need_s, None) == B.STATUS_BAD_SHAPE
    assert hs_(ok4, 0, ns, 64, 0, OUT, WS, need_s, None) == B.STATUS_BAD_SHAPE
    for bad_flags in (B.RS_UNQUANTIZED, B.RING_ORDER | B.RS_UNQUANTIZED, 16):
        assert hs_(ok4, 4, ns, 64, bad_flags, OUT, WS, need_s, None) == B.STATUS_BAD_SHAPE
    assert hs_(ok4, 4, ns, 64, B.SEMI_LOOP, OUT, WS, need_s - 1, None) == B.STATUS_WORKSPACE_TOO_SMALL
    assert hs_(ok4, 4, ns, 64, B.SEMI_LOOP, OUT, WS + 16, need_s, None) == B.STATUS_MISALIGNED
    assert hs_(table(A, A, OUT + 16, A), 4, ns, 64, 0, OUT, WS, need_s, None) == B.STATUS_BAD_SHAPE
    assert hs_(ok4, 4, ns, 64, 0, OUT, OUT, need_s, None) == B.STATUS_BAD_SHAPE                 # workspace = output
    assert hs_(ok4, 4, 0, 64, B.SEMI_LOOP, None, None, 0, None) == B.STATUS_OK
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


def test_overlapping_buffers_are_rejected_before_launch(lib):
    """Every buffer a call writes must be disjoint from the call's other buffers unless the header says the two may
    BE the same buffer: partial overlaps, an output inside an input, a workspace over the output -- all
    EQUARX_BAD_SHAPE, decided on the host from the addresses (none is ever dereferenced here)."""
    B = binding
    BAD = B.STATUS_BAD_SHAPE

    def table(*ptrs):
        return (ctypes.c_void_p * len(ptrs))(*ptrs)

    n, blk = 4096, 256                      # codes 4096 B, scales 64 B, bf16 8192 B
    X, C, S, OUT = A, A + 0x10000, A + 0x20000, A + 0x30000
    q, d, st = lib.equarx_quantize, lib.equarx_dequantize, lib.equarx_reduce_stage
    assert q(X, n, blk, X, S, None) == BAD                       # codes over the input
    assert q(X, n, blk, X + 8192 - 16, S, None) == BAD           # codes start inside the input's last 16 bytes
    assert q(X, n, blk, C, C + 4096 - 16, None) == BAD           # scales start inside the codes
    assert q(X, n, blk, C, X + 16, None) == BAD                  # scales inside the input
    assert d(C, S, n, blk, C, None) == BAD                       # output over the codes
    assert d(C, S, n, blk, S - 8192 + 16, None) == BAD           # output's tail reaches the scales
    C2, S2, L = A + 0x40000, A + 0x50000, A + 0x60000
    assert st(C, S, L, n, blk, C + 16, S2, None) == BAD          # wire updated "in place" but shifted
    assert st(C, S, L, n, blk, C2, S + 16, None) == BAD
    assert st(C, S, L, n, blk, L, S2, None) == BAD               # codes written over the local shard
    assert st(C, S, L, n, blk, C2, L + 4096, None) == BAD        # scales written into the local shard
    assert st(C, S, L, n, blk, S - 4096 + 16, S2, None) == BAD   # codes_out reaches into scales_in
    assert st(C, S, L, n, blk, C2, C2 + 1024, None) == BAD       # the two outputs overlap each other
    assert st(C, S, L, n, blk, S, C, None) == BAD                # outputs swapped onto the inputs: not the same role
    for fn in (lib.equarx_quantize_strided,):
        ns = 1024 * 64
        assert fn(X, ns, 64, X + 2 * ns - 16, S + 0x100000, None) == BAD
    ns = 1024 * 64
    assert lib.equarx_dequantize_strided(C, C + ns + 0x1000, ns, 64, C + 16, None) == BAD
    assert lib.equarx_reduce_stage_strided(C, A + 0x200000, A + 0x300000, ns, 64, C + 1024, A + 0x400000, None) == BAD

    need = B.workspace_bytes(4, n, blk)
    ok4 = table(A, A + 0x10000, A + 0x20000, A + 0x30000)
    OUT, WS = A + 0x100000, A + 0x200000
    chains = [
        lambda parts, out, ws: lib.equarx_reduce_quantized(parts, 4, n, blk, out, ws, need, None, None, None),
        lambda parts, out, ws: lib.equarx_reduce_quantized_fused_ends(parts, 4, n, blk, out, ws, need, None),
        lambda parts, out, ws: lib.equarx_reduce_variant_hops(parts, 4, n, blk, 0, out, ws, need, None),
        lambda parts, out, ws: lib.equarx_reduce_variant_hops(parts, 4, n, blk, B.AG_UNQUANTIZED, out, ws, need, None),
    ]
    for call in chains:
        assert call(ok4, OUT, OUT) == BAD                        # workspace = output
        assert call(ok4, OUT, OUT + 8192 - 256) == BAD           # workspace starts inside the output
        assert call(ok4, WS + need - 256, WS) == BAD             # output starts inside the workspace
        assert call(ok4, OUT, A + 0x20000) == BAD                # workspace over a partial
        assert call(ok4, OUT, A + 0x20000 - need + 256) == BAD   # workspace's tail reaches a partial
        assert call(table(A, A, OUT + 16, A), OUT, WS) == BAD    # output overlaps a partial without being it
    need3 = lib.equarx_variant_workspace_bytes(B.SEMI_LOOP, 4, n, blk)
    assert lib.equarx_reduce_variant_hops(ok4, 4, n, blk, B.SEMI_LOOP, OUT, OUT - need3 + 256, need3, None) == BAD
    ns = 1024 * 64
    needs = B.workspace_bytes(4, ns, 64)
    oks = table(A, A + 0x100000, A + 0x200000, A + 0x300000)
    assert lib.equarx_reduce_quantized_strided(oks, 4, ns, 64, A + 0x400000, A + 0x400000 + 2 * ns - 256, needs, None) == BAD
    assert lib.equarx_reduce_quantized_strided(oks, 4, ns, 64, A + 0x400000, A + 0x200000, needs, None) == BAD
    # kept wire: [P][row] arrays the chain writes
    rc, rs = B.wire_row_codes(n), B.wire_row_scales(n, blk)
    WC, WSC = A + 0x300000, A + 0x400000
    rq, rf = lib.equarx_reduce_quantized, lib.equarx_reduce_fused
    assert rq(ok4, 4, n, blk, OUT, None, 0, OUT, WSC, None) == BAD                       # wire codes over the output
    assert rq(ok4, 4, n, blk, OUT, None, 0, WC, WC + 4 * rc - 16, None) == BAD           # scales start inside the codes' last row
    assert rq(ok4, 4, n, blk, OUT, None, 0, A + 0x10000 - 4 * rc + 16, WSC, None) == BAD # wire codes reach into partial 1
    assert rq(ok4, 4, n, blk, WSC + 16, None, 0, WC, WSC, None) == BAD                   # output inside the wire scales
    assert rf(ok4, 4, n, blk, OUT, OUT + 4096, WSC, None) == BAD
    assert rf(ok4, 4, n, blk, OUT, WC, A + 0x30000 + 8192 - 16, None) == BAD             # wire scales over partial 3's end
    assert rf(ok4, 4, n, blk, OUT, WC, WC + 16, None) == BAD
    # flat: nothing written may share memory with anything read or with another output
    fl = lib.equarx_reduce_flat
    LOC = A + 0x40000
    ctab, stab = table(A, A + 0x10000), table(A + 0x20000, A + 0x30000)
    CO, SO = A + 0x500000, A + 0x600000
    assert fl(LOC, ctab, stab, 2, n, blk, LOC + 16, None, None, None) == BAD             # output overlaps the local shard
    assert fl(LOC, ctab, stab, 2, n, blk, A + 0x10000 - 8192 + 16, None, None, None) == BAD    # output's tail in codes[1]
    assert fl(LOC, ctab, stab, 2, n, blk, OUT, A, SO, None) == BAD                       # codes_out = a received shard
    assert fl(LOC, ctab, stab, 2, n, blk, OUT, A + 2048, SO, None) == BAD                # ... or half way into it
    assert fl(LOC, ctab, stab, 2, n, blk, OUT, CO, A + 0x30000, None) == BAD             # scales_out = received scales
    assert fl(LOC, ctab, stab, 2, n, blk, OUT, OUT + 4096, SO, None) == BAD              # two outputs overlap
    assert fl(LOC, ctab, stab, 2, n, blk, None, CO, CO + 4096 - 16, None) == BAD
    assert fl(LOC, ctab, stab, 2, n, blk, OUT, LOC + 4096, SO, None) == BAD              # codes_out in the local shard
    # batch quantize: every output against every input and every other output
    qb = lib.equarx_quantize_batch
    xs = table(A, A + 0x10000)
    assert qb(xs, table(A + 0x20000, A + 0x20000 + 2048), table(A + 0x40000, A + 0x50000), 2, n, blk, None) == BAD
    assert qb(xs, table(A + 0x20000, A + 0x30000), table(A + 0x40000, A + 0x40000 + 32), 2, n, blk, None) == BAD
    assert qb(xs, table(A + 0x20000, A + 0x10000 + 4096), table(A + 0x40000, A + 0x50000), 2, n, blk, None) == BAD
    assert qb(xs, table(A + 0x20000, A + 0x30000), table(A + 16, A + 0x50000), 2, n, blk, None) == BAD
    assert qb(xs, table(A + 0x20000, A + 0x30000), table(A + 0x30000 + 4096 - 16, A + 0x50000), 2, n, blk, None) == BAD
    # developer aids follow the same rule
    assert lib.equarx_calib_copy(A, A + 64, 128, None) == BAD and lib.equarx_calib_copy(A, A, 128, None) == BAD
    ht = lib.equarx_calib_hop_traffic
    C0, C1 = A + 0x300000, A + 0x400000
    assert ht(ok4, 4, n, blk, C0, C0 + 0x1000, C0 + 2048, C1 + 0x1000, None) == BAD
    assert ht(ok4, 4, n, blk, C0, C0 + 0x1000, C1, C0 + 0x1000 + 16, None) == BAD
    assert ht(ok4, 4, n, blk, A + 0x20000 + 4096, C0 + 0x1000, C1, C1 + 0x1000, None) == BAD


def test_timing_hooks_do_not_outlive_the_next_call(lib):
    """A span or launch hook armed before a call that fails validation is dropped by that call: nothing stays
    pending for a later, unrelated call (checked through the library's own bookkeeping: arming, a rejected call,
    and equarx_time_cancel all return, and a second rejected call behaves the same)."""
    E0, E1 = A + 0x700000, A + 0x700100     # never used as events: every call below fails validation first
    lib.equarx_time_launch_span(0, 3, E0, E1)
    lib.equarx_time_next_launch(E0, E1)
    assert lib.equarx_quantize(A, 4096, 100, A, A, None) == binding.STATUS_BAD_BLOCK       # consumes and drops the hooks
    assert lib.equarx_quantize(None, 4096, 256, A, A, None) == binding.STATUS_NULL_POINTER
    lib.equarx_time_launch_span(2, 1, E0, E1)          # invalid: cancels
    lib.equarx_time_cancel()


def test_missing_library_is_an_error(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(build, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load()


def test_header_is_plain_c(tmp_path):
    """include/equarx.h is a C header: a C99 translation unit that includes it and takes the address of every
    declared function compiles with gcc (no C++, no HIP, no torch types in the signatures)."""
    import subprocess
    names = declared_functions() + declared_functions(DEVTOOLS_HEADER)
    src = tmp_path / "use_header.c"
    body = "\n".join(f"    p[{i}] = (void (*)(void))&{n};" for i, n in enumerate(names))
    src.write_text(f'#include "equarx.h"\n#include "equarx_devtools.h"\nvoid (*p[{len(names)}])(void);\n'
                   f'void take(void) {{\n{body}\n}}\n')
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-c", str(src), "-I", os.path.dirname(HEADER),
                    "-o", str(tmp_path / "use_header.o")], check=True)


def test_plain_c_client_builds_and_links():
    """A C99 program that uses nothing but include/equarx.h and the HIP runtime's C API compiles and links against
    the library (it runs in the GPU tests)."""
    from tests import build_abi_client
    binding.load()      # the library must be there to link against
    path = build_abi_client.build(force=True)
    assert os.path.exists(path) and os.access(path, os.X_OK)
