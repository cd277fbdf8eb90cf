"""Thin Python binding of libequarx.so: argument marshalling only.

Every function has the name and meaning of the C entry point declared in
``include/equarx.h``; tensors are torch CUDA tensors used purely as device
memory, and work is enqueued on torch's current stream.  There is no CPU
fallback: if the HIP library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

_lib = None

STATUS_OK = 0
STATUS_NULL_POINTER = 1
STATUS_BAD_SHAPE = 2
STATUS_BAD_BLOCK = 3
STATUS_MISALIGNED = 4
STATUS_WORKSPACE_TOO_SMALL = 5
STATUS_DEVICE_ERROR = 6
MAX_PARTIALS = 64
BLOCK_SIZES = (32, 64, 128, 256, 512)
SEMI_LOOP, RS_UNQUANTIZED, AG_UNQUANTIZED, RING_ORDER = 1, 2, 4, 8

# name -> (restype, argtypes); SIGNATURES mirrors include/equarx.h, DEVTOOLS_SIGNATURES include/equarx_devtools.h
_vp, _i64, _i32, _sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
SIGNATURES = {
    "equarx_quantize": (ctypes.c_int, [_vp, _i64, _i32, _vp, _vp, _vp]),
    "equarx_quantize_batch": (ctypes.c_int, [ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.POINTER(_vp), _i32, _i64,
                                             _i32, _vp]),
    "equarx_dequantize": (ctypes.c_int, [_vp, _vp, _i64, _i32, _vp, _vp]),
    "equarx_reduce_stage": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i32, _vp, _vp, _vp]),
    "equarx_reduce_quantized": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i64, _i32, _vp, _vp, _sz, _vp, _vp, _vp]),
    "equarx_reduce_quantized_static": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i64, _i32, _vp, _vp]),
    "equarx_reduce_quantized_fused_ends": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i64, _i32, _vp, _vp, _sz, _vp]),
    "equarx_reduce_fused": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i64, _i32, _vp, _vp, _vp, _vp]),
    "equarx_reduce_variant": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i64, _i32, ctypes.c_uint32, _vp, _vp]),
    "equarx_reduce_variant_hops": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i64, _i32, ctypes.c_uint32, _vp, _vp, _sz, _vp]),
    "equarx_variant_workspace_bytes": (_sz, [ctypes.c_uint32, _i32, _i64, _i32]),
    "equarx_reduce_flat": (ctypes.c_int, [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _i32, _i64, _i32, _vp, _vp, _vp,
                                          _vp]),
    "equarx_quantize_strided": (ctypes.c_int, [_vp, _i64, _i32, _vp, _vp, _vp]),
    "equarx_dequantize_strided": (ctypes.c_int, [_vp, _vp, _i64, _i32, _vp, _vp]),
    "equarx_reduce_stage_strided": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i32, _vp, _vp, _vp]),
    "equarx_reduce_quantized_strided": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i64, _i32, _vp, _vp, _sz, _vp]),
    "equarx_reduce_fused_strided": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i64, _i32, _vp, _vp]),
    "equarx_reduce_variant_strided": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i64, _i32, ctypes.c_uint32, _vp, _vp]),
    "equarx_reduce_variant_hops_strided": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i64, _i32, ctypes.c_uint32, _vp, _vp,
                                                          _sz, _vp]),
    "equarx_workspace_bytes": (_sz, [_i32, _i64, _i32]),
    "equarx_num_blocks": (_i64, [_i64, _i32]),
    "equarx_wire_row_codes": (_i64, [_i64]),
    "equarx_wire_row_scales": (_i64, [_i64, _i32]),
    "equarx_status_string": (ctypes.c_char_p, [ctypes.c_int]),
}
DEVTOOLS_SIGNATURES = {
    "equarx_calib_hop_traffic": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i64, _i32, _vp, _vp, _vp, _vp, _vp]),
    "equarx_calib_copy": (ctypes.c_int, [_vp, _vp, _sz, _vp]),
    "equarx_calib_empty_launches": (ctypes.c_int, [_i32, _i32, _vp]),
    "equarx_calib_interleaved_chains": (ctypes.c_int, [ctypes.POINTER(_vp), _i32, _i32, _i64, _i32, ctypes.POINTER(_vp),
                                                       ctypes.POINTER(_vp), _sz, _i32, _vp]),
    "equarx_selftest_quotients": (ctypes.c_int, [ctypes.c_uint32, ctypes.c_uint64, _vp, _vp]),
    "equarx_selftest_rounding": (ctypes.c_int, [ctypes.c_uint32, ctypes.c_uint64, _vp, _vp]),
    "equarx_eval_quotients": (ctypes.c_int, [_vp, _i64, _vp, _vp, _vp]),
    "equarx_time_launch_span": (None, [_i32, _i32, _vp, _vp]),
    "equarx_time_next_launch": (None, [_vp, _vp]),
    "equarx_time_cancel": (None, []),
}


class EquarxError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__(f"{where}: status {status} ({status_string(status)})")


def lib_path() -> str:
    return _build.LIB_PATH


def load() -> ctypes.CDLL:
    """Open libequarx.so (built in-tree by ``build.build()``); raises if it is not there."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(
                f"{path} is missing: build it first (python -m paper_2506_17615_amd.build); "
                "there is no fallback path")
        lib = ctypes.CDLL(path)
        for name, (res, args) in {**SIGNATURES, **DEVTOOLS_SIGNATURES}.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().equarx_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != STATUS_OK:
        raise EquarxError(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _need(t, dtype, count: int, what: str) -> None:
    """Host-side guard: a buffer handed to a kernel is a CUDA tensor of the right type, contiguous, long enough."""
    if count == 0:
        return
    if t is None or not t.is_cuda or t.dtype != dtype or not t.is_contiguous() or t.numel() < count:
        raise ValueError(f"{what}: need a contiguous CUDA {dtype} tensor of at least {count} elements")


def num_blocks(n: int, block: int) -> int:
    return int(load().equarx_num_blocks(n, block))


def workspace_bytes(P: int, n: int, block: int) -> int:
    return int(load().equarx_workspace_bytes(P, n, block))


def wire_row_codes(n: int) -> int:
    return int(load().equarx_wire_row_codes(n))


def wire_row_scales(n: int, block: int) -> int:
    return int(load().equarx_wire_row_scales(n, block))


def equarx_quantize(x_bf16: torch.Tensor, block: int, codes: torch.Tensor, scales: torch.Tensor) -> None:
    """codes[n] int8, scales[nb] fp32 <- Q_B(x_bf16[n])."""
    n = x_bf16.numel()
    _need(x_bf16, torch.bfloat16, n, "x_bf16")
    _need(codes, torch.int8, n, "codes")
    _need(scales, torch.float32, num_blocks(n, block), "scales")
    _check(load().equarx_quantize(_ptr(x_bf16), x_bf16.numel(), block, _ptr(codes), _ptr(scales), _stream()),
           "equarx_quantize")


def equarx_quantize_batch(xs, block: int, codes_list, scales_list) -> None:
    """equarx_quantize on several bf16 tensors of equal length in one launch."""
    count = len(xs)
    if len(codes_list) != count or len(scales_list) != count:
        raise ValueError("xs, codes_list and scales_list differ in length")
    n = xs[0].numel() if count else 0
    nb = num_blocks(n, block) if count else 0
    for x, c, s in zip(xs, codes_list, scales_list):
        _need(x, torch.bfloat16, n, "x_bf16")
        if x.numel() != n:
            raise ValueError("tensors differ in length")
        _need(c, torch.int8, n, "codes")
        _need(s, torch.float32, nb, "scales")
    mk = lambda ts: (_vp * max(count, 1))(*[t.data_ptr() for t in ts])
    _check(load().equarx_quantize_batch(mk(xs), mk(codes_list), mk(scales_list), count, n, block, _stream()),
           "equarx_quantize_batch")


def equarx_dequantize(codes: torch.Tensor, scales: torch.Tensor, block: int, out_bf16: torch.Tensor) -> None:
    """out_bf16[n] <- bf16(codes * scales[block])."""
    n = codes.numel()
    _need(codes, torch.int8, n, "codes")
    _need(scales, torch.float32, num_blocks(n, block), "scales")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    _check(load().equarx_dequantize(_ptr(codes), _ptr(scales), codes.numel(), block, _ptr(out_bf16), _stream()),
           "equarx_dequantize")


def equarx_reduce_stage(codes_in, scales_in, local_bf16, block: int, codes_out, scales_out) -> None:
    """One hop: (codes_out, scales_out) <- Q_B(fma(codes_in, scales_in, local_bf16))."""
    n = local_bf16.numel()
    nb = num_blocks(n, block)
    _need(local_bf16, torch.bfloat16, n, "local_bf16")
    _need(codes_in, torch.int8, n, "codes_in")
    _need(codes_out, torch.int8, n, "codes_out")
    _need(scales_in, torch.float32, nb, "scales_in")
    _need(scales_out, torch.float32, nb, "scales_out")
    _check(load().equarx_reduce_stage(_ptr(codes_in), _ptr(scales_in), _ptr(local_bf16), local_bf16.numel(), block,
                                      _ptr(codes_out), _ptr(scales_out), _stream()), "equarx_reduce_stage")


def equarx_reduce_quantized(partials, block: int, out_bf16, workspace=None, wire_codes=None, wire_scales=None) -> None:
    """The whole chain over the partials (sequence of bf16 tensors of equal length, chain order)."""
    P = len(partials)
    n = partials[0].numel() if P else 0
    for p in partials:
        _need(p, torch.bfloat16, n, "partial")
        if p.numel() != n:
            raise ValueError("partials differ in length")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    if wire_codes is not None or wire_scales is not None:
        _need(wire_codes, torch.int8, P * wire_row_codes(n), "wire_codes")
        _need(wire_scales, torch.float32, P * wire_row_scales(n, block) if block in BLOCK_SIZES else 0, "wire_scales")
    if workspace is not None and not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace: need a contiguous CUDA tensor")
    table = (_vp * max(P, 1))(*[p.data_ptr() for p in partials])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().equarx_reduce_quantized(table, P, n, block, _ptr(out_bf16), _ptr(workspace), ws_bytes,
                                          _ptr(wire_codes), _ptr(wire_scales), _stream()), "equarx_reduce_quantized")


STATIC_WORKSPACE_BYTES = 80 << 20


def equarx_reduce_quantized_static(partials, block: int, out_bf16) -> None:
    """equarx_reduce_quantized with the wire buffers in the library's static device array (allocates nothing)."""
    P = len(partials)
    n = partials[0].numel() if P else 0
    for p in partials:
        _need(p, torch.bfloat16, n, "partial")
        if p.numel() != n:
            raise ValueError("partials differ in length")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    table = (_vp * max(P, 1))(*[p.data_ptr() for p in partials])
    _check(load().equarx_reduce_quantized_static(table, P, n, block, _ptr(out_bf16), _stream()),
           "equarx_reduce_quantized_static")


def equarx_reduce_quantized_fused_ends(partials, block: int, out_bf16, workspace=None) -> None:
    """The hop-by-hop chain with its first two and last two passes fused (P-1 launches, same bits)."""
    P = len(partials)
    n = partials[0].numel() if P else 0
    for p in partials:
        _need(p, torch.bfloat16, n, "partial")
        if p.numel() != n:
            raise ValueError("partials differ in length")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    if workspace is not None and not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace: need a contiguous CUDA tensor")
    table = (_vp * max(P, 1))(*[p.data_ptr() for p in partials])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().equarx_reduce_quantized_fused_ends(table, P, n, block, _ptr(out_bf16), _ptr(workspace), ws_bytes,
                                                     _stream()), "equarx_reduce_quantized_fused_ends")


def equarx_reduce_fused(partials, block: int, out_bf16, wire_codes=None, wire_scales=None) -> None:
    """The whole chain in one launch (same bits as equarx_reduce_quantized, no workspace)."""
    P = len(partials)
    n = partials[0].numel() if P else 0
    for p in partials:
        _need(p, torch.bfloat16, n, "partial")
        if p.numel() != n:
            raise ValueError("partials differ in length")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    if wire_codes is not None or wire_scales is not None:
        _need(wire_codes, torch.int8, P * wire_row_codes(n), "wire_codes")
        _need(wire_scales, torch.float32, P * wire_row_scales(n, block) if block in BLOCK_SIZES else 0, "wire_scales")
    table = (_vp * max(P, 1))(*[p.data_ptr() for p in partials])
    _check(load().equarx_reduce_fused(table, P, n, block, _ptr(out_bf16), _ptr(wire_codes), _ptr(wire_scales),
                                      _stream()), "equarx_reduce_fused")


def equarx_reduce_variant(partials, block: int, flags: int, out_bf16) -> None:
    """A variant of the chain in one launch; flags: SEMI_LOOP | RS_UNQUANTIZED | AG_UNQUANTIZED | RING_ORDER."""
    P = len(partials)
    n = partials[0].numel() if P else 0
    for p in partials:
        _need(p, torch.bfloat16, n, "partial")
        if p.numel() != n:
            raise ValueError("partials differ in length")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    table = (_vp * max(P, 1))(*[p.data_ptr() for p in partials])
    _check(load().equarx_reduce_variant(table, P, n, block, flags, _ptr(out_bf16), _stream()), "equarx_reduce_variant")


def alloc_variant_workspace(flags: int, P: int, n: int, block: int) -> torch.Tensor:
    nbytes = int(load().equarx_variant_workspace_bytes(flags, P, n, block))
    return torch.empty(max(nbytes, 1), dtype=torch.uint8, device="cuda")


def equarx_reduce_variant_hops(partials, block: int, flags: int, out_bf16, workspace) -> None:
    """equarx_reduce_variant's full-loop / semi-loop forms hop by hop (one launch per hop, same bits)."""
    P = len(partials)
    n = partials[0].numel() if P else 0
    for p in partials:
        _need(p, torch.bfloat16, n, "partial")
        if p.numel() != n:
            raise ValueError("partials differ in length")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    if workspace is not None and not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace: need a contiguous CUDA tensor")
    table = (_vp * max(P, 1))(*[p.data_ptr() for p in partials])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().equarx_reduce_variant_hops(table, P, n, block, flags, _ptr(out_bf16), _ptr(workspace), ws_bytes,
                                             _stream()), "equarx_reduce_variant_hops")


def equarx_reduce_flat(local_bf16, codes_list, scales_list, block: int, out_bf16=None, codes_out=None,
                       scales_out=None) -> None:
    """Flat one-shot reduce of a local bf16 shard and R received (codes, scales) pairs."""
    n = local_bf16.numel()
    nb = num_blocks(n, block)
    R = len(codes_list)
    if len(scales_list) != R:
        raise ValueError("codes and scales lists differ in length")
    _need(local_bf16, torch.bfloat16, n, "local_bf16")
    for c, s in zip(codes_list, scales_list):
        _need(c, torch.int8, n, "codes")
        _need(s, torch.float32, nb, "scales")
    if out_bf16 is not None:
        _need(out_bf16, torch.bfloat16, n, "out_bf16")
    if codes_out is not None or scales_out is not None:
        _need(codes_out, torch.int8, n, "codes_out")
        _need(scales_out, torch.float32, nb, "scales_out")
    ctab = (_vp * max(R, 1))(*[c.data_ptr() for c in codes_list])
    stab = (_vp * max(R, 1))(*[s.data_ptr() for s in scales_list])
    _check(load().equarx_reduce_flat(_ptr(local_bf16), ctab, stab, R, n, block, _ptr(out_bf16), _ptr(codes_out),
                                     _ptr(scales_out), _stream()), "equarx_reduce_flat")


STRIDED_CHUNKS = (32, 64, 128)


def _strided_scales(n: int, chunks: int) -> int:
    return n // chunks if chunks in STRIDED_CHUNKS else 0


def equarx_quantize_strided(x_bf16, chunks: int, codes, scales) -> None:
    """Q with the strided block geometry: scale m*1024+j covers position j of every chunk of minishard m."""
    n = x_bf16.numel()
    _need(x_bf16, torch.bfloat16, n, "x_bf16")
    _need(codes, torch.int8, n, "codes")
    _need(scales, torch.float32, _strided_scales(n, chunks), "scales")
    _check(load().equarx_quantize_strided(_ptr(x_bf16), n, chunks, _ptr(codes), _ptr(scales), _stream()),
           "equarx_quantize_strided")


def equarx_dequantize_strided(codes, scales, chunks: int, out_bf16) -> None:
    n = codes.numel()
    _need(codes, torch.int8, n, "codes")
    _need(scales, torch.float32, _strided_scales(n, chunks), "scales")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    _check(load().equarx_dequantize_strided(_ptr(codes), _ptr(scales), n, chunks, _ptr(out_bf16), _stream()),
           "equarx_dequantize_strided")


def equarx_reduce_stage_strided(codes_in, scales_in, local_bf16, chunks: int, codes_out, scales_out) -> None:
    n = local_bf16.numel()
    ns = _strided_scales(n, chunks)
    _need(local_bf16, torch.bfloat16, n, "local_bf16")
    _need(codes_in, torch.int8, n, "codes_in")
    _need(codes_out, torch.int8, n, "codes_out")
    _need(scales_in, torch.float32, ns, "scales_in")
    _need(scales_out, torch.float32, ns, "scales_out")
    _check(load().equarx_reduce_stage_strided(_ptr(codes_in), _ptr(scales_in), _ptr(local_bf16), n, chunks,
                                              _ptr(codes_out), _ptr(scales_out), _stream()), "equarx_reduce_stage_strided")


def equarx_reduce_quantized_strided(partials, chunks: int, out_bf16, workspace) -> None:
    P = len(partials)
    n = partials[0].numel() if P else 0
    for p in partials:
        _need(p, torch.bfloat16, n, "partial")
        if p.numel() != n:
            raise ValueError("partials differ in length")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    if workspace is not None and not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace: need a contiguous CUDA tensor")
    table = (_vp * max(P, 1))(*[p.data_ptr() for p in partials])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().equarx_reduce_quantized_strided(table, P, n, chunks, _ptr(out_bf16), _ptr(workspace), ws_bytes,
                                                  _stream()), "equarx_reduce_quantized_strided")


def equarx_reduce_fused_strided(partials, chunks: int, out_bf16) -> None:
    """The strided chain in one launch (same bits as equarx_reduce_quantized_strided)."""
    P = len(partials)
    n = partials[0].numel() if P else 0
    for p in partials:
        _need(p, torch.bfloat16, n, "partial")
        if p.numel() != n:
            raise ValueError("partials differ in length")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    table = (_vp * max(P, 1))(*[p.data_ptr() for p in partials])
    _check(load().equarx_reduce_fused_strided(table, P, n, chunks, _ptr(out_bf16), _stream()),
           "equarx_reduce_fused_strided")


def equarx_reduce_variant_strided(partials, chunks: int, flags: int, out_bf16) -> None:
    """Semi-loop / stage-knob flavours of the chain in the strided geometry, one launch."""
    P = len(partials)
    n = partials[0].numel() if P else 0
    for p in partials:
        _need(p, torch.bfloat16, n, "partial")
        if p.numel() != n:
            raise ValueError("partials differ in length")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    table = (_vp * max(P, 1))(*[p.data_ptr() for p in partials])
    _check(load().equarx_reduce_variant_strided(table, P, n, chunks, flags, _ptr(out_bf16), _stream()),
           "equarx_reduce_variant_strided")


def equarx_reduce_variant_hops_strided(partials, chunks: int, flags: int, out_bf16, workspace) -> None:
    """Full loop or semi-loop, all-gather quantized or not, hop by hop in the strided geometry."""
    P = len(partials)
    n = partials[0].numel() if P else 0
    for p in partials:
        _need(p, torch.bfloat16, n, "partial")
        if p.numel() != n:
            raise ValueError("partials differ in length")
    _need(out_bf16, torch.bfloat16, n, "out_bf16")
    if not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous CUDA tensor")
    table = (_vp * max(P, 1))(*[p.data_ptr() for p in partials])
    _check(load().equarx_reduce_variant_hops_strided(table, P, n, chunks, flags, _ptr(out_bf16), _ptr(workspace),
                                                     workspace.numel() * workspace.element_size(), _stream()),
           "equarx_reduce_variant_hops_strided")


def equarx_calib_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
            and dst.numel() * dst.element_size() >= nbytes):
        raise ValueError("calib_copy: need contiguous CUDA tensors, dst at least as large as src")
    _check(load().equarx_calib_copy(_ptr(src), _ptr(dst), nbytes, _stream()), "equarx_calib_copy")


def equarx_calib_empty_launches(count: int, workgroups: int) -> None:
    """`count` back-to-back launches of a kernel that does nothing (`workgroups` workgroups each)."""
    _check(load().equarx_calib_empty_launches(count, workgroups, _stream()), "equarx_calib_empty_launches")


def equarx_calib_hop_traffic(partials, block: int, codes0, scales0, codes1, scales1) -> None:
    """The chain's P-1 hops as memory traffic only (XOR of what each launch read), ping-pong between two wires."""
    P = len(partials)
    n = partials[0].numel() if P else 0
    nb = num_blocks(n, block) if block in BLOCK_SIZES else 0
    for p in partials:
        _need(p, torch.bfloat16, n, "partial")
    for c, s in ((codes0, scales0), (codes1, scales1)):
        _need(c, torch.int8, n, "codes")
        _need(s, torch.float32, nb, "scales")
    table = (_vp * max(P, 1))(*[p.data_ptr() for p in partials])
    _check(load().equarx_calib_hop_traffic(table, P, n, block, _ptr(codes0), _ptr(scales0), _ptr(codes1),
                                           _ptr(scales1), _stream()), "equarx_calib_hop_traffic")


def equarx_calib_interleaved_chains(partial_sets, block: int, outs, workspaces, streaming: bool = False) -> None:
    """len(partial_sets) independent hop-by-hop chains, interleaved pass by pass (every wire read M-1 launches after
    it was written); chain m reduces partial_sets[m] into outs[m] using workspaces[m].  streaming: the wire is
    accessed with non-temporal hints, as the per-step entry points access it."""
    M = len(partial_sets)
    P = len(partial_sets[0]) if M else 0
    n = partial_sets[0][0].numel() if P else 0
    if len(outs) != M or len(workspaces) != M or any(len(ps) != P for ps in partial_sets):
        raise ValueError("one output, one workspace and P partials per chain")
    need = workspace_bytes(P, n, block) if P else 0
    for ps, o, w in zip(partial_sets, outs, workspaces):
        for p in ps:
            _need(p, torch.bfloat16, n, "partial")
            if p.numel() != n:
                raise ValueError("partials differ in length")
        _need(o, torch.bfloat16, n, "out_bf16")
        _need(w, torch.uint8, need, "workspace")
    flat = [p.data_ptr() for ps in partial_sets for p in ps]
    ptab = (_vp * max(len(flat), 1))(*flat)
    otab = (_vp * max(M, 1))(*[o.data_ptr() for o in outs])
    wtab = (_vp * max(M, 1))(*[w.data_ptr() for w in workspaces])
    _check(load().equarx_calib_interleaved_chains(ptab, M, P, n, block, otab, wtab, need, int(bool(streaming)), _stream()),
           "equarx_calib_interleaved_chains")


def equarx_time_launch_span(first: int, last: int, start_event, stop_event) -> None:
    """Raw hipEvent_t handles recorded before launch `first` and after launch `last` (from 0) of this thread's
    next call."""
    load().equarx_time_launch_span(first, last, start_event, stop_event)


def equarx_time_next_launch(start_event, stop_event) -> None:
    """start/stop: raw hipEvent_t handles (ints); the first launch of this thread's next call records its begin and
    end there."""
    load().equarx_time_next_launch(start_event, stop_event)


def equarx_time_cancel() -> None:
    load().equarx_time_cancel()


def equarx_selftest_quotients(first_bits: int, count: int, mismatches: torch.Tensor) -> None:
    """mismatches: CUDA int64[2], zeroed by the caller; receives the counts of differing scales / reciprocals."""
    _need(mismatches, torch.int64, 2, "mismatches")
    _check(load().equarx_selftest_quotients(first_bits, count, _ptr(mismatches), _stream()), "equarx_selftest_quotients")


def equarx_selftest_rounding(first_bits: int, count: int, mismatches: torch.Tensor) -> None:
    """mismatches: CUDA int64[1], zeroed by the caller; receives the number of |p| patterns whose codes differ."""
    _need(mismatches, torch.int64, 1, "mismatches")
    _check(load().equarx_selftest_rounding(first_bits, count, _ptr(mismatches), _stream()), "equarx_selftest_rounding")


def equarx_eval_quotients(absmax: torch.Tensor, scale: torch.Tensor, inv: torch.Tensor) -> None:
    n = absmax.numel()
    _need(absmax, torch.float32, n, "absmax")
    _need(scale, torch.float32, n, "scale")
    _need(inv, torch.float32, n, "inv")
    _check(load().equarx_eval_quotients(_ptr(absmax), n, _ptr(scale), _ptr(inv), _stream()), "equarx_eval_quotients")


def alloc_workspace(P: int, n: int, block: int, device="cuda") -> torch.Tensor:
    """Device buffer of the size the chain needs (torch is the allocator; the library never allocates)."""
    return torch.empty(max(workspace_bytes(P, n, block), 256), dtype=torch.uint8, device=device)
