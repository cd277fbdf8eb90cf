"""numpy front end of the CPU oracle -- TEST INFRASTRUCTURE ONLY.

Loads ``libequarx_oracle.so`` (built from ``equarx_oracle.c`` with gcc) and
exposes its functions on numpy arrays.  bf16 tensors travel as ``uint16``
arrays holding the raw bit patterns.  Nothing here touches the GPU or the HIP
library; only tests, the smoke check and the benchmark's cpu_baseline leg may
import this module.

The arithmetic lives in the C file; this module only marshals arguments.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "equarx_oracle.c")
_LIB = os.path.join(_HERE, "libequarx_oracle.so")

# Every rounding is written out in the source; the flags keep the compiler from
# changing any of them (no contraction into FMAs, no value-changing shortcuts).
_CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC", "-std=c11"]


def build(force: bool = False, src: str = _SRC, lib: str = _LIB, extra_flags=()) -> str:
    """Compile the C oracle with gcc.  Returns the path of the shared library."""
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(src):
        return lib
    cmd = ["gcc", *_CFLAGS, *extra_flags, src, "-o", lib, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


_c_i8p = ctypes.POINTER(ctypes.c_int8)
_c_u16p = ctypes.POINTER(ctypes.c_uint16)
_c_f32p = ctypes.POINTER(ctypes.c_float)
_c_f64p = ctypes.POINTER(ctypes.c_double)


def _declare(lib: ctypes.CDLL) -> ctypes.CDLL:
    i64, i32 = ctypes.c_int64, ctypes.c_int32
    pp = ctypes.POINTER(_c_u16p)
    lib.equarx_oracle_set_threads.argtypes = [ctypes.c_int]
    lib.equarx_oracle_set_threads.restype = None
    lib.equarx_oracle_get_threads.argtypes = []
    lib.equarx_oracle_get_threads.restype = ctypes.c_int
    lib.equarx_oracle_has_openmp.argtypes = []
    lib.equarx_oracle_has_openmp.restype = ctypes.c_int
    lib.equarx_oracle_bf16_to_f32.argtypes = [_c_u16p, i64, _c_f32p]
    lib.equarx_oracle_f32_to_bf16.argtypes = [_c_f32p, i64, _c_u16p]
    lib.equarx_oracle_quantize_f32.argtypes = [_c_f32p, i64, i32, _c_i8p, _c_f32p]
    lib.equarx_oracle_quantize_bf16.argtypes = [_c_u16p, i64, i32, _c_i8p, _c_f32p]
    lib.equarx_oracle_dequantize_f32.argtypes = [_c_i8p, _c_f32p, i64, i32, _c_f32p]
    lib.equarx_oracle_dequantize_bf16.argtypes = [_c_i8p, _c_f32p, i64, i32, _c_u16p]
    lib.equarx_oracle_hop.argtypes = [_c_i8p, _c_f32p, _c_u16p, i64, i32, _c_i8p, _c_f32p]
    lib.equarx_oracle_reduce_chain.argtypes = [pp, i32, i64, i32, _c_u16p, _c_i8p, _c_f32p]
    lib.equarx_oracle_exact_sum_f64.argtypes = [pp, i32, i64, _c_f64p]
    lib.equarx_oracle_sum_f32.argtypes = [pp, i32, i64, _c_f32p]
    lib.equarx_oracle_reduce_stages.argtypes = [pp, i32, i64, i32, ctypes.c_int, ctypes.c_int, _c_u16p]
    lib.equarx_oracle_reduce_semi_loop.argtypes = [pp, i32, i64, i32, ctypes.c_int, _c_u16p]
    lib.equarx_oracle_reduce_flat.argtypes = [_c_u16p, ctypes.POINTER(_c_i8p), ctypes.POINTER(_c_f32p), i32, i64, i32,
                                              _c_u16p, _c_i8p, _c_f32p]
    for name in ("bf16_to_f32", "f32_to_bf16", "quantize_f32", "quantize_bf16", "dequantize_f32",
                 "dequantize_bf16", "hop", "reduce_chain", "exact_sum_f64", "sum_f32", "reduce_stages",
                 "reduce_semi_loop", "reduce_flat"):
        getattr(lib, "equarx_oracle_" + name).restype = None
    return lib


def load(lib_path: str | None = None) -> ctypes.CDLL:
    """Load (building first if needed) the oracle library."""
    path = lib_path or build()
    return _declare(ctypes.CDLL(path))


_lib = None


def _L() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = load()
    return _lib


def _arr(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a.reshape(-1)


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctype)


def _check_block(B: int) -> int:
    B = int(B)
    if B < 1:
        raise ValueError("block size must be >= 1")
    return B


def num_blocks(n: int, B: int) -> int:
    return (int(n) + int(B) - 1) // int(B)


def set_threads(threads: int) -> None:
    _L().equarx_oracle_set_threads(int(threads))


def get_threads() -> int:
    return int(_L().equarx_oracle_get_threads())


def bf16_to_f32(x_u16) -> np.ndarray:
    x = _arr(x_u16, np.uint16)
    out = np.empty(x.size, np.float32)
    _L().equarx_oracle_bf16_to_f32(_ptr(x, _c_u16p), x.size, _ptr(out, _c_f32p))
    return out


def f32_to_bf16(v) -> np.ndarray:
    v = _arr(v, np.float32)
    out = np.empty(v.size, np.uint16)
    _L().equarx_oracle_f32_to_bf16(_ptr(v, _c_f32p), v.size, _ptr(out, _c_u16p))
    return out


def quantize_f32(v, B: int, lib=None):
    """Q_B of an fp32 tensor -> (codes int8 [n], scales fp32 [ceil(n/B)])."""
    B = _check_block(B)
    v = _arr(v, np.float32)
    codes = np.empty(v.size, np.int8)
    scales = np.empty(num_blocks(v.size, B), np.float32)
    (lib or _L()).equarx_oracle_quantize_f32(_ptr(v, _c_f32p), v.size, B, _ptr(codes, _c_i8p), _ptr(scales, _c_f32p))
    return codes, scales


def quantize_bf16(x_u16, B: int, lib=None):
    """Q_B of a bf16 tensor (uint16 bit patterns) -> (codes, scales)."""
    B = _check_block(B)
    x = _arr(x_u16, np.uint16)
    codes = np.empty(x.size, np.int8)
    scales = np.empty(num_blocks(x.size, B), np.float32)
    (lib or _L()).equarx_oracle_quantize_bf16(_ptr(x, _c_u16p), x.size, B, _ptr(codes, _c_i8p), _ptr(scales, _c_f32p))
    return codes, scales


def dequantize_f32(codes, scales, B: int, lib=None) -> np.ndarray:
    B = _check_block(B)
    c = _arr(codes, np.int8)
    s = _arr(scales, np.float32)
    assert s.size == num_blocks(c.size, B)
    out = np.empty(c.size, np.float32)
    (lib or _L()).equarx_oracle_dequantize_f32(_ptr(c, _c_i8p), _ptr(s, _c_f32p), c.size, B, _ptr(out, _c_f32p))
    return out


def dequantize_bf16(codes, scales, B: int, lib=None) -> np.ndarray:
    B = _check_block(B)
    c = _arr(codes, np.int8)
    s = _arr(scales, np.float32)
    assert s.size == num_blocks(c.size, B)
    out = np.empty(c.size, np.uint16)
    (lib or _L()).equarx_oracle_dequantize_bf16(_ptr(c, _c_i8p), _ptr(s, _c_f32p), c.size, B, _ptr(out, _c_u16p))
    return out


def hop(codes_in, scales_in, local_u16, B: int, lib=None):
    """One receive step: dequantize, add the local bf16 shard in fp32, requantize."""
    B = _check_block(B)
    c = _arr(codes_in, np.int8)
    s = _arr(scales_in, np.float32)
    x = _arr(local_u16, np.uint16)
    assert x.size == c.size and s.size == num_blocks(c.size, B)
    codes = np.empty(c.size, np.int8)
    scales = np.empty(s.size, np.float32)
    (lib or _L()).equarx_oracle_hop(_ptr(c, _c_i8p), _ptr(s, _c_f32p), _ptr(x, _c_u16p), c.size, B,
                                    _ptr(codes, _c_i8p), _ptr(scales, _c_f32p))
    return codes, scales


def _pointer_table(partials):
    arrs = [_arr(p, np.uint16) for p in partials]
    if not arrs:
        raise ValueError("need at least one partial")
    n = arrs[0].size
    if any(a.size != n for a in arrs):
        raise ValueError("partials differ in length")
    table = (_c_u16p * len(arrs))(*[_ptr(a, _c_u16p) for a in arrs])
    return arrs, table, n


def reduce_chain(partials, B: int, keep_wire: bool = False, lib=None):
    """The full-loop adder chain with reduce-scatter and all-gather both quantized.

    partials: sequence of P bf16 tensors (uint16), in chain order.
    Returns out (uint16 [n]); with keep_wire also (wire_codes [P, n], wire_scales [P, nb]).
    """
    B = _check_block(B)
    arrs, table, n = _pointer_table(partials)
    P = len(arrs)
    nb = num_blocks(n, B)
    out = np.empty(n, np.uint16)
    if keep_wire:
        wc = np.empty((P, n), np.int8)
        ws = np.empty((P, nb), np.float32)
        wcp, wsp = _ptr(wc, _c_i8p), _ptr(ws, _c_f32p)
    else:
        wc = ws = None
        wcp, wsp = None, None
    (lib or _L()).equarx_oracle_reduce_chain(table, P, n, B, _ptr(out, _c_u16p), wcp, wsp)
    if keep_wire:
        return out, wc, ws
    return out


def exact_sum_f64(partials, lib=None) -> np.ndarray:
    arrs, table, n = _pointer_table(partials)
    ref = np.empty(n, np.float64)
    (lib or _L()).equarx_oracle_exact_sum_f64(table, len(arrs), n, _ptr(ref, _c_f64p))
    return ref


def sum_f32(partials, lib=None) -> np.ndarray:
    arrs, table, n = _pointer_table(partials)
    ref = np.empty(n, np.float32)
    (lib or _L()).equarx_oracle_sum_f32(table, len(arrs), n, _ptr(ref, _c_f32p))
    return ref


def reduce_stages(partials, B: int, quantize_rs: bool = True, quantize_ag: bool = True, lib=None) -> np.ndarray:
    """Full-loop chain with the stage knob: which of reduce-scatter / all-gather is quantized."""
    B = _check_block(B)
    arrs, table, n = _pointer_table(partials)
    out = np.empty(n, np.uint16)
    (lib or _L()).equarx_oracle_reduce_stages(table, len(arrs), n, B, int(bool(quantize_rs)), int(bool(quantize_ag)),
                                              _ptr(out, _c_u16p))
    return out


def reduce_semi_loop(partials, B: int, quantize_ag: bool = True, lib=None) -> np.ndarray:
    """Semi-loop chain: partials[0] is the owner, the others follow in ring order around it."""
    B = _check_block(B)
    arrs, table, n = _pointer_table(partials)
    out = np.empty(n, np.uint16)
    (lib or _L()).equarx_oracle_reduce_semi_loop(table, len(arrs), n, B, int(bool(quantize_ag)), _ptr(out, _c_u16p))
    return out


def reduce_flat(local_u16, codes_list, scales_list, B: int, lib=None):
    """Flat one-shot reduce of a local bf16 shard and R received (codes, scales) pairs.

    Returns (out bf16 [n], codes_out [n], scales_out [nb])."""
    B = _check_block(B)
    x = _arr(local_u16, np.uint16)
    n = x.size
    nb = num_blocks(n, B)
    cs = [_arr(c, np.int8) for c in codes_list]
    ss = [_arr(s, np.float32) for s in scales_list]
    assert len(cs) == len(ss) and all(c.size == n for c in cs) and all(s.size == nb for s in ss)
    R = len(cs)
    ctab = (_c_i8p * max(R, 1))(*[_ptr(c, _c_i8p) for c in cs])
    stab = (_c_f32p * max(R, 1))(*[_ptr(s, _c_f32p) for s in ss])
    out = np.empty(n, np.uint16)
    co = np.empty(n, np.int8)
    so = np.empty(nb, np.float32)
    (lib or _L()).equarx_oracle_reduce_flat(_ptr(x, _c_u16p), ctab, stab, R, n, B, _ptr(out, _c_u16p),
                                            _ptr(co, _c_i8p), _ptr(so, _c_f32p))
    return out, co, so


def ring_order(P: int, shard: int):
    """Order in which a ring reduce-scatter visits the devices for the shard that ends on device `shard`
    (Sec. 3): the chain starts at the next device and walks once around the ring.  The direction is a
    convention; the paper's figure is what would fix it."""
    return [(shard + 1 + i) % P for i in range(P)]


def shard_bounds(n: int, B: int, P: int):
    """Split [0, n) into P shards on block boundaries: ceil(nb/P) blocks each, the last ones possibly short or empty."""
    nb = num_blocks(n, B)
    per = (nb + P - 1) // P
    return [(min(n, k * per * B), min(n, (k + 1) * per * B)) for k in range(P)]


def reduce_ring(partials, B: int, semi: bool = False, quantize_rs: bool = True, quantize_ag: bool = True,
                lib=None) -> np.ndarray:
    """The reduction as a real ring lays it out: shard k ends on device k.

    Full loop: shard k is reduced in the rotated order ring_order(P, k).  Semi-loop: device k is the owner
    and the devices k+1, k+2, ... follow in ring order around it."""
    arrs = [_arr(p, np.uint16) for p in partials]
    P, n = len(arrs), arrs[0].size
    out = np.empty(n, np.uint16)
    for k, (lo, hi) in enumerate(shard_bounds(n, B, P)):
        if hi <= lo:
            continue
        if semi:
            order = [(k + j) % P for j in range(P)]
            out[lo:hi] = reduce_semi_loop([arrs[d][lo:hi] for d in order], B, quantize_ag, lib=lib)
        else:
            out[lo:hi] = reduce_stages([arrs[d][lo:hi] for d in ring_order(P, k)], B, quantize_rs, quantize_ag, lib=lib)
    return out


# ---------------------------------------------------------------------------------------------------------
# The paper's own block geometry (Sec. 3.2, "VPU-friendly"): a minishard of `chunks` consecutive chunks of
# CHUNK = 8 x 128 = 1024 elements gets 1024 scales; scale j covers the elements at position j of every chunk,
# i.e. a block of `chunks` entries 1024 apart.  Transposing each minishard from [chunks, 1024] to
# [1024, chunks] turns those strided blocks into contiguous blocks of B = chunks, so every strided function
# below IS the contiguous one applied between that transposition and its inverse; scale number
# minishard * 1024 + j is then simply block number minishard * 1024 + j of the transposed tensor.

CHUNK = 1024


def _check_strided(n: int, chunks: int) -> None:
    if chunks < 1 or n % (CHUNK * chunks) != 0:
        raise ValueError("strided layout needs n to be a multiple of 1024 * chunks")


def to_block_major(a, chunks: int) -> np.ndarray:
    """[minishards, chunks, 1024] -> [minishards, 1024, chunks], flattened."""
    a = np.asarray(a).reshape(-1)
    _check_strided(a.size, chunks)
    return np.ascontiguousarray(a.reshape(-1, chunks, CHUNK).transpose(0, 2, 1)).reshape(-1)


def from_block_major(a, chunks: int) -> np.ndarray:
    a = np.asarray(a).reshape(-1)
    _check_strided(a.size, chunks)
    return np.ascontiguousarray(a.reshape(-1, CHUNK, chunks).transpose(0, 2, 1)).reshape(-1)


def quantize_bf16_strided(x_u16, chunks: int, lib=None):
    c, s = quantize_bf16(to_block_major(_arr(x_u16, np.uint16), chunks), chunks, lib=lib)
    return from_block_major(c, chunks), s


def dequantize_bf16_strided(codes, scales, chunks: int, lib=None) -> np.ndarray:
    out = dequantize_bf16(to_block_major(_arr(codes, np.int8), chunks), scales, chunks, lib=lib)
    return from_block_major(out, chunks)


def hop_strided(codes_in, scales_in, local_u16, chunks: int, lib=None):
    c, s = hop(to_block_major(_arr(codes_in, np.int8), chunks), scales_in,
               to_block_major(_arr(local_u16, np.uint16), chunks), chunks, lib=lib)
    return from_block_major(c, chunks), s


def reduce_chain_strided(partials, chunks: int, keep_wire: bool = False, lib=None):
    """The full-loop chain (RS and AG quantized) with the strided block geometry."""
    moved = [to_block_major(_arr(p, np.uint16), chunks) for p in partials]
    if keep_wire:
        out, wc, ws = reduce_chain(moved, chunks, keep_wire=True, lib=lib)
        wc = np.stack([from_block_major(row, chunks) for row in wc])
        return from_block_major(out, chunks), wc, ws
    return from_block_major(reduce_chain(moved, chunks, lib=lib), chunks)


def reduce_stages_strided(partials, chunks: int, quantize_rs: bool = True, quantize_ag: bool = True, lib=None) -> np.ndarray:
    """The full-loop chain with the stage knob (Sec. 3.4) in the strided block geometry (Sec. 3.2)."""
    moved = [to_block_major(_arr(p, np.uint16), chunks) for p in partials]
    return from_block_major(reduce_stages(moved, chunks, quantize_rs, quantize_ag, lib=lib), chunks)


def reduce_semi_loop_strided(partials, chunks: int, quantize_ag: bool = True, lib=None) -> np.ndarray:
    """The semi-loop chain (Sec. 3.3; partials[0] owns the result) in the strided block geometry (Sec. 3.2)."""
    moved = [to_block_major(_arr(p, np.uint16), chunks) for p in partials]
    return from_block_major(reduce_semi_loop(moved, chunks, quantize_ag, lib=lib), chunks)


def reduce_ring_strided(partials, chunks: int, semi: bool = False, quantize_rs: bool = True, quantize_ag: bool = True,
                        lib=None) -> np.ndarray:
    """The ring layout (Sec. 3) with the blocks of Sec. 3.2: a device's shard is cut into minishards, so shards
    are whole minishards here -- ceil(M/P) of the M minishards each, the last ones possibly short or empty --
    and shard k ends on device k: reduced in the order ring_order(P, k), or with device k as the semi-loop's
    owner and the devices k+1, k+2, ... around it."""
    arrs = [_arr(p, np.uint16) for p in partials]
    P, n = len(arrs), arrs[0].size
    _check_strided(n, chunks)
    out = np.empty(n, np.uint16)
    for k, (lo, hi) in enumerate(shard_bounds(n, CHUNK * chunks, P)):
        if hi <= lo:
            continue
        if not semi:
            shard = [arrs[d][lo:hi] for d in ring_order(P, k)]
            out[lo:hi] = reduce_stages_strided(shard, chunks, quantize_rs, quantize_ag, lib=lib)
        else:
            around = [arrs[(k + step) % P][lo:hi] for step in range(P)]
            out[lo:hi] = reduce_semi_loop_strided(around, chunks, quantize_ag, lib=lib)
    return out
