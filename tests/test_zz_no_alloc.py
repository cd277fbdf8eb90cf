"""The entry point that allocates nothing (equarx_reduce_quantized_static), through the C ABI, against the entry
point it is a variant of (equarx_reduce_quantized with a caller-owned workspace) and against the CPU oracle:
bit-exact, on two calls in a row, the second with a smaller input that leaves most of the static array holding
the first call's wire."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2506_17615_amd import binding as eq


def _partials(seed, P, n):
    rng = np.random.default_rng(seed)
    vals = [(rng.standard_normal(n) * np.exp(rng.standard_normal(n))).astype(np.float32) for _ in range(P)]
    return [torch.from_numpy(v).to(torch.bfloat16).cuda() for v in vals]


def _u16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.gpu
def test_static_workspace_matches_caller_workspace(oracle):
    assert torch.cuda.is_available()
    from paper_2506_17615_amd import build
    build.ensure_built()
    lib = eq.load()
    calls = ((8, 2048 * 3 * 37 + 2048 + 300, 64, 11),      # many workgroups, a ragged last tile and block
             (5, 2048 + 24, 256, 12))                      # much smaller, other block size, odd chain length
    for P, n, B, seed in calls:
        parts = _partials(seed, P, n)
        want = torch.full((n,), 7.0, dtype=torch.bfloat16, device="cuda")
        eq.equarx_reduce_quantized(parts, B, want, eq.alloc_workspace(P, n, B))
        got = torch.full((n,), -3.0, dtype=torch.bfloat16, device="cuda")
        table = (ctypes.c_void_p * P)(*[p.data_ptr() for p in parts])
        status = lib.equarx_reduce_quantized_static(table, P, n, B, got.data_ptr(),
                                                    torch.cuda.current_stream().cuda_stream)
        assert status == eq.STATUS_OK, eq.status_string(status)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (P, n, B)
        assert (_u16(got) == oracle.reduce_chain([_u16(p) for p in parts], B)).all(), (P, n, B)
    # in place, as an AllReduce is usually called, and once more on the first size: the array's stale content
    # (the smaller call's wire at its start, the larger call's beyond) changes nothing
    P, n, B, seed = calls[0]
    parts = _partials(seed, P, n)
    want = oracle.reduce_chain([_u16(p) for p in parts], B)
    eq.equarx_reduce_quantized_static(parts, B, parts[3])
    torch.cuda.synchronize()
    assert (_u16(parts[3]) == want).all()


@pytest.mark.gpu
def test_static_workspace_under_graph_capture(oracle):
    """What the entry point is for: captured in a HIP graph (after one eager call has looked the array's address up),
    replayed several times on changing inputs with eager calls in between; every replay equals the eager result."""
    assert torch.cuda.is_available()
    P, n, B = 6, 2048 * 3 * 9 + 1000, 128
    parts = [torch.zeros(n, dtype=torch.bfloat16, device="cuda") for _ in range(P)]
    out = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    eager = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    eq.equarx_reduce_quantized_static(parts, B, out)           # outside capture: resolves the static array's address
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        eq.equarx_reduce_quantized_static(parts, B, out)
    for rep in range(4):
        fresh = _partials(40 + rep, P, n)
        for d, f in zip(parts, fresh):
            d.copy_(f)
        eq.equarx_reduce_quantized(parts, B, eager, eq.alloc_workspace(P, n, B))      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), rep
        assert (_u16(out) == oracle.reduce_chain([_u16(p) for p in parts], B)).all(), rep
        if rep == 1:        # an eager call of another size on the same array between two replays
            small = _partials(77, 3, 4096)
            o2 = torch.zeros(4096, dtype=torch.bfloat16, device="cuda")
            eq.equarx_reduce_quantized_static(small, 256, o2)
            torch.cuda.synchronize()
            assert (_u16(o2) == oracle.reduce_chain([_u16(p) for p in small], 256)).all()


def test_static_workspace_limit_is_enforced():
    """Sizes whose wire buffers do not fit the static array are rejected on the host, before any launch."""
    lib = eq.load()
    A = 0x7F0000001000
    table = (ctypes.c_void_p * 2)(A, A + (1 << 32))
    n_fit = (eq.STATIC_WORKSPACE_BYTES // 2) * 32 // 36 // 256 * 256      # 2 * (n + 4n/32) <= limit
    assert eq.workspace_bytes(2, n_fit, 32) <= eq.STATIC_WORKSPACE_BYTES
    n_big = n_fit + (1 << 20)
    assert eq.workspace_bytes(2, n_big, 32) > eq.STATIC_WORKSPACE_BYTES
    # every configuration of the benchmark list fits, the 64 MiB message at block 32 included
    for n, B in ((4096, 256), (2048 * 3840, 256), (4096 * 5376, 256), (64 * 5376, 128), (33_554_432, 32), (33_554_432, 512)):
        assert 0 < eq.workspace_bytes(8, n, B) <= eq.STATIC_WORKSPACE_BYTES
    assert lib.equarx_reduce_quantized_static(table, 2, n_big, 32, A + (1 << 33), None) == eq.STATUS_WORKSPACE_TOO_SMALL
    assert lib.equarx_reduce_quantized_static(table, 2, 1 << 30, 512, A + (1 << 33), None) == eq.STATUS_WORKSPACE_TOO_SMALL
    assert lib.equarx_reduce_quantized_static(table, 2, 4096, 256, None, None) == eq.STATUS_NULL_POINTER
    assert lib.equarx_reduce_quantized_static(table, 2, 4096, 256, A + 16, None) == eq.STATUS_BAD_SHAPE   # overlaps partial 0
    assert lib.equarx_reduce_quantized_static(table, 2, 0, 256, None, None) == eq.STATUS_OK
