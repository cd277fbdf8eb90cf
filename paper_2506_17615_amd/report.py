"""Speed and error of every flavour of the quantized reduction on one workload (python -m paper_2506_17615_amd.report).

The paper's Sec. 4.1 / Fig. 7 compares its flavours -- full-loop or semi-loop, reduce-scatter and/or all-gather
quantized -- by speedup and by mean squared error against the unquantized bf16 AllReduce, on a (4096, 4096)
N(0,1) tensor over 8 devices with block size 64.  This prints the same comparison for the entry points of this
library on one MI355X: time per reduction (all partials resident in HBM) and error against the exact sum.
"""
from __future__ import annotations

import argparse
import sys
import time

import torch

from . import binding as eq
from . import build
from . import workloads as wl

FIG7 = wl.FIG7


def _time_us(fn, sets, reps: int) -> float:
    """Wall clock per call, calls back to back, the resident input sets used in turn (as bench.py does)."""
    for k in range(5):
        fn(sets[k % len(sets)])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(reps):
        fn(sets[k % len(sets)])
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps * 1e6


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="fig7", help="fig7 or an id of workloads.WORKLOADS")
    ap.add_argument("--block", type=int, default=0, help="block size instead of the workload's own")
    ap.add_argument("--reps", type=int, default=50)
    args = ap.parse_args()
    build.ensure_built()
    eq.load()
    w = FIG7 if args.workload == "fig7" else wl.WORKLOADS[args.workload]
    if args.block:
        w = w.with_block(args.block)
    P, n, B = w.P, w.n, w.block
    parts = [p.reshape(-1).cuda() for p in wl.make_partials(w)]
    sets = [parts, [p.clone() for p in parts]]      # two sets, together larger than the 256 MB Infinity Cache
    ref = torch.zeros(n, dtype=torch.float64, device="cuda")
    for p in parts:
        ref += p.double()
    base = ref.float().to(torch.bfloat16).double()          # what an unquantized bf16 AllReduce returns
    out = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    work = eq.alloc_workspace(P, n, B)
    work3 = eq.alloc_variant_workspace(eq.SEMI_LOOP, P, n, B)
    work4 = eq.alloc_variant_workspace(eq.SEMI_LOOP | eq.RING_ORDER, P, n, B)
    nb = eq.num_blocks(n, B)
    qc = [torch.empty(n, dtype=torch.int8, device="cuda") for _ in range(P - 1)]
    qs = [torch.empty(nb, dtype=torch.float32, device="cuda") for _ in range(P - 1)]

    def flat(ps):
        eq.equarx_quantize_batch(ps[1:], B, qc, qs)
        eq.equarx_reduce_flat(ps[0], qc, qs, B, out)

    wire_c = torch.empty((P, eq.wire_row_codes(n)), dtype=torch.int8, device="cuda")
    wire_s = torch.empty((P, eq.wire_row_scales(n, B)), dtype=torch.float32, device="cuda")

    rows = [
        ("full-loop RS+AG, hop by hop (P+1 launches)", lambda ps: eq.equarx_reduce_quantized(ps, B, out, work)),
        ("full-loop RS+AG, hop by hop, ends fused (P-1 launches)",
         lambda ps: eq.equarx_reduce_quantized_fused_ends(ps, B, out, work)),
        ("full-loop RS+AG, one launch", lambda ps: eq.equarx_reduce_fused(ps, B, out)),
        ("full-loop RS+AG, one launch, every hop's wire written out",
         lambda ps: eq.equarx_reduce_fused(ps, B, out, wire_c, wire_s)),
        ("full-loop RS only", lambda ps: eq.equarx_reduce_variant(ps, B, eq.AG_UNQUANTIZED, out)),
        ("full-loop AG only", lambda ps: eq.equarx_reduce_variant(ps, B, eq.RS_UNQUANTIZED, out)),
        ("full-loop RS only, hop by hop (P launches)",
         lambda ps: eq.equarx_reduce_variant_hops(ps, B, eq.AG_UNQUANTIZED, out, work3)),
        ("semi-loop RS+AG, hop by hop (P launches)",
         lambda ps: eq.equarx_reduce_variant_hops(ps, B, eq.SEMI_LOOP, out, work3)),
        ("semi-loop RS only, hop by hop (P launches)",
         lambda ps: eq.equarx_reduce_variant_hops(ps, B, eq.SEMI_LOOP | eq.AG_UNQUANTIZED, out, work3)),
        ("semi-loop RS+AG", lambda ps: eq.equarx_reduce_variant(ps, B, eq.SEMI_LOOP, out)),
        ("semi-loop RS only", lambda ps: eq.equarx_reduce_variant(ps, B, eq.SEMI_LOOP | eq.AG_UNQUANTIZED, out)),
        ("full-loop RS+AG, ring order per shard", lambda ps: eq.equarx_reduce_variant(ps, B, eq.RING_ORDER, out)),
        ("full-loop RS+AG, ring order, hop by hop (P launches)",
         lambda ps: eq.equarx_reduce_variant_hops(ps, B, eq.RING_ORDER, out, work3)),
        ("semi-loop RS+AG, ring order per shard", lambda ps: eq.equarx_reduce_variant(ps, B, eq.SEMI_LOOP | eq.RING_ORDER, out)),
        ("semi-loop RS+AG, ring order, hop by hop (P/2+1 launches)",
         lambda ps: eq.equarx_reduce_variant_hops(ps, B, eq.SEMI_LOOP | eq.RING_ORDER, out, work4)),
        ("all-to-all: batched quantize + flat reduce", flat),
    ]
    if B in eq.STRIDED_CHUNKS and n % (1024 * B) == 0:
        rows.append(("full-loop RS+AG, strided 8x128-chunk blocks, hop by hop",
                     lambda ps: eq.equarx_reduce_quantized_strided(ps, B, out, work)))
        rows.append(("full-loop RS+AG, strided 8x128-chunk blocks, one launch",
                     lambda ps: eq.equarx_reduce_fused_strided(ps, B, out)))
        for label, flags in (("full-loop RS only", eq.AG_UNQUANTIZED), ("full-loop AG only", eq.RS_UNQUANTIZED),
                             ("semi-loop RS+AG", eq.SEMI_LOOP), ("semi-loop RS only", eq.SEMI_LOOP | eq.AG_UNQUANTIZED),
                             ("full-loop RS+AG, ring order", eq.RING_ORDER),
                             ("semi-loop RS+AG, ring order", eq.SEMI_LOOP | eq.RING_ORDER)):
            rows.append((label + ", strided 8x128-chunk blocks",
                         lambda ps, flags=flags: eq.equarx_reduce_variant_strided(ps, B, flags, out)))
            if not flags & eq.RS_UNQUANTIZED:
                ws = work3 if flags & eq.SEMI_LOOP else work
                rows.append((label + ", strided, hop by hop",
                             lambda ps, flags=flags, ws=ws: eq.equarx_reduce_variant_hops_strided(ps, B, flags, out, ws)))

    print(f"workload {w.name}: P={P}, n={n} ({w.rows} x {w.hidden}), block {B}, {w.dist}; MI355X, one GPU")
    print(f"{'flavour':58s} {'us':>8s} {'eff. input GB/s':>16s} {'MSE vs bf16 sum':>16s} {'rel-L2 vs exact':>16s}")
    with torch.cuda.stream(torch.cuda.Stream()):
        for name, fn in rows:
            us = _time_us(fn, sets, args.reps)
            fn(parts)
            torch.cuda.synchronize()
            got = out.double()
            mse = float(((got - base) ** 2).mean())
            rel = float((got - ref).norm() / ref.norm())
            print(f"{name:58s} {us:8.1f} {2.0 * P * n / us / 1e3:16.0f} {mse:16.3e} {rel:16.4f}", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
