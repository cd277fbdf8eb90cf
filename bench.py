#!/usr/bin/env python3
"""Benchmark of the quantized P-way reduction on one MI355X.

A step is one pass of the whole hot path -- quantize, P-1 fused dequantize-add-requantize hops, final
dequantize (equarx_reduce_quantized) -- over one batch of synthetic partial sums already resident in HBM.
Prints ONE JSON line:

  value      effective input GB/s (bf16 bytes reduced per second): 2*P*n / (mean wall-clock time of a step over
             the K timed steps, between two device synchronisations).  Inputs are COLD (two resident input sets
             used in turn, more than the 256 MB Infinity Cache); the wire is WARM (each hop reads what the launch
             before it wrote, which that cache still holds).
  roofline   the dominant kernel (the hop), its duration measured with HIP events recorded on the stream around
             runs of hops inside the real call.  `achieved`/`frac` are the warm-wire figures of the timed chain;
             `cold_wire` holds the same kernel's figures when every wire it reads was written several launches
             earlier (independent chains interleaved pass by pass), which is what a wire arriving from another
             device looks like.
  chain, other_schedules   every schedule with its own byte count, wall-clock figures and kernel figures kept apart.
  cpu_baseline   the CPU oracle timed on the host as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0            # MI355X HBM3E, published peak
INFINITY_CACHE_BYTES = 256 << 20
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hop_kernel_c3_traffic.txt")


def hop_bytes(n: int, block: int) -> float:
    """Algorithmic bytes of one hop launch: bf16 shard in, codes+scales in, codes+scales out."""
    return n * (2.0 + 2.0 * (1.0 + 4.0 / block))


def chain_bytes(P: int, n: int, block: int) -> float:
    """Algorithmic bytes of the hop-by-hop schedule: every wire buffer written once and read once."""
    return n * (2.0 * P + 2.0 * P * (1.0 + 4.0 / block) + 2.0)


def fused_bytes(P: int, n: int) -> float:
    """Algorithmic bytes of the single-launch chain: every partial read once, the output written once."""
    return n * (2.0 * P + 2.0)


def ends_bytes(P: int, n: int, block: int) -> float:
    """Hop by hop with both ends fused: P-2 wire buffers written once and read once."""
    return fused_bytes(P, n) + 2.0 * max(P - 2, 0) * n * (1.0 + 4.0 / block)


def input_sets(P: int, n: int) -> int:
    """Resident copies of the inputs to rotate over: enough that together they are at least twice the Infinity
    Cache, so that a set has left it when its turn comes again; between 2 and 64."""
    return int(min(64, max(2, -(-2 * INFINITY_CACHE_BYTES // (2 * P * n)))))


def wire_bytes(n: int, block: int) -> float:
    """Bytes of one wire buffer: int8 codes and fp32 scales."""
    return n * (1.0 + 4.0 / block)


def cold_chains(n: int, block: int) -> int:
    """Independent chains to interleave so that a wire is cold when it is read: between its write and its read
    the other chains write M-1 wires of their own, and those ALONE exceed the 256 MB Infinity Cache by a quarter
    (counting only wire writes makes the arrangement safe whatever that cache does with the streamed bf16 inputs).
    0 if that takes more than 64 chains (small messages: nothing about them is ever cold; no figure is reported)."""
    m = int(-(-1.25 * INFINITY_CACHE_BYTES // wire_bytes(n, block))) + 1
    return m if m <= 64 else 0


def cold_flat_pipelines(P: int, n: int, block: int) -> int:
    """Independent all-to-all pipelines to interleave (all batched quantizes, then all flat reduces) so that the
    P-1 wires of one are cold when its reduce reads them: the other pipelines' wire writes in between exceed the
    Infinity Cache by a quarter.  0 if that takes more than 16 pipelines."""
    m = int(-(-1.25 * INFINITY_CACHE_BYTES // ((P - 1) * wire_bytes(n, block)))) + 1
    return m if m <= 16 else 0


def read_traffic(library_digest: str):
    """Bytes per hop launch between L2 and the memory fabric, from the committed rocprofv3 counter summary, if that
    summary was made with the library as it is built now; else None.  A profile, not a live measurement."""
    try:
        vals = {}
        with open(TRAFFIC_FILE) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 2 and parts[0] in ("hbm_bytes_per_launch", "l2_fabric_bytes_per_launch"):
                    vals["bytes"] = float(parts[1])
                if len(parts) >= 2 and parts[0] == "library_digest":
                    vals["digest"] = parts[1]
        if "bytes" not in vals:
            return None
        if vals.get("digest") != library_digest:
            return None
        return vals["bytes"]
    except OSError:
        return None


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, host_u16, budget_s: float):
    """The oracle as it stands, timed on this machine's host cores on the same workload: on as many threads as the box
    grants (its OMP_NUM_THREADS share, else every CPU it shows), then on one."""
    import numpy as np

    from oracle import equarx_oracle as orc
    orc.build()
    shown = os.cpu_count() or 1
    granted = int(os.environ.get("OMP_NUM_THREADS", "0") or 0)
    threads = max(1, min(shown, granted)) if granted > 0 else shown

    def timed(nthreads, budget, most):
        orc.set_threads(nthreads)
        times = []
        t_end = time.perf_counter() + budget
        while len(times) < most and (not times or time.perf_counter() + times[-1] < t_end):
            t0 = time.perf_counter()
            out = orc.reduce_chain(host_u16, w.block)
            times.append(time.perf_counter() - t0)
        return statistics.median(times), len(times), out

    best, reps, out = timed(threads, 0.7 * budget_s, 10)
    used = orc.get_threads()
    one, reps1, _ = timed(1, 0.3 * budget_s, 3)
    orc.set_threads(1)
    ref = orc.exact_sum_f64(host_u16)
    got = orc.bf16_to_f32(out).astype(np.float64)
    rel = float(np.linalg.norm(got - ref) / np.linalg.norm(ref))
    return {
        "value": round(2.0 * w.P * w.n / best / 1e9, 4),
        "unit": "GB/s effective input",
        "cores": used,
        "kind": "oracle",
        "sample": f"whole workload ({w.P} x {w.n} bf16), median of {reps} full chains, {best * 1e3:.0f} ms each",
        "cpu_model": cpu_model(),
        "host_cpus_shown": shown,
        "threads_granted_by_OMP_NUM_THREADS": granted or None,
        "single_thread_value": round(2.0 * w.P * w.n / one / 1e9, 4),
        "single_thread_sample": f"median of {reps1} full chains, {one * 1e3:.0f} ms each",
        "rel_l2_vs_exact_sum": rel,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c3_gemma3_27b")
    ap.add_argument("--block", type=int, default=0, help="override the workload's block size")
    ap.add_argument("--rows", type=int, default=0,
                    help="override the workload's row count (e.g. rows/8: the share of one GPU of an 8-GPU node)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the oracle timing; 0 skips it")
    ap.add_argument("--schedule", choices=("hop", "ends", "fused"), default="hop",
                    help="which schedule `value` reports.  hop: P+1 launches, the wire written and read back (default, "
                         "the schedule a ring imposes); ends: the same with the first two and the last two passes "
                         "sharing a launch; fused: the chain in one launch")
    ap.add_argument("--only", choices=("all", "chain", "cold"), default="all",
                    help="chain: run nothing but the timed steps of --schedule (for a clean kernel trace); "
                         "cold: nothing but the interleaved cold-wire chains")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all P partials live in one MI355X's HBM); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch

    from paper_2506_17615_amd import binding as eq
    from paper_2506_17615_amd import build as hip_build
    from paper_2506_17615_amd import workloads as wl

    hip_build.ensure_built()
    eq.load()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    w = wl.WORKLOADS[args.workload]
    if args.block:
        w = w.with_block(args.block)
    if args.rows:
        w = w.with_rows(args.rows)
    K, W = args.steps, args.warmup
    P, n, B = w.P, w.n, w.block
    everything = args.only == "all"

    host = wl.make_partials(w)
    # resident input sets, used in turn, so that no step finds its inputs in the 256 MB Infinity Cache: as many as it
    # takes for the sets together to be twice that cache (two for the 27B shape, five for the 12B shape), at most 64
    S = input_sets(P, n)
    sets = [[p.reshape(-1).cuda() for p in host]]
    for _ in range(S - 1):
        sets.append([p.clone() for p in sets[0]])
    out = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    work = eq.alloc_workspace(P, n, B)
    nb = eq.num_blocks(n, B)

    def gbps(nbytes, ms):
        return nbytes / (ms * 1e-3) / 1e9

    def frac(nbytes, ms):
        return round(gbps(nbytes, ms) / HBM_PEAK_GBPS, 4)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):

        def timed_steps(call):
            """W untimed calls, then exactly K between two synchronisations: mean wall-clock ms per step."""
            for k in range(W):
                call(k)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k in range(K):
                call(k)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / K

        def event_pairs(count):
            made = []
            for _ in range(count):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                b.record(stream)          # creates the underlying hipEvent_t handles
                made.append((a, b))
            torch.cuda.synchronize()
            return made

        def per_launch_ms(call, first, count, group=1, reps=None):
            """Mean duration of one of `count * group` consecutive launches (from launch `first`) of call(k).  Spans of
            two lengths are timed on alternate calls and subtracted, which cancels what the two event records cost."""
            reps = reps or K
            short = count // 2 if count >= 3 and reps >= 4 else 0
            for k in range(min(W, 10)):     # untimed: first touches of fresh buffers, clocks
                call(k)
            pairs = event_pairs(reps)
            for k, (a, b) in enumerate(pairs):
                length = short if (short and k % 2) else count
                eq.equarx_time_launch_span(first, first + length * group - 1, a.cuda_event, b.cuda_event)
                call(k)
            torch.cuda.synchronize()
            times = [a.elapsed_time(b) for a, b in pairs]
            if not short:
                return statistics.fmean(times) / (count * group), len(times) * count * group
            long_ms, short_ms = statistics.fmean(times[0::2]), statistics.fmean(times[1::2])
            return ((long_ms - short_ms) / ((count - short) * group),
                    (len(times[0::2]) * count + len(times[1::2]) * short) * group)

        def single_kernel_ms(call, reps):
            """Mean duration of the one kernel call(k) launches, from an event pair the launch itself carries."""
            pairs = event_pairs(reps)
            for k, (a, b) in enumerate(pairs):
                eq.equarx_time_next_launch(a.cuda_event, b.cuda_event)
                call(k)
            torch.cuda.synchronize()
            return statistics.fmean(a.elapsed_time(b) for a, b in pairs)

        calls = {
            "hop": lambda k: eq.equarx_reduce_quantized(sets[k % S], B, out, work),
            "ends": lambda k: eq.equarx_reduce_quantized_fused_ends(sets[k % S], B, out, work),
            "fused": lambda k: eq.equarx_reduce_fused(sets[k % S], B, out),
        }
        descriptions = {
            "hop": "hop-by-hop, P+1 launches, wire written once and read once",
            "ends": "hop-by-hop with both ends fused: max(P-1, 1) launches, P-2 wire buffers written once and read once",
            "fused": "single launch, chain in registers, no wire traffic",
        }
        own_bytes = {"hop": chain_bytes(P, n, B), "ends": ends_bytes(P, n, B), "fused": fused_bytes(P, n)}

        infos = {}
        results = {}
        wanted = list(calls) if everything else ([args.schedule] if args.only == "chain" else [])
        for name in wanted:
            calls[name](0)      # not a step: the first call of a process loads the code object (tens of ms), also with --warmup 0
            torch.cuda.synchronize()
            ms = timed_steps(calls[name])
            results[name] = out.clone()
            infos[name] = {
                "schedule": descriptions[name],
                "ms_per_step": round(ms, 5),
                "effective_input_GBps": round(gbps(2.0 * P * n, ms), 1),
                "algorithmic_bytes": own_bytes[name],
                "frac_of_hbm_peak": frac(own_bytes[name], ms),
                "inputs": f"cold ({S} input sets in turn)",
                "wire": "none" if name == "fused" else "warm (read by the launch after the one that wrote it)",
            }
        if everything:
            # the same launches replayed from HIP graphs (one captured call per input set, at most 8): what a caller
            # with a fixed set of buffers saves in launch cost; the entry points enqueue kernels only, so they capture
            for name in wanted:
                if name == "fused":
                    continue
                graphs = []
                for k in range(min(S, 8)):
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=stream):
                        calls[name](k)
                    graphs.append(g)
                gms = timed_steps(lambda k: graphs[k % len(graphs)].replay())
                infos[name]["graph_replay"] = {
                    "ms_per_step": round(gms, 5),
                    "frac_of_hbm_peak": frac(own_bytes[name], gms),
                    "graphs": len(graphs),
                    "same_bits": bool(torch.equal(out.view(torch.int16), results[name].view(torch.int16)))
                    if (K - 1) % len(graphs) == (K - 1) % S else None,
                }
                del graphs
        if "hop" in infos:
            # spread of single steps: the same K steps once more, each between two events on the stream (the records
            # themselves cost a microsecond or two per step, so the median sits slightly above ms_per_step)
            marks = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
            marks[0].record(stream)
            for k in range(K):
                calls["hop"](k)
                marks[k + 1].record(stream)
            torch.cuda.synchronize()
            step_us = sorted(marks[k].elapsed_time(marks[k + 1]) * 1e3 for k in range(K))
            infos["hop"]["single_step_us"] = {"p10": round(step_us[int(0.1 * (K - 1))], 2),
                                              "median": round(step_us[(K - 1) // 2], 2),
                                              "p90": round(step_us[int(0.9 * (K - 1))], 2)}
        if "fused" in infos and everything:
            kms = single_kernel_ms(calls["fused"], min(K, 50))
            infos["fused"]["kernel_avg_launch_us"] = round(kms * 1e3, 3)
            infos["fused"]["kernel_frac_of_hbm_peak"] = frac(fused_bytes(P, n), kms)

        # all-to-all form: every non-owner quantizes its shard once, the owner reduces all of them in one kernel
        flat_info = None
        if P > 1 and everything:
            qc = [torch.empty(n, dtype=torch.int8, device="cuda") for _ in range(P - 1)]
            qs = [torch.empty(nb, dtype=torch.float32, device="cuda") for _ in range(P - 1)]

            def flat_pipeline(k):
                eq.equarx_quantize_batch(sets[k % S][1:], B, qc, qs)
                eq.equarx_reduce_flat(sets[k % S][0], qc, qs, B, out)

            flat_ms = timed_steps(flat_pipeline)
            # the same pipelines with every wire cold when it is read: M of them side by side, wires of their own
            flat_cold_ms, Mf = None, cold_flat_pipelines(P, n, B)
            if Mf:
                fc = [[torch.empty(n, dtype=torch.int8, device="cuda") for _ in range(P - 1)] for _ in range(Mf)]
                fs = [[torch.empty(nb, dtype=torch.float32, device="cuda") for _ in range(P - 1)] for _ in range(Mf)]

                def flat_round(k):
                    for m in range(Mf):
                        eq.equarx_quantize_batch(sets[(k * Mf + m) % S][1:], B, fc[m], fs[m])
                    for m in range(Mf):
                        eq.equarx_reduce_flat(sets[(k * Mf + m) % S][0], fc[m], fs[m], B, out)

                for k in range(2):
                    flat_round(k)
                torch.cuda.synchronize()
                rounds = max(2, K // Mf)
                t0 = time.perf_counter()
                for k in range(rounds):
                    flat_round(k)
                torch.cuda.synchronize()
                flat_cold_ms = (time.perf_counter() - t0) * 1e3 / (rounds * Mf)
                del fc, fs
            flat_kernel_ms = single_kernel_ms(lambda k: eq.equarx_reduce_flat(sets[k % S][0], qc, qs, B, out), min(K, 50))
            flat_kernel_bytes = n * (2.0 + (P - 1) * (1.0 + 4.0 / B) + 2.0)
            flat_pipe_bytes = flat_kernel_bytes + (P - 1) * n * (2.0 + 1.0 + 4.0 / B)
            ref = torch.zeros(n, dtype=torch.float64, device="cuda")
            flat_pipeline(0)
            for p in sets[0]:
                ref += p.double()
            flat_rel = float((out.double() - ref).norm() / ref.norm())
            del ref, qc, qs
            flat_info = {
                "schedule": "all-to-all form: one batched quantize of the P-1 sent shards, then one flat reduce + requantize kernel",
                "ms_per_step": round(flat_ms, 5),
                "effective_input_GBps": round(gbps(2.0 * P * n, flat_ms), 1),
                "algorithmic_bytes": flat_pipe_bytes,
                "frac_of_hbm_peak": frac(flat_pipe_bytes, flat_ms),
                "cold_wire": None if flat_cold_ms is None else {
                    "arrangement": f"{Mf} independent pipelines side by side: all batched quantizes, then all flat "
                                   "reduces; between a wire's write and its read the others write more than the "
                                   "Infinity Cache holds",
                    "ms_per_step": round(flat_cold_ms, 5),
                    "frac_of_hbm_peak": frac(flat_pipe_bytes, flat_cold_ms)},
                "wire_access": "non-temporal (the wires cross devices in an all-to-all)",
                "flat_kernel_avg_launch_us": round(flat_kernel_ms * 1e3, 3),
                "flat_kernel_frac_of_hbm_peak": frac(flat_kernel_bytes, flat_kernel_ms),
                "rel_l2_vs_exact_sum": flat_rel,
            }

        # error of the result against the exact sum (fp64), computed with torch on the GPU; all schedules agree bit for bit
        rel_l2 = mse = max_abs = None
        if everything:
            calls["hop"](0)
            torch.cuda.synchronize()
            first = out.clone()
            for name, got in results.items():
                calls[name](0)
                torch.cuda.synchronize()
                assert torch.equal(out.view(torch.int16), first.view(torch.int16)), f"schedule {name} disagrees"
            ref = torch.zeros(n, dtype=torch.float64, device="cuda")
            for p in sets[0]:
                ref += p.double()
            diff = first.double() - ref
            rel_l2 = float(diff.norm() / ref.norm())
            mse = float((diff * diff).mean())
            max_abs = float(diff.abs().max())
            del ref, diff, first
        results.clear()

        # the dominant kernel inside the real chain: events recorded on the stream around its hops (launches 1..P-1 of
        # the call), back to back as they run there, nothing attached to the kernels themselves
        kernel_ms = launches_timed = traffic_only_ms = copy_gbps = None
        if everything and P > 1:
            kernel_ms, launches_timed = per_launch_ms(calls["hop"], 1, P - 1)
            if n % B == 0:      # calibration: the hops' loads and stores without their arithmetic, same ping-pong, same cadence
                codes = [torch.empty(n, dtype=torch.int8, device="cuda") for _ in range(2)]
                scales = [torch.empty(nb, dtype=torch.float32, device="cuda") for _ in range(2)]
                traffic_only_ms, _ = per_launch_ms(
                    lambda k: eq.equarx_calib_hop_traffic(sets[k % S], B, codes[0], scales[0], codes[1], scales[1]),
                    0, P - 1)
                del codes, scales
        elif everything:
            kernel_ms, launches_timed = per_launch_ms(calls["hop"], 0, 1)
        empty_us = None
        if everything:      # calibration: the stream time of a launch that does nothing, at the hop kernel's grid size
            grid = -(-n // (2048 * 3))
            for _ in range(3):
                eq.equarx_calib_empty_launches(64, grid)
            ev = event_pairs(10)
            for a, b in ev:
                a.record(stream)
                eq.equarx_calib_empty_launches(256, grid)
                b.record(stream)
            torch.cuda.synchronize()
            empty_us = statistics.median(a.elapsed_time(b) for a, b in ev) * 1e3 / 256
        if empty_us:        # what the launches alone cost each schedule, and the time no such schedule can beat
            launches = {"hop": P + 1, "ends": max(P - 1, 1), "fused": 1}
            for name, info in infos.items():
                floor_us = launches[name] * empty_us
                bound_us = floor_us + own_bytes[name] / (HBM_PEAK_GBPS * 1e9) * 1e6
                info["launches"] = launches[name]
                info["launch_floor_us"] = round(floor_us, 2)
                info["floor_plus_bytes_at_hbm_peak_us"] = round(bound_us, 2)
                info["frac_of_that_bound"] = round(bound_us / (info["ms_per_step"] * 1e3), 4)
        if everything:      # calibration: what a plain 16-byte copy reaches on this device over the same footprint
            src = torch.empty(2 * P * n // 2, dtype=torch.uint8, device="cuda")
            dst = torch.empty_like(src)
            for _ in range(3):
                eq.equarx_calib_copy(src, dst)
            copy_ms = single_kernel_ms(lambda k: eq.equarx_calib_copy(src, dst), 10)
            copy_gbps = 2.0 * src.numel() / (copy_ms * 1e-3) / 1e9
            del src, dst

        # cold wire: M independent chains interleaved pass by pass, every wire read M-1 launches after it was written
        cold = None
        M = cold_chains(n, B) if P > 1 and args.only in ("all", "cold") else 0
        if M:
            more = (sets + [[p.clone() for p in sets[0]] for _ in range(max(M - S, 0))])[:M]
            outs = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(M)]
            works = [eq.alloc_workspace(P, n, B) for _ in range(M)]
            rounds = max(2, -(-K // M))

            def cold_ms(streaming):
                for _ in range(2):
                    eq.equarx_calib_interleaved_chains(more, B, outs, works, streaming)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(rounds):
                    eq.equarx_calib_interleaved_chains(more, B, outs, works, streaming)
                torch.cuda.synchronize()
                return (time.perf_counter() - t0) * 1e3 / (rounds * M)

            # hops are launches M .. P*M-1 of the call: (P-1) groups of M launches, all of them cold-wire hops
            def cold_hop(streaming):
                return per_launch_ms(lambda k: eq.equarx_calib_interleaved_chains(more, B, outs, works, streaming),
                                     M, P - 1, group=M, reps=max(4, 2 * rounds))

            stream_ms = cold_ms(True)
            stream_hop_ms, cold_launches = cold_hop(True)
            # the same arrangement with the chain entry points' cacheable wire accesses: only with --only cold, so that
            # in the default run each kernel symbol stands for one situation (hop_kernel<.., false>: warm wire inside
            # the timed chain; hop_kernel<.., true>: cold wire) and a kernel trace of the run can be read directly
            cached_ms = cached_hop_ms = None
            if args.only == "cold":
                cached_ms = cold_ms(False)
                cached_hop_ms, _ = cold_hop(False)
            calls["hop"](0)
            torch.cuda.synchronize()
            assert all(torch.equal(o.view(torch.int16), out.view(torch.int16)) for o in outs), "cold chains disagree"
            cold = {
                "how": f"{M} independent chains interleaved pass by pass: every wire is read {M - 1} launches after it was "
                       f"written, behind {(M - 1) * wire_bytes(n, B) / 1e6:.0f} MB of other wires written and "
                       f"{(M - 1) * hop_bytes(n, B) / 1e6:.0f} MB of traffic in all; inputs cold as well; wire accessed "
                       f"with non-temporal hints, as the per-step entry points (equarx_quantize, equarx_reduce_stage, "
                       f"equarx_dequantize) access it",
                "chains_interleaved": M,
                "ms_per_step": round(stream_ms, 5),
                "effective_input_GBps": round(gbps(2.0 * P * n, stream_ms), 1),
                "frac_of_hbm_peak": frac(chain_bytes(P, n, B), stream_ms),
                "cacheable_wire_ms_per_step": round(cached_ms, 5) if cached_ms else None,
                "cacheable_wire_frac_of_hbm_peak": frac(chain_bytes(P, n, B), cached_ms) if cached_ms else None,
                "hop_kernel_us": round(stream_hop_ms * 1e3, 3),
                "hop_kernel_frac_of_hbm_peak": frac(hop_bytes(n, B), stream_hop_ms),
                "hop_kernel_cacheable_wire_us": round(cached_hop_ms * 1e3, 3) if cached_hop_ms else None,
                "hop_launches_timed": cold_launches,
            }
            del more, outs, works

    chosen = infos.get(args.schedule)
    if chosen is None:          # --only cold
        print(json.dumps({"config": {"workload": w.name, "P": P, "n": n, "block": B}, "cold_wire": cold}), flush=True)
        return 0
    ms_per_step = chosen["ms_per_step"]
    value = 2.0 * P * n / (ms_per_step * 1e-3) / 1e9
    if args.schedule == "fused":
        dominant = "chain (all hops in one launch)"
        per_launch = fused_bytes(P, n)
        kernel_ms = (chosen.get("kernel_avg_launch_us") or 0) * 1e-3 or None
        launches_timed = min(K, 50) if kernel_ms else None
    else:
        dominant = "hop (dequantize + fp32 add + requantize)" if P > 1 else "quantize"
        per_launch = hop_bytes(n, B) if P > 1 else n * (2.0 + 1.0 + 4.0 / B)
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": None, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": None,
                "traffic": None, "bytes_per_launch": per_launch}
    if kernel_ms:
        achieved = per_launch / (kernel_ms * 1e-3) / 1e9
        roofline.update({
            "achieved": round(achieved, 1), "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "avg_launch_us": round(kernel_ms * 1e3, 3), "launches_timed": launches_timed,
            "measured": "HIP events on the stream around runs of this kernel inside the timed entry point; inputs cold, "
                        "wire warm (written by the previous launch, still in the 256 MB Infinity Cache)",
        })
    if args.schedule != "fused":
        traffic = read_traffic(hip_build.source_digest()) if (w.name, B) == ("c3_gemma3_27b", 256) else None
        roofline.update({
            "traffic": traffic,
            "traffic_source": ("profiles/hop_kernel_c3_traffic.txt: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE per dispatch, "
                               "each scaled by the same counter's reading for a copy of known size; a committed profile "
                               "of this library build, not measured by this run") if traffic else None,
            "traffic_level": "bytes between L2 and the memory fabric (Infinity Cache + HBM together; not DRAM bytes)",
            "same_traffic_no_arithmetic_us": round(traffic_only_ms * 1e3, 3) if traffic_only_ms else None,
            "cold_wire": ({"avg_launch_us": cold["hop_kernel_us"],
                           "achieved": round(hop_bytes(n, B) / (cold["hop_kernel_us"] * 1e-6) / 1e9, 1),
                           "frac": cold["hop_kernel_frac_of_hbm_peak"], "launches_timed": cold["hop_launches_timed"],
                           "cacheable_wire_avg_launch_us": cold["hop_kernel_cacheable_wire_us"],
                           "measured": cold["how"]} if cold else None),
        })
    if copy_gbps:
        roofline["copy_kernel_GBps"] = round(copy_gbps, 1)
    if empty_us:
        roofline["empty_launch_pitch_us"] = round(empty_us, 3)

    if cold:
        chosen = dict(chosen, cold_wire={k: v for k, v in cold.items() if not k.startswith("hop_")})
    result = {
        "metric": "effective input GB/s (bf16 bytes reduced/sec)",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "value_is": "mean over the K timed steps (wall clock between two device synchronisations); inputs cold, wire warm",
        "config": {"workload": w.name, "P": P, "rows": w.rows, "hidden": w.hidden, "n": n, "block": B,
                   "distribution": w.dist, "schedule": chosen["schedule"]},
        "chain": chosen,
        "other_schedules": [v for k, v in infos.items() if k != args.schedule] + ([flat_info] if flat_info else []),
        "roofline": roofline,
        "error_vs_exact_sum": {"rel_l2": rel_l2, "mse": mse, "max_abs": max_abs},
    }
    if args.cpu_seconds > 0 and everything:
        result["cpu_baseline"] = cpu_baseline(w, [wl.as_u16(p) for p in host], args.cpu_seconds)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
