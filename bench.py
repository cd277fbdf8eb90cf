#!/usr/bin/env python3
"""Benchmark of the quantized P-way reduction on one MI355X.

A step is one pass of the whole hot path -- quantize, P-1 fused dequantize-add-requantize hops, final
dequantize (equarx_reduce_quantized) -- over one batch of synthetic partial sums already resident in HBM.
Prints ONE JSON line: effective input GB/s (bf16 bytes reduced per second), the roofline of the dominant
kernel (the hop) from HIP events recorded around runs of hops inside the real call, the other schedules with
their own byte counts, and the CPU oracle timed on the host as a reported baseline.
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


def read_traffic():
    """HBM bytes per hop launch from the committed rocprofv3 counter summary, or None."""
    try:
        vals = {}
        with open(TRAFFIC_FILE) as f:
            for line in f:
                if line.startswith("hbm_bytes_per_launch"):
                    vals["t"] = float(line.split()[1])
        return vals.get("t")
    except OSError:
        return None


def cpu_baseline(w, host_u16, budget_s: float):
    """The oracle as it stands, timed on this machine's host cores on the same workload (all cores, then one)."""
    import numpy as np

    from oracle import equarx_oracle as orc
    orc.build()
    threads = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16") or 16)))

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
        "single_thread_value": round(2.0 * w.P * w.n / one / 1e9, 4),
        "single_thread_sample": f"median of {reps1} full chains, {one * 1e3:.0f} ms each",
        "rel_l2_vs_exact_sum": rel,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c3_gemma3_27b")
    ap.add_argument("--block", type=int, default=0, help="override the workload's block size")
    ap.add_argument("--rows", type=int, default=0,
                    help="override the workload's row count (e.g. rows/8: the share of one GPU of an 8-GPU node)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the oracle timing; 0 skips it")
    ap.add_argument("--schedule", choices=("hop", "fused"), default="hop",
                    help="hop: P+1 launches, the wire written and read back (default, the schedule a ring imposes); "
                         "fused: the same chain in one launch (equarx_reduce_fused)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all P partials live in one MI355X's HBM); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch

    from paper_2506_17615_amd import binding as eq
    from paper_2506_17615_amd import workloads as wl

    from paper_2506_17615_amd import build as hip_build
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

    host = wl.make_partials(w)
    # two resident input sets, used in turn, so that no step finds its inputs in the 256 MB Infinity Cache
    sets = [[p.reshape(-1).cuda() for p in host]]
    sets.append([p.clone() for p in sets[0]])
    out = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    work = eq.alloc_workspace(P, n, B)
    nb = eq.num_blocks(n, B)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for k in range(W):
            eq.equarx_reduce_quantized(sets[k % 2], B, out, work)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(K):
            eq.equarx_reduce_quantized(sets[k % 2], B, out, work)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        hop_ms_per_step = (t1 - t0) * 1e3 / K

        # spread of single steps: the same K steps once more, each between two events on the stream (the records
        # themselves cost a microsecond or two per step, so the median sits slightly above ms_per_step)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
        marks[0].record(stream)
        for k in range(K):
            eq.equarx_reduce_quantized(sets[k % 2], B, out, work)
            marks[k + 1].record(stream)
        torch.cuda.synchronize()
        step_us = sorted(marks[k].elapsed_time(marks[k + 1]) * 1e3 for k in range(K))
        spread = {"p10": round(step_us[int(0.1 * (K - 1))], 2), "median": round(step_us[(K - 1) // 2], 2),
                  "p90": round(step_us[int(0.9 * (K - 1))], 2)}

        # hop by hop with the first two and the last two passes sharing a launch: same bits, P-1 launches
        for k in range(W):
            eq.equarx_reduce_quantized_fused_ends(sets[k % 2], B, out, work)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(K):
            eq.equarx_reduce_quantized_fused_ends(sets[k % 2], B, out, work)
        torch.cuda.synchronize()
        ends_ms_per_step = (time.perf_counter() - t0) * 1e3 / K
        out_ends = out.clone()

        # the same chain in one launch: same bits, no wire traffic
        for k in range(W):
            eq.equarx_reduce_fused(sets[k % 2], B, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(K):
            eq.equarx_reduce_fused(sets[k % 2], B, out)
        torch.cuda.synchronize()
        fused_ms_per_step = (time.perf_counter() - t0) * 1e3 / K
        fused_pairs = []
        for _ in range(min(K, 50)):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            b.record(stream)
            fused_pairs.append((a, b))
        torch.cuda.synchronize()
        for k, (a, b) in enumerate(fused_pairs):
            eq.equarx_time_next_launch(a.cuda_event, b.cuda_event)
            eq.equarx_reduce_fused(sets[k % 2], B, out)
        torch.cuda.synchronize()
        fused_kernel_ms = statistics.fmean(a.elapsed_time(b) for a, b in fused_pairs)
        out_fused = out.clone()

        # all-to-all form: every non-owner quantizes its shard once, the owner reduces all of them in one kernel
        flat_info = None
        if P > 1:
            qc = [torch.empty(n, dtype=torch.int8, device="cuda") for _ in range(P - 1)]
            qs = [torch.empty(nb, dtype=torch.float32, device="cuda") for _ in range(P - 1)]

            def flat_pipeline(parts):
                eq.equarx_quantize_batch(parts[1:], B, qc, qs)
                eq.equarx_reduce_flat(parts[0], qc, qs, B, out)

            for k in range(W):
                flat_pipeline(sets[k % 2])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k in range(K):
                flat_pipeline(sets[k % 2])
            torch.cuda.synchronize()
            flat_ms = (time.perf_counter() - t0) * 1e3 / K
            fp = []
            for _ in range(min(K, 50)):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                b.record(stream)
                fp.append((a, b))
            torch.cuda.synchronize()
            for k, (a, b) in enumerate(fp):
                eq.equarx_time_next_launch(a.cuda_event, b.cuda_event)
                eq.equarx_reduce_flat(sets[k % 2][0], qc, qs, B, out)
            torch.cuda.synchronize()
            flat_kernel_ms = statistics.fmean(a.elapsed_time(b) for a, b in fp)
            flat_kernel_bytes = n * (2.0 + (P - 1) * (1.0 + 4.0 / B) + 2.0)
            flat_pipe_bytes = flat_kernel_bytes + (P - 1) * n * (2.0 + 1.0 + 4.0 / B)
            ref = torch.zeros(n, dtype=torch.float64, device="cuda")
            flat_pipeline(sets[0])
            for p in sets[0]:
                ref += p.double()
            flat_rel = float((out.double() - ref).norm() / ref.norm())
            del ref
            flat_info = {
                "schedule": "all-to-all form: one batched quantize of the P-1 sent shards, then one flat reduce + requantize kernel",
                "ms_per_step": round(flat_ms, 5),
                "effective_input_GBps": round(2.0 * P * n / (flat_ms * 1e-3) / 1e9, 1),
                "algorithmic_bytes": flat_pipe_bytes,
                "frac_of_hbm_peak": round(flat_pipe_bytes / (flat_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "flat_kernel_avg_launch_us": round(flat_kernel_ms * 1e3, 3),
                "flat_kernel_frac_of_hbm_peak": round(flat_kernel_bytes / (flat_kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "rel_l2_vs_exact_sum": flat_rel,
            }

        # error of the result against the exact sum (fp64), computed with torch on the GPU
        eq.equarx_reduce_fused(sets[0], B, out_fused)
        eq.equarx_reduce_quantized(sets[0], B, out, work)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), out_fused.view(torch.int16)), "schedules disagree"
        assert torch.equal(out.view(torch.int16), out_ends.view(torch.int16)), "schedules disagree"
        ref = torch.zeros(n, dtype=torch.float64, device="cuda")
        for p in sets[0]:
            ref += p.double()
        diff = out.double() - ref
        rel_l2 = float(diff.norm() / ref.norm())
        mse = float((diff * diff).mean())
        max_abs = float(diff.abs().max())
        del ref, diff

        # the same K steps once more, each call with a pair of HIP events recorded on the stream around its hops
        # (launches 1..P-1 of the call): the dominant kernel's duration inside the real chain, back to back as it
        # runs there, nothing attached to the kernels themselves
        codes = [torch.empty(n, dtype=torch.int8, device="cuda") for _ in range(2)]
        scales = [torch.empty(nb, dtype=torch.float32, device="cuda") for _ in range(2)]

        def event_pairs(count):
            made = []
            for _ in range(count):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                b.record(stream)          # creates the underlying hipEvent_t handles
                made.append((a, b))
            torch.cuda.synchronize()
            return made

        def per_launch_ms(call, first, count):
            """Mean duration of one of `count` consecutive launches (from launch `first`) of call(k).  Spans of two
            lengths are timed on alternate steps and subtracted, which cancels what the two event records cost."""
            short = count // 2 if count >= 3 and K >= 4 else 0
            pairs = event_pairs(K)
            for k, (a, b) in enumerate(pairs):
                length = short if (short and k % 2) else count
                eq.equarx_time_launch_span(first, first + length - 1, a.cuda_event, b.cuda_event)
                call(k)
            torch.cuda.synchronize()
            times = [a.elapsed_time(b) for a, b in pairs]
            if not short:
                return statistics.fmean(times) / count, len(times) * count
            long_ms, short_ms = statistics.fmean(times[0::2]), statistics.fmean(times[1::2])
            return (long_ms - short_ms) / (count - short), len(times[0::2]) * count + len(times[1::2]) * short

        kernel_ms, launches_timed = per_launch_ms(lambda k: eq.equarx_reduce_quantized(sets[k % 2], B, out, work),
                                                  1 if P > 1 else 0, max(P - 1, 1))

        # calibration: the hops' loads and stores without their arithmetic, same ping-pong, same cadence
        traffic_only_ms = None
        if P > 1 and n % B == 0:
            traffic_only_ms, _ = per_launch_ms(
                lambda k: eq.equarx_calib_hop_traffic(sets[k % 2], B, codes[0], scales[0], codes[1], scales[1]),
                0, P - 1)

        # calibration: what a plain 16-byte copy reaches on this device over the same footprint
        src = torch.empty(2 * P * n // 2, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            eq.equarx_calib_copy(src, dst)
        cp = []
        for _ in range(10):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            b.record(stream)
            torch.cuda.synchronize()
            eq.equarx_time_next_launch(a.cuda_event, b.cuda_event)
            eq.equarx_calib_copy(src, dst)
            torch.cuda.synchronize()
            cp.append(a.elapsed_time(b))
        copy_gbps = 2.0 * src.numel() / (statistics.median(cp) * 1e-3) / 1e9

    def gbps(nbytes, ms):
        return nbytes / (ms * 1e-3) / 1e9

    hop_info = {
        "schedule": "hop-by-hop, P+1 launches, wire written once and read once",
        "ms_per_step": round(hop_ms_per_step, 5),
        "effective_input_GBps": round(gbps(2.0 * P * n, hop_ms_per_step), 1),
        "algorithmic_bytes": chain_bytes(P, n, B),
        "frac_of_hbm_peak": round(gbps(chain_bytes(P, n, B), hop_ms_per_step) / HBM_PEAK_GBPS, 4),
        "single_step_us": spread,
    }
    fused_info = {
        "schedule": "single launch, chain in registers, no wire traffic",
        "ms_per_step": round(fused_ms_per_step, 5),
        "effective_input_GBps": round(gbps(2.0 * P * n, fused_ms_per_step), 1),
        "algorithmic_bytes": fused_bytes(P, n),
        "frac_of_hbm_peak": round(gbps(fused_bytes(P, n), fused_ms_per_step) / HBM_PEAK_GBPS, 4),
        "kernel_avg_launch_us": round(fused_kernel_ms * 1e3, 3),
    }
    ends_bytes = fused_bytes(P, n) + 2.0 * max(P - 2, 0) * n * (1.0 + 4.0 / B)
    ends_info = {
        "schedule": "hop-by-hop with both ends fused: max(P-1, 1) launches, P-2 wire buffers written once and read once",
        "ms_per_step": round(ends_ms_per_step, 5),
        "effective_input_GBps": round(gbps(2.0 * P * n, ends_ms_per_step), 1),
        "algorithmic_bytes": ends_bytes,
        "frac_of_hbm_peak": round(gbps(ends_bytes, ends_ms_per_step) / HBM_PEAK_GBPS, 4),
    }
    if args.schedule == "hop":
        ms_per_step, chosen, other = hop_ms_per_step, hop_info, fused_info
        dominant = "hop (dequantize + fp32 add + requantize)" if P > 1 else "quantize"
        per_launch = hop_bytes(n, B) if P > 1 else n * (2.0 + 1.0 + 4.0 / B)
        traffic = read_traffic() if (w.name, B) == ("c3_gemma3_27b", 256) else None
    else:
        ms_per_step, chosen, other = fused_ms_per_step, fused_info, hop_info
        dominant = "chain (all hops in one launch)"
        per_launch = fused_bytes(P, n)
        kernel_ms, launches_timed = fused_kernel_ms, len(fused_pairs)
        traffic = None
    achieved = per_launch / (kernel_ms * 1e-3) / 1e9
    value = 2.0 * P * n / (ms_per_step * 1e-3) / 1e9

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
        "config": {"workload": w.name, "P": P, "rows": w.rows, "hidden": w.hidden, "n": n, "block": B,
                   "distribution": w.dist, "schedule": chosen["schedule"]},
        "chain": chosen,
        "other_schedules": [x for x in (ends_info, other, flat_info) if x],
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "bytes_per_launch": per_launch, "avg_launch_us": round(kernel_ms * 1e3, 3),
                     "launches_timed": launches_timed, "copy_kernel_GBps": round(copy_gbps, 1),
                     "same_traffic_no_arithmetic_us": (round(traffic_only_ms * 1e3, 3)
                                                       if traffic_only_ms and args.schedule == "hop" else None)},
        "error_vs_exact_sum": {"rel_l2": rel_l2, "mse": mse, "max_abs": max_abs},
    }
    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(w, [wl.as_u16(p) for p in host], args.cpu_seconds)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
