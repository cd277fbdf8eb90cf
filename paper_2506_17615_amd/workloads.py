"""Seeded synthetic inputs for the quantized P-way reduction.

This module holds input recipes only -- no quantization, no reduction, none of
the method's arithmetic -- so that the HIP path's tests, the benchmark and the
CPU oracle's tests can all draw the very same tensors from it.

Each workload is P partial-sum tensors of identical shape, bf16, generated in
fp32 on the CPU from a seeded ``torch.Generator`` and cast to bf16
(round-to-nearest-even).  The shapes and value distributions stand in for the
AllReduce inputs of the paper's microbenchmarks (Sec. 4: N(0,1) tensors, a
sweep over message sizes) and of its Gemma 3 prefill experiment (Sec. 5:
activations of [tokens, hidden] summed over the model-parallel group); no
model weights or datasets are involved.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str            # short id used in reports
    P: int               # number of partial sums in the chain
    rows: int            # tokens (1 for flat messages)
    hidden: int          # elements per row; blocks run along this dimension
    block: int           # quantization block size B
    dist: str            # "normal" | "row_lognormal" | "row_lognormal_outliers" | "student_t3"
    seed: int
    note: str = ""

    @property
    def n(self) -> int:
        return self.rows * self.hidden

    def with_rows(self, rows: int) -> "Workload":
        """Same recipe on fewer (or more) rows -- for tests the oracle must finish quickly."""
        return replace(self, rows=int(rows))

    def with_block(self, block: int) -> "Workload":
        return replace(self, block=int(block))


# Index = position in the benchmark's config list; seed = 1000 + index.
WORKLOADS = {
    "c1_small": Workload("c1_small", P=4, rows=1, hidden=4096, block=256, dist="normal", seed=1000,
                         note="correctness-sized message, N(0,1)"),
    "c2_gemma3_12b": Workload("c2_gemma3_12b", P=8, rows=2048, hidden=3840, block=256, dist="row_lognormal",
                              seed=1001, note="12B-shaped prefill activation, 2048 tokens x 3840 hidden"),
    "c3_gemma3_27b": Workload("c3_gemma3_27b", P=8, rows=4096, hidden=5376, block=256,
                              dist="row_lognormal_outliers", seed=1002,
                              note="27B-shaped prefill activation, 4096 tokens x 5376 hidden, outlier channels"),
    "c4_decode": Workload("c4_decode", P=16, rows=64, hidden=5376, block=128, dist="normal", seed=1003,
                          note="decode-sized message, latency regime"),
    "c5_large": Workload("c5_large", P=8, rows=1, hidden=33_554_432, block=128, dist="student_t3", seed=1004,
                         note="64 MiB per partial, heavy tails; block swept over 32/128/512"),
}

# The tensor of the paper's own accuracy/speed comparison of its flavours (Sec. 4.1, Fig. 7): (4096, 4096), N(0,1),
# 8 devices, block size 64.  Not one of the benchmark's configs; used by the report tool and the parity tests.
FIG7 = Workload("fig7", P=8, rows=4096, hidden=4096, block=64, dist="normal", seed=1007,
                note="the (4096, 4096) N(0,1) tensor of Sec. 4.1 / Fig. 7: 8 devices, block 64")

OUTLIER_FRACTION = 0.001   # share of hidden channels scaled up in the outlier recipe
OUTLIER_GAIN = 50.0


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def _shared_row_factors(w: Workload) -> torch.Tensor:
    """Per-row lognormal(0,1) factors, drawn once and shared by all partials."""
    return torch.exp(torch.randn(w.rows, 1, generator=_gen(w.seed * 100 + 90), dtype=torch.float32))


def outlier_channels(w: Workload) -> torch.Tensor:
    """Indices of the hidden channels that carry the x50 gain (same for all partials)."""
    k = max(1, round(OUTLIER_FRACTION * w.hidden))
    perm = torch.randperm(w.hidden, generator=_gen(w.seed * 100 + 91))
    return perm[:k].sort().values


def make_partial(w: Workload, p: int) -> torch.Tensor:
    """Partial sum number p of workload w: a bf16 CPU tensor of shape [rows, hidden]."""
    g = _gen(w.seed * 100 + p)
    shape = (w.rows, w.hidden)
    if w.dist == "normal":
        v = torch.randn(shape, generator=g, dtype=torch.float32)
    elif w.dist in ("row_lognormal", "row_lognormal_outliers"):
        v = torch.randn(shape, generator=g, dtype=torch.float32) * _shared_row_factors(w)
        if w.dist == "row_lognormal_outliers":
            v[:, outlier_channels(w)] *= OUTLIER_GAIN
    elif w.dist == "student_t3":
        z = torch.randn(shape, generator=g, dtype=torch.float32)
        chi2 = torch.zeros(shape, dtype=torch.float32)
        for _ in range(3):
            chi2 += torch.randn(shape, generator=g, dtype=torch.float32) ** 2
        v = z / torch.sqrt(chi2 / 3.0)
    else:
        raise ValueError(f"unknown distribution {w.dist!r}")
    return v.to(torch.bfloat16)


def make_partials(w: Workload) -> list[torch.Tensor]:
    """All P partials of workload w, in chain order."""
    return [make_partial(w, p) for p in range(w.P)]


def as_u16(t: torch.Tensor):
    """Raw bf16 bit patterns of a CPU tensor as a flat numpy uint16 array."""
    return t.contiguous().view(torch.uint16).reshape(-1).numpy()
