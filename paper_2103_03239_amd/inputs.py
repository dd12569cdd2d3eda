"""Seeded synthetic inputs and the five workload configurations.

This module holds no arithmetic of the averaging method: it only draws random
peer vectors with the shapes, sizes and value scales of the paper's workloads
and names the failure-schedule parameters.  Both the GPU tests/benchmark and
the CPU-oracle tests take their inputs from here, so the two sides always see
the same bytes.

The paper's datasets and trained weights are not used anywhere; only shapes are
taken from it: a ResNet-50-sized flat parameter vector (Sec. 4.2), the
N=1024, M=32, d=2 averaging experiment (Sec. 4.1), 16 servers on a 4x4 grid
(Sec. 4.2) and a large swarm of peers that leave and return (Sec. 4.1, App. I).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch

F32, BF16 = 0, 1                       # storage dtype codes (same as the C header)
KIND_NONE, KIND_IID, KIND_REJOIN = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    M: int
    d: int
    P: int
    dtype: int            # F32 or BF16
    init: str             # "normal" | "peer_mean" | "small" | "peer_offset"
    kind: int             # failure schedule kind
    p: float              # per-round failure probability
    down: int             # rounds a failed peer stays away (kind 2)
    rounds: int
    data_seed: int
    mask_seed: int

    @property
    def elem_size(self) -> int:
        return 4 if self.dtype == F32 else 2

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == F32 else torch.bfloat16

    def scaled(self, P: int, name: str | None = None) -> "Workload":
        """Same grid and schedule, shorter vectors (for CPU-sized parity runs)."""
        return replace(self, P=P, name=name or f"{self.name}-P{P}")


CONFIGS = {
    1: Workload("cfg1-4x4-f32", 16, 4, 2, 65_536, F32, "normal", KIND_NONE, 0.0, 0, 2, 1001, 2001),
    2: Workload("cfg2-16x16-f32", 256, 16, 2, 1_048_576, F32, "peer_mean", KIND_IID, 0.05, 0, 10, 1002, 2002),
    3: Workload("cfg3-4x4x4-resnet50-f32", 64, 4, 3, 25_557_032, F32, "small", KIND_IID, 0.1, 0, 6, 1003, 2003),
    4: Workload("cfg4-32x32-f32", 1024, 32, 2, 4_194_304, F32, "peer_offset", KIND_IID, 0.2, 0, 8, 1004, 2004),
    5: Workload("cfg5-16x16x16-bf16", 4096, 16, 3, 262_144, BF16, "normal", KIND_REJOIN, 0.1, 2, 12, 1005, 2005),
}


def aligned_row_stride(P: int, dtype: int) -> int:
    """Smallest row stride (in elements) >= P whose rows start on 128-byte boundaries, the
    cache-line size of the GPU: measured worth about 5 % of HBM throughput on rows that
    are not (25,557,032 binary32 parameters are 96 bytes short of one)."""
    per_line = 128 // (4 if dtype == F32 else 2)
    return -(-P // per_line) * per_line


def make_state(w: Workload, device: str | torch.device = "cpu", row_stride: int | None = None,
               progress=None) -> torch.Tensor:
    """Draw the [N, P] peer-state matrix of a workload in its storage dtype.

    Rows are filled one at a time so no temporary larger than a row exists.
    With ``row_stride`` > P the result is a view into a padded [N, row_stride]
    buffer (padding filled with a sentinel the kernels must never touch).
    ``progress(rows_done, N)``, if given, is called every 512 rows (a run under a
    profiler that serialises launches spends minutes here).
    """
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(w.data_seed)
    stride = w.P if row_stride is None else row_stride
    if stride < w.P:
        raise ValueError("row_stride must be >= P")
    buf = torch.full((w.N, stride), 12345.0, dtype=w.torch_dtype, device=device)
    X = buf[:, : w.P]
    offsets = None
    if w.init == "peer_offset":
        offsets = torch.rand(w.N, generator=gen, device=device, dtype=torch.float32) * 2.0 - 1.0
    row = torch.empty(w.P, dtype=torch.float32, device=device)
    for i in range(w.N):
        row.normal_(0.0, 1.0, generator=gen)
        if w.init == "peer_mean":
            row.add_(0.01 * i)
        elif w.init == "small":
            row.mul_(0.02)
        elif w.init == "peer_offset":
            row.add_(offsets[i])
        elif w.init != "normal":
            raise ValueError(f"unknown init {w.init!r}")
        X[i].copy_(row)          # fp32 -> storage dtype, round-to-nearest-even
        if progress is not None and (i + 1) % 512 == 0:
            progress(i + 1, w.N)
    return X
