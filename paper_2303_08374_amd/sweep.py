"""The op sweep (allreduce, reduce_scatter, allgather, alltoall; fp32 and bf16; 4 KiB to
256 MiB per rank; P simulated ranks) as a list of launchable cells over one device arena.

Stands in for the OSU micro-benchmark sweeps the paper uses to compare backends and to
build its tuning tables (Sec. II "Motivation" figure, Sec. V-B).  "Message size" M is one
rank's send buffer in bytes for all four ops.

Cold-cache policy: every launch takes its buffers from a cursor that walks cyclically
through an arena much larger than the last-level cache, so a buffer is touched again only
after gigabytes of other traffic.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import torch

from . import mcr

OPS = {"allreduce": mcr.OP_ALLREDUCE, "reduce_scatter": mcr.OP_REDUCE_SCATTER,
       "allgather": mcr.OP_ALLGATHER, "alltoall": mcr.OP_ALLTOALL}
DTYPES = {"f32": mcr.F32, "bf16": mcr.BF16}
ELEM = {"f32": 4, "bf16": 2}
ALIGN = 256


def algorithmic_bytes(op: str, P: int, M: int) -> int:
    """Bytes the op must read plus write once (no cache reuse assumed)."""
    if op == "allreduce":
        return 2 * P * M                 # P reads + P writes
    if op == "reduce_scatter":
        return (P + 1) * M               # P reads + P slices of M/P written
    if op == "allgather":
        return (P + P * P) * M           # P reads + P outputs of P*M
    if op == "alltoall":
        return 2 * P * M
    raise ValueError(op)


def _round_up(x: int, a: int = ALIGN) -> int:
    return (x + a - 1) // a * a


@dataclass
class Cell:
    op: str
    dtype: str
    P: int
    M: int                                    # bytes of one rank's send buffer
    in_bytes: int = 0                         # per rank
    out_bytes: int = 0                        # per rank (0: in place)
    footprint: int = 0
    alg_bytes: int = 0
    count: int = 0

    def __post_init__(self):
        self.count = self.M // ELEM[self.dtype]
        self.in_bytes = self.M
        self.out_bytes = {"allreduce": 0, "reduce_scatter": self.M // self.P,
                          "allgather": self.M * self.P, "alltoall": self.M}[self.op]
        self.footprint = self.P * (_round_up(self.in_bytes) + _round_up(self.out_bytes))
        self.alg_bytes = algorithmic_bytes(self.op, self.P, self.M)

    @property
    def key(self) -> str:
        return f"{self.op}/{self.dtype}/{self.M}"

    def pointers(self, base: int):
        ins = [base + p * _round_up(self.in_bytes) for p in range(self.P)]
        obase = base + self.P * _round_up(self.in_bytes)
        outs = [obase + p * _round_up(self.out_bytes) for p in range(self.P)]
        return ins, outs

    def launch(self, ctx, base: int, variant: int = mcr.AUTO, stream=None) -> None:
        ins, outs = self.pointers(base)
        dt = DTYPES[self.dtype]
        if self.op == "allreduce":
            mcr.mcr_allreduce(ctx, ins, self.count, dt, mcr.SUM, self.P, variant, stream)
        elif self.op == "reduce_scatter":
            mcr.mcr_reduce_scatter(ctx, outs, ins, self.count, dt, mcr.SUM, self.P, variant, stream)
        elif self.op == "allgather":
            mcr.mcr_allgather(ctx, outs, ins, self.count, dt, self.P, variant, stream)
        else:
            mcr.mcr_alltoall(ctx, outs, ins, self.count, dt, self.P, variant, stream)

    def auto_variant(self, ctx) -> int:
        return mcr.mcr_auto_variant(ctx, OPS[self.op], DTYPES[self.dtype], self.P, self.M, True)


def make_cells(P: int, ops: Sequence[str], dtypes: Sequence[str], sizes: Sequence[int]) -> List[Cell]:
    return [Cell(op, dt, P, M) for dt in dtypes for op in ops for M in sizes]


class Arena:
    """One device allocation that every cell carves its rank buffers from."""

    def __init__(self, nbytes: int, seed: int = 0):
        self.nbytes = _round_up(nbytes)
        self.buf = torch.empty(self.nbytes // 2, dtype=torch.bfloat16, device="cuda")
        self.base = self.buf.data_ptr()
        assert self.base % ALIGN == 0
        self.cursor = 0
        self.seed = seed
        self.refill()

    def refill(self) -> None:
        """uniform[-1,1) bf16 patterns; two of them read as one fp32 are again a finite value
        of magnitude below 1, so the same fill serves both dtypes."""
        g = torch.Generator(device="cuda")
        g.manual_seed(self.seed)
        step = 1 << 28
        for i in range(0, self.buf.numel(), step):
            self.buf[i:i + step].uniform_(-1.0, 1.0, generator=g)

    def take(self, footprint: int) -> int:
        """Device address of the next `footprint` bytes, wrapping at the end."""
        assert footprint <= self.nbytes
        if self.cursor + footprint > self.nbytes:
            self.cursor = 0
        addr = self.base + self.cursor
        self.cursor = _round_up(self.cursor + footprint)
        return addr


def time_launches(fn, reps: int) -> float:
    """Mean milliseconds per call of `fn` over `reps` back-to-back calls on the current
    stream, between two events (the paper's "end-to-end time on a set of overlapped
    communication operations" read as one batch on one stream)."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(reps):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / reps
