"""The tuning suite (paper Sec. IV-E and V-B): micro-benchmarks every kernel variant of every
op over the message-size sweep, picks the variant with the least time per (op, dtype, P,
size) and writes the static tuning table that MCR_AUTO consults.

    python -m paper_2303_08374_amd.tune [--out paper_2303_08374_amd/tuning/mi355x.tbl]
                                        [--report tune_report.json] [--ranks 4,8,16]

One table cell = one batch of identical launches on one stream over cold buffers, mean time
per launch.  Ties go to the lower variant id.  Besides the per-size ("fine", the paper's
MCR-DL-T) table the report holds the best single variant per op ("coarse", the paper's
MCR-DL) and the gap between the two.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import torch

from . import inputs, mcr, sweep, workloads

HERE = os.path.dirname(os.path.abspath(__file__))
DEFAULT_TABLE = os.path.join(HERE, "tuning", "mi355x.tbl")


def tie_window_us(floor_us: float, graph_timed: bool = False) -> float:
    """Times within this many microseconds of the least one count as a tie (the lowest variant id
    then wins): 2 % of the least time while a launch is shorter than 100 us, 0.5 % from there on
    (where a batch mean repeats to a few tenths of a percent), and never less than half a
    microsecond, which is what two batches of the same launch-bound kernel issued from the host
    differ by; a tenth of a microsecond for a batch replayed from a graph, which repeats to a few
    hundredths."""
    return max(0.1 if graph_timed else 0.5, floor_us * (0.02 if floor_us < 100.0 else 0.005))


def pick(times_us: dict, graph_timed: bool = False):
    """The table's choice among {variant: microseconds per launch}, the figures as they are
    recorded (two decimals): least time, ties to the variant listed first (the lowest id)."""
    floor = min(times_us.values())
    for v, t in times_us.items():
        if t <= floor + tie_window_us(floor, graph_timed):
            return v


def variants_of(ctx, op_id: int):
    """The variants worth timing for an op: every 128-bit shape (the element path is only the
    fallback); for the reductions not the "v2", "v4", "ln" and "sn" ids, which run the "nt" kernels."""
    n_var = len(mcr.mcr_get_variants(ctx, op_id))
    if op_id in (mcr.OP_ALLREDUCE, mcr.OP_REDUCE_SCATTER):
        return [v for v in range(1, n_var) if v not in (2, 3) and not 7 <= v <= 12]
    return list(range(1, n_var))


GRAPH_BELOW_MS = 0.03


def graph_batch_ms(launch, bases) -> float:
    """Milliseconds per launch of `launch(base, stream)` over `bases`, captured once into a HIP
    graph (the entry points only enqueue kernels) and replayed: the least of three replays."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        launch(bases[0], None)                                # nothing is loaded for the first time inside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        stream = torch.cuda.current_stream().cuda_stream
        for b in bases:
            launch(b, stream)
    graph.replay()
    torch.cuda.synchronize()
    ms = min(sweep.time_launches(graph.replay, 1) for _ in range(3)) / len(bases)
    del graph
    return ms


def reps_for(alg_bytes: int) -> int:
    # about 160 GiB of traffic per batch (tens of milliseconds), between 5 and 50 launches
    return int(max(5, min(50, (160 << 30) // max(alg_bytes, 1))))


def tune_workload_ops(ctx, verbose: bool = True):
    """One table row per (op, dtype, P) of the ops the application-shaped workloads use beyond the
    swept collectives: all_to_allv, pack, unpack (MoE: bf16, P=16; DLRM: fp32, P=8), fuse, unfuse and
    the fused multi-tensor allreduce (gradient buckets: bf16, P=8).  Every stage of a workload is an
    independent launch timed on its own, so one run with all stages on variant v gives v's time for
    each of them."""
    n_var = len(mcr.mcr_get_variants(ctx, mcr.OP_ALLTOALLV))
    names = mcr.mcr_get_variants(ctx, mcr.OP_ALLTOALLV)
    variants = list(range(1, n_var))
    moe, dlrm, gb = inputs.MoEWorkload(), inputs.DLRMWorkload(), inputs.GradBucketWorkload()
    plans = [
        # (label, runner, {op id: [stage names]}, dtype, P, table bytes)
        ("moe", lambda vv: workloads.moe_dispatch_combine(ctx, reps=5, variants=vv),
         {mcr.OP_PACK: ["pack"], mcr.OP_ALLTOALLV: ["alltoallv_dispatch", "alltoallv_return"], mcr.OP_UNPACK: ["unpack_combine"],
          mcr.OP_MOE_DISPATCH: ["fused/moe_dispatch"], mcr.OP_MOE_COMBINE: ["fused/moe_combine"],
          mcr.OP_MOE_DISPATCH_BY_EXPERT: ["by_expert/moe_dispatch_by_expert"],
          mcr.OP_MOE_COMBINE_BY_EXPERT: ["by_expert/moe_combine_by_expert"]},
         mcr.BF16, moe.P, moe.T * moe.H * 2),
        ("dlrm", lambda vv: workloads.dlrm_shuffle(ctx, reps=5, variants=vv),
         {mcr.OP_PACK: ["fwd_pack_send_order", "bwd_pack_permute"], mcr.OP_ALLTOALLV: ["fwd_alltoallv", "bwd_alltoallv"],
          mcr.OP_UNPACK: ["fwd_unpack_permute", "bwd_unpack_table_order"],
          mcr.OP_DLRM_SHUFFLE: ["fused/fwd_dlrm_shuffle", "fused/bwd_dlrm_shuffle"]},
         mcr.F32, dlrm.P, (dlrm.batch // dlrm.P) * dlrm.n_tables * dlrm.dim * 4),
        ("grad_buckets", lambda vv: workloads.grad_buckets(ctx, reps=2, variants=vv, per_tensor=False),
         {mcr.OP_FUSE: ["fuse"], mcr.OP_UNFUSE: ["unfuse"], mcr.OP_ALLREDUCE_MULTI: ["allreduce_multi_one_launch"]},
         mcr.BF16, gb.P, 1 << 20),
    ]
    key_of = {mcr.OP_PACK: "pack", mcr.OP_ALLTOALLV: "alltoallv", mcr.OP_UNPACK: "unpack", mcr.OP_FUSE: "fuse",
              mcr.OP_UNFUSE: "unfuse", mcr.OP_ALLREDUCE_MULTI: "allreduce_multi", mcr.OP_MOE_DISPATCH: "moe_dispatch",
              mcr.OP_MOE_COMBINE: "moe_combine", mcr.OP_DLRM_SHUFFLE: "dlrm_shuffle",
              mcr.OP_MOE_DISPATCH_BY_EXPERT: "moe_dispatch_by_expert", mcr.OP_MOE_COMBINE_BY_EXPERT: "moe_combine_by_expert"}

    def stage_us(rep, path):
        for part in path.split("/"):
            rep = rep[part]
        return rep["us"]
    # the multi-tensor all_reduce has two kernels, plain and nontemporal: the other ids run the second one
    distinct = {mcr.OP_ALLREDUCE_MULTI: (1, 4)}
    report = {}
    for label, runner, ops, dtype, P, nbytes in plans:
        times = {op: {} for op in ops}
        for v in variants:
            rep = runner({key_of[op]: v for op in ops})
            for op, stages in ops.items():
                if v in distinct.get(op, variants):
                    times[op][v] = sum(stage_us(rep, st) for st in stages)
            torch.cuda.empty_cache()
        for op in ops:
            us = {v: round(t, 2) for v, t in times[op].items()}
            best = pick(us)
            mcr.mcr_tune_set(ctx, op, dtype, P, nbytes, best)
            report.setdefault("_rows", []).append((mcr.OP_NAMES[op], dtype, P, nbytes, names[best],
                                                   {names[v]: t for v, t in us.items()}))
            report[f"{label}/{mcr.OP_NAMES[op]}"] = {"best": names[best], "us": {names[v]: round(t, 1) for v, t in times[op].items()}}
            if verbose:
                print(f"{label}/{mcr.OP_NAMES[op]:18s} best={names[best]:6s} " +
                      " ".join(f"{names[v]}={t:.0f}" for v, t in times[op].items()), flush=True)
    return report


_NAMES = {}


def names_of(ctx, op_id: int):
    if op_id not in _NAMES:
        _NAMES[op_id] = mcr.mcr_get_variants(ctx, op_id)
    return _NAMES[op_id]


TIMES_HEADER = ("# every variant's time, in microseconds per launch, behind each row of the tuning table next to it\n"
                "# (written by python -m paper_2303_08374_amd.tune --times-out): op dtype P bytes chosen how-timed | variant=us ...\n")


def write_times(path: str, rows, coarse_vs_fine=None) -> None:
    dt = {mcr.F32: "f32", mcr.BF16: "bf16", mcr.F16: "f16", mcr.I32: "i32"}
    with open(path, "w") as f:
        f.write(TIMES_HEADER)
        for op, dtype, P, nbytes, best, us, *how in rows:
            f.write(f"{op} {dt[dtype]} {P} {nbytes} {best} {how[0] if how else 'batch'} | " + " ".join(f"{k}={v}" for k, v in us.items()) + "\n")
        if coarse_vs_fine:
            f.write("# one variant per (op, dtype, scale) for every size (the paper's MCR-DL) against one per size (MCR-DL-T):\n"
                    "# sum over the 17 sizes of the time per launch, in microseconds\n")
            for key, v in coarse_vs_fine.items():
                f.write(f"# {key}: best single variant {v['variant']} {v['sum_us']} us, per-size table {v['fine_sum_us']} us "
                        f"(x{v['fine_gain']})\n")


def read_times(path: str):
    """[(op, dtype name, P, bytes, chosen, {variant name: us}, "batch" | "graph")] of a file written by
    write_times; the last field says how the row's launches were timed (back to back from the host,
    or replayed from a captured graph)."""
    rows = []
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            head, tail = line.split("|")
            op, dt, P, nbytes, best, how = head.split()
            rows.append((op, dt, int(P), int(nbytes), best, {k: float(v) for k, v in (kv.split("=") for kv in tail.split())}, how))
    return rows


def run(out_path: str, report_path: str | None, scales, max_bytes: int, arena_gib: float, verbose: bool = True,
        times_path: str | None = None):
    """`scales`: the rank counts (world sizes) to tune the swept collectives for; the table is keyed by
    scale first, then by message size."""
    ctx = mcr.mcr_init(0)
    mcr.mcr_tune_clear(ctx)
    sizes = [m for m in inputs.SWEEP_BYTES if m <= max_bytes]
    names = mcr.mcr_get_variants(ctx, mcr.OP_ALLGATHER)                  # the longest list; a prefix serves the others
    report = {"scales": list(scales), "variants": names, "cells": {}, "coarse_vs_fine": {}}
    for P in scales:
        _tune_sweep(ctx, P, sizes, arena_gib, names, report, verbose)
    report["workload_ops"] = tune_workload_ops(ctx, verbose)
    rows = report.pop("_rows", []) + report["workload_ops"].pop("_rows", [])
    os.makedirs(os.path.dirname(out_path) or ".", exist_ok=True)
    mcr.mcr_tune_save(ctx, out_path)
    if times_path:
        write_times(times_path, rows, report["coarse_vs_fine"])
    if report_path:
        os.makedirs(os.path.dirname(report_path) or ".", exist_ok=True)
        with open(report_path, "w") as f:
            json.dump(report, f, indent=1)
    n = mcr.mcr_tune_count(ctx)
    mcr.mcr_finalize(ctx)
    return n, report


def _tune_sweep(ctx, P: int, sizes, arena_gib: float, names, full_report, verbose: bool):
    cells = sweep.make_cells(P, inputs.SWEEP_OPS, inputs.SWEEP_DTYPES, sizes)
    need = max(c.footprint for c in cells)
    arena = sweep.Arena(max(int(arena_gib * (1 << 30)), need + (1 << 20)))
    report = {"cells": {}}
    for cell in cells:
        variants = variants_of(ctx, sweep.OPS[cell.op])
        reps = reps_for(cell.alg_bytes)
        times = {}
        graph_timed = None
        for v in variants:
            cell.launch(ctx, arena.take(cell.footprint), v)              # first-launch effects out of the way
            ms = sweep.time_launches(lambda: cell.launch(ctx, arena.take(cell.footprint), v), reps)
            if graph_timed is None:
                graph_timed = ms < GRAPH_BELOW_MS                         # one way of timing per cell, decided by its first variant
            if graph_timed:
                # the host's cost per call (8 to 10 us from Python) hides what a kernel this short takes: time the
                # same batch replayed from a captured graph, where only the device's own launch floor is left
                ms = graph_batch_ms(lambda base, stream: cell.launch(ctx, base, v, stream),
                                    [arena.take(cell.footprint) for _ in range(reps)])
            elif ms < 0.1:
                # the least of three batches, which is what the kernel costs when nothing else interferes
                for _ in range(2):
                    ms = min(ms, sweep.time_launches(lambda: cell.launch(ctx, arena.take(cell.footprint), v), reps))
            times[v] = ms
        # least time wins; anything within the tie window of it counts as a tie and the lowest id
        # is taken, so that launch-bound sizes do not pick a variant by noise
        names = names_of(ctx, sweep.OPS[cell.op])
        us = {v: round(times[v] * 1e3, 2) for v in variants}              # ascending ids
        best = pick(us, graph_timed)
        mcr.mcr_tune_set(ctx, sweep.OPS[cell.op], sweep.DTYPES[cell.dtype], P, cell.M, best)
        full_report.setdefault("_rows", []).append((cell.op, sweep.DTYPES[cell.dtype], P, cell.M, names[best],
                                                    {names[v]: t for v, t in us.items()}, "graph" if graph_timed else "batch"))
        report["cells"][cell.key] = {
            "alg_bytes": cell.alg_bytes, "best": names[best],
            "us": {names[v]: round(times[v] * 1e3, 3) for v in variants},
            "GBps": {names[v]: round(cell.alg_bytes / (times[v] * 1e-3) / 1e9, 1) for v in variants},
        }
        if verbose:
            print(f"P={P:2d} {cell.key:34s} best={names[best]:6s} {times[best]*1e3:10.2f} us "
                  f"{cell.alg_bytes / (times[best] * 1e-3) / 1e9:8.1f} GB/s", flush=True)
    # coarse (one variant per op and dtype) versus fine (one per size)
    coarse = {}
    for op in inputs.SWEEP_OPS:
        variants = variants_of(ctx, sweep.OPS[op])
        names = names_of(ctx, sweep.OPS[op])
        for dt in inputs.SWEEP_DTYPES:
            keys = [c.key for c in cells if c.op == op and c.dtype == dt]
            tot = {v: sum(report["cells"][k]["us"][names[v]] for k in keys) for v in variants}
            fine = sum(min(report["cells"][k]["us"].values()) for k in keys)
            bv = min(variants, key=lambda v: (tot[v], v))
            coarse[f"{op}/{dt}"] = {"variant": names[bv], "sum_us": round(tot[bv], 2), "fine_sum_us": round(fine, 2),
                                    "fine_gain": round(tot[bv] / fine, 4)}
    for k, v in report["cells"].items():
        full_report["cells"][f"P{P}/{k}"] = v
    for k, v in coarse.items():
        full_report["coarse_vs_fine"][f"P{P}/{k}"] = v
    del arena
    torch.cuda.empty_cache()


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=DEFAULT_TABLE)
    ap.add_argument("--report", default=None)
    ap.add_argument("--ranks", default="4,8,16", help="rank counts to tune the swept collectives for")
    ap.add_argument("--max-bytes", type=int, default=inputs.SWEEP_BYTES[-1])
    ap.add_argument("--arena-gib", type=float, default=20.0)
    ap.add_argument("--times-out", default=None, help="write every variant's time behind every table row here")
    a = ap.parse_args(argv)
    if not torch.cuda.is_available():
        print("the tuning suite needs a GPU", file=sys.stderr)
        return 2
    n, _ = run(a.out, a.report, [int(x) for x in a.ranks.split(",")], a.max_bytes, a.arena_gib, times_path=a.times_out)
    print(f"wrote {n} rows to {a.out}")
    return 0


if __name__ == "__main__":
    sys.exit(main())
