"""Hardware-counter evidence for the large-message kernels: a short, fixed list of launches to run
under `rocprofv3 --pmc`, and the summary of what the counters read.

    rocprofv3 --pmc <counters> -d <dir> -o pmc --output-format csv -- \\
        python3 -m paper_2303_08374_amd.counters run [--mib 256] [--reps 3]
    python3 -m paper_2303_08374_amd.counters summarize <dir> [<dir> ...] [--out FILE]

`run` launches, over buffers the caches have not seen (a cursor walking a large arena), `reps`
times each: the plain copy of 1 GiB (all_to_all_single at P=1: the kernel of known size every
reading is compared with), then at P=8 and `mib` MiB per rank, fp32, through MCR_AUTO with the
shipped tuning table: all_reduce, reduce_scatter, all_to_all_single, all_gather, and two launches
that bracket the read/write mix: reduce_scatter at P=16 (16 reads to 1 write) and bcast at P=8
(1 read to 7 writes).  rocprofv3 collects one set of counters per run; `summarize` reads the
`*_counter_collection.csv` of several runs and prints, per kernel, every counter's mean per
dispatch and the rates that follow from them.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import os
import re
import sys

HERE = os.path.dirname(os.path.abspath(__file__))

# label -> what is launched; the summary names kernels by the label whose launch produced them
LAUNCHES = ("copy_1GiB_P1", "allreduce", "reduce_scatter", "alltoall", "allgather", "reduce_scatter_P16", "bcast")


def run(mib: int, reps: int) -> int:
    import torch
    from . import inputs, mcr, sweep
    if not torch.cuda.is_available():
        print("counters run needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    ctx = mcr.mcr_init(0)
    mcr.mcr_tune_load(ctx, mcr.SHIPPED_TABLE)
    M = mib << 20
    P = 8
    n = M // 4
    arena = sweep.Arena(max(P * (M + P * M), 2 << 30) + (2 << 30), seed=inputs.SWEEP_SEED)
    torch.cuda.synchronize()

    def ptrs(base, k, nbytes):
        return [base + i * nbytes for i in range(k)]

    for _ in range(reps):
        base = arena.take(2 << 30)
        mcr.mcr_alltoall(ctx, [base + (1 << 30)], [base], (1 << 30) // 4, mcr.F32, 1, 4)       # v1nt at P=1: a plain copy
    for _ in range(reps):
        mcr.mcr_allreduce(ctx, ptrs(arena.take(P * M), P, M), n, mcr.F32, mcr.SUM, P)
    for _ in range(reps):
        base = arena.take(P * M + M)
        mcr.mcr_reduce_scatter(ctx, ptrs(base + P * M, P, M // P), ptrs(base, P, M), n, mcr.F32, mcr.SUM, P)
    for _ in range(reps):
        base = arena.take(2 * P * M)
        mcr.mcr_alltoall(ctx, ptrs(base + P * M, P, M), ptrs(base, P, M), n, mcr.F32, P)
    for _ in range(reps):
        base = arena.take(P * M + P * P * M)
        mcr.mcr_allgather(ctx, ptrs(base + P * M, P, P * M), ptrs(base, P, M), n, mcr.F32, P)
    Mh = M // 2                                                                          # 16 ranks of half the size: same input bytes
    for _ in range(reps):
        base = arena.take(16 * Mh + Mh)
        mcr.mcr_reduce_scatter(ctx, ptrs(base + 16 * Mh, 16, Mh // 16), ptrs(base, 16, Mh), Mh // 4, mcr.F32, mcr.SUM, 16)
    for _ in range(reps):
        mcr.mcr_bcast(ctx, ptrs(arena.take(P * M), P, M), n, mcr.F32, 0, P)
    torch.cuda.synchronize()
    mcr.mcr_finalize(ctx)
    print(f"counters run: {len(LAUNCHES)} kinds of launch x {reps}, {mib} MiB per rank")
    return 0


def _short(name: str) -> str:
    name = re.sub(r"void mcr::\(anonymous namespace\)::", "", name)
    name = re.sub(r"\(mcr::.*$", "", name)
    name = re.sub(r"\(.*$", "", name)
    return name


def _read(dirs):
    """{kernel: {counter: [values per dispatch]}}, {kernel: [durations ns]}, kernel order, grid sizes."""
    vals = collections.OrderedDict()
    for d in dirs:
        files = sorted(glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True))
        if not files:
            raise SystemExit(f"no *_counter_collection.csv under {d}")
        for path in files:
            with open(path) as f:
                for r in csv.DictReader(f):
                    if "mcr::" not in r["Kernel_Name"]:
                        continue
                    key = (_short(r["Kernel_Name"]), int(r["Grid_Size"]))
                    vals.setdefault(key, collections.OrderedDict()).setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    return vals


def _label(kernel: str, grid: int, copy_grid: int) -> str:
    if kernel.startswith("alltoall_kernel") and grid == copy_grid:
        return "plain copy, 1 GiB (all_to_all_single at P=1)"
    return kernel


def summarize(dirs, out_path):
    vals = _read(dirs)
    lines = []
    counters = []
    for per in vals.values():
        for c in per:
            if c not in counters:
                counters.append(c)
    copy_grid = (1 << 30) // 16                                        # one 16-byte vector per thread
    lines.append("per dispatch: mean over the dispatches of each kernel (the first dispatch of a kernel is left out when there are more)")
    lines.append("")
    for (kernel, grid), per in vals.items():
        lines.append(f"{_label(kernel, grid, copy_grid)}   grid {grid} threads")
        mean = {}
        for c in counters:
            if c not in per:
                continue
            v = per[c][1:] if len(per[c]) > 1 else per[c]
            mean[c] = sum(v) / len(v)
            lines.append(f"    {c:44s} {mean[c]:18.1f}   (n={len(v)})")
        derived = _derived(mean)
        for k, v in derived:
            lines.append(f"    -> {k:50s} {v}")
        lines.append("")
    text = "\n".join(lines)
    if out_path:
        with open(out_path, "w") as f:
            f.write(text + "\n")
    print(text)
    return 0


def _derived(m):
    """Rates that need two counters of the same run."""
    out = []
    g = m.get("GRBM_GUI_ACTIVE")

    def have(*names):
        return all(n in m and m[n] > 0 for n in names)
    if have("TCC_EA0_RDREQ_sum", "TCC_EA0_RDREQ_LEVEL_sum"):
        out.append(("mean read latency seen by L2, cycles (RDREQ_LEVEL / RDREQ)", f"{m['TCC_EA0_RDREQ_LEVEL_sum'] / m['TCC_EA0_RDREQ_sum']:.0f}"))
    if have("TCC_EA0_WRREQ_sum", "TCC_EA0_WRREQ_LEVEL_sum"):
        out.append(("mean write latency seen by L2, cycles (WRREQ_LEVEL / WRREQ)", f"{m['TCC_EA0_WRREQ_LEVEL_sum'] / m['TCC_EA0_WRREQ_sum']:.0f}"))
    if g:
        for name, what in (("TCC_EA0_RDREQ_sum", "read requests per active cycle (all L2 channels)"),
                           ("TCC_EA0_WRREQ_sum", "write requests per active cycle (all L2 channels)"),
                           ("TCC_EA0_RDREQ_LEVEL_sum", "read requests in flight, L2 to memory (mean)"),
                           ("TCC_EA0_WRREQ_LEVEL_sum", "write requests in flight, L2 to memory (mean)"),
                           ("TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum", "read credit-stall cycles per active cycle, summed over channels"),
                           ("TCC_EA0_WRREQ_DRAM_CREDIT_STALL_sum", "write credit-stall cycles per active cycle, summed over channels"),
                           ("TCC_EA0_WRREQ_STALL_sum", "write-request stall cycles per active cycle, summed over channels"),
                           ("TCC_TOO_MANY_EA_WRREQS_STALL_sum", "too-many-writes stall cycles per active cycle, summed over channels"),
                           ("TCC_TAG_STALL_sum", "tag stall cycles per active cycle, summed over channels"),
                           ("TCC_REQ_sum", "L2 requests per active cycle (all channels)"),
                           ("SQ_BUSY_CYCLES", "SQ busy cycles per active cycle")):
            if name in m:
                out.append((what, f"{m[name] / g:.3f}"))
    if have("SQ_WAVE_CYCLES", "SQ_BUSY_CYCLES"):
        out.append(("wavefronts resident per busy SQ cycle (WAVE_CYCLES / BUSY_CYCLES)", f"{m['SQ_WAVE_CYCLES'] / m['SQ_BUSY_CYCLES']:.2f}"))
    if have("SQ_WAIT_INST_ANY", "SQ_WAVE_CYCLES"):
        out.append(("share of wavefront cycles spent waiting for an instruction's data", f"{m['SQ_WAIT_INST_ANY'] / m['SQ_WAVE_CYCLES']:.3f}"))
    if have("TCP_TCC_READ_REQ_sum", "TCP_TCC_READ_REQ_LATENCY_sum"):
        out.append(("mean read latency seen by the vector L1, cycles", f"{m['TCP_TCC_READ_REQ_LATENCY_sum'] / m['TCP_TCC_READ_REQ_sum']:.0f}"))
    if have("TCP_TCC_WRITE_REQ_sum", "TCP_TCC_WRITE_REQ_LATENCY_sum"):
        out.append(("mean write latency seen by the vector L1, cycles", f"{m['TCP_TCC_WRITE_REQ_LATENCY_sum'] / m['TCP_TCC_WRITE_REQ_sum']:.0f}"))
    return out


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    r = sub.add_parser("run")
    r.add_argument("--mib", type=int, default=256)
    r.add_argument("--reps", type=int, default=3)
    s = sub.add_parser("summarize")
    s.add_argument("dirs", nargs="+")
    s.add_argument("--out", default=None)
    a = ap.parse_args(argv)
    if a.cmd == "run":
        return run(a.mib, a.reps)
    return summarize(a.dirs, a.out)


if __name__ == "__main__":
    sys.exit(main())
