"""Hardware-counter evidence for the large-message kernels: a fixed list of launches to run under
`rocprofv3 --pmc`, and the summary of what the counters read.

    rocprofv3 --pmc <counters> -d <dir> -o pmc --output-format csv -- \\
        python3 -m paper_2303_08374_amd.counters run [--ops ...] [--mibs 256] [--reps 3]
    python3 -m paper_2303_08374_amd.counters summarize <dir> [<dir> ...] [--ops ...] [--mibs ...] [--reps 3]
                                                       [--out FILE] [--traffic-json FILE]

`run` launches, over buffers the caches have not seen (a cursor walking a large arena), `reps`
times each: first the plain copy of 1 GiB (all_to_all_single at P=1: the kernel of known size that
every reading is compared with), then for every size of `--mibs` (MiB per rank; or `--kibs`) the
`--ops`, fp32 (`allgather_bf16`: all_gather on bf16), through MCR_AUTO with the shipped tuning table: all_reduce, reduce_scatter, all_to_all_single and
all_gather at P=8, and two launches that bracket the read / write mix: reduce_scatter at P=16 on
half the message (16 reads to 1 write) and bcast at P=8 (1 read to 7 writes).  Every launch is one
kernel, so the dispatches of the library's kernels in a run are this list in this order;
`summarize`, given the same options, labels them by that order.  rocprofv3 collects one set of
counters per run; `summarize` reads the `*_counter_collection.csv` of several runs and prints, per
launch kind and size, every counter's mean per dispatch and the rates that follow from them; with
FETCH_SIZE and WRITE_SIZE among the counters it also prints the HBM traffic, each counter scaled by
its reading for the plain copy, next to the algorithmic bytes.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ALL_OPS = ("allreduce", "reduce_scatter", "alltoall", "allgather", "reduce_scatter_P16", "bcast")   # also: "allgather_bf16"
N_XCD = 8            # GRBM_GUI_ACTIVE is summed over the accelerator dies of the MI355X
P = 8
GIB = 1 << 30


def _human(nbytes: int) -> str:
    return f"{nbytes >> 20} MiB" if nbytes % (1 << 20) == 0 else f"{nbytes >> 10} KiB"


def _bytes_of(label: str) -> int:
    _, n, unit = label.split()
    return int(n) << (20 if unit == "MiB" else 10)


def plan(ops, sizes, reps):
    """[(label, algorithmic bytes)] in launch order; `sizes` in bytes per rank."""
    out = [("plain copy 1 GiB (all_to_all_single at P=1)", 2 * GIB)] * reps
    for M in sizes:
        alg = {"allreduce": 2 * P * M, "reduce_scatter": (P + 1) * M, "alltoall": 2 * P * M, "allgather": (P + P * P) * M,
               "allgather_bf16": (P + P * P) * M, "reduce_scatter_P16": 17 * (M // 2), "bcast": P * M}
        for op in ops:
            out += [(f"{op} {_human(M)}", alg[op])] * reps
    return out


def run(ops, sizes, reps: int) -> int:
    import torch
    from . import inputs, mcr, sweep
    if not torch.cuda.is_available():
        print("counters run needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    ctx = mcr.mcr_init(0)
    mcr.mcr_tune_load(ctx, mcr.SHIPPED_TABLE)
    top = max(sizes)
    need = max(2 * GIB, 2 * P * top, (P + P * P) * top if any(o.startswith("allgather") for o in ops) else 0)
    arena = sweep.Arena(need + 2 * GIB, seed=inputs.SWEEP_SEED)
    torch.cuda.synchronize()

    def ptrs(base, k, nbytes):
        return [base + i * nbytes for i in range(k)]

    for _ in range(reps):
        base = arena.take(2 * GIB)
        mcr.mcr_alltoall(ctx, [base + GIB], [base], GIB // 4, mcr.F32, 1, 4)       # v1nt at P=1: a plain copy
    for M in sizes:
        n = M // 4
        for op in ops:
            for _ in range(reps):
                if op == "allreduce":
                    mcr.mcr_allreduce(ctx, ptrs(arena.take(P * M), P, M), n, mcr.F32, mcr.SUM, P)
                elif op == "reduce_scatter":
                    base = arena.take(P * M + M)
                    mcr.mcr_reduce_scatter(ctx, ptrs(base + P * M, P, M // P), ptrs(base, P, M), n, mcr.F32, mcr.SUM, P)
                elif op == "alltoall":
                    base = arena.take(2 * P * M)
                    mcr.mcr_alltoall(ctx, ptrs(base + P * M, P, M), ptrs(base, P, M), n, mcr.F32, P)
                elif op == "allgather":
                    base = arena.take(P * M + P * P * M)
                    mcr.mcr_allgather(ctx, ptrs(base + P * M, P, P * M), ptrs(base, P, M), n, mcr.F32, P)
                elif op == "allgather_bf16":                                       # the table may choose differently per element type
                    base = arena.take(P * M + P * P * M)
                    mcr.mcr_allgather(ctx, ptrs(base + P * M, P, P * M), ptrs(base, P, M), M // 2, mcr.BF16, P)
                elif op == "reduce_scatter_P16":
                    Mh = M // 2                                                    # 16 ranks of half the size: the same input bytes
                    base = arena.take(16 * Mh + Mh)
                    mcr.mcr_reduce_scatter(ctx, ptrs(base + 16 * Mh, 16, Mh // 16), ptrs(base, 16, Mh), Mh // 4, mcr.F32, mcr.SUM, 16)
                elif op == "bcast":
                    mcr.mcr_bcast(ctx, ptrs(arena.take(P * M), P, M), n, mcr.F32, 0, P)
                else:
                    raise SystemExit(f"unknown op {op}")
    torch.cuda.synchronize()
    mcr.mcr_finalize(ctx)
    print(f"counters run: plain copy + {len(ops)} kinds of launch x {len(sizes)} sizes x {reps}")
    return 0


def _short(name: str) -> str:
    name = re.sub(r"^(void )?mcr::\(anonymous namespace\)::", "", name)
    name = re.sub(r"\(mcr::.*$", "", name)
    return re.sub(r"\(.*$", "", name)


def _read(dirs, labels):
    """{label: {"kernel": name, counter: [values per dispatch]}} with the dispatches of the library's
    kernels of every run matched to `labels` by order."""
    vals = collections.OrderedDict()
    groups = []
    for d in dirs:
        files = sorted(glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True))
        if not files:
            raise SystemExit(f"no *_counter_collection.csv under {d}")
        per_dispatch = collections.OrderedDict()
        for path in files:
            with open(path) as f:
                for r in csv.DictReader(f):
                    if "mcr::" in r["Kernel_Name"]:
                        per_dispatch.setdefault(int(r["Dispatch_Id"]), []).append(r)
        order = sorted(per_dispatch)
        seen = []
        for rows in per_dispatch.values():
            for r in rows:
                if r["Counter_Name"] not in seen:
                    seen.append(r["Counter_Name"])
        groups.append(seen)
        if len(order) != len(labels):
            raise SystemExit(f"{d}: {len(order)} library dispatches, the launch list has {len(labels)}: pass the options of the run")
        for disp, (label, _) in zip(order, labels):
            for r in per_dispatch[disp]:
                e = vals.setdefault(label, collections.OrderedDict())
                e["kernel"] = _short(r["Kernel_Name"])
                e.setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    return vals, groups


def summarize(dirs, ops, sizes, reps, out_path, traffic_json, opts):
    labels = plan(ops, sizes, reps)
    alg = dict(labels)
    vals, groups = _read(dirs, labels)
    lines = ["Hardware counters of the library's kernels on one MI355X, fp32, MCR_AUTO with the shipped tuning table, cold buffers.",
             "Commands (from /tmp, TMPDIR=/tmp; rocprofv3 collects one group of counters per run):"]
    for i, g in enumerate(groups):
        lines.append(f"  rocprofv3 --pmc {' '.join(g)} -d pmc_{i} -o pmc --output-format csv -- python3 -m paper_2303_08374_amd.counters run {opts}")
    lines.append(f"  python3 -m paper_2303_08374_amd.counters summarize {' '.join(f'pmc_{i}' for i in range(len(groups)))} {opts}")
    lines += ["", "per dispatch: mean over the dispatches of each launch (the first one left out)", ""]
    mean = collections.OrderedDict()
    for label, per in vals.items():
        m = collections.OrderedDict()
        for c, v in per.items():
            if c == "kernel":
                continue
            vv = v[1:] if len(v) > 1 else v
            m[c] = sum(vv) / len(vv)
        mean[label] = m
    copy = mean[labels[0][0]]
    scale = {c: (GIB / 1024.0) / copy[c] for c in ("FETCH_SIZE", "WRITE_SIZE") if copy.get(c)}
    for c, s in scale.items():
        lines.append(f"{c}: the plain copy of 1 GiB reads {copy[c]:.1f} KiB per dispatch, expected 1048576: scale factor {s:.5f}")
    if scale:
        lines.append("")
    traffic = {}
    for label, m in mean.items():
        lines.append(f"{label}   [{vals[label]['kernel']}]")
        for c, v in m.items():
            lines.append(f"    {c:44s} {v:18.1f}")
        if len(scale) == 2 and "FETCH_SIZE" in m and "WRITE_SIZE" in m:
            fe, wr = m["FETCH_SIZE"] * scale["FETCH_SIZE"] * 1024, m["WRITE_SIZE"] * scale["WRITE_SIZE"] * 1024
            traffic[label] = round(fe + wr)
            lines.append(f"    -> HBM traffic: {fe / GIB:.3f} GiB fetched + {wr / GIB:.3f} GiB written = {(fe + wr) / GIB:.3f} GiB; "
                         f"algorithmic {alg[label] / GIB:.3f} GiB; ratio {(fe + wr) / alg[label]:.3f}")
        for k, v in _derived(m):
            lines.append(f"    -> {k:66s} {v}")
        lines.append("")
    text = "\n".join(lines)
    if out_path:
        with open(out_path, "w") as f:
            f.write(text + "\n")
    if traffic_json:
        sys.path.insert(0, os.path.dirname(HERE))
        import bench
        per_size = {str(_bytes_of(label)): t for label, t in traffic.items()
                    if label.startswith("allgather") and "superchunk" in vals[label]["kernel"]}
        with open(traffic_json, "w") as f:
            json.dump({"sources_digest": bench.kernel_sources_digest(), "scale": {c: round(s, 5) for c, s in scale.items()},
                       "kernels": {"allgather/superchunk": per_size}}, f, indent=1)
    print(text)
    return 0


def _derived(m):
    """Rates that need two counters of the same run; per cycle of one accelerator die."""
    out = []
    g = m.get("GRBM_GUI_ACTIVE")
    cyc = g / N_XCD if g else None

    def have(*names):
        return all(n in m and m[n] > 0 for n in names)
    if have("TCC_EA0_RDREQ_sum", "TCC_EA0_RDREQ_LEVEL_sum"):
        out.append(("mean read latency L2 -> memory, cycles (RDREQ_LEVEL / RDREQ)", f"{m['TCC_EA0_RDREQ_LEVEL_sum'] / m['TCC_EA0_RDREQ_sum']:.0f}"))
    if have("TCC_EA0_WRREQ_sum", "TCC_EA0_WRREQ_LEVEL_sum"):
        out.append(("mean write latency L2 -> memory, cycles (WRREQ_LEVEL / WRREQ)", f"{m['TCC_EA0_WRREQ_LEVEL_sum'] / m['TCC_EA0_WRREQ_sum']:.0f}"))
    if cyc:
        out.append(("kernel cycles (GRBM_GUI_ACTIVE / 8 dies)", f"{cyc:.0f}"))
        for name, what in (("TCC_EA0_RDREQ_sum", "read requests L2 -> memory per cycle, whole chip"),
                           ("TCC_EA0_WRREQ_sum", "write requests L2 -> memory per cycle, whole chip"),
                           ("TCC_EA0_RDREQ_LEVEL_sum", "read requests in flight L2 -> memory, whole chip (mean)"),
                           ("TCC_EA0_WRREQ_LEVEL_sum", "write requests in flight L2 -> memory, whole chip (mean)"),
                           ("TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum", "L2 channels (of 128) stalled for a read credit, mean"),
                           ("TCC_EA0_WRREQ_DRAM_CREDIT_STALL_sum", "L2 channels (of 128) stalled for a write credit, mean"),
                           ("TCC_TAG_STALL_sum", "L2 channels (of 128) in a tag stall, mean"),
                           ("TCC_REQ_sum", "L2 requests per cycle, whole chip"),
                           ("TCP_PENDING_STALL_CYCLES_sum", "vector L1s (of 256) waiting for data from L2, mean"),
                           ("TA_DATA_STALLED_BY_TC_CYCLES_sum", "address units (of 256) whose store data the L1 does not take, mean"),
                           ("TA_ADDR_STALLED_BY_TC_CYCLES_sum", "address units (of 256) whose addresses the L1 does not take, mean"),
                           ("TCP_TCC_READ_REQ_sum", "read requests L1 -> L2 per cycle and compute unit"),
                           ("TCP_TCC_WRITE_REQ_sum", "write requests L1 -> L2 per cycle and compute unit")):
            if name in m:
                v = m[name] / cyc
                if name.startswith("TCP_TCC_"):
                    v /= 256.0
                out.append((what, f"{v:.4f}" if v < 1 else f"{v:.1f}"))
    if have("SQ_WAVE_CYCLES", "SQ_BUSY_CYCLES"):
        out.append(("wavefronts resident per busy SQ cycle (WAVE_CYCLES / BUSY_CYCLES)", f"{m['SQ_WAVE_CYCLES'] / m['SQ_BUSY_CYCLES']:.1f}"))
    if have("SQ_WAIT_INST_ANY", "SQ_WAVE_CYCLES"):
        out.append(("share of wavefront cycles spent waiting for an instruction's data", f"{m['SQ_WAIT_INST_ANY'] / m['SQ_WAVE_CYCLES']:.3f}"))
    if have("TCP_TCC_READ_REQ_sum", "TCP_TCC_READ_REQ_LATENCY_sum"):
        lat = m["TCP_TCC_READ_REQ_LATENCY_sum"] / m["TCP_TCC_READ_REQ_sum"]
        out.append(("mean read latency seen by the vector L1, cycles", f"{lat:.0f}"))
        if cyc:
            out.append(("read requests in flight per compute unit (rate x latency)", f"{m['TCP_TCC_READ_REQ_sum'] / cyc / 256.0 * lat:.0f}"))
    if have("TCP_TCC_WRITE_REQ_sum", "TCP_TCC_WRITE_REQ_LATENCY_sum"):
        lat = m["TCP_TCC_WRITE_REQ_LATENCY_sum"] / m["TCP_TCC_WRITE_REQ_sum"]
        out.append(("mean write latency seen by the vector L1, cycles", f"{lat:.0f}"))
        if cyc:
            out.append(("write requests in flight per compute unit (rate x latency)", f"{m['TCP_TCC_WRITE_REQ_sum'] / cyc / 256.0 * lat:.0f}"))
    return out


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    for name in ("run", "summarize"):
        s = sub.add_parser(name)
        s.add_argument("--ops", default=",".join(ALL_OPS))
        s.add_argument("--mibs", default="256", help="message sizes per rank in MiB")
        s.add_argument("--kibs", default=None, help="message sizes per rank in KiB (instead of --mibs)")
        s.add_argument("--reps", type=int, default=3)
        if name == "summarize":
            s.add_argument("dirs", nargs="+")
            s.add_argument("--out", default=None)
            s.add_argument("--traffic-json", default=None,
                           help="write the all_gather traffic per message size here, for bench.py's roofline.traffic")
    a = ap.parse_args(argv)
    ops = [o for o in a.ops.split(",") if o]
    sizes = [int(x) << 10 for x in a.kibs.split(",")] if a.kibs else [int(x) << 20 for x in a.mibs.split(",")]
    if a.cmd == "run":
        return run(ops, sizes, a.reps)
    opts = f"--ops {','.join(ops)} " + (f"--kibs {a.kibs}" if a.kibs else f"--mibs {a.mibs}") + f" --reps {a.reps}"
    return summarize(a.dirs, ops, sizes, a.reps, a.out, a.traffic_json, opts)


if __name__ == "__main__":
    sys.exit(main())
