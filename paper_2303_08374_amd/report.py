"""Text summaries of bench.py's measurements (the tables kept under profiles/).

    python3 bench.py --cells-out CELLS.json --cells-md profiles/op_sweep_cells.md   # per-cell table + workloads
    rocprofv3 --kernel-trace --output-format csv -d DIR -o trace -- python3 bench.py --trace-passes 5
    python3 -m paper_2303_08374_amd.report kernel-times DIR --passes 5 --cells CELLS.json \\
        --out profiles/op_sweep_kernel_times.md                       # kernel-only durations per cell
"""
from __future__ import annotations

import argparse
import csv
import glob
import json
import os
import re
import sys

from . import inputs, sweep

OPS = ["allreduce", "reduce_scatter", "allgather", "alltoall"]


def human(b: int) -> str:
    return f"{b >> 20} MiB" if b >= 1 << 20 else f"{b >> 10} KiB"


def cells_markdown(cells: dict, line: dict, command: str) -> str:
    """`cells`: bench.py's per-cell table; `line`: the JSON line it printed."""
    out = ["# Op sweep on one MI355X: per-cell results of bench.py", "",
           f"Command: `{command}` (P=8 simulated ranks, MCR_AUTO dispatch with the shipped tuning table, cold buffers: every",
           "launch takes its rank buffers from a cursor walking a 20 GiB arena; median of 5 passes, events on the launch stream).",
           "GB/s = algorithmic bytes / time; % = of 8000 GB/s. Message size M = one rank's send buffer.", ""]
    ceil = line.get("ceilings")
    if ceil:
        out += ["Ceilings measured in the same run with library calls (cold buffers, median of 5 launches):", ""]
        for k, v in ceil.items():
            out.append(f"- {k}: {v['GBps']} GB/s ({v['what']})")
        out.append("")
    per_op = line.get("roofline_per_op")
    if per_op:
        out += ["Messages of 16 MiB per rank and more, per op and element type (bytes summed / times summed):", "",
                "| op / dtype | GB/s | % of 8000 GB/s | % of the copy ceiling | worst cell | best cell |", "|---|---|---|---|---|---|"]
        for k, v in per_op.items():
            out.append(f"| {k} | {v['GBps']} | {100 * v['frac_of_peak']:.1f} | {100 * v['frac_of_copy_ceiling']:.1f} | "
                       f"{100 * v['min_frac']:.1f} % | {100 * v['max_frac']:.1f} % |")
        out += ["", f"Worst of them: {line.get('worst_op')}.", ""]
    for dt in ("f32", "bf16"):
        out += ["", f"## {dt}", "",
                "| M per rank | " + " | ".join(f"{o} variant | us | GB/s | %" for o in OPS) + " |",
                "|" + "---|" * (1 + 4 * len(OPS))]
        sizes = sorted({int(k.split("/")[2]) for k in cells if k.split("/")[1] == dt})
        for m in sizes:
            row = [human(m)]
            for o in OPS:
                c = cells[f"{o}/{dt}/{m}"]
                row += [c["variant"], f"{c['us']:.1f}", f"{c['GBps']:.0f}", f"{100 * c['frac_of_peak']:.1f}"]
            out.append("| " + " | ".join(row) + " |")
    st = line.get("stages")
    if st:
        out += ["", "", "## Application-shaped workloads (same run)", ""] + _stage_lines(st)
    cb = line.get("cpu_baseline")
    if cb:
        out += ["", f"CPU oracle beside it: {cb['value']} GB/s on {cb['cores']} core ({cb['sample']}).", ""]
    return "\n".join(out) + "\n"


def _sg(d):
    return f"{d['us']} us" + (f", {d['GBps']} GB/s" if d.get("GBps") else "")


def _stage_lines(st: dict):
    m, d, g, sm = st["moe_dispatch_combine"], st["dlrm_shuffle"], st["grad_buckets"], st["small_tensor_path"]
    a = st["allreduce_small"]
    gr = st["small_cells_graph_replay"]
    lines = [
        f"- small allreduce (P=4, 2^20 fp32, 32 MiB traffic): cold {_sg(a['cold'])}; warm (cache resident, not an HBM figure) {_sg(a['warm'])}",
        f"- MoE (P=16, T=16384, H=2048 bf16, E=64, Zipf 1.2, C=320, kept {m['kept_fraction']}): route {m['route']['us']} us; pack {_sg(m['pack'])}; "
        f"alltoallv dispatch {_sg(m['alltoallv_dispatch'])}; alltoallv return {_sg(m['alltoallv_return'])}; unpack+combine {_sg(m['unpack_combine'])}; "
        f"chain end to end {_sg(m['end_to_end'])}",
        f"  - fused: moe_dispatch {_sg(m['fused']['moe_dispatch'])}; moe_combine {_sg(m['fused']['moe_combine'])}; end to end {_sg(m['fused']['end_to_end'])} "
        f"= {m['fused']['speedup_vs_chain']}x the chain",
        f"  - expert-major receive layout: expert_layout {m['by_expert']['expert_layout']['us']} us; dispatch {_sg(m['by_expert']['moe_dispatch_by_expert'])}; "
        f"combine {_sg(m['by_expert']['moe_combine_by_expert'])}; end to end {_sg(m['by_expert']['end_to_end'])}",
        f"  - the chain's own (source-major) layout through the table-driven calls: source_layout {m['source_major_by_table']['source_layout']['us']} us; "
        f"dispatch {_sg(m['source_major_by_table']['moe_dispatch_by_expert'])}; combine {_sg(m['source_major_by_table']['moe_combine_by_expert'])}; "
        f"end to end {_sg(m['source_major_by_table']['end_to_end'])} = {m['source_major_by_table']['speedup_vs_chain']}x the chain",
        f"  - top-2 gating on the same tokens (capacity 640, kept {m['top2']['kept_fraction']}): route {m['top2']['route']['us']} us; "
        f"dispatch {_sg(m['top2']['moe_dispatch_by_expert'])}; combine {_sg(m['top2']['moe_combine_by_expert'])}; end to end {_sg(m['top2']['end_to_end'])}",
    ]
    if "odd_rows" in m:
        o = m["odd_rows"]
        lines.append(f"  - the same workload with H = {o['H']} (rows of {o['row_bytes']} bytes, not a multiple of 16): " +
                     "; ".join(f"{k} {_sg(v)} ({v['vs_aligned']}x the H = 2048 time)" for k, v in o["stages"].items()))
    lines += [
        f"- DLRM shuffle (P=8, 26 tables x [16384,128] fp32): fwd pack {_sg(d['fwd_pack_send_order'])}, alltoallv {_sg(d['fwd_alltoallv'])}, "
        f"unpack {_sg(d['fwd_unpack_permute'])}; bwd {_sg(d['bwd_pack_permute'])}, {_sg(d['bwd_alltoallv'])}, {_sg(d['bwd_unpack_table_order'])}; "
        f"chain end to end {_sg(d['end_to_end'])}",
        f"  - fused single pass: fwd {_sg(d['fused']['fwd_dlrm_shuffle'])}; bwd {_sg(d['fused']['bwd_dlrm_shuffle'])}; end to end {_sg(d['fused']['end_to_end'])} "
        f"= {d['fused']['speedup_vs_chain']}x the chain",
    ]
    if "odd_rows" in d:
        o = d["odd_rows"]
        lines.append(f"  - the same workload with dim = {o['dim']} (rows of {o['row_bytes']} bytes, not a multiple of 16): " +
                     "; ".join(f"{k} {_sg(v)} ({v['per_byte_vs_aligned']}x the time per byte of dim = 128)" for k, v in o["stages"].items()))
    lines += [
        f"- gradient buckets ({g['tensors']} bf16 tensors, {g['elements_per_rank'] / 1e9:.3f} G elements per rank, P=8, {g['buckets']} buckets; minimum traffic "
        f"{g['fuse']['alg_bytes'] / 1e9:.1f} GB = {g['fuse']['alg_bytes'] / 8e6:.0f} us at 8 TB/s): fuse {_sg(g['fuse'])}; allreduce(flat, AVG) {_sg(g['allreduce_flat'])}; "
        f"unfuse {_sg(g['unfuse'])}; pipeline of {g['pipeline_fuse_allreduce_unfuse']['launches']} launches {g['pipeline_fuse_allreduce_unfuse']['us']} us; "
        f"multi-tensor allreduce in one launch {_sg(g['allreduce_multi_one_launch'])}; one launch per tensor {_sg(g['allreduce_per_tensor'])}",
        f"- small-message path: the {sm['tensors']} gradients of at most 8192 elements ({sm['bytes_per_rank']} bytes per rank): one fused launch "
        f"{sm['allreduce_multi_one_launch_us']} us vs one launch per tensor {sm['allreduce_per_tensor_us']} us ({sm['speedup']}x)",
        "- dispatch overhead of all_to_all_single through MCR_AUTO against bare launches of the same kernel (C loop inside the library): "
        + "; ".join(f"{human(int(k))}: dispatch layer alone {v['dispatch_only_us']} us per call = "
                    f"{round(100 * v['dispatch_only_us'] / min(v['auto_us'], v['direct_us']), 2)} % of one operation; end to end through the entry point vs "
                    f"bare launches {v['auto_us']} vs {v['direct_us']} us" for k, v in st["dispatch_overhead_alltoall"].items()),
    ]
    rc = st.get("rooted_collectives")
    if rc:
        lines.append(f"- rooted and vector collectives (P={rc['P']}, fp32, {human(rc['bytes_per_rank'])} per rank, cold buffers): " +
                     "; ".join(f"{k} {_sg(rc[k])}" for k in ("reduce", "bcast", "gather", "scatter", "allgatherv")))
    lines += [
        f"- HIP graph: the {gr['launches']} sweep cells of at most 1 MiB per rank issued call by call from Python {gr['eager_us']} us "
        f"({gr['eager_us_per_launch']} us per launch), replayed from one captured graph {gr['graph_us']} us ({gr['graph_us_per_launch']} us per launch)",
    ]
    return lines


def kernel_times(trace_dir: str, passes: int, cells_json: str | None) -> str:
    """Kernel-only duration of every sweep cell from a rocprofv3 kernel trace of
    `bench.py --trace-passes N`: that run ends with N passes over the cells in a fixed order, one
    kernel per cell, so the last N * (number of cells) library kernels of the trace are those
    passes; the median over the passes is reported next to the event-pair time of the cell table."""
    files = sorted(glob.glob(os.path.join(trace_dir, "**", "*kernel_trace.csv"), recursive=True))
    if not files:
        raise SystemExit(f"no *_kernel_trace.csv under {trace_dir}")
    rows = []
    with open(files[0]) as f:
        for r in csv.DictReader(f):
            if "mcr::" in r["Kernel_Name"]:
                rows.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), r["Kernel_Name"]))
    rows.sort()
    cells = sweep.make_cells(inputs.SWEEP_P, inputs.SWEEP_OPS, inputs.SWEEP_DTYPES, inputs.SWEEP_BYTES)
    n = len(cells)
    if len(rows) < passes * n:
        raise SystemExit(f"the trace holds {len(rows)} library kernels, fewer than {passes} passes of {n} cells")
    rows = rows[-passes * n:]
    table = json.load(open(cells_json)) if cells_json else {}
    out = ["# Op sweep: kernel-only durations per cell (rocprofv3 kernel trace)", "",
           f"Commands: `rocprofv3 --kernel-trace --output-format csv -d DIR -o trace -- python3 bench.py --trace-passes {passes}`, then",
           f"`python3 -m paper_2303_08374_amd.report kernel-times DIR --passes {passes} --cells CELLS.json`.",
           "Median over the passes of the kernel's own begin-to-end time; \"events\" is the event-pair time of the same cell in",
           "`op_sweep_cells.md` (two events around one launch cost about 6 us by themselves, which is all a small cell shows there).",
           "GB/s and % of 8000 GB/s from the kernel-only time.", ""]
    for dt in inputs.SWEEP_DTYPES:
        out += ["", f"## {dt}", "", "| M per rank | " + " | ".join(f"{o} kernel us | events us | GB/s | %" for o in OPS) + " |",
                "|" + "---|" * (1 + 4 * len(OPS))]
        for m in inputs.SWEEP_BYTES:
            line = [human(m)]
            for o in OPS:
                i = next(k for k, c in enumerate(cells) if c.op == o and c.dtype == dt and c.M == m)
                durs = sorted(rows[p * n + i][1] - rows[p * n + i][0] for p in range(passes))
                us = durs[len(durs) // 2] / 1e3
                gbps = cells[i].alg_bytes / us / 1e3
                ev = table.get(cells[i].key, {}).get("us")
                line += [f"{us:.1f}", f"{ev:.1f}" if ev is not None else "-", f"{gbps:.0f}", f"{gbps / 80:.1f}"]
            out.append("| " + " | ".join(line) + " |")
    return "\n".join(out) + "\n"


def _short_kernel(n: str) -> str:
    n = n.replace("void ", "").replace("mcr::(anonymous namespace)::", "")
    return re.sub(r"\(.*$", "", n)


def kernel_stats(stats_dir: str, log_path: str, command: str, what: str) -> str:
    """The library's kernels of a `rocprofv3 --kernel-trace --stats` run of bench.py (calls, average,
    least and largest duration, share of the library's kernel time) and, from the JSON line bench.py
    printed in that run, what its own events measured for the dominant kernel."""
    files = sorted(glob.glob(os.path.join(stats_dir, "**", "*kernel_stats.csv"), recursive=True))
    if not files:
        raise SystemExit(f"no *_kernel_stats.csv under {stats_dir}")
    with open(files[0]) as f:
        rows = [r for r in csv.DictReader(f) if "mcr::" in r["Name"]]
    line = None
    with open(log_path) as f:
        for l in f:
            if l.startswith('{"metric"'):
                line = json.loads(l)
    out = [f"rocprofv3 kernel statistics of {what}, one MI355X.", "", "command (from /tmp, TMPDIR=/tmp):", f"  {command}", "",
           f"{'kernel':84s} {'calls':>6s} {'avg_us':>10s} {'min_us':>9s} {'max_us':>10s} {'share%':>7s}"]
    tot = sum(int(r["TotalDurationNs"]) for r in rows)
    for r in rows:
        share = 100.0 * int(r["TotalDurationNs"]) / tot
        if share < 0.05:
            continue
        out.append(f"{_short_kernel(r['Name'])[:84]:84s} {r['Calls']:>6s} {float(r['AverageNs']) / 1e3:10.2f} {int(r['MinNs']) / 1e3:9.2f} "
                   f"{int(r['MaxNs']) / 1e3:10.2f} {share:7.2f}")
    if line:
        rl = line["roofline"]
        out += ["", f"bench.py in the same run (events on the launch stream, timed region only): dominant kernel {rl['kernel']}, "
                    f"{rl['launches']} launches, average {rl['avg_launch_us']} us, {rl['avg_launch_alg_bytes']} algorithmic bytes per launch on "
                    f"average => {rl['achieved']} GB/s = {rl['frac']} of 8000 GB/s.",
                f"whole step: {line['ms_per_step']} ms for {line['config']['algorithmic_bytes_per_step']} algorithmic bytes => {line['value']} GB/s."]
        st = line.get("stages")
        if st:
            m = st["moe_dispatch_combine"]
            out += ["", "bench.py's own stage times in the same run (events around each call, us): "
                        f"pack {m['pack']['us']}, all_to_allv {m['alltoallv_dispatch']['us']} / {m['alltoallv_return']['us']}, unpack + combine {m['unpack_combine']['us']}; "
                        f"fused pair: dispatch {m['fused']['moe_dispatch']['us']}, combine {m['fused']['moe_combine']['us']}; "
                        f"by expert: dispatch {m['by_expert']['moe_dispatch_by_expert']['us']}, combine {m['by_expert']['moe_combine_by_expert']['us']}; "
                        f"top-2: dispatch {m['top2']['moe_dispatch_by_expert']['us']}, combine {m['top2']['moe_combine_by_expert']['us']}; "
                        f"DLRM fused shuffle fwd {st['dlrm_shuffle']['fused']['fwd_dlrm_shuffle']['us']}, bwd {st['dlrm_shuffle']['fused']['bwd_dlrm_shuffle']['us']}; "
                        f"allreduce_multi {st['grad_buckets']['allreduce_multi_one_launch']['us']}."]
    return "\n".join(out) + "\n"


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    ks = sub.add_parser("kernel-stats")
    ks.add_argument("stats_dir")
    ks.add_argument("--log", required=True, help="stdout of the profiled bench.py run")
    ks.add_argument("--command", required=True, help="the full profiling command, for the header")
    ks.add_argument("--what", default="the op sweep (bench.py)")
    ks.add_argument("--out", default=None)
    k = sub.add_parser("kernel-times")
    k.add_argument("trace_dir")
    k.add_argument("--passes", type=int, required=True)
    k.add_argument("--cells", default=None)
    k.add_argument("--out", default=None)
    a = ap.parse_args(argv)
    if a.cmd == "kernel-stats":
        text = kernel_stats(a.stats_dir, a.log, a.command, a.what)
    else:
        text = kernel_times(a.trace_dir, a.passes, a.cells)
    if a.out:
        with open(a.out, "w") as f:
            f.write(text)
    print(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
