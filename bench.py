#!/usr/bin/env python3
"""Benchmark of the collectives' local data movement on one MI355X.

A step is one pass of the op sweep: allreduce, reduce_scatter, allgather and equal-split
alltoall over P=8 simulated ranks, fp32 and bf16 (fp32 accumulate), per-rank message sizes
4 KiB ... 256 MiB, every call dispatched through MCR_AUTO (the static tuning table).  Inputs
are synthetic (uniform[-1,1)), resident in HBM before the clock starts, and every launch
takes buffers the caches have not seen for gigabytes of traffic.

Prints ONE JSON line: whole-step effective GB/s (algorithmic bytes / time), the roofline of
the kernel that dominates the step (measured with events on the launch stream inside the
timed region), the rate of every (op, element type) group on messages of 16 MiB and more
next to the ceilings that plain library launches reach in the same run, and the CPU oracle
timed on a bounded sample of the same sweep.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--cells-out", default=None, help="write the per-cell table (JSON) here")
    ap.add_argument("--cells-md", default=None, help="write the per-cell table and the workloads as markdown here")
    ap.add_argument("--trace-passes", type=int, default=0,
                    help="for a kernel trace: after the warm-up run this many plain passes over the cells and stop")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-stages", action="store_true",
                    help="skip the application-shaped workloads (small allreduce, MoE, DLRM, gradient buckets)")
    ap.add_argument("--cpu-max-bytes", type=int, default=128 << 20)
    ap.add_argument("--calibrate", action="store_true",
                    help="finish with three plain 1 GiB copies (alltoall at P=1): the known-size kernel that "
                         "hardware-counter readings are scaled by")
    return ap.parse_args()


SWEEP_KERNEL_SOURCES = ("csrc/mcr_allreduce_impl.hpp", "csrc/mcr_reduce_scatter_impl.hpp", "csrc/mcr_copy.hip",
                        "csrc/mcr_device.hpp", "csrc/mcr_dispatch.hpp", "csrc/mcr_reduce_tile.hpp", "tuning/mi355x.tbl")


def kernel_sources_digest():
    """Digest of what decides the sweep's device code and launch shapes (the kernel files of the
    four swept ops, the device headers they include, the shipped tuning table): stored counter
    readings are only reported while it matches."""
    h = hashlib.sha256()
    for name in SWEEP_KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2303_08374_amd", name), "rb") as f:
            h.update(name.encode())
            h.update(f.read())
    return h.hexdigest()[:16]


def stored_traffic(kernel_key, message_sizes):
    """Mean HBM bytes per launch of `kernel_key` over launches with the given per-rank message
    sizes, from the committed rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE, each scaled by
    its reading for a plain copy of known size); None when there is no reading for this kernel
    or the kernel sources have changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    if rec.get("sources_digest") != kernel_sources_digest():
        return None
    per_size = rec.get("kernels", {}).get(kernel_key)
    if not per_size or any(str(m) not in per_size for m in message_sizes):
        return None
    return round(sum(per_size[str(m)] for m in message_sizes) / len(message_sizes))


def kernel_group(op, dtype, variant_name):
    """One name per kernel function, the way a profiler groups launches: the reductions are
    compiled per dtype, the copies are not, and the super-chunk all_gather is one kernel
    whatever its super-chunk size."""
    if op == "allgather" and variant_name.startswith("sc"):
        return "allgather/superchunk"
    if op in ("allreduce", "reduce_scatter"):
        return f"{op}/{dtype}/{variant_name}"
    return f"{op}/{variant_name}"


def measure_ceilings(ctx, arena, torch, mcr):
    """What plain library launches reach on this GPU in this run, over cold buffers, median of 5:
    a copy (all_to_all_single at P=1: one read and one write stream), a read-dominated launch
    (reduce_scatter at P=16: 16 read streams to 1 write stream) and a write-dominated one (bcast
    to 7 receivers: 1 read to 7 writes)."""
    G = 1 << 30

    def timed(launch, footprint, alg_bytes):
        ms = []
        for i in range(7):
            base = arena.take(footprint)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            launch(base)
            e1.record()
            e1.synchronize()
            if i >= 2:
                ms.append(e0.elapsed_time(e1))
        t = sorted(ms)[len(ms) // 2]
        return round(alg_bytes / (t * 1e-3) / 1e9, 1), round(t * 1e3, 1)

    out = {}
    g, us = timed(lambda b: mcr.mcr_alltoall(ctx, [b + G], [b], G // 4, mcr.F32, 1, 4), 2 * G, 2 * G)
    out["copy"] = {"GBps": g, "us": us, "what": "mcr_alltoall at P=1, 1 GiB, variant v1nt: 1 GiB read + 1 GiB written"}
    M = 128 << 20
    g, us = timed(lambda b: mcr.mcr_reduce_scatter(ctx, [b + 16 * M + r * (M // 16) for r in range(16)], [b + p * M for p in range(16)],
                                                   M // 4, mcr.F32, mcr.SUM, 16), 17 * M, 17 * M)
    out["read_dominated"] = {"GBps": g, "us": us, "what": "mcr_reduce_scatter at P=16, 128 MiB per rank, fp32: 2 GiB read + 128 MiB written"}
    M = 256 << 20
    g, us = timed(lambda b: mcr.mcr_bcast(ctx, [b + p * M for p in range(8)], M // 4, mcr.F32, 0, 8), 8 * M, 8 * M)
    out["write_dominated"] = {"GBps": g, "us": us, "what": "mcr_bcast at P=8, 256 MiB, fp32: 256 MiB read + 1.75 GiB written"}
    return out


def cpu_baseline(max_bytes):
    """The oracle as it stands, one thread, on the sweep cells up to `max_bytes` per rank."""
    import numpy as np
    import oracle
    from paper_2303_08374_amd import inputs, sweep
    P = inputs.SWEEP_P
    sizes = [m for m in inputs.SWEEP_BYTES if m <= max_bytes]
    total_bytes, total_s = 0, 0.0
    for dt_name, dt in (("f32", oracle.F32), ("bf16", oracle.BF16)):
        for M in sizes:
            n = M // sweep.ELEM[dt_name]
            bufs = inputs.rank_buffers(P, n, inputs.SWEEP_SEED, "uniform", bf16=(dt == oracle.BF16))
            for op in inputs.SWEEP_OPS:
                t0 = time.perf_counter()
                if op == "allreduce":
                    oracle.allreduce([b.copy() for b in bufs], dt, oracle.SUM)
                elif op == "reduce_scatter":
                    oracle.reduce_scatter(bufs, dt, oracle.SUM)
                elif op == "allgather":
                    oracle.allgather(bufs, dt)
                else:
                    oracle.alltoall(bufs, dt)
                total_s += time.perf_counter() - t0
                total_bytes += sweep.algorithmic_bytes(op, P, M)
    return {"value": round(total_bytes / total_s / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"the same sweep (4 ops x fp32,bf16, P={P}) restricted to messages <= {max_bytes >> 20} MiB "
                      f"per rank: {total_bytes / 1e9:.2f} GB algorithmic in {total_s:.1f} s, single thread "
                      f"(allocation of outputs and the in-place copy included)",
            "host_cpus": os.cpu_count()}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the P ranks are simulated inside one MI355X's HBM and nothing here "
              "uses a second device; run with --gpus 1", file=sys.stderr)
        return 2
    import torch
    from paper_2303_08374_amd import inputs, mcr, sweep
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    ctx = mcr.mcr_init(0)
    table = os.environ.get("MCR_TUNING_TABLE") or os.path.join(ROOT, "paper_2303_08374_amd", "tuning", "mi355x.tbl")
    table_rows = 0
    if os.path.exists(table):
        mcr.mcr_tune_load(ctx, table)
        table_rows = mcr.mcr_tune_count(ctx)
    P = inputs.SWEEP_P
    cells = sweep.make_cells(P, inputs.SWEEP_OPS, inputs.SWEEP_DTYPES, inputs.SWEEP_BYTES)
    need = max(c.footprint for c in cells)
    arena = sweep.Arena(need + (2 << 30), seed=inputs.SWEEP_SEED)
    variant_names = {op: mcr.mcr_get_variants(ctx, sweep.OPS[op]) for op in inputs.SWEEP_OPS}
    variant_of = {c.key: c.auto_variant(ctx) for c in cells}
    step_bytes = sum(c.alg_bytes for c in cells)

    def run_step(instrument=None):
        """One pass of the sweep.  `instrument`: set of cell keys whose launches get an event pair."""
        evs = []
        for c in cells:
            base = arena.take(c.footprint)
            if instrument is not None and c.key in instrument:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                c.launch(ctx, base, mcr.AUTO)
                e1.record()
                evs.append((c, e0, e1))
            else:
                c.launch(ctx, base, mcr.AUTO)
        return evs

    all_keys = {c.key for c in cells}
    for _ in range(max(args.warmup, 1)):
        run_step()
    torch.cuda.synchronize()
    if args.trace_passes > 0:
        for _ in range(args.trace_passes):
            run_step()
            torch.cuda.synchronize()
        mcr.mcr_finalize(ctx)
        print(json.dumps({"trace_passes": args.trace_passes, "cells_per_pass": len(cells)}))
        return 0
    # one instrumented pass decides which kernel dominates the step
    evs = run_step(all_keys)
    torch.cuda.synchronize()
    group_ms = {}
    group_of = {c.key: kernel_group(c.op, c.dtype, variant_names[c.op][variant_of[c.key]]) for c in cells}
    for c, e0, e1 in evs:
        g = group_of[c.key]
        group_ms[g] = group_ms.get(g, 0.0) + e0.elapsed_time(e1)
    dom = max(group_ms, key=group_ms.get)
    dom_keys = {c.key for c in cells if group_of[c.key] == dom}
    arena.refill()
    torch.cuda.synchronize()

    # ---- timed region -------------------------------------------------------------------
    dom_evs = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dom_evs += run_step(dom_keys)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # ---------------------------------------------------------------------------------------
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    dom_ms = sum(e0.elapsed_time(e1) for _, e0, e1 in dom_evs)
    dom_bytes = sum(c.alg_bytes for c, _, _ in dom_evs)
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": stored_traffic(dom, [c.M for c, _, _ in dom_evs]),
                "kernel": dom, "launches": len(dom_evs),
                "avg_launch_us": round(dom_ms * 1e3 / len(dom_evs), 2),
                "avg_launch_alg_bytes": dom_bytes // len(dom_evs)}

    # ---- per-cell table (cold buffers, median of 5 instrumented passes) -------------------
    per_cell = {c.key: [] for c in cells}
    smallest = min(cells, key=lambda c: c.M)
    # (not a launch of the dominant kernel, so that a profiler's average for that kernel over the
    # whole process still covers the same mix of launches as the timed region)
    largest = max((c for c in cells if group_of[c.key] != dom), key=lambda c: c.alg_bytes)
    for _ in range(5):
        # One large launch keeps the GPU busy while the host enqueues what follows; otherwise the
        # first small cells of a pass are timed with the GPU waiting for the host between the two
        # events.  The small launches after it keep the first launches after an idle gap, which
        # run slow, out of the table.
        largest.launch(ctx, arena.take(largest.footprint), mcr.AUTO)
        for _ in range(20):
            smallest.launch(ctx, arena.take(smallest.footprint), mcr.AUTO)
        evs = run_step(all_keys)
        torch.cuda.synchronize()
        for c, e0, e1 in evs:
            per_cell[c.key].append(e0.elapsed_time(e1))
    ceilings = measure_ceilings(ctx, arena, torch, mcr)
    table_out, large = {}, {}
    for c in cells:
        ms = sorted(per_cell[c.key])[len(per_cell[c.key]) // 2]
        gbps = c.alg_bytes / (ms * 1e-3) / 1e9
        table_out[c.key] = {"variant": variant_names[c.op][variant_of[c.key]], "us": round(ms * 1e3, 2), "GBps": round(gbps, 1),
                            "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4)}
        if c.M >= (16 << 20):
            g = large.setdefault(f"{c.op}/{c.dtype}", {"bytes": 0, "ms": 0.0, "fracs": []})
            g["bytes"] += c.alg_bytes
            g["ms"] += ms
            g["fracs"].append(gbps / HBM_PEAK_GBPS)
    # per (op, element type), messages of 16 MiB and more: bytes summed over times summed
    per_op = {}
    for k, g in large.items():
        gbps = g["bytes"] / (g["ms"] * 1e-3) / 1e9
        per_op[k] = {"GBps": round(gbps, 1), "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4),
                     "frac_of_copy_ceiling": round(gbps / ceilings["copy"]["GBps"], 4),
                     "min_frac": round(min(g["fracs"]), 4), "max_frac": round(max(g["fracs"]), 4)}
    worst = min(per_op, key=lambda k: per_op[k]["frac_of_peak"])
    small_us = {f"{c.op}/{c.dtype}": table_out[c.key]["us"] for c in cells if c.M == inputs.SWEEP_BYTES[0]}
    if args.cells_out:
        os.makedirs(os.path.dirname(args.cells_out) or ".", exist_ok=True)
        with open(args.cells_out, "w") as f:
            json.dump(table_out, f, indent=1)

    out = {
        "metric": "effective GB/s and % of HBM peak per op vs message size (4 KB-256 MB)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "element_types": ["f32", "bf16"], "data": "synthetic",
        "config": {"workload": "op sweep: allreduce, reduce_scatter, allgather, alltoall x {fp32, bf16 with fp32 "
                               "accumulate} x 17 per-rank message sizes 4 KiB..256 MiB, P=8 simulated ranks, "
                               "uniform[-1,1), MCR_AUTO dispatch, cold buffers",
                   "P": P, "launches_per_step": len(cells), "algorithmic_bytes_per_step": step_bytes,
                   "tuning_table_rows": table_rows},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "roofline": roofline,
        "ceilings": ceilings,
        "roofline_per_op": per_op,
        "worst_op": f"{worst}: {per_op[worst]['GBps']} GB/s = {100 * per_op[worst]['frac_of_peak']:.1f} % of 8000 GB/s, "
                    f"{100 * per_op[worst]['frac_of_copy_ceiling']:.1f} % of the copy ceiling",
        "smallest_message_us": small_us,
    }
    if not args.no_stages:
        from paper_2303_08374_amd import workloads
        out["stages"] = workloads.run_all(ctx)
    if args.calibrate:
        n = (1 << 30) // 4
        src = arena.base
        dst = arena.base + (1 << 30)
        for _ in range(3):
            mcr.mcr_alltoall(ctx, [dst], [src], n, mcr.F32, 1, 4)          # variant v1nt, P=1: a plain copy
        torch.cuda.synchronize()
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(args.cpu_max_bytes)
    if args.cells_md:
        from paper_2303_08374_amd import report
        os.makedirs(os.path.dirname(args.cells_md) or ".", exist_ok=True)
        with open(args.cells_md, "w") as f:
            f.write(report.cells_markdown(table_out, out, "python3 bench.py " + " ".join(sys.argv[1:])))
    mcr.mcr_finalize(ctx)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
