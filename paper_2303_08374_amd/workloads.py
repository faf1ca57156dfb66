"""Device-side drivers of the application-shaped workloads: the small allreduce, MoE token
dispatch/combine, the DLRM embedding shuffle and dense gradient buckets.  Each returns
per-stage times measured with events on the launch stream, with the algorithmic bytes of the
stage (bytes that must be read plus written once).

They stand in for the paper's DS-MoE, DLRM and Megatron-DeepSpeed runs (Sec. V-A4), whose
models and datasets are not needed for the data movement itself.  Inputs are generated on the
device here (timing only; the parity tests use the host generators of ``inputs``).
"""
from __future__ import annotations

from typing import Dict, List, Optional

import math

import numpy as np
import torch

from . import inputs, mcr


def _v(variants: Optional[Dict[str, int]], key: str) -> int:
    """Variant for one stage: MCR_AUTO unless the tuning suite asks for a specific one."""
    return mcr.AUTO if not variants else variants.get(key, mcr.AUTO)


def _events(n):
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def _stage_report(names, alg_bytes, ev_rows):
    """ev_rows: one list of len(names)+1 events per repetition."""
    out = {}
    for i, name in enumerate(names):
        ms = sorted(r[i].elapsed_time(r[i + 1]) for r in ev_rows)
        med = ms[len(ms) // 2]
        out[name] = {"us": round(med * 1e3, 2), "alg_bytes": int(alg_bytes[i]),
                     "GBps": round(alg_bytes[i] / (med * 1e-3) / 1e9, 1) if alg_bytes[i] else None}
    tot = sorted(r[0].elapsed_time(r[-1]) for r in ev_rows)
    med = tot[len(tot) // 2]
    out["end_to_end"] = {"us": round(med * 1e3, 2), "alg_bytes": int(sum(alg_bytes)),
                         "GBps": round(sum(alg_bytes) / (med * 1e-3) / 1e9, 1)}
    return out


# ---- workload 1 ---------------------------------------------------------------------------
def allreduce_small(ctx, reps: int = 50) -> Dict:
    """P=4, 2^20 fp32 per rank (32 MiB of traffic per call).  `cold`: 32 buffer sets in rotation
    (512 MiB, beyond the last-level cache); `warm`: the same buffers every time (cache resident,
    not an HBM figure)."""
    w = inputs.AllreduceSmall()
    sets = 32
    arena = torch.empty(sets * w.P * w.n, dtype=torch.float32, device="cuda").normal_()
    base = arena.data_ptr()
    ptrs = [[base + (s * w.P + p) * w.n * 4 for p in range(w.P)] for s in range(sets)]
    alg = 2 * w.P * w.n * 4
    out = {}
    for label, pick in (("cold", lambda i: ptrs[i % sets]), ("warm", lambda i: ptrs[0])):
        for i in range(sets):
            mcr.mcr_allreduce(ctx, pick(i), w.n, mcr.F32, mcr.SUM, w.P)
        e = _events(2)
        e[0].record()
        for i in range(reps):
            mcr.mcr_allreduce(ctx, pick(i), w.n, mcr.F32, mcr.SUM, w.P)
        e[1].record()
        e[1].synchronize()
        ms = e[0].elapsed_time(e[1]) / reps
        out[label] = {"us": round(ms * 1e3, 2), "alg_bytes": alg, "GBps": round(alg / (ms * 1e-3) / 1e9, 1)}
        arena.normal_()
    return out


# ---- workload 3 ---------------------------------------------------------------------------
def moe_dispatch_combine(ctx, reps: int = 10, w: inputs.MoEWorkload = inputs.MoEWorkload(),
                         variants: Optional[Dict[str, int]] = None, odd_hidden: int = 0) -> Dict:
    """`odd_hidden`: a second hidden size (say 2052: rows of 4104 bytes, not a multiple of 16) to run
    the row kernels on as well; their times are reported against the ones at w.H."""
    P, T, H, E, C = w.P, w.T, w.H, w.E, w.C
    row = H * 2
    d_ids = [torch.from_numpy(w.ids(p)).cuda() for p in range(P)]
    d_tok = [torch.empty(T * H, dtype=torch.bfloat16, device="cuda").normal_() for _ in range(P)]
    d_gate = [torch.rand(T, dtype=torch.float32, device="cuda") for _ in range(P)]
    d_slot = [torch.empty(T, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_cnt = [torch.empty(E, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_S = torch.empty(P * P, dtype=torch.int64, device="cuda")
    mk = lambda rows: [torch.zeros(rows * H, dtype=torch.bfloat16, device="cuda") for _ in range(P)]
    d_packed, d_recv, d_back, d_out = mk(T), mk(w.recv_rows), mk(T), mk(T)
    rows = []
    for it in range(reps + 2):
        e = _events(6)
        e[0].record()
        mcr.mcr_moe_route(ctx, d_ids, T, E, P, C, d_slot, d_cnt, d_S)
        e[1].record()
        mcr.mcr_pack(ctx, d_packed, d_tok, d_slot, T, T, H, mcr.BF16, P, _v(variants, "pack"))
        e[2].record()
        mcr.mcr_alltoallv(ctx, d_recv, d_packed, d_S, mcr.SPLITS_ON_DEVICE, T, w.recv_rows, H, mcr.BF16, P, _v(variants, "alltoallv"))
        e[3].record()
        mcr.mcr_alltoallv(ctx, d_back, d_recv, d_S, mcr.SPLITS_ON_DEVICE | mcr.SPLITS_TRANSPOSED, w.recv_rows, T, H, mcr.BF16, P,
                          _v(variants, "alltoallv"))
        e[4].record()
        mcr.mcr_unpack(ctx, d_out, d_back, d_slot, d_gate, T, T, H, mcr.BF16, P, _v(variants, "unpack"))
        e[5].record()
        if it >= 2:
            rows.append(e)
    torch.cuda.synchronize()
    kept = int(d_S.sum().item())
    alg = [0,                                  # routing: a few KB of integers, latency bound
           2 * kept * row + P * T * 4,         # pack: kept rows read and written, slots read
           2 * kept * row,                     # dispatch alltoallv
           2 * kept * row,                     # return alltoallv
           kept * row + P * T * row + P * T * 8]   # combine: kept rows read, all T rows written, slot + gate read
    rep = _stage_report(["route", "pack", "alltoallv_dispatch", "alltoallv_return", "unpack_combine"], alg, rows)
    rep["kept_rows"] = kept
    rep["kept_fraction"] = round(kept / (P * T), 4)
    # the same result with the fused calls: tokens go straight into the receive buffers and come
    # straight back out of them (identity experts in between)
    rows = []
    for it in range(reps + 2):
        e = _events(4)
        e[0].record()
        mcr.mcr_moe_route(ctx, d_ids, T, E, P, C, d_slot, d_cnt, d_S)
        e[1].record()
        mcr.mcr_moe_dispatch(ctx, d_recv, d_tok, d_slot, d_S, T, w.recv_rows, H, mcr.BF16, P, _v(variants, "moe_dispatch"))
        e[2].record()
        mcr.mcr_moe_combine(ctx, d_out, d_recv, d_slot, d_gate, d_S, T, w.recv_rows, H, mcr.BF16, P, _v(variants, "moe_combine"))
        e[3].record()
        if it >= 2:
            rows.append(e)
    torch.cuda.synchronize()
    falg = [0, 2 * kept * row + P * T * 4, kept * row + P * T * row + P * T * 8]
    rep["fused"] = _stage_report(["route", "moe_dispatch", "moe_combine"], falg, rows)
    rep["fused"]["speedup_vs_chain"] = round(rep["end_to_end"]["us"] / rep["fused"]["end_to_end"]["us"], 2)
    # the expert-major receive layout (every expert's tokens in one block), same row traffic; routing
    # by several workgroups per rank with a workspace
    K_MAX = 2
    d_tab = torch.empty(P * E, dtype=torch.int64, device="cuda")
    d_first = torch.empty(E, dtype=torch.int64, device="cuda")
    d_rows = torch.empty(E, dtype=torch.int64, device="cuda")
    ws_bytes = mcr.mcr_moe_route_workspace_bytes(K_MAX * T, E, P)
    d_ws = torch.empty(max(ws_bytes, 4) // 4, dtype=torch.int32, device="cuda")
    rows = []
    for it in range(reps + 2):
        e = _events(5)
        e[0].record()
        mcr.mcr_moe_route_ws(ctx, d_ids, T, E, P, C, d_slot, d_cnt, d_S, d_ws, ws_bytes)
        e[1].record()
        mcr.mcr_moe_expert_layout(ctx, d_cnt, E, P, d_tab, d_first, d_rows)
        e[2].record()
        mcr.mcr_moe_dispatch_by_expert(ctx, d_recv, d_tok, d_ids, d_slot, d_tab, T, 1, E, w.recv_rows, H, mcr.BF16, P,
                                       _v(variants, "moe_dispatch_by_expert"))
        e[3].record()
        mcr.mcr_moe_combine_by_expert(ctx, d_out, d_recv, d_ids, d_slot, d_gate, d_tab, T, 1, E, w.recv_rows, H, mcr.BF16, P,
                                      _v(variants, "moe_combine_by_expert"))
        e[4].record()
        if it >= 2:
            rows.append(e)
    torch.cuda.synchronize()
    ealg = [0, 0, 2 * kept * row + P * T * 8, kept * row + P * T * row + P * T * 12]
    rep["by_expert"] = _stage_report(["route", "expert_layout", "moe_dispatch_by_expert", "moe_combine_by_expert"], ealg, rows)
    # the chain's own (source-major) layout through the same table-driven calls
    rows = []
    for it in range(reps + 2):
        e = _events(5)
        e[0].record()
        mcr.mcr_moe_route_ws(ctx, d_ids, T, E, P, C, d_slot, d_cnt, d_S, d_ws, ws_bytes)
        e[1].record()
        mcr.mcr_moe_source_layout(ctx, d_cnt, E, P, d_tab)
        e[2].record()
        mcr.mcr_moe_dispatch_by_expert(ctx, d_recv, d_tok, d_ids, d_slot, d_tab, T, 1, E, w.recv_rows, H, mcr.BF16, P,
                                       _v(variants, "moe_dispatch_by_expert"))
        e[3].record()
        mcr.mcr_moe_combine_by_expert(ctx, d_out, d_recv, d_ids, d_slot, d_gate, d_tab, T, 1, E, w.recv_rows, H, mcr.BF16, P,
                                      _v(variants, "moe_combine_by_expert"))
        e[4].record()
        if it >= 2:
            rows.append(e)
    torch.cuda.synchronize()
    rep["source_major_by_table"] = _stage_report(["route", "source_layout", "moe_dispatch_by_expert", "moe_combine_by_expert"],
                                                 ealg, rows)
    rep["source_major_by_table"]["speedup_vs_chain"] = round(rep["end_to_end"]["us"] / rep["source_major_by_table"]["end_to_end"]["us"], 2)
    # top-2 gating on the same tokens: second choice = the id stream rotated by 17 tokens, capacity doubled
    K = 2
    A, C2 = K * T, int(math.ceil(w.capacity_factor * K * T / E))
    rows2 = P * min(A, (E // P) * C2)
    d_ids2 = [torch.cat([x, torch.roll(x, 17)]) for x in d_ids]
    d_gate2 = [torch.rand(A, dtype=torch.float32, device="cuda") for _ in range(P)]
    d_slot2 = [torch.empty(A, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_recv2 = mk(rows2)
    rows = []
    for it in range(reps + 2):
        e = _events(5)
        e[0].record()
        mcr.mcr_moe_route_ws(ctx, d_ids2, A, E, P, C2, d_slot2, d_cnt, d_S, d_ws, ws_bytes)
        e[1].record()
        mcr.mcr_moe_expert_layout(ctx, d_cnt, E, P, d_tab, d_first, d_rows)
        e[2].record()
        mcr.mcr_moe_dispatch_by_expert(ctx, d_recv2, d_tok, d_ids2, d_slot2, d_tab, T, K, E, rows2, H, mcr.BF16, P,
                                       _v(variants, "moe_dispatch_by_expert"))
        e[3].record()
        mcr.mcr_moe_combine_by_expert(ctx, d_out, d_recv2, d_ids2, d_slot2, d_gate2, d_tab, T, K, E, rows2, H, mcr.BF16, P,
                                      _v(variants, "moe_combine_by_expert"))
        e[4].record()
        if it >= 2:
            rows.append(e)
    torch.cuda.synchronize()
    kept2 = int(d_S.sum().item())
    # dispatch reads a token row once if any of its choices is kept and writes it once per kept choice
    tokens_sent = sum(int((s.view(K, T) >= 0).any(dim=0).sum().item()) for s in d_slot2)
    talg = [0, 0, (tokens_sent + kept2) * row + P * A * 8, kept2 * row + P * T * row + P * A * 12]
    rep["top2"] = _stage_report(["route", "expert_layout", "moe_dispatch_by_expert", "moe_combine_by_expert"], talg, rows)
    rep["top2"]["kept_assignments"] = kept2
    rep["top2"]["tokens_with_a_kept_choice"] = tokens_sent
    rep["top2"]["kept_fraction"] = round(kept2 / (P * A), 4)
    if odd_hidden:
        import dataclasses
        del d_tok, d_packed, d_recv, d_back, d_out, d_recv2
        torch.cuda.empty_cache()
        odd = moe_dispatch_combine(ctx, reps, dataclasses.replace(w, H=odd_hidden), variants)
        pairs = [("pack", ("pack",)), ("alltoallv_dispatch", ("alltoallv_dispatch",)), ("unpack_combine", ("unpack_combine",)),
                 ("moe_dispatch", ("fused", "moe_dispatch")), ("moe_combine", ("fused", "moe_combine")),
                 ("moe_dispatch_by_expert", ("by_expert", "moe_dispatch_by_expert")),
                 ("moe_combine_by_expert", ("by_expert", "moe_combine_by_expert")),
                 ("top2 moe_dispatch_by_expert", ("top2", "moe_dispatch_by_expert")),
                 ("top2 moe_combine_by_expert", ("top2", "moe_combine_by_expert"))]

        def at(r, path):
            for k in path:
                r = r[k]
            return r
        rep["odd_rows"] = {"H": odd_hidden, "row_bytes": odd_hidden * 2, "stages": {
            name: {"us": at(odd, path)["us"], "GBps": at(odd, path).get("GBps"),
                   "vs_aligned": round(at(odd, path)["us"] / at(rep, path)["us"], 2)} for name, path in pairs}}
    return rep


# ---- workload 4 ---------------------------------------------------------------------------
def dlrm_shuffle(ctx, reps: int = 10, w: inputs.DLRMWorkload = inputs.DLRMWorkload(), sets: int = 3,
                 variants: Optional[Dict[str, int]] = None, odd_dim: int = 0) -> Dict:
    """Forward: pooled [T_p, B, D] -> destination-major send order (pack) -> alltoallv ->
    [B/P, n_tables, D] (unpack with the table permutation).  Backward: the inverse chain.
    `sets` independent buffer sets are used in rotation so that a stage does not find its
    input in the last-level cache.  `odd_dim`: a second embedding width (say 130: rows of 520
    bytes, not a multiple of 16) to run the same stages on; their times per byte against the
    first width's go under "odd_rows"."""
    P, NT, D, B = w.P, w.n_tables, w.dim, w.batch
    bl = B // P
    n_local = [len(w.tables_on(p)) for p in range(P)]
    max_rows = max(n_local) * B
    S = w.splits()
    send_slot = []
    for p in range(P):
        lt, r, b = np.meshgrid(np.arange(n_local[p]), np.arange(P), np.arange(bl), indexing="ij")
        full = np.full(max_rows, -1, dtype=np.int32)
        full[: lt.size] = ((r * n_local[p] + lt) * bl + b).reshape(-1)
        send_slot.append(torch.from_numpy(full).cuda())
    order = [t for p in range(P) for t in w.tables_on(p)]
    pos = np.empty(NT, dtype=np.int64)
    pos[order] = np.arange(NT)
    perm = (pos[None, :] * bl + np.arange(bl)[:, None]).reshape(-1).astype(np.int32)
    d_perm = [torch.from_numpy(perm).cuda() for _ in range(P)]
    f32 = lambda rows: [torch.empty(rows * D, dtype=torch.float32, device="cuda").normal_() for _ in range(P)]
    bufs = [dict(src=f32(max_rows), send=f32(max_rows), recv=f32(NT * bl), out=f32(bl * NT), grecv=f32(NT * bl),
                 gsend=f32(max_rows), gsrc=f32(max_rows)) for _ in range(sets)]
    ST = S.T.copy()
    rows = []
    for it in range(reps + sets):
        x = bufs[it % sets]
        e = _events(7)
        e[0].record()
        mcr.mcr_pack(ctx, x["send"], x["src"], send_slot, max_rows, max_rows, D, mcr.F32, P, _v(variants, "pack"))
        e[1].record()
        mcr.mcr_alltoallv(ctx, x["recv"], x["send"], S, False, max_rows, NT * bl, D, mcr.F32, P, _v(variants, "alltoallv"))
        e[2].record()
        mcr.mcr_unpack(ctx, x["out"], x["recv"], d_perm, None, bl * NT, NT * bl, D, mcr.F32, P, _v(variants, "unpack"))
        e[3].record()
        mcr.mcr_pack(ctx, x["grecv"], x["out"], d_perm, bl * NT, NT * bl, D, mcr.F32, P, _v(variants, "pack"))
        e[4].record()
        mcr.mcr_alltoallv(ctx, x["gsend"], x["grecv"], ST, False, NT * bl, max_rows, D, mcr.F32, P, _v(variants, "alltoallv"))
        e[5].record()
        mcr.mcr_unpack(ctx, x["gsrc"], x["gsend"], send_slot, None, max_rows, max_rows, D, mcr.F32, P, _v(variants, "unpack"))
        e[6].record()
        if it >= sets:
            rows.append(e)
    torch.cuda.synchronize()
    data = NT * B * D * 4                                   # 208 MiB of pooled rows
    pad = (P * max_rows - NT * B) * D * 4                   # zero rows written for the ranks that own fewer tables
    alg = [2 * data + P * max_rows * 4, 2 * data, 2 * data + NT * B * 4,
           2 * data + NT * B * 4, 2 * data, 2 * data + pad + P * max_rows * 4]
    rep = _stage_report(["fwd_pack_send_order", "fwd_alltoallv", "fwd_unpack_permute",
                         "bwd_pack_permute", "bwd_alltoallv", "bwd_unpack_table_order"], alg, rows)
    # the fused single-pass shuffle
    rows = []
    for it in range(reps + sets):
        x = bufs[it % sets]
        e = _events(3)
        e[0].record()
        mcr.mcr_dlrm_shuffle(ctx, x["out"], x["src"], NT, B, D, mcr.F32, P, False, _v(variants, "dlrm_shuffle"))
        e[1].record()
        mcr.mcr_dlrm_shuffle(ctx, x["gsrc"], x["out"], NT, B, D, mcr.F32, P, True, _v(variants, "dlrm_shuffle"))
        e[2].record()
        if it >= sets:
            rows.append(e)
    torch.cuda.synchronize()
    rep["fused"] = _stage_report(["fwd_dlrm_shuffle", "bwd_dlrm_shuffle"], [2 * data, 2 * data], rows)
    rep["fused"]["speedup_vs_chain"] = round(rep["end_to_end"]["us"] / rep["fused"]["end_to_end"]["us"], 2)
    if odd_dim:
        import dataclasses
        del bufs
        torch.cuda.empty_cache()
        odd = dlrm_shuffle(ctx, reps, dataclasses.replace(w, dim=odd_dim), sets, variants)
        names = [(k, (k,)) for k in ("fwd_pack_send_order", "fwd_alltoallv", "fwd_unpack_permute", "bwd_pack_permute", "bwd_alltoallv",
                                     "bwd_unpack_table_order")] + [(k, ("fused", k)) for k in ("fwd_dlrm_shuffle", "bwd_dlrm_shuffle")]

        def at(r, path):
            for k in path:
                r = r[k]
            return r
        rep["odd_rows"] = {"dim": odd_dim, "row_bytes": odd_dim * 4, "stages": {
            name: {"us": at(odd, path)["us"], "GBps": at(odd, path).get("GBps"),
                   "per_byte_vs_aligned": round(at(odd, path)["us"] / at(rep, path)["us"] * D / odd_dim, 2)} for name, path in names}}
    return rep


# ---- workload 5 ---------------------------------------------------------------------------
def grad_buckets(ctx, reps: int = 3, w: inputs.GradBucketWorkload = inputs.GradBucketWorkload(),
                 variants: Optional[Dict[str, int]] = None, per_tensor: bool = True) -> Dict:
    """bf16 gradients of the GPT-style list on P ranks.  Three ways to all-reduce (average) them:
    per bucket fuse -> allreduce(flat) -> unfuse; the fused multi-tensor allreduce in one launch
    over the whole list; and one allreduce launch per tensor (no fusion)."""
    P = w.P
    numel = w.numel()
    total = sum(numel)
    plan = mcr.mcr_fuse_plan_create(ctx, numel, w.bucket_elems, mcr.BF16)
    try:
        bn, tb, to = mcr.mcr_fuse_plan_info(plan, len(numel))
        arenas = [torch.empty(total, dtype=torch.bfloat16, device="cuda").normal_(0.0, w.std) for _ in range(P)]
        offs = np.concatenate([[0], np.cumsum(numel)[:-1]]).tolist()
        ptrs = [arenas[p].data_ptr() + offs[i] * 2 for p in range(P) for i in range(len(numel))]
        mcr.mcr_fuse_plan_bind(ctx, plan, ptrs, P)
        flats = [torch.empty(max(bn), dtype=torch.bfloat16, device="cuda") for _ in range(P)]
        s = 2
        rows_pipe, rows_multi, rows_each = [], [], []
        for it in range(reps + 1):
            e = _events(2)
            stage_ev = []
            e[0].record()
            for k in range(len(bn)):
                se = _events(4)
                se[0].record()
                mcr.mcr_fuse(ctx, plan, k, flats, P, _v(variants, "fuse"))
                se[1].record()
                mcr.mcr_allreduce(ctx, flats, bn[k], mcr.BF16, mcr.AVG, P)
                se[2].record()
                mcr.mcr_unfuse(ctx, plan, k, flats, P, _v(variants, "unfuse"))
                se[3].record()
                stage_ev.append(se)
            e[1].record()
            if it >= 1:
                rows_pipe.append((e, stage_ev))
        for it in range(reps + 1):
            e = _events(2)
            e[0].record()
            mcr.mcr_allreduce_multi(ctx, plan, -1, mcr.AVG, _v(variants, "allreduce_multi"))
            e[1].record()
            if it >= 1:
                rows_multi.append(e)
        for it in range(reps + 1 if per_tensor else 0):
            e = _events(2)
            e[0].record()
            for i, n in enumerate(numel):
                mcr.mcr_allreduce(ctx, [ptrs[p * len(numel) + i] for p in range(P)], n, mcr.BF16, mcr.AVG, P)
            e[1].record()
            if it >= 1:
                rows_each.append(e)
        torch.cuda.synchronize()
        minimum = 2 * P * total * s                          # read every gradient once, write it once
        med = lambda xs: sorted(xs)[len(xs) // 2]
        rep = {}
        for name, idx, alg in (("fuse", 0, 2 * P * total * s), ("allreduce_flat", 1, 2 * P * total * s),
                               ("unfuse", 2, 2 * P * total * s)):
            ms = med([sum(se[idx].elapsed_time(se[idx + 1]) for se in stage_ev) for _, stage_ev in rows_pipe])
            rep[name] = {"us": round(ms * 1e3, 1), "alg_bytes": alg, "GBps": round(alg / (ms * 1e-3) / 1e9, 1)}
        ms = med([e[0].elapsed_time(e[1]) for e, _ in rows_pipe])
        rep["pipeline_fuse_allreduce_unfuse"] = {"us": round(ms * 1e3, 1), "launches": 3 * len(bn), "traffic_bytes": 3 * minimum,
                                                 "GBps_of_minimum": round(minimum / (ms * 1e-3) / 1e9, 1),
                                                 "GBps_of_traffic": round(3 * minimum / (ms * 1e-3) / 1e9, 1)}
        ms = med([e[0].elapsed_time(e[1]) for e in rows_multi])
        rep["allreduce_multi_one_launch"] = {"us": round(ms * 1e3, 1), "launches": 1, "alg_bytes": minimum,
                                             "GBps": round(minimum / (ms * 1e-3) / 1e9, 1)}
        if per_tensor:
            ms = med([e[0].elapsed_time(e[1]) for e in rows_each])
            rep["allreduce_per_tensor"] = {"us": round(ms * 1e3, 1), "launches": len(numel), "alg_bytes": minimum,
                                           "GBps": round(minimum / (ms * 1e-3) / 1e9, 1)}
        rep["tensors"], rep["buckets"], rep["elements_per_rank"] = len(numel), len(bn), total
        return rep
    finally:
        mcr.mcr_fuse_plan_destroy(plan)


def small_tensor_path(ctx, reps: int = 5, w: inputs.GradBucketWorkload = inputs.GradBucketWorkload()) -> Dict:
    """The small-message path on its own: only the gradients of at most 8192 elements (LayerNorm
    weights and biases, linear biases: 194 tensors of 4-16 KiB per rank), averaged over P ranks
    either with one launch per tensor or with the fused multi-tensor launch."""
    P = w.P
    numel = [n for n in w.numel() if n <= 8192]
    total = sum(numel)
    plan = mcr.mcr_fuse_plan_create(ctx, numel, 1 << 40, mcr.BF16)
    try:
        arenas = [torch.empty(total, dtype=torch.bfloat16, device="cuda").normal_(0.0, w.std) for _ in range(P)]
        offs = np.concatenate([[0], np.cumsum(numel)[:-1]]).tolist()
        ptrs = [arenas[p].data_ptr() + offs[i] * 2 for p in range(P) for i in range(len(numel))]
        mcr.mcr_fuse_plan_bind(ctx, plan, ptrs, P)
        per_tensor = [[ptrs[p * len(numel) + i] for p in range(P)] for i in range(len(numel))]
        t_multi, t_each = [], []
        for it in range(reps + 1):
            e = _events(3)
            e[0].record()
            mcr.mcr_allreduce_multi(ctx, plan, -1, mcr.AVG)
            e[1].record()
            for i, n in enumerate(numel):
                mcr.mcr_allreduce(ctx, per_tensor[i], n, mcr.BF16, mcr.AVG, P)
            e[2].record()
            e[2].synchronize()
            if it >= 1:
                t_multi.append(e[0].elapsed_time(e[1]))
                t_each.append(e[1].elapsed_time(e[2]))
        med = lambda xs: sorted(xs)[len(xs) // 2]
        alg = 2 * P * total * 2
        return {"tensors": len(numel), "bytes_per_rank": total * 2, "alg_bytes": alg,
                "allreduce_multi_one_launch_us": round(med(t_multi) * 1e3, 2),
                "allreduce_per_tensor_us": round(med(t_each) * 1e3, 2),
                "launches_saved": len(numel) - 1,
                "speedup": round(med(t_each) / med(t_multi), 1)}
    finally:
        mcr.mcr_fuse_plan_destroy(plan)


def dispatch_overhead(ctx, P: int = inputs.SWEEP_P) -> Dict:
    """Cost of the dispatch layer per all_to_all_single operation against bare launches of the same
    kernel, over message sizes (the paper's overhead-over-OMB figure, Sec. V-B)."""
    out = {}
    for M, iters in ((4 << 10, 500), (64 << 10, 500), (1 << 20, 500), (16 << 20, 200), (128 << 20, 30)):
        src = [torch.empty(M // 4, dtype=torch.float32, device="cuda").uniform_(-1, 1) for _ in range(P)]
        dst = [torch.empty(M // 4, dtype=torch.float32, device="cuda") for _ in range(P)]
        a, d, ha, hd, do = mcr.mcr_dispatch_overhead(ctx, dst, src, M // 4, mcr.F32, P, iters)
        # overhead_pct: the dispatch layer's own CPU time against one operation (the faster of the two
        # end-to-end loops, which differ by up to a microsecond per launch either way with the state of
        # the runtime's queue, far more than the layer costs)
        out[str(M)] = {"dispatch_only_us": round(do, 4), "direct_us": round(d, 3), "auto_us": round(a, 3),
                       "overhead_pct": round(100.0 * do / min(a, d), 2), "end_to_end_diff_pct": round(100.0 * (a - d) / d, 2),
                       "host_auto_us": round(ha, 3), "host_direct_us": round(hd, 3)}
        del src, dst
    return out


def graph_replay(ctx, P: int = inputs.SWEEP_P, max_bytes: int = 1 << 20, reps: int = 20) -> Dict:
    """The launch-bound part of the op sweep (every cell up to `max_bytes` per rank) issued call by
    call and replayed from one HIP graph: the entry points only enqueue kernels, so the whole batch
    can be captured once and replayed without the per-call host cost."""
    from . import sweep
    cells = [c for c in sweep.make_cells(P, inputs.SWEEP_OPS, inputs.SWEEP_DTYPES, inputs.SWEEP_BYTES) if c.M <= max_bytes]
    arena = sweep.Arena(max(c.footprint for c in cells) * 2 + (64 << 20), seed=inputs.SWEEP_SEED)
    bases = [arena.take(c.footprint) for c in cells]

    def batch(stream):
        for c, b in zip(cells, bases):
            c.launch(ctx, b, mcr.AUTO, stream)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        batch(None)                                           # warm every kernel up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        batch(torch.cuda.current_stream().cuda_stream)
    eager_ms = sweep.time_launches(lambda: batch(None), reps)
    graph_ms = sweep.time_launches(graph.replay, reps)
    return {"launches": len(cells), "max_bytes_per_rank": max_bytes, "eager_us": round(eager_ms * 1e3, 1),
            "graph_us": round(graph_ms * 1e3, 1), "eager_us_per_launch": round(eager_ms * 1e3 / len(cells), 2),
            "graph_us_per_launch": round(graph_ms * 1e3 / len(cells), 2), "speedup": round(eager_ms / graph_ms, 2)}


def rooted_collectives(ctx, P: int = inputs.SWEEP_P, M: int = 32 << 20, reps: int = 12) -> Dict:
    """reduce, bcast, gather, scatter and all_gatherv (the rooted and vector collectives of the API
    listing) on fp32 messages of `M` bytes per rank over cold buffers: a batch of `reps` launches
    back to back, microseconds per launch and GB/s of the bytes the operation has to move."""
    from . import sweep
    n = M // 4
    arena = sweep.Arena(max(20 * (P + P * P) * M // 8, 4 << 30), seed=inputs.SWEEP_SEED)

    def ptrs(base, k, nbytes):
        return [base + i * nbytes for i in range(k)]

    def reduce_():
        mcr.mcr_reduce(ctx, ptrs(arena.take(P * M), P, M), n, mcr.F32, mcr.SUM, 0, P)

    def bcast():
        mcr.mcr_bcast(ctx, ptrs(arena.take(P * M), P, M), n, mcr.F32, 0, P)

    def gather():
        base = arena.take(2 * P * M)
        mcr.mcr_gather(ctx, base + P * M, ptrs(base, P, M), n, mcr.F32, P)

    def scatter():
        base = arena.take(2 * P * M)
        mcr.mcr_scatter(ctx, ptrs(base + P * M, P, M), base, n, mcr.F32, P)

    def allgatherv():
        base = arena.take(P * M + P * P * M)
        mcr.mcr_allgatherv(ctx, ptrs(base + P * M, P, P * M), ptrs(base, P, M), [n] * P, mcr.F32, P)
    out = {"P": P, "bytes_per_rank": M}
    for name, fn, alg in (("reduce", reduce_, (P + 1) * M), ("bcast", bcast, P * M), ("gather", gather, 2 * P * M),
                          ("scatter", scatter, 2 * P * M), ("allgatherv", allgatherv, (P + P * P) * M)):
        fn()
        ms = sweep.time_launches(fn, reps)
        out[name] = {"us": round(ms * 1e3, 2), "alg_bytes": alg, "GBps": round(alg / (ms * 1e-3) / 1e9, 1)}
    return out


def run_all(ctx) -> Dict:
    out = {"allreduce_small": allreduce_small(ctx)}
    torch.cuda.empty_cache()
    out["moe_dispatch_combine"] = moe_dispatch_combine(ctx, odd_hidden=2052)
    torch.cuda.empty_cache()
    out["dlrm_shuffle"] = dlrm_shuffle(ctx, odd_dim=130)
    torch.cuda.empty_cache()
    out["grad_buckets"] = grad_buckets(ctx)
    torch.cuda.empty_cache()
    out["small_tensor_path"] = small_tensor_path(ctx)
    torch.cuda.empty_cache()
    out["dispatch_overhead_alltoall"] = dispatch_overhead(ctx)
    torch.cuda.empty_cache()
    out["small_cells_graph_replay"] = graph_replay(ctx)
    torch.cuda.empty_cache()
    out["rooted_collectives"] = rooted_collectives(ctx)
    torch.cuda.empty_cache()
    torch.cuda.empty_cache()
    return out
