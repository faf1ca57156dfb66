"""Every operation entry point only enqueues kernels on the stream it is given (no allocation, no
synchronisation, no host round trip), so a sequence of them can be captured in a HIP graph and
replayed.  Each replay is checked against the eager result, with eager work and synchronisation
between the replays."""
import numpy as np
import pytest
import torch

import oracle
from paper_2303_08374_amd import inputs, mcr
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def test_collectives_and_moe_chain_replay_from_a_graph():
    c = gu.ctx()
    P, n = 4, 16 * 1024
    src = [gu.to_dev(x) for x in inputs.rank_buffers(P, n, 3100, "normal")]
    ar = [torch.empty_like(s) for s in src]
    ag = [gu.dev_empty(P * n, mcr.F32, 0) for _ in range(P)]
    a2a = [gu.dev_empty(n, mcr.F32, 0) for _ in range(P)]
    rs = [gu.dev_empty(n // P, mcr.F32, 0) for _ in range(P)]
    w = inputs.MoEWorkload(P=4, T=2000, H=64, E=8)
    T, H, E, C = w.T, w.H, w.E, w.C
    ids = [w.ids(p) for p in range(P)]
    toks = [w.tokens(p) for p in range(P)]
    gates = [w.gate(p) for p in range(P)]
    d_ids = [torch.from_numpy(x).cuda() for x in ids]
    d_tok = [gu.to_dev(t) for t in toks]
    d_gate = [torch.from_numpy(g).cuda() for g in gates]
    d_slot = [torch.empty(T, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_cnt = [torch.empty(E, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_S = torch.empty(P * P, dtype=torch.int64, device="cuda")
    d_tab = torch.empty(P * E, dtype=torch.int64, device="cuda")
    d_first = torch.empty(E, dtype=torch.int64, device="cuda")
    d_rows = torch.empty(E, dtype=torch.int64, device="cuda")
    d_recv = [gu.dev_empty(w.recv_rows * H, mcr.BF16, 0) for _ in range(P)]
    d_out = [gu.dev_empty(T * H, mcr.BF16, 1) for _ in range(P)]

    def sequence(stream):
        mcr.mcr_allreduce(c, ar, n, mcr.F32, mcr.SUM, P, mcr.AUTO, stream)
        mcr.mcr_allgather(c, ag, src, n, mcr.F32, P, mcr.AUTO, stream)
        mcr.mcr_alltoall(c, a2a, src, n, mcr.F32, P, mcr.AUTO, stream)
        mcr.mcr_reduce_scatter(c, rs, src, n, mcr.F32, mcr.AVG, P, mcr.AUTO, stream)
        mcr.mcr_moe_route(c, d_ids, T, E, P, C, d_slot, d_cnt, d_S, stream)
        mcr.mcr_moe_expert_layout(c, d_cnt, E, P, d_tab, d_first, d_rows, stream)
        mcr.mcr_moe_dispatch_by_expert(c, d_recv, d_tok, d_ids, d_slot, d_tab, T, 1, E, w.recv_rows, H, mcr.BF16, P, mcr.AUTO, stream)
        mcr.mcr_moe_combine_by_expert(c, d_out, d_recv, d_ids, d_slot, d_gate, d_tab, T, 1, E, w.recv_rows, H, mcr.BF16, P,
                                      mcr.AUTO, stream)

    outputs = lambda: [t.clone() for t in ar + ag + a2a + rs + d_slot + d_cnt + [d_S, d_tab, d_first, d_rows] + d_recv + d_out]

    def reset():
        for a, s in zip(ar, src):
            a.copy_(s)                      # all_reduce is in place: every run starts from the same values
        for t in ag + a2a + rs + d_recv:
            t.zero_()
        for t in d_out:
            t.fill_(1)

    reset()
    sequence(None)
    gu.sync()
    eager = outputs()
    # the eager result itself against the oracle, once
    host = [s.cpu().numpy().copy() for s in src]
    oracle.allreduce(host, oracle.F32, oracle.SUM)
    gu.assert_bits_equal(ar[2].cpu().numpy(), host[2], "eager all_reduce")

    graph = torch.cuda.CUDAGraph()
    reset()
    gu.sync()
    with torch.cuda.graph(graph):
        sequence(torch.cuda.current_stream().cuda_stream)
    for replay in range(4):
        reset()
        gu.sync()
        graph.replay()
        gu.sync()
        for k, (a, b) in enumerate(zip(outputs(), eager)):
            assert torch.equal(a, b), f"replay {replay}: output {k} differs from the eager run"
        # eager work of the same kind between the replays
        mcr.mcr_alltoall(c, a2a, src, n, mcr.F32, P)
        gu.sync()
