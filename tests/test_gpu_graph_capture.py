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


def test_moe_chain_and_fused_pair_on_wide_rows_replay_from_a_graph():
    """Rows wide enough for the one-row kernels: the fused pair then keeps its displacement tables in
    a slot of the context's ring, which the captured graph holds on to while eager calls between the
    replays move the ring on.  The chain (pack, all_to_allv there and back with the matrix read
    transposed, unpack) and the fused pair must leave the same bits, eager and replayed."""
    c = gu.ctx()
    w = inputs.MoEWorkload(P=4, T=300, H=1040, E=8, capacity_factor=0.8)
    P, T, H, E, C = w.P, w.T, w.H, w.E, w.C
    R = w.recv_rows
    d_ids = [torch.from_numpy(w.ids(p, True)).cuda() for p in range(P)]
    d_tok = [gu.to_dev(w.tokens(p)) for p in range(P)]
    d_gate = [torch.from_numpy(w.gate(p)).cuda() for p in range(P)]
    d_slot = [torch.empty(T, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_cnt = [torch.empty(E, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_S = torch.empty(P * P, dtype=torch.int64, device="cuda")
    mk = lambda rows, fill: [gu.dev_empty(rows * H, mcr.BF16, fill) for _ in range(P)]
    d_packed, d_recv, d_back, d_out = mk(T, 0), mk(R, 0), mk(T, 0), mk(T, 1)
    f_recv, f_out = mk(R, 0), mk(T, 1)
    dev = mcr.SPLITS_ON_DEVICE

    def sequence(stream):
        mcr.mcr_moe_route(c, d_ids, T, E, P, C, d_slot, d_cnt, d_S, stream)
        mcr.mcr_pack(c, d_packed, d_tok, d_slot, T, T, H, mcr.BF16, P, mcr.AUTO, stream)
        mcr.mcr_alltoallv(c, d_recv, d_packed, d_S, dev, T, R, H, mcr.BF16, P, mcr.AUTO, stream)
        mcr.mcr_alltoallv(c, d_back, d_recv, d_S, dev | mcr.SPLITS_TRANSPOSED, R, T, H, mcr.BF16, P, mcr.AUTO, stream)
        mcr.mcr_unpack(c, d_out, d_back, d_slot, d_gate, T, T, H, mcr.BF16, P, mcr.AUTO, stream)
        mcr.mcr_moe_dispatch(c, f_recv, d_tok, d_slot, d_S, T, R, H, mcr.BF16, P, mcr.AUTO, stream)
        mcr.mcr_moe_combine(c, f_out, f_recv, d_slot, d_gate, d_S, T, R, H, mcr.BF16, P, mcr.AUTO, stream)

    def reset():
        for t in d_packed + d_recv + d_back + f_recv:
            t.zero_()
        for t in d_out + f_out:
            t.fill_(1)

    outputs = lambda: [t.clone() for t in d_slot + [d_S] + d_recv + d_out + f_recv + f_out]
    reset()
    sequence(None)
    gu.sync()
    eager = outputs()
    for p in range(P):
        assert torch.equal(d_out[p], f_out[p]) and torch.equal(d_recv[p], f_recv[p]), "the fused pair against the chain"
    # the eager result against the oracle, once
    slot0, _, _ = oracle.moe_route(w.ids(0, True), E, P, C)
    gu.assert_bits_equal(d_slot[0].cpu().numpy(), slot0, "eager routing")

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
        # eager fused calls between the replays take further slots of the ring
        for _ in range(3 + replay):
            mcr.mcr_moe_dispatch(c, f_recv, d_tok, d_slot, d_S, T, R, H, mcr.BF16, P)
        gu.sync()
