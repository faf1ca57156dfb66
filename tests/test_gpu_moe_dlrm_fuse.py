"""GPU parity of MoE routing / pack / unpack / combine, the DLRM embedding shuffle and tensor
fusion against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2303_08374_amd import inputs, mcr
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


# ------------------------------------------------------------------------ routing
def _route_gpu(ids_per_rank, E, C):
    P = len(ids_per_rank)
    T = len(ids_per_rank[0])
    d_ids = [_i32(x) for x in ids_per_rank]
    d_slot = [torch.full((max(T, 1),), -77, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_cnt = [torch.full((E,), -77, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_S = torch.full((P * P,), -77, dtype=torch.int64, device="cuda")
    mcr.mcr_moe_route(gu.ctx(), d_ids, T, E, P, C, d_slot, d_cnt, d_S)
    gu.sync()
    return [s.cpu().numpy()[:T] for s in d_slot], [c.cpu().numpy() for c in d_cnt], d_S.cpu().numpy().reshape(P, P)


@pytest.mark.parametrize("T", [0, 1, 63, 64, 65, 1000, 16384, 20001])
@pytest.mark.parametrize("E,P", [(1, 1), (4, 2), (64, 16), (512, 8), (48, 3)])
def test_moe_route_matches_oracle(T, E, P):
    g = np.random.Generator(np.random.Philox(key=T * 1000 + E))
    for C in (0, 1, max(1, int(np.ceil(1.25 * T / E))), 1 << 30):
        ids = [g.integers(0, E, size=T).astype(np.int32) for _ in range(P)]
        if T > 10:
            ids[0][::7] = -1                # out-of-range ids are dropped
            ids[P - 1][3] = E
            ids[P - 1][:] = np.where(g.random(T) < 0.7, 0, ids[P - 1])     # a very hot expert
        slot, cnt, S = _route_gpu(ids, E, C)
        for p in range(P):
            es, ec, er = oracle.moe_route(ids[p], E, P, C)
            assert np.array_equal(slot[p], es), (T, E, P, C, p)
            assert np.array_equal(cnt[p], ec), (T, E, P, C, p)
            assert np.array_equal(S[p], er), (T, E, P, C, p)


@pytest.mark.parametrize("T", [2049, 4096, 16384, 20001, 70000, 150001])
@pytest.mark.parametrize("E,P", [(4, 2), (64, 16), (512, 8), (48, 3)])
def test_moe_route_with_workspace_matches_oracle(T, E, P):
    """Several workgroups per rank: the same slots, counts and splits as the definition."""
    rng = np.random.Generator(np.random.Philox(key=4000 + T + E))
    ids = [rng.integers(-1, E + 1, size=T).astype(np.int32) for _ in range(P)]           # a few ids out of range
    ids[0][: T // 2] = 1                                                              # one expert far over capacity
    C = int(np.ceil(1.25 * T / E))
    need = mcr.mcr_moe_route_workspace_bytes(T, E, P)
    assert need > 0
    d_ids = [_i32(x) for x in ids]
    d_slot = [torch.full((T,), -77, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_cnt = [torch.full((E,), -77, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_S = torch.full((P * P,), -77, dtype=torch.int64, device="cuda")
    ws = torch.full((need // 4 + 3,), -5, dtype=torch.int32, device="cuda")            # stale contents must not matter
    mcr.mcr_moe_route_ws(gu.ctx(), d_ids, T, E, P, C, d_slot, d_cnt, d_S, ws, need)
    gu.sync()
    assert (ws[need // 4:].cpu().numpy() == -5).all()                                # nothing past the stated size is touched
    for p in range(P):
        slot, counts, srow = oracle.moe_route(ids[p], E, P, C)
        assert np.array_equal(d_slot[p].cpu().numpy(), slot), f"slots rank {p}"
        assert np.array_equal(d_cnt[p].cpu().numpy(), counts)
        assert np.array_equal(d_S.cpu().numpy().reshape(P, P)[p], srow)
    with pytest.raises(mcr.McrError) as e:
        mcr.mcr_moe_route_ws(gu.ctx(), d_ids, T, E, P, C, d_slot, d_cnt, d_S, ws, need - 4)
    assert e.value.status == mcr.EINVAL


def test_moe_route_with_workspace_small_inputs_take_the_one_workgroup_path():
    T, E, P = 1000, 8, 4
    assert mcr.mcr_moe_route_workspace_bytes(T, E, P) == 0
    ids = [inputs.zipf_ids(T, E, 1.2, 11, p) for p in range(P)]
    d_slot = [torch.empty(T, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_cnt = [torch.empty(E, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_S = torch.empty(P * P, dtype=torch.int64, device="cuda")
    mcr.mcr_moe_route_ws(gu.ctx(), [_i32(x) for x in ids], T, E, P, 300, d_slot, d_cnt, d_S, None, 0)
    gu.sync()
    for p in range(P):
        assert np.array_equal(d_slot[p].cpu().numpy(), oracle.moe_route(ids[p], E, P, 300)[0])


def test_moe_route_zipf_workload():
    w = inputs.MoEWorkload()
    for permute in (False, True):
        ids = [w.ids(p, permute) for p in range(w.P)]
        slot, cnt, S = _route_gpu(ids, w.E, w.C)
        for p in range(w.P):
            es, ec, er = oracle.moe_route(ids[p], w.E, w.P, w.C)
            assert np.array_equal(slot[p], es) and np.array_equal(cnt[p], ec) and np.array_equal(S[p], er)


# ----------------------------------------------------------------- pack / unpack
@pytest.mark.parametrize("dtype,w", [(mcr.F32, 1), (mcr.F32, 4), (mcr.F32, 128), (mcr.BF16, 5), (mcr.BF16, 8),
                                      (mcr.BF16, 2048), (mcr.BF16, 24), (mcr.F32, 1028), (mcr.BF16, 1040), (mcr.F32, 516),
                                      (mcr.BF16, 8200), (mcr.BF16, 2052), (mcr.BF16, 2049), (mcr.F32, 1027), (mcr.F32, 515),
                                      (mcr.BF16, 1031), (mcr.BF16, 1), (mcr.BF16, 33), (mcr.F32, 17), (mcr.F32, 130),
                                      (mcr.BF16, 1021), (mcr.BF16, 516)])
def test_pack_unpack_combine(dtype, w):
    P, T, E = 3, 777, 12
    g = np.random.Generator(np.random.Philox(key=w))
    ids = [g.integers(0, E, size=T).astype(np.int32) for _ in range(P)]
    routes = [oracle.moe_route(ids[p], E, P, 40) for p in range(P)]
    slots = [r[0] for r in routes]
    out_rows = max(int(r[1].sum()) for r in routes) + 1
    toks = [inputs.normal(T * w, 800 + w, p, bf16=(dtype == mcr.BF16)) for p in range(P)]
    gates = [inputs.uniform01(T, 900 + w, p) for p in range(P)]
    fillv = 0x1111 if dtype == mcr.BF16 else 3.5
    exp_packed, exp_plain, exp_comb = [], [], []
    for p in range(P):
        buf = np.full(out_rows * w, fillv, dtype=gu.NPDT[dtype])
        oracle.pack(toks[p], slots[p], w, dtype, buf)
        exp_packed.append(buf)
        exp_plain.append(oracle.unpack(buf, slots[p], None, w, dtype))
        exp_comb.append(oracle.unpack(buf, slots[p], gates[p], w, dtype))
    vec_ok = (w * gu.EB[dtype]) % 16 == 0
    d_slot = [_i32(s) for s in slots]
    d_gate = [torch.from_numpy(x).cuda() for x in gates]
    for variant in [mcr.AUTO, 0] + ([1, 5] if vec_ok else []):
        d_tok = [gu.to_dev(t) for t in toks]
        d_packed = [gu.to_dev(np.full(out_rows * w, fillv, dtype=gu.NPDT[dtype])) for _ in range(P)]
        mcr.mcr_pack(gu.ctx(), d_packed, d_tok, d_slot, T, out_rows, w, dtype, P, variant)
        d_plain = [gu.dev_empty(T * w, dtype, 1) for _ in range(P)]
        d_comb = [gu.dev_empty(T * w, dtype, 1) for _ in range(P)]
        mcr.mcr_unpack(gu.ctx(), d_plain, d_packed, d_slot, None, T, out_rows, w, dtype, P, variant)
        mcr.mcr_unpack(gu.ctx(), d_comb, d_packed, d_slot, d_gate, T, out_rows, w, dtype, P, variant)
        gu.sync()
        for p in range(P):
            gu.assert_bits_equal(gu.to_host(d_packed[p], gu.NPDT[dtype]), exp_packed[p], f"pack w={w} v={variant}")
            gu.assert_bits_equal(gu.to_host(d_plain[p], gu.NPDT[dtype]), exp_plain[p], f"unpack w={w} v={variant}")
            gu.assert_bits_equal(gu.to_host(d_comb[p], gu.NPDT[dtype]), exp_comb[p], f"combine w={w} v={variant}")


def test_pack_skips_slots_beyond_capacity():
    T, w = 10, 4
    slot = np.array([0, 5, 2, 99, -1, 1, 3, 4, 7, -5], dtype=np.int32)      # 99 and 7 exceed out_rows=6
    tok = np.arange(T * w, dtype=np.float32)
    d_out = [gu.dev_empty(6 * w, mcr.F32, -1.0)]
    mcr.mcr_pack(gu.ctx(), d_out, [gu.to_dev(tok)], [_i32(slot)], T, 6, w, mcr.F32, 1, mcr.AUTO)
    gu.sync()
    got = gu.to_host(d_out[0], np.float32).reshape(6, w)
    for t, s in enumerate(slot):
        if 0 <= s < 6:
            assert np.array_equal(got[s], tok.reshape(T, w)[t])


def _moe_pipeline(w: inputs.MoEWorkload, permute=False, check_ranks=None, fused_variant=mcr.AUTO):
    """route -> pack -> alltoallv(S, device resident) -> [identity experts] -> alltoallv(S^T) ->
    gate-weighted combine, each stage compared with the oracle."""
    P, T, H, E, C = w.P, w.T, w.H, w.E, w.C
    ids = [w.ids(p, permute) for p in range(P)]
    toks = [w.tokens(p) for p in range(P)]
    gates = [w.gate(p) for p in range(P)]
    send_rows, recv_rows = T, w.recv_rows
    # device side
    d_ids = [_i32(x) for x in ids]
    d_tok = [gu.to_dev(t) for t in toks]
    d_gate = [torch.from_numpy(x).cuda() for x in gates]
    d_slot = [torch.empty(T, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_cnt = [torch.empty(E, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_S = torch.empty(P * P, dtype=torch.int64, device="cuda")
    d_packed = [gu.dev_empty(send_rows * H, mcr.BF16, 0) for _ in range(P)]
    d_recv = [gu.dev_empty(recv_rows * H, mcr.BF16, 0) for _ in range(P)]
    d_back = [gu.dev_empty(send_rows * H, mcr.BF16, 0) for _ in range(P)]
    d_out = [gu.dev_empty(T * H, mcr.BF16, 1) for _ in range(P)]
    c = gu.ctx()
    mcr.mcr_moe_route(c, d_ids, T, E, P, C, d_slot, d_cnt, d_S)
    mcr.mcr_pack(c, d_packed, d_tok, d_slot, T, send_rows, H, mcr.BF16, P)
    mcr.mcr_alltoallv(c, d_recv, d_packed, d_S, mcr.SPLITS_ON_DEVICE, send_rows, recv_rows, H, mcr.BF16, P)
    mcr.mcr_alltoallv(c, d_back, d_recv, d_S, mcr.SPLITS_ON_DEVICE | mcr.SPLITS_TRANSPOSED, recv_rows, send_rows, H, mcr.BF16, P)
    mcr.mcr_unpack(c, d_out, d_back, d_slot, d_gate, T, send_rows, H, mcr.BF16, P)
    gu.sync()
    # oracle side
    routes = [oracle.moe_route(ids[p], E, P, C) for p in range(P)]
    S = np.stack([r[2] for r in routes])
    assert np.array_equal(d_S.cpu().numpy().reshape(P, P), S)
    packed = []
    for p in range(P):
        buf = np.zeros(send_rows * H, dtype=np.uint16)
        oracle.pack(toks[p], routes[p][0], H, oracle.BF16, buf)
        packed.append(buf)
    recv = [np.zeros(recv_rows * H, dtype=np.uint16) for _ in range(P)]
    oracle.alltoallv(packed, S, H, oracle.BF16, recv)
    back = [np.zeros(send_rows * H, dtype=np.uint16) for _ in range(P)]
    oracle.alltoallv(recv, S, H, oracle.BF16, back, transposed=True)
    # the fused forms: dispatch = pack + alltoallv, combine = alltoallv(S^T) + gate-weighted unpack
    f_recv = [gu.dev_empty(recv_rows * H, mcr.BF16, 0) for _ in range(P)]
    f_out = [gu.dev_empty(T * H, mcr.BF16, 1) for _ in range(P)]
    f_plain = [gu.dev_empty(T * H, mcr.BF16, 1) for _ in range(P)]
    mcr.mcr_moe_dispatch(c, f_recv, d_tok, d_slot, d_S, T, recv_rows, H, mcr.BF16, P, fused_variant)
    mcr.mcr_moe_combine(c, f_out, f_recv, d_slot, d_gate, d_S, T, recv_rows, H, mcr.BF16, P, fused_variant)
    mcr.mcr_moe_combine(c, f_plain, f_recv, d_slot, None, d_S, T, recv_rows, H, mcr.BF16, P, fused_variant)
    # the same layout through the table-driven calls: source-major row table
    d_tab = torch.full((P * E,), -77, dtype=torch.int64, device="cuda")
    t_recv = [gu.dev_empty(recv_rows * H, mcr.BF16, 0) for _ in range(P)]
    t_out = [gu.dev_empty(T * H, mcr.BF16, 1) for _ in range(P)]
    mcr.mcr_moe_source_layout(c, d_cnt, E, P, d_tab)
    mcr.mcr_moe_dispatch_by_expert(c, t_recv, d_tok, d_ids, d_slot, d_tab, T, 1, E, recv_rows, H, mcr.BF16, P, fused_variant)
    mcr.mcr_moe_combine_by_expert(c, t_out, t_recv, d_ids, d_slot, d_gate, d_tab, T, 1, E, recv_rows, H, mcr.BF16, P, fused_variant)
    gu.sync()
    for p in (check_ranks if check_ranks is not None else range(P)):
        assert np.array_equal(d_slot[p].cpu().numpy(), routes[p][0])
        gu.assert_bits_equal(gu.to_host(d_packed[p], np.uint16), packed[p], f"packed r={p}")
        gu.assert_bits_equal(gu.to_host(d_recv[p], np.uint16), recv[p], f"recv r={p}")
        gu.assert_bits_equal(gu.to_host(d_back[p], np.uint16), back[p], f"back r={p}")
        exp = oracle.unpack(back[p], routes[p][0], gates[p], H, oracle.BF16)
        gu.assert_bits_equal(gu.to_host(d_out[p], np.uint16), exp, f"combine r={p}")
        gu.assert_bits_equal(gu.to_host(f_recv[p], np.uint16), recv[p], f"fused dispatch r={p}")
        gu.assert_bits_equal(gu.to_host(f_out[p], np.uint16), exp, f"fused combine r={p}")
        gu.assert_bits_equal(gu.to_host(t_recv[p], np.uint16), recv[p], f"table-driven source-major dispatch r={p}")
        gu.assert_bits_equal(gu.to_host(t_out[p], np.uint16), exp, f"table-driven source-major combine r={p}")
        gu.assert_bits_equal(gu.to_host(f_plain[p], np.uint16), oracle.unpack(back[p], routes[p][0], None, H, oracle.BF16),
                             f"fused combine without gate r={p}")


def test_moe_pipeline_small():
    _moe_pipeline(inputs.MoEWorkload(P=4, T=1000, H=72, E=8))
    _moe_pipeline(inputs.MoEWorkload(P=2, T=333, H=7, E=6), permute=True)     # rows not a multiple of 16 bytes
    _moe_pipeline(inputs.MoEWorkload(P=2, T=333, H=1, E=6), permute=True)     # one element per row
    _moe_pipeline(inputs.MoEWorkload(P=3, T=200, H=33, E=6), permute=True)
    for v in (0, 1, 4, 7, 10):
        _moe_pipeline(inputs.MoEWorkload(P=4, T=1000, H=72, E=8), fused_variant=v)
    _moe_pipeline(inputs.MoEWorkload(P=16, T=100, H=8, E=16, capacity_factor=0.5))   # heavy dropping, one-vector rows
    _moe_pipeline(inputs.MoEWorkload(P=1, T=65, H=16, E=3))
    # rows wider than half a workgroup: the one-row-per-workgroup forms of the fused pair (130 and 513 vectors per row)
    for v in (mcr.AUTO, 1, 6, 8, 11):
        _moe_pipeline(inputs.MoEWorkload(P=4, T=300, H=1040, E=8, capacity_factor=0.8), permute=True, fused_variant=v)
    _moe_pipeline(inputs.MoEWorkload(P=16, T=90, H=4104, E=16, capacity_factor=0.5))
    _moe_pipeline(inputs.MoEWorkload(P=1, T=65, H=2048, E=3))
    # wide rows that are not a multiple of 16 bytes (4104, 4098 and 2062 bytes): 16-byte pieces at
    # element-aligned addresses and a tail, in every stage of the chain and in the fused pair
    for H in (2052, 2049, 1031):
        _moe_pipeline(inputs.MoEWorkload(P=4, T=300, H=H, E=8, capacity_factor=0.8), permute=True)
    _moe_pipeline(inputs.MoEWorkload(P=16, T=90, H=2052, E=16, capacity_factor=0.5), fused_variant=0)


def test_moe_pipeline_config3_full_size():
    """P=16, T=16384, H=2048 bf16, E=64, Zipf(1.2), capacity 320: every stage, every rank."""
    _moe_pipeline(inputs.MoEWorkload())


def _moe_by_expert(w: inputs.MoEWorkload, permute=False, variant=mcr.AUTO, dtype=mcr.BF16, K=1):
    """route -> expert layout -> dispatch by expert -> [identity experts] -> combine by expert, with
    K choices per token (choice-major ids / slots / gates of K*T entries per rank)."""
    P, T, H, E = w.P, w.T, w.H, w.E
    A = K * T
    C = int(np.ceil(w.capacity_factor * A / E))
    npdt = gu.NPDT[dtype]
    # choice k of token t: the workload's id stream rotated by 17*k tokens (distinct experts are not required)
    ids = [np.concatenate([np.roll(w.ids(p, permute), 17 * k) for k in range(K)]).astype(np.int32) for p in range(P)]
    if dtype == mcr.BF16:
        toks = [w.tokens(p) for p in range(P)]
    else:
        toks = [inputs.bf16_bits_to_f32(w.tokens(p)) * np.float32(1.0009765625) for p in range(P)]
    gates = [inputs.uniform01(A, w.seed, p, 4) for p in range(P)]
    recv_rows = P * min(A, (E // P) * C)
    d_ids = [_i32(x) for x in ids]
    d_tok = [gu.to_dev(t) for t in toks]
    d_gate = [torch.from_numpy(x).cuda() for x in gates]
    d_slot = [torch.empty(max(A, 1), dtype=torch.int32, device="cuda") for _ in range(P)]
    d_cnt = [torch.empty(E, dtype=torch.int32, device="cuda") for _ in range(P)]
    d_S = torch.empty(P * P, dtype=torch.int64, device="cuda")
    d_tab = torch.full((P * E,), -77, dtype=torch.int64, device="cuda")
    d_first = torch.full((E,), -77, dtype=torch.int64, device="cuda")
    d_rows = torch.full((E,), -77, dtype=torch.int64, device="cuda")
    d_recv = [gu.dev_empty(max(recv_rows * H, 1), dtype, 0) for _ in range(P)]
    d_out = [gu.dev_empty(max(T * H, 1), dtype, 1) for _ in range(P)]
    d_plain = [gu.dev_empty(max(T * H, 1), dtype, 1) for _ in range(P)]
    c = gu.ctx()
    mcr.mcr_moe_route(c, d_ids, A, E, P, C, d_slot, d_cnt, d_S)
    mcr.mcr_moe_expert_layout(c, d_cnt, E, P, d_tab, d_first, d_rows)
    mcr.mcr_moe_dispatch_by_expert(c, d_recv, d_tok, d_ids, d_slot, d_tab, T, K, E, recv_rows, H, dtype, P, variant)
    mcr.mcr_moe_combine_by_expert(c, d_out, d_recv, d_ids, d_slot, d_gate, d_tab, T, K, E, recv_rows, H, dtype, P, variant)
    mcr.mcr_moe_combine_by_expert(c, d_plain, d_recv, d_ids, d_slot, None, d_tab, T, K, E, recv_rows, H, dtype, P, variant)
    gu.sync()
    routes = [oracle.moe_route(ids[p], E, P, C) for p in range(P)]
    slots = [r[0] for r in routes]
    counts = np.stack([r[1] for r in routes])
    bf, ef, er = oracle.moe_expert_layout(counts)
    assert np.array_equal(d_first.cpu().numpy(), ef) and np.array_equal(d_rows.cpu().numpy(), er)
    # the library's table is the oracle's block starts minus what each sender packs before the expert
    packed_before = np.cumsum(counts, axis=1) - counts
    assert np.array_equal(d_tab.cpu().numpy().reshape(P, E), bf - packed_before)
    recv = [np.zeros(max(recv_rows * H, 1), dtype=npdt) for _ in range(P)]
    oracle.moe_dispatch_by_expert(recv, toks, ids, slots, counts, H, dtype, K=K)
    exp_g = oracle.moe_combine_by_expert(recv, ids, slots, gates, counts, H, dtype, K=K)
    exp_p = oracle.moe_combine_by_expert(recv, ids, slots, None, counts, H, dtype, K=K)
    for p in range(P):
        gu.assert_bits_equal(gu.to_host(d_recv[p], npdt), recv[p], f"dispatch by expert r={p}")
        gu.assert_bits_equal(gu.to_host(d_out[p], npdt)[:T * H], exp_g[p], f"combine by expert r={p}")
        gu.assert_bits_equal(gu.to_host(d_plain[p], npdt)[:T * H], exp_p[p], f"combine by expert, no gate r={p}")


def test_moe_by_expert_small():
    _moe_by_expert(inputs.MoEWorkload(P=4, T=1000, H=72, E=8))
    _moe_by_expert(inputs.MoEWorkload(P=2, T=333, H=7, E=6), permute=True)        # rows not a multiple of 16 bytes
    _moe_by_expert(inputs.MoEWorkload(P=2, T=333, H=7, E=6), dtype=mcr.F32)
    _moe_by_expert(inputs.MoEWorkload(P=2, T=333, H=1, E=6), permute=True)        # one element per row
    for v in (0, 1, 4, 7, 10):
        _moe_by_expert(inputs.MoEWorkload(P=4, T=1000, H=72, E=8), variant=v)
        _moe_by_expert(inputs.MoEWorkload(P=3, T=500, H=256, E=48), variant=v, dtype=mcr.F32)   # rows a wavefront wide
    _moe_by_expert(inputs.MoEWorkload(P=16, T=100, H=8, E=16, capacity_factor=0.5))   # heavy dropping, one-vector rows
    _moe_by_expert(inputs.MoEWorkload(P=8, T=3000, H=16, E=512))                      # the largest expert count
    _moe_by_expert(inputs.MoEWorkload(P=1, T=65, H=16, E=3))
    _moe_by_expert(inputs.MoEWorkload(P=2, T=0, H=16, E=4))
    # rows wider than half a workgroup take the one-row-per-workgroup kernels: 130, 256, 257 and 1025 vectors per row
    for H, dt in ((1040, mcr.BF16), (2048, mcr.BF16), (1028, mcr.F32), (8200, mcr.BF16)):
        for v in (mcr.AUTO, 1, 6, 8, 11):
            _moe_by_expert(inputs.MoEWorkload(P=4, T=300, H=H, E=8, capacity_factor=0.8), variant=v, dtype=dt, permute=True)


def test_moe_by_expert_wide_rows_of_any_width():
    """Rows wider than half a workgroup whose width is not a multiple of 16 bytes: one row per
    workgroup, 16-byte pieces at element-aligned addresses and a tail of single elements."""
    for H, dt in ((2052, mcr.BF16), (2049, mcr.BF16), (1027, mcr.F32), (1031, mcr.BF16)):
        for K in (1, 2, 3):
            _moe_by_expert(inputs.MoEWorkload(P=4, T=300, H=H, E=8, capacity_factor=0.8), dtype=dt, K=K, permute=True)
    _moe_by_expert(inputs.MoEWorkload(P=16, T=90, H=2052, E=16, capacity_factor=0.5), variant=0)


@pytest.mark.parametrize("K", [2, 3, 4])
def test_moe_by_expert_top_k(K):
    _moe_by_expert(inputs.MoEWorkload(P=4, T=1000, H=72, E=8), K=K)
    _moe_by_expert(inputs.MoEWorkload(P=4, T=1000, H=72, E=8, capacity_factor=0.7), K=K, dtype=mcr.F32)   # many dropped choices
    _moe_by_expert(inputs.MoEWorkload(P=2, T=333, H=7, E=6), K=K, permute=True)                       # element path
    _moe_by_expert(inputs.MoEWorkload(P=2, T=333, H=7, E=6), K=K, dtype=mcr.F32, variant=0)
    for v in (1, 4, 7, 10):
        _moe_by_expert(inputs.MoEWorkload(P=3, T=500, H=256, E=48), variant=v, K=K)
    _moe_by_expert(inputs.MoEWorkload(P=2, T=0, H=16, E=4), K=K)
    _moe_by_expert(inputs.MoEWorkload(P=1, T=65, H=16, E=3), K=K)
    for H, dt in ((1040, mcr.BF16), (1028, mcr.F32), (4104, mcr.BF16)):                 # one row per workgroup
        for v in (mcr.AUTO, 7):
            _moe_by_expert(inputs.MoEWorkload(P=4, T=300, H=H, E=8, capacity_factor=0.8), variant=v, dtype=dt, K=K, permute=True)


def test_moe_by_expert_config3_full_size():
    """P=16, T=16384, H=2048 bf16, E=64, Zipf(1.2), capacity 320: every rank, every row."""
    _moe_by_expert(inputs.MoEWorkload())


def test_moe_top2_config3_full_size():
    """The same workload with two choices per token (capacity 640)."""
    _moe_by_expert(inputs.MoEWorkload(), K=2)


# ---------------------------------------------------------------------------- DLRM
def _dlrm_maps(w: inputs.DLRMWorkload):
    """Index maps for one rank's local permute between the alltoallv receive order
    [(owner, local) table order][b] and the batch-major layout [b][table]."""
    bl = w.batch // w.P
    order = [t for p in range(w.P) for t in w.tables_on(p)]          # receive order of tables
    pos = {t: k for k, t in enumerate(order)}
    b = np.arange(bl)[:, None]
    t = np.arange(w.n_tables)[None, :]
    recv_row = np.vectorize(pos.get)(t) * bl + b                      # [bl, n_tables] -> row in recv
    return recv_row.reshape(-1).astype(np.int32)


def _dlrm_roundtrip(w: inputs.DLRMWorkload, payload="normal"):
    P, NT, D, B = w.P, w.n_tables, w.dim, w.batch
    bl = B // P
    src = []
    for p in range(P):
        if payload == "normal":
            src.append(w.pooled(p))
        else:   # closed form: value = table * 2^14 + global batch index + column / 256
            tabs = w.tables_on(p)
            v = np.empty((len(tabs), B, D), dtype=np.float32)
            for li, t in enumerate(tabs):
                v[li] = (t * (1 << 14) + np.arange(B))[:, None] + np.arange(D)[None, :] / 256.0
            src.append(v.reshape(-1))
    S = w.splits()
    # the send buffer of rank p must be ordered by destination: [r][local table][b]; the pooled
    # source is [local table][B] = [local table][r][b], so this is itself an equal-block shuffle
    # of rows; done here with the same pack primitive (slot = destination-major row index).
    c = gu.ctx()
    n_local = [len(w.tables_on(p)) for p in range(P)]
    max_rows = max(n_local) * B
    send_slot = []
    for p in range(P):
        lt, r, b = np.meshgrid(np.arange(n_local[p]), np.arange(P), np.arange(bl), indexing="ij")
        s = (r * n_local[p] + lt) * bl + b
        full = np.full(max_rows, -1, dtype=np.int32)
        full[: s.size] = s.reshape(-1)
        send_slot.append(full)
    d_src = [gu.to_dev(np.concatenate([s, np.zeros(max_rows * D - s.size, dtype=np.float32)])) for s in src]
    d_send = [gu.dev_empty(max_rows * D, mcr.F32, 0) for _ in range(P)]
    d_recv = [gu.dev_empty(NT * bl * D, mcr.F32, 0) for _ in range(P)]
    d_out = [gu.dev_empty(bl * NT * D, mcr.F32, 0) for _ in range(P)]
    d_sslot = [_i32(s) for s in send_slot]
    perm = _dlrm_maps(w)
    d_perm = [_i32(perm) for _ in range(P)]
    mcr.mcr_pack(c, d_send, d_src, d_sslot, max_rows, max_rows, D, mcr.F32, P)
    mcr.mcr_alltoallv(c, d_recv, d_send, S, False, max_rows, NT * bl, D, mcr.F32, P)
    mcr.mcr_unpack(c, d_out, d_recv, d_perm, None, bl * NT, NT * bl, D, mcr.F32, P)
    gu.sync()
    exp = oracle.dlrm_forward(src, NT, B, D, oracle.F32)
    for r in range(P):
        gu.assert_bits_equal(gu.to_host(d_out[r], np.float32), exp[r], f"dlrm fwd r={r}")
    if payload != "normal":
        for r in range(P):
            o = gu.to_host(d_out[r], np.float32).reshape(bl, NT, D)
            b, t, col = np.meshgrid(np.arange(bl), np.arange(NT), np.arange(D), indexing="ij")
            assert np.array_equal(o, (t * (1 << 14) + r * bl + b + col / 256.0).astype(np.float32))
    # backward: the inverse permutation.  grad_out [bl][NT] -> recv order (pack with the same map),
    # alltoallv with S^T, then back to table-major (unpack with the send map).
    d_grecv = [gu.dev_empty(NT * bl * D, mcr.F32, 0) for _ in range(P)]
    d_gsend = [gu.dev_empty(max_rows * D, mcr.F32, 0) for _ in range(P)]
    d_gsrc = [gu.dev_empty(max_rows * D, mcr.F32, 0) for _ in range(P)]
    mcr.mcr_pack(c, d_grecv, d_out, d_perm, bl * NT, NT * bl, D, mcr.F32, P)
    mcr.mcr_alltoallv(c, d_gsend, d_grecv, S.T.copy(), False, NT * bl, max_rows, D, mcr.F32, P)
    mcr.mcr_unpack(c, d_gsrc, d_gsend, d_sslot, None, max_rows, max_rows, D, mcr.F32, P)
    gu.sync()
    gexp = oracle.dlrm_backward(exp, NT, B, D, oracle.F32)
    for p in range(P):
        got = gu.to_host(d_gsrc[p], np.float32)[: src[p].size]
        gu.assert_bits_equal(got, gexp[p], f"dlrm bwd r={p}")
        gu.assert_bits_equal(got, src[p], f"dlrm bwd(fwd) r={p}")
    # the fused single-pass shuffle, forward and backward
    for variant in (mcr.AUTO, 0, 1, 5, 8, 11):
        f_out = [gu.dev_empty(bl * NT * D, mcr.F32, 0) for _ in range(P)]
        f_src = [gu.dev_empty(max(src[p].size, 4), mcr.F32, 0) for p in range(P)]
        mcr.mcr_dlrm_shuffle(c, f_out, d_src, NT, B, D, mcr.F32, P, False, variant)
        mcr.mcr_dlrm_shuffle(c, f_src, f_out, NT, B, D, mcr.F32, P, True, variant)
        gu.sync()
        for r in range(P):
            gu.assert_bits_equal(gu.to_host(f_out[r], np.float32), exp[r], f"fused dlrm fwd v={variant} r={r}")
            gu.assert_bits_equal(gu.to_host(f_src[r], np.float32)[: src[r].size], gexp[r], f"fused dlrm bwd v={variant} r={r}")


def test_dlrm_small_closed_form():
    _dlrm_roundtrip(inputs.DLRMWorkload(P=4, n_tables=10, dim=8, batch=64), payload="closed")


def test_dlrm_fused_odd_shapes():
    """Fewer tables than ranks (some ranks own none), rows that are not a multiple of 16 bytes, bf16."""
    for P, NT, D, B, dtype in ((4, 3, 5, 16, mcr.F32), (8, 26, 12, 64, mcr.BF16), (1, 2, 8, 7, mcr.F32), (3, 7, 128, 9, mcr.BF16),
                               (8, 26, 130, 64, mcr.F32), (4, 5, 65, 32, mcr.BF16), (2, 3, 1, 8, mcr.BF16), (3, 4, 1027, 9, mcr.BF16),
                               (2, 3, 17, 10, mcr.F32), (4, 9, 2052, 8, mcr.BF16)):
        bf = dtype == mcr.BF16
        n_local = [len(range(p, NT, P)) for p in range(P)]
        src = [inputs.normal(max(n_local[p] * B * D, 0), 1300 + NT, p, bf16=bf) for p in range(P)]
        exp = oracle.dlrm_forward(src, NT, B, D, dtype)
        gexp = oracle.dlrm_backward(exp, NT, B, D, dtype)
        d_src = [gu.to_dev(s) if s.size else gu.dev_empty(8, dtype, 0) for s in src]
        for variant in (mcr.AUTO, 0):
            f_out = [gu.dev_empty((B // P) * NT * D, dtype, 0) for _ in range(P)]
            f_back = [gu.dev_empty(max(s.size, 8), dtype, 0) for s in src]
            mcr.mcr_dlrm_shuffle(gu.ctx(), f_out, d_src, NT, B, D, dtype, P, False, variant)
            mcr.mcr_dlrm_shuffle(gu.ctx(), f_back, f_out, NT, B, D, dtype, P, True, variant)
            gu.sync()
            for r in range(P):
                gu.assert_bits_equal(gu.to_host(f_out[r], gu.NPDT[dtype]), exp[r], f"fwd P={P} NT={NT} D={D} v={variant}")
                gu.assert_bits_equal(gu.to_host(f_back[r], gu.NPDT[dtype])[: src[r].size], gexp[r], f"bwd P={P} NT={NT} D={D}")


def test_dlrm_config4_full_size():
    """P=8, 26 tables x [16384, 128] fp32 round-robin, batch-sharded output [2048, 26, 128]."""
    _dlrm_roundtrip(inputs.DLRMWorkload(), payload="normal")
    _dlrm_roundtrip(inputs.DLRMWorkload(), payload="closed")


# ------------------------------------------------------------------- tensor fusion
def _fusion_case(numel, B, dtype, P, seed, variants):
    c = gu.ctx()
    plan = mcr.mcr_fuse_plan_create(c, numel, B, dtype)
    try:
        bn, tb, to = mcr.mcr_fuse_plan_info(plan, len(numel))
        otb, oto, obn = oracle.fuse_plan(numel, B)
        assert bn == obn.tolist() and tb == otb.tolist() and to == oto.tolist()
        bf = dtype == mcr.BF16
        host = [[inputs.normal(n, seed, p, i, std=1e-3, bf16=bf) for i, n in enumerate(numel)] for p in range(P)]
        # tensors live at odd offsets inside one arena per rank so that some are only element-aligned
        def arena(p):
            offs, cur = [], 1
            for n in numel:
                offs.append(cur)
                cur += n + (1 if n % 2 else 0)
            a = np.zeros(cur + 8, dtype=gu.NPDT[dtype])
            for i, n in enumerate(numel):
                a[offs[i]: offs[i] + n] = host[p][i]
            return a, offs
        for variant in variants:
            arenas, views = [], []
            for p in range(P):
                a, offs = arena(p)
                d = gu.to_dev(a)
                arenas.append(d)
                views += [d[offs[i]: offs[i] + numel[i]] for i in range(len(numel))]
            mcr.mcr_fuse_plan_bind(c, plan, views, P)
            for k in range(len(bn)):
                idx = [i for i in range(len(numel)) if tb[i] == k]
                flats = [gu.dev_empty(bn[k] + 3, dtype, 0) for _ in range(P)]
                fviews = [f[1:1 + bn[k]] if (k % 2) else f[:bn[k]] for f in flats]     # odd buckets: misaligned flat
                mcr.mcr_fuse(c, plan, k, fviews, P, variant)
                gu.sync()
                for p in range(P):
                    exp = oracle.fuse([host[p][i] for i in idx], [to[i] for i in idx], bn[k], dtype)
                    gu.assert_bits_equal(gu.to_host(fviews[p], gu.NPDT[dtype]), exp, f"fuse k={k} v={variant}")
                # reduce the flat buckets, then unfuse into the tensors
                mcr.mcr_allreduce(c, fviews, bn[k], dtype, mcr.AVG, P, mcr.AUTO)
                mcr.mcr_unfuse(c, plan, k, fviews, P, variant)
            gu.sync()
            exp_t = [[t.copy() for t in host[p]] for p in range(P)]
            for i in range(len(numel)):
                oracle.allreduce([exp_t[p][i] for p in range(P)], dtype, oracle.AVG)
            for p in range(P):
                for i in range(len(numel)):
                    gu.assert_reduced_equal(gu.to_host(views[p * len(numel) + i], gu.NPDT[dtype]), exp_t[p][i], dtype,
                                            f"fuse->allreduce->unfuse t={i} v={variant}")
            # the fused small-message path must give the same tensors without a flat buffer
            arenas2, views2 = [], []
            for p in range(P):
                a, offs = arena(p)
                d = gu.to_dev(a)
                arenas2.append(d)
                views2 += [d[offs[i]: offs[i] + numel[i]] for i in range(len(numel))]
            mcr.mcr_fuse_plan_bind(c, plan, views2, P)
            mcr.mcr_allreduce_multi(c, plan, -1, mcr.AVG, variant)
            gu.sync()
            for p in range(P):
                for i in range(len(numel)):
                    gu.assert_reduced_equal(gu.to_host(views2[p * len(numel) + i], gu.NPDT[dtype]), exp_t[p][i], dtype,
                                            f"allreduce_multi t={i} v={variant}")
                # nothing outside the tensors was written
                a, offs = arena(p)
                got = gu.to_host(arenas2[p], gu.NPDT[dtype])
                mask = np.ones(a.size, dtype=bool)
                for i, n in enumerate(numel):
                    mask[offs[i]: offs[i] + n] = False
                assert np.array_equal(got[mask], a[mask])
    finally:
        mcr.mcr_fuse_plan_destroy(plan)


@pytest.mark.parametrize("dtype", [mcr.F32, mcr.BF16])
def test_fusion_odd_sizes(dtype):
    _fusion_case([1, 3, 7, 8191, 2, 64, 20000, 5, 4096, 8192, 16385], 9000, dtype, P=3, seed=1000, variants=[mcr.AUTO, 0, 3, 5])


def test_fusion_scaled_down_gpt_list():
    w = inputs.GradBucketWorkload(layers=2, hidden=64, ffn=256, vocab=1000, bucket_elems=30000)
    _fusion_case(w.numel(), w.bucket_elems, mcr.BF16, P=8, seed=w.seed, variants=[mcr.AUTO])


def test_allreduce_multi_single_bucket():
    """bucket >= 0 reduces only that bucket's tensors."""
    numel = [100, 200, 5000, 50]
    c = gu.ctx()
    plan = mcr.mcr_fuse_plan_create(c, numel, 300, mcr.F32)
    try:
        bn, tb, to = mcr.mcr_fuse_plan_info(plan, len(numel))
        P = 2
        host = [[inputs.normal(n, 1100, p, i) for i, n in enumerate(numel)] for p in range(P)]
        dev = [[gu.to_dev(t) for t in host[p]] for p in range(P)]
        mcr.mcr_fuse_plan_bind(c, plan, [t for p in range(P) for t in dev[p]], P)
        mcr.mcr_allreduce_multi(c, plan, 0, mcr.SUM, mcr.AUTO)
        gu.sync()
        for i in range(len(numel)):
            exp = [host[p][i].copy() for p in range(P)]
            if tb[i] == 0:
                oracle.allreduce(exp, oracle.F32, oracle.SUM)
            for p in range(P):
                gu.assert_bits_equal(gu.to_host(dev[p][i], np.float32), exp[p], f"bucket-0 only t={i}")
    finally:
        mcr.mcr_fuse_plan_destroy(plan)


@pytest.mark.parametrize("H", [24, 2048])
def test_fused_moe_pair_with_hostile_splits_and_slots(H):
    """The split matrix and the slots are device data the library cannot check on the host: negative or huge split
    entries count as 0 / as T, slots outside the packed range and rows outside the receive buffer are skipped.  The
    result is what that rule says (modelled here in numpy), for the narrow-row and the one-row-per-workgroup kernels."""
    P, T, recv_rows = 4, 200, 150
    rng = np.random.Generator(np.random.Philox(key=5200 + H))
    S = rng.integers(0, 80, size=(P, P)).astype(np.int64)
    S[1, 2] = -5
    S[2, 0] = 1 << 40
    S[3, 3] = T + 7
    slots = [rng.integers(-3, T + 5, size=T).astype(np.int32) for _ in range(P)]
    # distinct destinations per sender are not guaranteed any more; make the slots of one sender distinct where valid
    for p in range(P):
        perm = rng.permutation(T + 8).astype(np.int32)[:T] - 3
        slots[p] = perm
    toks = [inputs.normal(T * H, 5201, p, 3, bf16=True) for p in range(P)]
    gates = [inputs.uniform01(T, 5202, p) for p in range(P)]
    Sc = np.clip(S, 0, T)
    sd = np.concatenate([np.zeros((P, 1), dtype=np.int64), np.cumsum(Sc, axis=1)], axis=1)       # sd[p][r]
    rd = np.cumsum(Sc, axis=0) - Sc                                                                 # rd[p][r]: rows above p in column r
    exp_recv = [np.zeros(recv_rows * H, dtype=np.uint16) for _ in range(P)]
    where = [[None] * T for _ in range(P)]
    for p in range(P):
        for t in range(T):
            s = int(slots[p][t])
            if s < 0 or s >= sd[p][P] or s >= T:
                continue
            r = int(sum(1 for q in range(1, P) if sd[p][q] <= s))
            row = int(rd[p][r] + (s - sd[p][r]))
            if row >= recv_rows:
                continue
            where[p][t] = (r, row)
    # two senders may now claim one row; keep the model simple by checking only rows claimed once
    claims = {}
    for p in range(P):
        for t in range(T):
            if where[p][t]:
                claims.setdefault(where[p][t], []).append((p, t))
    d_recv = [gu.dev_empty(recv_rows * H, mcr.BF16, 0) for _ in range(P)]
    d_slot = [torch.from_numpy(s).cuda() for s in slots]
    d_S = torch.from_numpy(S.reshape(-1)).cuda()
    d_tok = [gu.to_dev(x) for x in toks]
    mcr.mcr_moe_dispatch(gu.ctx(), d_recv, d_tok, d_slot, d_S, T, recv_rows, H, mcr.BF16, P)
    d_out = [gu.dev_empty(T * H, mcr.BF16, 1) for _ in range(P)]
    mcr.mcr_moe_combine(gu.ctx(), d_out, d_recv, d_slot, [torch.from_numpy(g).cuda() for g in gates], d_S, T, recv_rows, H,
                        mcr.BF16, P)
    gu.sync()
    got_recv = [gu.to_host(d, np.uint16).reshape(recv_rows, H) for d in d_recv]
    touched = [np.zeros(recv_rows, dtype=bool) for _ in range(P)]
    for (r, row), who in claims.items():
        touched[r][row] = True
        if len(who) == 1:
            p, t = who[0]
            assert np.array_equal(got_recv[r][row], toks[p].reshape(T, H)[t]), f"dispatch ({p},{t}) -> ({r},{row})"
        else:
            assert any(np.array_equal(got_recv[r][row], toks[p].reshape(T, H)[t]) for p, t in who)
    for r in range(P):
        assert (got_recv[r][~touched[r]] == 0).all(), "a row nobody claimed was written"
    for p in range(P):
        got = gu.to_host(d_out[p], np.uint16).reshape(T, H)
        for t in range(T):
            if where[p][t] is None:
                assert (got[t] == 0).all(), f"combine ({p},{t}) should be zeros"
            else:
                r, row = where[p][t]
                exp = oracle.unpack(got_recv[r][row].copy(), np.array([0], dtype=np.int32), gates[p][t:t + 1], H, oracle.BF16)
                assert np.array_equal(got[t], exp), f"combine ({p},{t})"
