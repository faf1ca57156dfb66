"""Pins of the CPU oracle against things other than itself: hand-worked fixtures,
closed forms, involutions, brute force on tiny inputs and library routines
(numpy transposes / stable sorts, torch's CPU bf16 conversion).  CPU only.

Each check is a plain function so that the mutation test can re-run all of
them against a deliberately broken oracle build.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2303_08374_amd import inputs
from tests import golden_io as gio

F32, BF16, SUM, AVG = oracle.F32, oracle.BF16, oracle.SUM, oracle.AVG


def bits32(x):
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)


def is_bf16_nan(h):
    h = np.asarray(h, dtype=np.uint16)
    return ((h & 0x7F80) == 0x7F80) & ((h & 0x007F) != 0)


# =============================== bf16 rounding ================================
def check_bf16_golden():
    for s in gio.lines("bf16_rne_cases.txt"):
        a, b = s.split()[:2]
        x = np.array([int(a, 16)], dtype=np.uint32).view(np.float32)
        got = oracle.f32_to_bf16(x)[0]
        if b == "nan":
            assert is_bf16_nan(got), (a, hex(got))
        else:
            assert got == int(b, 16), (a, hex(got), b)


def check_bf16_vs_torch():
    # torch's CPU conversion is an independent round-to-nearest-even routine
    g = np.random.Generator(np.random.Philox(key=7))
    pats = g.integers(0, 1 << 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    # add every pattern whose discarded half is a tie or next to one, over a spread of upper halves
    hi = g.integers(0, 1 << 16, size=4096, dtype=np.uint64).astype(np.uint32) << 16
    near = np.concatenate([hi | lo for lo in (0x7FFF, 0x8000, 0x8001, 0x0000, 0xFFFF)])
    pats = np.concatenate([pats, near])
    x = pats.view(np.float32)
    got = oracle.f32_to_bf16(x)
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], ref[~nan])
    assert is_bf16_nan(got[nan]).all()


def check_bf16_widen_exact():
    h = np.arange(1 << 16, dtype=np.uint16)
    got = oracle.bf16_to_f32(h)
    ref = torch.from_numpy(h.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(bits32(got), bits32(ref))
    # widening then rounding is the identity on every non-NaN bf16 value
    back = oracle.f32_to_bf16(got)
    nan = is_bf16_nan(h)
    assert np.array_equal(back[~nan], h[~nan])


# ================================ all_reduce =================================
def check_allreduce_golden():
    for s in gio.lines("allreduce_cases.txt"):
        op, vals, exp = [t.strip() for t in s.split("|")]
        xs = [gio.f32_from_token(t) for t in vals.split()]
        bufs = [np.array([x], dtype=np.float32) for x in xs]
        oracle.allreduce(bufs, F32, SUM if op == "sum" else AVG)
        for b in bufs:
            if exp == "nan":
                assert np.isnan(b[0]), s
            else:
                assert bits32(b)[0] == bits32([gio.f32_from_token(exp)])[0], (s, hex(bits32(b)[0]))


def check_reduce_ops_golden_and_closed_form():
    ops = {"max": oracle.MAX, "min": oracle.MIN, "prod": oracle.PROD}
    for s in gio.lines("reduce_op_cases.txt"):
        op, vals, exp = [t.strip() for t in s.split("|")]
        bufs = [np.array([gio.f32_from_token(t)], dtype=np.float32) for t in vals.split()]
        with np.errstate(all="ignore"):
            oracle.allreduce(bufs, F32, ops[op])
        for b in bufs:
            if exp == "nan":
                assert np.isnan(b[0]), s
            else:
                assert bits32(b)[0] == bits32([gio.f32_from_token(exp)])[0], (s, hex(bits32(b)[0]))
    # numpy's reductions on NaN-free data; small-integer products are exact
    for dtype in (F32, BF16):
        P = 6
        bufs = inputs.rank_buffers(P, 5000, seed=81, dist="normal", bf16=(dtype == BF16))
        wide = np.stack([b if dtype == F32 else inputs.bf16_bits_to_f32(b) for b in bufs])
        for op, ref in ((oracle.MAX, wide.max(axis=0)), (oracle.MIN, wide.min(axis=0))):
            got = [b.copy() for b in bufs]
            oracle.allreduce(got, dtype, op)
            g = got[2] if dtype == F32 else inputs.bf16_bits_to_f32(got[2])
            assert np.array_equal(g, ref)
    i = np.arange(1000)
    bufs = [((i + p) % 3 + 1).astype(np.float32) for p in range(5)]          # factors 1..3, product <= 243
    expect = np.prod(np.stack(bufs).astype(np.int64), axis=0)
    oracle.allreduce(bufs, F32, oracle.PROD)
    assert np.array_equal(bufs[4], expect.astype(np.float32))
    # reduce_scatter and reduce take the same ops
    bufs = inputs.rank_buffers(4, 64, seed=82)
    rs = oracle.reduce_scatter(bufs, F32, oracle.MAX)
    assert np.array_equal(np.concatenate(rs), np.stack(bufs).max(axis=0))


def check_allreduce_closed_form():
    # small integers are exact in binary32 (and here in bf16) under any association
    for dtype in (F32, BF16):
        for P in (1, 2, 3, 4, 8, 16):
            n = 1000
            i = np.arange(n)
            # bf16 holds integers up to 256 exactly: keep the largest sum within that
            mod = 251 if dtype == F32 else max(2, 256 // (P * (P + 1) // 2))
            vals = [((p + 1) * (i % mod)).astype(np.float32) for p in range(P)]
            expect = (P * (P + 1) // 2) * (i % mod)
            if dtype == BF16:
                bufs = [inputs.f32_bits_to_bf16_trunc(v) for v in vals]   # exact: integers <= 256
            else:
                bufs = [v.copy() for v in vals]
            oracle.allreduce(bufs, dtype, SUM)
            for b in bufs:
                got = b if dtype == F32 else inputs.bf16_bits_to_f32(b)
                assert np.array_equal(got, expect.astype(np.float32)), (dtype, P)


def check_allreduce_loop_interchange():
    # rank-outer vectorised numpy accumulation must agree bit for bit with the
    # element-outer scalar loop of the oracle
    for P in (2, 3, 5, 8):
        bufs = inputs.rank_buffers(P, 4099, seed=11, dist="normal")
        acc = bufs[0].copy()
        for p in range(1, P):
            acc = acc + bufs[p]
        oracle.allreduce(bufs, F32, SUM)
        for b in bufs:
            assert np.array_equal(bits32(b), bits32(acc))


def check_allreduce_fp64_bound():
    for dtype, P in ((F32, 8), (F32, 16), (BF16, 8)):
        bufs = inputs.rank_buffers(P, 1 << 14, seed=12, dist="normal", bf16=(dtype == BF16))
        ref, mag = oracle.allreduce_ref64(bufs, dtype, SUM)
        # the reference itself against numpy's float64 sum
        wide = [b.astype(np.float64) if dtype == F32 else inputs.bf16_bits_to_f32(b).astype(np.float64) for b in bufs]
        assert np.allclose(ref, np.sum(wide, axis=0), rtol=1e-15, atol=0)
        assert np.allclose(mag, np.sum(np.abs(wide), axis=0), rtol=1e-15, atol=0)
        oracle.allreduce(bufs, dtype, SUM)
        if dtype == F32:
            err = np.abs(bufs[0].astype(np.float64) - ref)
            assert (err <= (P - 1) * 2.0 ** -24 * mag).all()
        else:
            # one rounding of an fp32 sum: within 1 bf16 ulp of the rounded exact sum
            exact = oracle.f32_to_bf16(ref.astype(np.float32))
            d = np.abs(bufs[0].astype(np.int32) - exact.astype(np.int32))
            assert d.max() <= 1
        for b in bufs[1:]:
            assert np.array_equal(b, bufs[0])


SPECIALS = np.array([0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x7FC00000, 0x7F7FFFFF,
                     0x00000001, 0x3F800000, 0xBF800000, 0x33800000], dtype=np.uint32).view(np.float32)


def check_allreduce_bruteforce_p2():
    # P=2: the reduction is a single IEEE addition; numpy's binary32 add is the library routine
    with np.errstate(all="ignore"):
        for n in (1, 2, 3, 8):
            for combo in itertools.islice(itertools.product(range(len(SPECIALS)), repeat=2), 0, None):
                a = np.full(n, SPECIALS[combo[0]], dtype=np.float32)
                b = np.full(n, SPECIALS[combo[1]], dtype=np.float32)
                a[n // 2] = SPECIALS[combo[1]]
                expect = a + b
                bufs = [a.copy(), b.copy()]
                oracle.allreduce(bufs, F32, SUM)
                for out in bufs:
                    nan = np.isnan(expect)
                    assert np.array_equal(np.isnan(out), nan)
                    assert np.array_equal(bits32(out)[~nan], bits32(expect)[~nan])


# ====================== rooted and vector collectives ==========================
def check_reduce_and_bcast():
    for dtype in (F32, BF16):
        P, n = 5, 333
        bufs = inputs.rank_buffers(P, n, seed=71, dist="normal", bf16=(dtype == BF16))
        for root in (0, 3):
            full = [b.copy() for b in bufs]
            oracle.allreduce(full, dtype, AVG)
            red = [b.copy() for b in bufs]
            oracle.reduce(red, dtype, AVG, root)
            for r in range(P):
                # the root holds what all_reduce gives everyone; the others are untouched
                assert np.array_equal(red[r], full[r] if r == root else bufs[r])
            bc = [b.copy() for b in bufs]
            oracle.bcast(bc, dtype, root)
            for r in range(P):
                assert np.array_equal(bc[r], bufs[root])
    # closed form
    bufs = [np.full(10, p + 1, dtype=np.float32) for p in range(4)]
    oracle.reduce(bufs, F32, SUM, 2)
    assert (bufs[2] == 10).all() and (bufs[0] == 1).all() and (bufs[3] == 4).all()


def check_gatherv_scatterv_allgatherv():
    # hand-worked: counts 2,0,3 -> displacements 0,2,2
    ins = [np.array([1, 2], dtype=np.float32), np.zeros(0, dtype=np.float32), np.array([7, 8, 9], dtype=np.float32)]
    g = oracle.gatherv(ins, [2, 0, 3], F32)
    assert g.tolist() == [1, 2, 7, 8, 9]
    sc = oracle.scatterv(g, [2, 0, 3], F32)
    assert [x.tolist() for x in sc] == [[1, 2], [], [7, 8, 9]]
    ag = oracle.allgatherv(ins, [2, 0, 3], F32)
    assert all(a.tolist() == [1, 2, 7, 8, 9] for a in ag)
    rng = np.random.Generator(np.random.Philox(key=72))
    for dtype in (F32, BF16):
        for P in (1, 3, 8):
            counts = rng.integers(0, 50, size=P).tolist()
            ins = [inputs.uniform_pm1(c, 73, p, bf16=(dtype == BF16)) for p, c in enumerate(counts)]
            g = oracle.gatherv(ins, counts, dtype)
            assert np.array_equal(g, np.concatenate(ins))                     # numpy's concatenation
            back = oracle.scatterv(g, counts, dtype)
            for p in range(P):
                assert np.array_equal(back[p], ins[p])                        # scatterv inverts gatherv
            for a in oracle.allgatherv(ins, counts, dtype):
                assert np.array_equal(a, g)
            # equal counts: all_gatherv is all_gather
            eq = [inputs.uniform_pm1(17, 74, p, bf16=(dtype == BF16)) for p in range(P)]
            a1 = oracle.allgatherv(eq, [17] * P, dtype)
            a2 = oracle.allgather(eq, dtype)
            for r in range(P):
                assert np.array_equal(a1[r], a2[r])


# ========================= reduce_scatter / all_gather =========================
def check_rs_ag_compose():
    for dtype in (F32, BF16):
        for P in (2, 4, 8):
            n = P * 131
            bufs = inputs.rank_buffers(P, n, seed=21, dist="uniform", bf16=(dtype == BF16))
            rs = oracle.reduce_scatter(bufs, dtype, SUM)
            ag = oracle.allgather(rs, dtype)
            ar = [b.copy() for b in bufs]
            oracle.allreduce(ar, dtype, SUM)
            for r in range(P):
                assert np.array_equal(ag[r].view(np.uint8), ar[r].view(np.uint8))


def check_reduce_scatter_closed_form():
    P, b = 4, 300
    n = P * b
    i = np.arange(n)
    bufs = [((p + 1) * (i % 251)).astype(np.float32) for p in range(P)]
    rs = oracle.reduce_scatter(bufs, F32, SUM)
    for r in range(P):
        j = np.arange(b)
        assert np.array_equal(rs[r], (10 * ((r * b + j) % 251)).astype(np.float32))


def check_allgather_closed_form():
    P, m = 5, 77
    ins = [(p * m + np.arange(m)).astype(np.float32) for p in range(P)]
    outs = oracle.allgather(ins, F32)
    for r in range(P):
        assert np.array_equal(outs[r], np.arange(P * m, dtype=np.float32))
    # bit copy: NaN payloads and -0 survive
    pats = np.array([0x7FC01234, 0x80000000, 0x7F800001, 0x00000001], dtype=np.uint32)
    outs = oracle.allgather([pats.view(np.float32), pats[::-1].copy().view(np.float32)], F32)
    assert np.array_equal(outs[1].view(np.uint32), np.concatenate([pats, pats[::-1]]))


# ================================= all_to_all =================================
def check_alltoall_transpose():
    for dtype in (F32, BF16):
        for P, b in ((2, 1), (3, 5), (8, 64), (16, 3)):
            n = P * b
            if dtype == F32:
                ins = [(p * (1 << 16) + np.arange(n)).astype(np.float32) for p in range(P)]
            else:
                ins = [((p * n + np.arange(n)) % 65536).astype(np.uint16) for p in range(P)]
            outs = oracle.alltoall(ins, dtype)
            # textbook: a P x P transpose of blocks
            ref = np.stack(ins).reshape(P, P, b).transpose(1, 0, 2).reshape(P, n)
            for r in range(P):
                assert np.array_equal(outs[r], ref[r])
            if dtype == F32:  # closed form: out[r][p*b+k] = p*2^16 + r*b + k
                for r in range(P):
                    p, k = np.divmod(np.arange(n), b)
                    assert np.array_equal(outs[r], (p * (1 << 16) + r * b + k).astype(np.float32))


def check_alltoallv_golden():
    g = gio.keyed_ints("alltoallv_case.txt")
    S = np.array(g["S"], dtype=np.int64).reshape(2, 2)
    ins = [np.array(g["in0"], dtype=np.float32), np.array(g["in1"], dtype=np.float32)]
    outs = oracle.alltoallv(ins, S, 1, F32)
    assert outs[0].tolist() == g["out0"] and outs[1].tolist() == g["out1"]


def _random_splits(P, max_rows, seed):
    g = np.random.Generator(np.random.Philox(key=seed))
    S = g.integers(0, max_rows + 1, size=(P, P), dtype=np.int64)
    S[g.random((P, P)) < 0.2] = 0
    return S


def check_alltoallv_properties():
    for P, w, seed in ((2, 1, 1), (4, 3, 2), (8, 16, 3), (16, 2, 4)):
        S = _random_splits(P, 9, seed)
        # payload encodes (source rank, source row, column)
        ins = []
        for p in range(P):
            rows = int(S[p].sum())
            v = (p << 20) + (np.arange(rows)[:, None] << 6) + np.arange(w)[None, :]
            ins.append(v.astype(np.float32).reshape(-1))
        outs = oracle.alltoallv(ins, S, w, F32)
        # slicing definition written with numpy cumsum / concatenate
        sd = np.concatenate([np.zeros((P, 1), dtype=np.int64), np.cumsum(S, axis=1)], axis=1)
        for r in range(P):
            ref = np.concatenate([ins[p].reshape(-1, w)[sd[p, r]:sd[p, r + 1]] for p in range(P)]).reshape(-1)
            assert np.array_equal(outs[r], ref)
        # every input row appears exactly once
        assert sorted(np.concatenate(ins).tolist()) == sorted(np.concatenate(outs).tolist())
        # involution with the transposed split matrix
        back = oracle.alltoallv(outs, S.T.copy(), w, F32)
        for p in range(P):
            assert np.array_equal(back[p], ins[p])


def check_alltoallv_transposed():
    """The way back (S[p][r] rows go from rank r to rank p): the hand-worked example returns to its
    inputs; on random matrices it is the forward exchange with the numpy-transposed matrix, the numpy
    slicing definition of that, and the inverse of the forward exchange."""
    g = gio.keyed_ints("alltoallv_case.txt")
    S = np.array(g["S"], dtype=np.int64).reshape(2, 2)
    outs = [np.array(g["out0"], dtype=np.float32), np.array(g["out1"], dtype=np.float32)]
    back = oracle.alltoallv(outs, S, 1, F32, transposed=True)
    assert back[0].tolist() == g["in0"] and back[1].tolist() == g["in1"]
    for P, w, seed in ((2, 1, 11), (3, 2, 12), (8, 4, 13), (16, 1, 14)):
        S = _random_splits(P, 7, seed)
        T = S.T.copy()
        ins = []
        for a in range(P):                      # rank a sends T[a][b] = S[b][a] rows to rank b
            rows = int(T[a].sum())
            v = (a << 20) + (np.arange(rows)[:, None] << 6) + np.arange(w)[None, :]
            ins.append(v.astype(np.float32).reshape(-1))
        got = oracle.alltoallv(ins, S, w, F32, transposed=True)
        via_forward = oracle.alltoallv(ins, T, w, F32)
        sd = np.concatenate([np.zeros((P, 1), dtype=np.int64), np.cumsum(T, axis=1)], axis=1)
        for b in range(P):
            ref = np.concatenate([ins[a].reshape(-1, w)[sd[a, b]:sd[a, b + 1]] for a in range(P)]).reshape(-1)
            assert np.array_equal(got[b], ref) and np.array_equal(got[b], via_forward[b])
        # forward with S, then the way back with the same S, is the identity
        fwd_in = [np.arange(int(S[p].sum()) * w, dtype=np.float32) + 1000 * p for p in range(P)]
        there = oracle.alltoallv(fwd_in, S, w, F32)
        home = oracle.alltoallv(there, S, w, F32, transposed=True)
        for p in range(P):
            assert np.array_equal(home[p], fwd_in[p])


def check_alltoallv_equal_is_alltoall():
    P, b, w = 4, 6, 5
    ins = inputs.rank_buffers(P, P * b * w, seed=31, dist="uniform")
    S = np.full((P, P), b, dtype=np.int64)
    a = oracle.alltoallv(ins, S, w, F32)
    e = oracle.alltoall(ins, F32)
    for r in range(P):
        assert np.array_equal(bits32(a[r]), bits32(e[r]))


def check_alltoallv_untouched_tail():
    P, w = 3, 2
    S = np.array([[1, 0, 2], [0, 0, 1], [2, 1, 0]], dtype=np.int64)
    ins = [np.arange(int(S[p].sum()) * w, dtype=np.float32) + 100 * p for p in range(P)]
    outs = [np.full(10 * w, -7.0, dtype=np.float32) for _ in range(P)]
    oracle.alltoallv(ins, S, w, F32, outs)
    for r in range(P):
        used = int(S[:, r].sum()) * w
        assert (outs[r][used:] == -7.0).all() and (outs[r][:used] != -7.0).all()


# ================================== MoE route =================================
def route_bruteforce(ids, E, P, C):
    """O(T^2) literal definition in Python."""
    T = len(ids)
    pos = [sum(1 for u in range(t) if ids[u] == ids[t]) for t in range(T)]
    total = [sum(1 for t in range(T) if ids[t] == e) for e in range(E)]
    cnt = [min(x, C) for x in total]
    base = [sum(cnt[:e]) for e in range(E)]
    slot = [base[ids[t]] + pos[t] if pos[t] < C else -1 for t in range(T)]
    per = E // P
    srow = [sum(cnt[r * per:(r + 1) * per]) for r in range(P)]
    return slot, cnt, srow


def check_route_golden():
    g = gio.keyed_ints("moe_route_case.txt")
    slot, cnt, srow = oracle.moe_route(np.array(g["ids"]), g["E"][0], g["P"][0], g["C"][0])
    assert slot.tolist() == g["slot"] and cnt.tolist() == g["counts"] and srow.tolist() == g["srow"]


def check_route_bruteforce():
    g = np.random.Generator(np.random.Philox(key=41))
    for T, E, P, C in ((0, 4, 2, 2), (1, 1, 1, 1), (17, 4, 2, 3), (64, 8, 4, 5), (64, 8, 8, 0), (50, 6, 3, 100)):
        ids = g.integers(0, E, size=T).astype(np.int32)
        slot, cnt, srow = oracle.moe_route(ids, E, P, C)
        bs, bc, br = route_bruteforce(ids.tolist(), E, P, C)
        assert slot.tolist() == bs and cnt.tolist() == bc and srow.tolist() == br


def check_route_invariants_and_sort():
    w = inputs.MoEWorkload(T=4096)
    for rank in (0, 5):
        for permute in (False, True):
            ids = w.ids(rank, permute)
            slot, cnt, srow = oracle.moe_route(ids, w.E, w.P, w.C)
            kept = slot >= 0
            nk = int(kept.sum())
            assert cnt.sum() == nk and (cnt <= w.C).all() and srow.sum() == nk
            assert sorted(slot[kept].tolist()) == list(range(nk))            # bijection onto [0, kept)
            assert np.array_equal(cnt, np.minimum(np.bincount(ids, minlength=w.E), w.C))
            # textbook: stable sort by expert id, truncate each group to C
            order = np.argsort(ids, kind="stable")
            rank_in_group = np.arange(len(ids)) - np.searchsorted(ids[order], ids[order], side="left")
            kept_sorted = order[rank_in_group < w.C]
            assert np.array_equal(np.argsort(np.where(kept, slot, 1 << 30), kind="stable")[:nk], kept_sorted)
            assert np.array_equal(srow, cnt.reshape(w.P, -1).sum(axis=1))


def check_route_out_of_range_ids():
    ids = np.array([0, -1, 1, 7, 0, 1], dtype=np.int32)
    slot, cnt, srow = oracle.moe_route(ids, 2, 2, 4)
    assert slot.tolist() == [0, -1, 2, -1, 1, 3] and cnt.tolist() == [2, 2] and srow.tolist() == [2, 2]


# ============================ fp16 and int32 =====================================
def check_f16_widening_is_numpy_float16_for_every_pattern():
    h = np.arange(65536, dtype=np.uint16)
    got = oracle.f16_bits_to_f32(h)
    exp = h.view(np.float16).astype(np.float32)
    nan = np.isnan(exp)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), exp[~nan].view(np.uint32))
    # NaN payloads keep their place (fraction << 13)
    assert np.array_equal(got[nan].view(np.uint32) & 0x7fffff, (h[nan].astype(np.uint32) & 0x3ff) << 13)


def check_f16_rounding_against_numpy_and_by_hand():
    F16 = np.float16
    rng = np.random.default_rng(5)
    # random binary32 patterns over the whole range, and dense samples around every fp16 value and midpoint
    pats = rng.integers(0, 2**32, size=400000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    halves = np.arange(0x7c00, dtype=np.uint16).view(F16).astype(np.float64)          # all finite non-negative
    mids = (halves[:-1] + halves[1:]) / 2
    around = np.concatenate([halves, mids, np.nextafter(mids.astype(np.float32), np.float32(np.inf)).astype(np.float64),
                             np.nextafter(mids.astype(np.float32), np.float32(-np.inf)).astype(np.float64),
                             [65504.0, 65519.99, 65520.0, 65536.0, 1e30, 2.0**-24, 2.0**-25, 2.0**-25 * 1.0000001, 2.0**-26, 0.0]])
    xs = np.concatenate([pats, around.astype(np.float32), -around.astype(np.float32), [np.float32(np.inf), -np.float32(np.inf)]]).astype(np.float32)
    finite_or_inf = ~np.isnan(xs)
    with np.errstate(over="ignore"):
        exp = xs.astype(F16).view(np.uint16)
    got = oracle.f32_to_f16_bits(xs)
    assert np.array_equal(got[finite_or_inf], exp[finite_or_inf])
    nan_in = np.isnan(xs)
    assert ((got[nan_in] & 0x7c00) == 0x7c00).all() and ((got[nan_in] & 0x3ff) != 0).all()
    # by hand: ties to even at 1 + 2^-11 (down to 1.0) and 1 + 3*2^-11 (up to 1 + 2^-9); 65520 overflows; 2^-25 is a tie to 0
    by_hand = {1.0 + 2.0**-11: 0x3c00, 1.0 + 3 * 2.0**-11: 0x3c02, 65520.0: 0x7c00, 65519.0: 0x7bff, 2.0**-25: 0x0000,
               3 * 2.0**-25: 0x0002, 2.0**-14 - 2.0**-25: 0x0400, -2.0: 0xc000}
    for x, bits in by_hand.items():
        assert int(oracle.f32_to_f16_bits(np.array([x], dtype=np.float32))[0]) == bits, x


def check_f16_allreduce_brute_force():
    """P=2 and 3: numpy's own float16 -> float32, binary32 add in rank order, -> float16."""
    rng = np.random.default_rng(6)
    special = np.array([0.0, -0.0, 1.0, -1.0, 65504.0, -65504.0, 6.1e-5, 6e-8, np.inf, -np.inf, 1000.0, 0.333], dtype=np.float16)
    for P in (2, 3):
        bufs = [np.concatenate([rng.standard_normal(500).astype(np.float16) * np.float16(100), rng.permutation(np.tile(special, 4))]) for _ in range(P)]
        for op, f in ((SUM, None), (AVG, None), (oracle.MAX, None), (oracle.PROD, None)):
            acc = bufs[0].astype(np.float32)
            with np.errstate(all="ignore"):
                for b in bufs[1:]:
                    x = b.astype(np.float32)
                    if op in (SUM, AVG):
                        acc = (acc + x).astype(np.float32)
                    elif op == oracle.PROD:
                        acc = (acc * x).astype(np.float32)
                    else:
                        acc = np.where((x > acc) | np.isnan(x), x, acc)
                if op == AVG:
                    acc = (acc * (np.float32(1.0) / np.float32(P))).astype(np.float32)
                exp = acc.astype(np.float16)
            work = [b.copy() for b in bufs]
            oracle.allreduce(work, oracle.F16, op)
            nan = np.isnan(exp)
            for wbuf in work:
                assert np.array_equal(np.isnan(wbuf), nan)
                assert np.array_equal(wbuf[~nan].view(np.uint16), exp[~nan].view(np.uint16)), (P, op)


def check_i32_reductions_wrap_like_numpy():
    rng = np.random.default_rng(8)
    for P in (1, 2, 5):
        bufs = [rng.integers(-2**31, 2**31, size=300, dtype=np.int64).astype(np.int32) for _ in range(P)]
        for b in bufs:
            b[:4] = [2**31 - 1, -2**31, -1, 0]
        with np.errstate(over="ignore"):
            exp = {SUM: np.sum(np.stack(bufs).astype(np.int64), axis=0).astype(np.int32),            # mod 2^32 of the exact sum
                   oracle.MAX: np.max(np.stack(bufs), axis=0), oracle.MIN: np.min(np.stack(bufs), axis=0),
                   oracle.PROD: np.array([int(np.prod([int(b[i]) for b in bufs], dtype=object)) & 0xffffffff for i in range(300)],
                                         dtype=np.uint32).view(np.int32)}
        for op, e in exp.items():
            work = [b.copy() for b in bufs]
            oracle.allreduce(work, oracle.I32, op)
            assert all(np.array_equal(wb, e) for wb in work), (P, op)
            if 300 % P == 0:
                rs = oracle.reduce_scatter(bufs, oracle.I32, op)
                assert np.array_equal(np.concatenate(rs), e)
        with pytest.raises(ValueError):
            oracle.allreduce([b.copy() for b in bufs], oracle.I32, AVG)


# ============================ displacements chosen by the caller ================
def check_alltoallv_displs_golden():
    g = gio.keyed_ints("alltoallv_displs_case.txt")
    P = g["P"][0]
    ins = [np.array(g[f"send{p}"], dtype=np.float32) for p in range(P)]
    outs = [np.full(len(g[f"recv{r}"]), -1, dtype=np.float32) for r in range(P)]
    sq = lambda k: np.array(g[k], dtype=np.int64).reshape(P, P)
    oracle.alltoallv_displs(outs, ins, sq("counts"), sq("sdispls"), sq("rdispls"), 1, F32)
    for r in range(P):
        assert outs[r].tolist() == g[f"recv{r}"]


def check_displs_reduce_to_the_packed_forms_and_to_numpy_slicing():
    rng = np.random.default_rng(11)
    for P, dtype, re in ((3, F32, 1), (4, BF16, 5), (1, F32, 2)):
        npdt = oracle.np_dtype(dtype)
        mk = lambda n: rng.integers(0, 60000, size=n).astype(npdt)
        # packed displacements give what the packed functions (pinned elsewhere) give
        S = rng.integers(0, 6, size=(P, P)).astype(np.int64)
        S[0, P - 1] = 0
        ins = [mk(int(S[p].sum()) * re) for p in range(P)]
        SD = np.cumsum(S, axis=1) - S
        RD = (np.cumsum(S, axis=0) - S).T.copy()                 # RD[r, p] = rows of senders before p at receiver r
        outs = [np.full(int(S[:, r].sum()) * re, 7, dtype=npdt) for r in range(P)]
        oracle.alltoallv_displs(outs, ins, S, SD, RD, re, dtype)
        for a, b in zip(outs, oracle.alltoallv(ins, S, re, dtype)):
            assert np.array_equal(a, b)
        counts = rng.integers(0, 9, size=P)
        counts[P // 2] = 0
        packed = np.cumsum(counts) - counts
        gin = [mk(int(c)) for c in counts]
        out = np.full(int(counts.sum()), 7, dtype=npdt)
        oracle.gatherv_displs(out, gin, counts, packed, dtype)
        assert np.array_equal(out, oracle.gatherv(gin, counts, dtype))
        root = mk(int(counts.sum()))
        for a, b in zip(oracle.scatterv_displs(root, counts, packed, dtype), oracle.scatterv(root, counts, dtype)):
            assert np.array_equal(a, b)
        # blocks in reverse order with a gap of 2 between them: numpy slicing says where everything is
        displs = np.zeros(P, dtype=np.int64)
        at = 1
        for p in reversed(range(P)):
            displs[p] = at
            at += int(counts[p]) + 2
        out = np.full(at, 7, dtype=npdt)
        oracle.gatherv_displs(out, gin, counts, displs, dtype)
        exp = np.full(at, 7, dtype=npdt)
        for p in range(P):
            exp[displs[p]: displs[p] + counts[p]] = gin[p]
        assert np.array_equal(out, exp)
        outs = [np.full(at, 9, dtype=npdt) for _ in range(P)]
        oracle.allgatherv_displs(outs, gin, counts, displs, dtype)
        exp9 = np.full(at, 9, dtype=npdt)
        for p in range(P):
            exp9[displs[p]: displs[p] + counts[p]] = gin[p]
        assert all(np.array_equal(o, exp9) for o in outs)
        src = mk(at)
        for r, o in enumerate(oracle.scatterv_displs(src, counts, displs, dtype)):
            assert np.array_equal(o, src[displs[r]: displs[r] + counts[r]])


# ============================ expert-major receive layout =======================
def check_expert_layout_golden():
    g = gio.keyed_ints("moe_expert_layout_case.txt")
    E, P = g["E"][0], g["P"][0]
    bf, ef, er = oracle.moe_expert_layout(np.array(g["counts"], dtype=np.int32).reshape(P, E))
    assert er.tolist() == g["expert_rows"] and ef.tolist() == g["expert_first"] and bf.reshape(-1).tolist() == g["block_first"]


def check_dispatch_by_expert_is_a_stable_regroup():
    """The expert-major receive buffer holds the rows of the source-major one (pack + all_to_allv),
    stably re-sorted by local expert; every expert's rows form one block of expert_rows[e] rows."""
    for w, permute in ((inputs.MoEWorkload(P=4, T=300, H=4, E=8), False), (inputs.MoEWorkload(P=2, T=77, H=3, E=6, capacity_factor=0.6), True),
                       (inputs.MoEWorkload(P=1, T=40, H=2, E=3), False)):
        P, T, H, E = w.P, w.T, w.H, w.E
        ids = [w.ids(p, permute) for p in range(P)]
        routes = [oracle.moe_route(ids[p], E, P, w.C) for p in range(P)]
        slots = [r[0] for r in routes]
        counts = np.stack([r[1] for r in routes])
        S = np.stack([r[2] for r in routes])
        # payload: float(p * 2^16 + t) in column 0, the expert id in column 1
        toks = []
        for p in range(P):
            v = np.zeros((T, H), dtype=np.float32)
            v[:, 0] = p * 65536 + np.arange(T)
            v[:, 1] = ids[p]
            toks.append(v.reshape(-1))
        # source-major reference through the already pinned chain
        packed = []
        for p in range(P):
            buf = np.zeros(int(S[p].sum()) * H, dtype=np.float32)
            oracle.pack(toks[p], slots[p], H, F32, buf)
            packed.append(buf)
        src_major = oracle.alltoallv(packed, S, H, F32)
        bf, ef, er = oracle.moe_expert_layout(counts)
        assert np.array_equal(er, counts.sum(axis=0))
        recv = [np.full(int(S[:, r].sum()) * H, -1.0, dtype=np.float32) for r in range(P)]
        oracle.moe_dispatch_by_expert(recv, toks, ids, slots, counts, H, F32)
        per = E // P
        for r in range(P):
            a = src_major[r].reshape(-1, H)
            b = recv[r].reshape(-1, H)
            order = np.argsort(a[:, 1], kind="stable")            # numpy's stable sort by expert id
            assert np.array_equal(b, a[order])
            for e in range(r * per, (r + 1) * per):
                blk = b[ef[e]: ef[e] + er[e]]
                assert (blk[:, 1] == e).all()
        # combine with gate 1 returns the kept tokens, zeros elsewhere; gate 2^-1 halves them exactly
        back = oracle.moe_combine_by_expert(recv, ids, slots, None, counts, H, F32)
        half = oracle.moe_combine_by_expert(recv, ids, slots, [np.full(T, 0.5, dtype=np.float32)] * P, counts, H, F32)
        for p in range(P):
            kept = slots[p] >= 0
            exp = np.where(kept[:, None], toks[p].reshape(T, H), 0)
            assert np.array_equal(back[p].reshape(T, H), exp)
            assert np.array_equal(half[p].reshape(T, H), exp * np.float32(0.5))


def check_top2_golden():
    g = gio.keyed_ints("moe_top2_case.txt")
    E, P, T, K, C = (g[k][0] for k in "EPTKC")
    ids = np.array(g["ids"], dtype=np.int32)
    slot, counts, _ = oracle.moe_route(ids, E, P, C)                # routing walks the K*T assignments in order
    assert slot.tolist() == g["slot"] and counts.tolist() == g["counts"]
    tok = np.array(g["tokens"], dtype=np.float32)
    recv = [np.full(len(g["recv"]), -1, dtype=np.float32)]
    oracle.moe_dispatch_by_expert(recv, [tok], [ids], [slot], counts[None, :], 2, F32, K=K)
    assert recv[0].tolist() == g["recv"]
    gate = np.array(g["gate_x16"], dtype=np.float32) / 16
    out = oracle.moe_combine_by_expert(recv, [ids], [slot], [gate], counts[None, :], 2, F32, K=K)
    assert (out[0] * 16).tolist() == g["out_x16"]


def check_topk_combine_against_numpy_binary32():
    """K = 3: the weighted sum is binary32 multiply, binary32 add in choice order, one rounding
    (numpy float32 arithmetic as the library routine); dropped assignments add nothing; the order
    matters for K = 3, so a sum taken in another order fails here."""
    for dtype, K, w in ((F32, 3, inputs.MoEWorkload(P=2, T=200, H=5, E=4, capacity_factor=2.2)),
                        (BF16, 3, inputs.MoEWorkload(P=2, T=200, H=5, E=4, capacity_factor=2.2)),
                        (BF16, 2, inputs.MoEWorkload(P=4, T=150, H=3, E=8, capacity_factor=1.6))):
        P, T, H, E = w.P, w.T, w.H, w.E
        C = int(np.ceil(w.capacity_factor * T / E))
        rng = np.random.default_rng(7 + K)
        ids = [np.concatenate([np.roll(w.ids(p, True), 17 * k) for k in range(K)]).astype(np.int32) for p in range(P)]
        gates = [rng.random(K * T, dtype=np.float32) for p in range(P)]
        routes = [oracle.moe_route(ids[p], E, P, C) for p in range(P)]
        slots = [r[0] for r in routes]
        counts = np.stack([r[1] for r in routes])
        assert any((s < 0).any() for s in slots) and any((s >= 0).all(axis=0).any() for s in [x.reshape(K, T) for x in slots])
        if dtype == F32:
            toks = [rng.standard_normal(T * H).astype(np.float32) for p in range(P)]
            for x in toks:
                x[::7] = np.float32(-0.0)                         # a sum that starts from +0 would lose the sign
            as_f32 = lambda x: x
            to_dt = lambda x: x.astype(np.float32)
        else:
            toks = [w.tokens(p) for p in range(P)]
            as_f32 = inputs.bf16_bits_to_f32
            to_dt = lambda x: torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        bf, ef, er = oracle.moe_expert_layout(counts)
        rows = int(er.reshape(P, -1).sum(axis=1).max())
        recv = [np.zeros(rows * H, dtype=toks[0].dtype) for _ in range(P)]
        oracle.moe_dispatch_by_expert(recv, toks, ids, slots, counts, H, dtype, K=K)
        got = oracle.moe_combine_by_expert(recv, ids, slots, gates, counts, H, dtype, K=K)
        for p in range(P):
            x = as_f32(toks[p]).reshape(T, H)                     # identity experts: the row that comes back is the token
            kept = (slots[p] >= 0).reshape(K, T)
            g = gates[p].reshape(K, T)
            acc = np.zeros((T, H), dtype=np.float32)
            started = np.zeros(T, dtype=bool)
            for k in range(K):
                term = (g[k][:, None] * x).astype(np.float32)
                summed = (acc + term).astype(np.float32)
                nxt = np.where(started[:, None], summed, term)
                acc = np.where(kept[k][:, None], nxt, acc)
                started |= kept[k]
            exp = to_dt(np.where(started[:, None], acc, np.float32(0)))
            assert np.array_equal(got[p].view(np.uint8), np.ascontiguousarray(exp).reshape(-1).view(np.uint8)), (dtype, K, p)


# ============================ pack / unpack / combine ==========================
def check_pack_unpack_identity():
    for dtype, w in ((F32, 5), (BF16, 8)):
        T = 200
        g = np.random.Generator(np.random.Philox(key=51))
        ids = g.integers(0, 8, size=T).astype(np.int32)
        slot, cnt, _ = oracle.moe_route(ids, 8, 4, 20)
        nk = int(cnt.sum())
        tok = inputs.normal(T * w, 52, 0, bf16=(dtype == BF16))
        packed = np.full(nk * w, 0xAB, dtype=oracle.np_dtype(dtype)) if dtype == BF16 else np.full(nk * w, np.nan, dtype=np.float32)
        oracle.pack(tok, slot, w, dtype, packed)
        # numpy fancy-index definition
        ref = np.empty((nk, w), dtype=tok.dtype)
        ref[slot[slot >= 0]] = tok.reshape(T, w)[slot >= 0]
        assert np.array_equal(packed.view(np.uint8), ref.reshape(-1).view(np.uint8))
        back = oracle.unpack(packed, slot, None, w, dtype).reshape(T, w)
        assert np.array_equal(back[slot >= 0].view(np.uint8), tok.reshape(T, w)[slot >= 0].view(np.uint8))
        assert (back[slot < 0].view(np.uint8) == 0).all()


def check_combine_gate():
    T, w = 64, 16
    slot = np.arange(T, dtype=np.int32)
    slot[::5] = -1
    slot[slot >= 0] = np.random.Generator(np.random.Philox(key=53)).permutation(int((slot >= 0).sum())).astype(np.int32)
    nk = int((slot >= 0).sum())
    packed = inputs.normal(nk * w, 54, 0, bf16=True)
    # powers of two: exact scaling
    gate = np.float32(2.0) ** np.random.Generator(np.random.Philox(key=55)).integers(-3, 3, size=T).astype(np.float32)
    out = oracle.unpack(packed, slot, gate, w, BF16).reshape(T, w)
    pf = inputs.bf16_bits_to_f32(packed).reshape(nk, w)
    for t in range(T):
        if slot[t] < 0:
            assert (out[t] == 0).all()
        else:
            assert np.array_equal(inputs.bf16_bits_to_f32(out[t]), pf[slot[t]] * gate[t])
    # general gates: torch's fp32 multiply + bf16 conversion is the library routine
    gate = inputs.uniform01(T, 56, 0)
    out = oracle.unpack(packed, slot, gate, w, BF16).reshape(T, w)
    tp = torch.from_numpy(packed.view(np.int16).copy()).view(torch.bfloat16).reshape(nk, w).float()
    keep = torch.from_numpy(slot >= 0)
    idx = torch.from_numpy(np.where(slot >= 0, slot, 0).astype(np.int64))
    ref = (torch.from_numpy(gate)[:, None] * tp[idx]).to(torch.bfloat16)
    ref = torch.where(keep[:, None], ref, torch.zeros_like(ref)).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(out, ref)
    # fp32: plain product, no further rounding
    pk32 = inputs.normal(nk * w, 57, 0)
    out32 = oracle.unpack(pk32, slot, gate, w, F32).reshape(T, w)
    ref32 = np.where((slot >= 0)[:, None], gate[:, None] * pk32.reshape(nk, w)[np.where(slot >= 0, slot, 0)], np.float32(0))
    assert np.array_equal(bits32(out32), bits32(ref32.astype(np.float32)))


def check_moe_roundtrip():
    """dispatch -> alltoallv(S) -> identity experts -> alltoallv(S^T) -> combine with gate 1
    returns the kept tokens, zeros elsewhere."""
    w = inputs.MoEWorkload(P=4, T=128, H=8, E=8)
    P, T, H = w.P, w.T, w.H
    toks = [w.tokens(p) for p in range(P)]
    routes = [oracle.moe_route(w.ids(p), w.E, P, w.C) for p in range(P)]
    S = np.stack([r[2] for r in routes])
    packed = []
    for p in range(P):
        buf = np.zeros(int(S[p].sum()) * H, dtype=np.uint16)
        oracle.pack(toks[p], routes[p][0], H, BF16, buf)
        packed.append(buf)
    recv = oracle.alltoallv(packed, S, H, BF16)
    back = oracle.alltoallv(recv, S.T.copy(), H, BF16)
    for p in range(P):
        assert np.array_equal(back[p], packed[p])
        out = oracle.unpack(back[p], routes[p][0], np.ones(T, dtype=np.float32), H, BF16).reshape(T, H)
        kept = routes[p][0] >= 0
        assert np.array_equal(out[kept], toks[p].reshape(T, H)[kept]) and (out[~kept] == 0).all()


# =================================== DLRM =====================================
def check_dlrm_closed_form_and_composition():
    w = inputs.DLRMWorkload(P=4, n_tables=10, dim=4, batch=32)
    P, NT, D, B = w.P, w.n_tables, w.dim, w.batch
    bl = B // P
    src = []
    for p in range(P):
        tabs = w.tables_on(p)
        v = np.empty((len(tabs), B, D), dtype=np.float32)
        for li, t in enumerate(tabs):
            v[li] = (t * (1 << 14) + np.arange(B))[:, None] + np.arange(D)[None, :] / 8.0
        src.append(v.reshape(-1))
    outs = oracle.dlrm_forward(src, NT, B, D, F32)
    for r in range(P):
        o = outs[r].reshape(bl, NT, D)
        b, t, c = np.meshgrid(np.arange(bl), np.arange(NT), np.arange(D), indexing="ij")
        assert np.array_equal(o, (t * (1 << 14) + r * bl + b + c / 8.0).astype(np.float32))
    # composition: plain alltoallv, then a local permute from (owner, local, b) to (b, t)
    sends = []
    for p in range(P):   # send buffer of rank p ordered by destination: [r][local][b]
        v = src[p].reshape(len(w.tables_on(p)), P, bl, D).transpose(1, 0, 2, 3)
        sends.append(np.ascontiguousarray(v).reshape(-1))
    recv = oracle.alltoallv(sends, w.splits(), D, F32)
    for r in range(P):
        rows = recv[r].reshape(-1, bl, D)          # tables in (owner, local) order
        order = [t for p in range(P) for t in w.tables_on(p)]
        o = np.empty((bl, NT, D), dtype=np.float32)
        for k, t in enumerate(order):
            o[:, t, :] = rows[k]
        assert np.array_equal(o.reshape(-1), outs[r])
    # backward is the inverse
    back = oracle.dlrm_backward(outs, NT, B, D, F32)
    for p in range(P):
        assert np.array_equal(back[p], src[p])


# ================================ tensor fusion ================================
def check_fuse_plan_golden():
    g = gio.keyed_ints("fuse_plan_case.txt")
    tb, to, bn = oracle.fuse_plan(g["numel"], g["B"][0])
    assert tb.tolist() == g["tensor_bucket"] and to.tolist() == g["tensor_offset"] and bn.tolist() == g["bucket_numel"]


def check_fuse_plan_invariants():
    w = inputs.GradBucketWorkload()
    for numel in (w.numel(), w.numel()[::-1], [1, 3, 7, 8191, 2, 25_000_000, 1, 25_000_001, 5]):
        B = w.bucket_elems
        tb, to, bn = oracle.fuse_plan(numel, B)
        numel = np.array(numel, dtype=np.uint64)
        assert bn.sum() == numel.sum()
        assert (np.diff(tb) >= 0).all() and set(np.diff(tb).tolist()) <= {0, 1} and tb[0] == 0 and tb[-1] == len(bn) - 1
        for k in range(len(bn)):
            idx = np.nonzero(tb == k)[0]
            assert len(idx) >= 1
            assert to[idx[0]] == 0
            assert np.array_equal(to[idx], np.concatenate([[0], np.cumsum(numel[idx])[:-1]]))
            assert bn[k] == numel[idx].sum()
            assert bn[k] <= B or len(idx) == 1
            if k + 1 < len(bn) and bn[k] <= B:     # greedy: the next tensor did not fit
                nxt = numel[idx[-1] + 1]
                assert bn[k] + nxt > B
    # the dense 1.3B-parameter list: 292 tensors, 1,315,819,520 elements, 73 buckets either way,
    # and the 50304 x 2048 embedding (103,022,592 > B) sits alone
    n = w.numel()
    assert len(n) == 292 and sum(n) == 1_315_819_520
    for lst in (n, n[::-1]):
        tb, to, bn = oracle.fuse_plan(lst, w.bucket_elems)
        assert len(bn) == 73
        k = tb[lst.index(103_022_592)]
        assert bn[k] == 103_022_592 and (tb == k).sum() == 1


def check_fuse_roundtrip_and_allreduce_commutes():
    numel = [1, 3, 7, 100, 2, 64, 5]
    B = 70
    P = 3
    tb, to, bn = oracle.fuse_plan(numel, B)
    tens = [[inputs.normal(n, 61, p, i, bf16=True) for i, n in enumerate(numel)] for p in range(P)]
    per_tensor = [[t.copy() for t in tens[p]] for p in range(P)]
    for i in range(len(numel)):
        oracle.allreduce([per_tensor[p][i] for p in range(P)], BF16, AVG)
    for k in range(len(bn)):
        idx = np.nonzero(tb == k)[0]
        flats = [oracle.fuse([tens[p][i] for i in idx], to[idx], int(bn[k]), BF16) for p in range(P)]
        # concatenation by numpy
        assert np.array_equal(flats[0], np.concatenate([tens[0][i] for i in idx]))
        un = oracle.unfuse(flats[0], [numel[i] for i in idx], to[idx], BF16)
        for j, i in enumerate(idx):
            assert np.array_equal(un[j], tens[0][i])
        oracle.allreduce(flats, BF16, AVG)
        for p in range(P):
            un = oracle.unfuse(flats[p], [numel[i] for i in idx], to[idx], BF16)
            for j, i in enumerate(idx):
                assert np.array_equal(un[j], per_tensor[p][i])


# ================================ tuning table ================================
def check_tune_table2():
    rows = [s.split() for s in gio.lines("table2_allgather.txt")]
    sizes = [int(r[0]) for r in rows]
    names = sorted(set(r[1] for r in rows))
    choice = [names.index(r[1]) for r in rows]
    look = lambda b: names[oracle.tune_lookup(sizes, choice, b)]
    for r in rows:                       # exact hits reproduce the table
        assert look(int(r[0])) == r[1]
    assert look(1) == "MVAPICH2-GDR" and look(255) == "MVAPICH2-GDR"          # below the first row
    assert look(4095) == "MVAPICH2-GDR" and look(4097) == "NCCL"               # between rows: floor
    assert look(16383) == "NCCL" and look(16384) == "SCCL"
    assert look(1 << 30) == "SCCL"                                             # above the last row
    assert oracle.tune_lookup([], [], 4096) == 0                               # empty table


ALL_CHECKS = [v for k, v in sorted(globals().items()) if k.startswith("check_") and callable(v)]


@pytest.mark.parametrize("check", ALL_CHECKS, ids=[c.__name__ for c in ALL_CHECKS])
def test_pin(check):
    check()
