"""Parity at the benchmark's full sizes and in the launch configuration bench.py times (MCR_AUTO
with the shipped tuning table): the op sweep at 64 and 256 MiB per rank and the 1.3 B-parameter
gradient list.  Whole outputs are too large for the CPU oracle, so windows of the output are
checked: the inputs of each window are downloaded, the oracle runs on them, and the result must
match the downloaded output bit for bit.  Windows include the first and last elements, tile and
super-chunk boundaries, and random places."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2303_08374_amd import inputs, mcr
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TABLE = os.path.join(ROOT, "paper_2303_08374_amd", "tuning", "mi355x.tbl")
P = inputs.SWEEP_P
W = 2048                      # elements per window


@pytest.fixture(scope="module")
def tuned_ctx():
    c = mcr.mcr_init(0)
    if os.path.exists(TABLE):
        mcr.mcr_tune_load(c, TABLE)
    yield c
    mcr.mcr_finalize(c)


def _fill(n, dtype, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    td = torch.float32 if dtype == mcr.F32 else torch.bfloat16
    return torch.empty(n, dtype=td, device="cuda").uniform_(-1.0, 1.0, generator=g)


def _host(t, s, w, dtype):
    a = t[s:s + w]
    if dtype == mcr.BF16:
        return a.view(torch.int16).cpu().numpy().view(np.uint16).copy()
    return a.cpu().numpy().copy()


def _bits(t):
    """A tensor as integers of its element size: equality of bit patterns, NaN and -0 included."""
    return t.view(torch.int16 if t.element_size() == 2 else torch.int32)


def _starts(n, rng, extra=()):
    """Window starts in [0, n - W]: both ends, boundaries of 4 KiB tiles and of 4/8/16 MiB super-chunks
    (in elements of either dtype), and random places."""
    cand = [0, n - W, 1024 - 7, (1 << 20) - W // 2, (2 << 20) - 3, (4 << 20) - 1000, (8 << 20) - 5] + list(extra)
    cand += [int(x) for x in rng.integers(0, max(n - W, 1), size=12)]
    return sorted({min(max(c, 0), n - W) for c in cand})


@pytest.mark.parametrize("ranks", [8, 16, 6])
@pytest.mark.parametrize("dtype", [mcr.F32, mcr.BF16])
def test_rows_of_the_shipped_table_whole_outputs(tuned_ctx, dtype, ranks):
    """MCR_AUTO with the shipped table at small and middle sizes, every element against the oracle:
    the rows of a tuned scale (8, 16) and of a scale that borrows its neighbour's table (6); sizes
    a little off the table's own so that tails are in play."""
    bf = dtype == mcr.BF16
    eb = 2 if bf else 4
    for M in (4 << 10, 72 << 10, (1 << 20) + 4 * ranks * eb, 3 << 20, 8 << 20, (16 << 20) + 16 * ranks):
        n = M // eb // ranks * ranks
        host = [inputs.uniform_pm1(n, 4100 + ranks, p, bf16=bf) for p in range(ranks)]
        names = {op: mcr.mcr_get_variants(tuned_ctx, op)[mcr.mcr_auto_variant(tuned_ctx, op, dtype, ranks, n * eb, True)]
                 for op in (mcr.OP_ALLREDUCE, mcr.OP_REDUCE_SCATTER, mcr.OP_ALLGATHER, mcr.OP_ALLTOALL)}
        what = f"P={ranks} M={n * eb} dtype={dtype} table picks {names}"
        d_in = [gu.to_dev(h) for h in host]
        d_out = [gu.dev_empty(n // ranks, dtype, 1) for _ in range(ranks)]
        mcr.mcr_reduce_scatter(tuned_ctx, d_out, d_in, n, dtype, mcr.SUM, ranks)
        exp = oracle.reduce_scatter(host, dtype)
        for r in range(ranks):
            gu.assert_reduced_equal(gu.to_host(d_out[r], gu.NPDT[dtype]), exp[r], dtype, "reduce_scatter " + what)
        d_out = [gu.dev_empty(n, dtype, 1) for _ in range(ranks)]
        mcr.mcr_alltoall(tuned_ctx, d_out, d_in, n, dtype, ranks)
        exp = oracle.alltoall(host, dtype)
        for r in range(ranks):
            gu.assert_bits_equal(gu.to_host(d_out[r], gu.NPDT[dtype]), exp[r], "alltoall " + what)
        if n * eb * ranks * ranks <= (1 << 30):
            d_out = [gu.dev_empty(n * ranks, dtype, 1) for _ in range(ranks)]
            mcr.mcr_allgather(tuned_ctx, d_out, d_in, n, dtype, ranks)
            exp = oracle.allgather(host, dtype)
            for r in range(ranks):
                gu.assert_bits_equal(gu.to_host(d_out[r], gu.NPDT[dtype]), exp[r], "allgather " + what)
            del d_out, exp
        mcr.mcr_allreduce(tuned_ctx, d_in, n, dtype, mcr.SUM, ranks)
        bufs = [h.copy() for h in host]
        oracle.allreduce(bufs, dtype)
        for r in range(ranks):
            gu.assert_reduced_equal(gu.to_host(d_in[r], gu.NPDT[dtype]), bufs[r], dtype, "allreduce " + what)


@pytest.mark.parametrize("M", [64 << 20, 256 << 20])
@pytest.mark.parametrize("dtype", [mcr.F32, mcr.BF16])
def test_sweep_ops_sampled(tuned_ctx, dtype, M):
    s = gu.EB[dtype]
    n = M // s
    b = n // P
    rng = np.random.Generator(np.random.Philox(key=M + dtype))
    ins = [_fill(n, dtype, 2000 + p) for p in range(P)]

    # reduce_scatter: out[r][j] = sum_p in[p][r*b + j]
    outs = [torch.zeros(b, dtype=ins[0].dtype, device="cuda") for _ in range(P)]
    mcr.mcr_reduce_scatter(tuned_ctx, outs, ins, n, dtype, mcr.SUM, P)
    gu.sync()
    for r in (0, 3, P - 1):
        for st in _starts(b, rng):
            win = [_host(ins[p], r * b + st, W, dtype) for p in range(P)]
            oracle.allreduce(win, dtype, oracle.SUM)
            gu.assert_bits_equal(_host(outs[r], st, W, dtype), win[0], f"reduce_scatter M={M} r={r} at {st}")
    del outs

    # all_to_all: out[r][p*b + k] = in[p][r*b + k]
    outs = [torch.zeros(n, dtype=ins[0].dtype, device="cuda") for _ in range(P)]
    mcr.mcr_alltoall(tuned_ctx, outs, ins, n, dtype, P)
    gu.sync()
    for r in (0, 5):
        for p in (0, 2, P - 1):
            for st in _starts(b, rng)[::3]:
                gu.assert_bits_equal(_host(outs[r], p * b + st, W, dtype), _host(ins[p], r * b + st, W, dtype),
                                     f"alltoall M={M} r={r} p={p} at {st}")
    # and the whole output, on the device: every (r, p) block is a bit copy of its source block
    for r in range(P):
        for p in range(P):
            assert torch.equal(_bits(outs[r][p * b:(p + 1) * b]), _bits(ins[p][r * b:(r + 1) * b])), f"alltoall M={M} block ({r}, {p})"
    del outs

    # all_gather: out[r][p*n + j] = in[p][j]  (P*M per output: 2 GiB each at the top size)
    outs = [torch.zeros(P * n, dtype=ins[0].dtype, device="cuda") for _ in range(P)]
    mcr.mcr_allgather(tuned_ctx, outs, ins, n, dtype, P)
    gu.sync()
    for r in (0, 6):
        for p in (0, 3, P - 1):
            for st in _starts(n, rng)[::2]:
                gu.assert_bits_equal(_host(outs[r], p * n + st, W, dtype), _host(ins[p], st, W, dtype),
                                     f"allgather M={M} r={r} p={p} at {st}")
    # and the whole output, on the device: every (r, p) slice is a bit copy of rank p's input
    for r in range(P):
        for p in range(P):
            assert torch.equal(_bits(outs[r][p * n:(p + 1) * n]), _bits(ins[p])), f"allgather M={M} slice ({r}, {p})"
    del outs

    # all_reduce, in place: download the windows first
    starts = _starts(n, rng)
    before = {st: [_host(ins[p], st, W, dtype) for p in range(P)] for st in starts}
    mcr.mcr_allreduce(tuned_ctx, ins, n, dtype, mcr.SUM, P)
    gu.sync()
    for st in starts:
        exp = before[st]
        oracle.allreduce(exp, dtype, oracle.SUM)
        for r in (0, P - 1):
            gu.assert_bits_equal(_host(ins[r], st, W, dtype), exp[r], f"allreduce M={M} r={r} at {st}")
    # every rank holds the same bits everywhere (a property that needs no oracle)
    for r in range(1, P):
        assert torch.equal(ins[r].view(torch.int16 if dtype == mcr.BF16 else torch.int32),
                           ins[0].view(torch.int16 if dtype == mcr.BF16 else torch.int32))


@pytest.mark.parametrize("variant,mib", [(13, 9), (14, 20), (15, 40), (16, 40), (16, 7)])
def test_allgather_superchunk_forms_with_several_superchunks(variant, mib):
    """The super-chunk forms of all_gather (4, 8 and 16 MiB per source and super-chunk; 16 MiB with
    the tiles renumbered in units per XCD) on messages of two super-chunks and a ragged third one,
    and the renumbering form on a message shorter than one group of units (where it must fall back),
    every element against the oracle."""
    Pn = 2
    n = ((mib << 20) + 4096 + 48) // 4                                  # fp32 elements: not a whole tile either
    host = inputs.rank_buffers(Pn, n, seed=4400 + variant, dist="uniform")
    exp = oracle.allgather(host, oracle.F32)
    dev_out = [gu.dev_empty(Pn * n, mcr.F32, 0) for _ in range(Pn)]
    mcr.mcr_allgather(gu.ctx(), dev_out, [gu.to_dev(h) for h in host], n, mcr.F32, Pn, variant)
    gu.sync()
    for r in range(Pn):
        gu.assert_bits_equal(gu.to_host(dev_out[r], np.float32), exp[r], f"super-chunk form {variant}, {mib} MiB, r={r}")


def test_gradient_buckets_full_size_sampled(tuned_ctx):
    """292 bf16 tensors, 1,315,819,520 elements per rank, 8 ranks: the fused multi-tensor average,
    and fuse -> allreduce -> unfuse of the largest and of a mixed bucket."""
    w = inputs.GradBucketWorkload()
    numel = w.numel()
    total = sum(numel)
    n_t = len(numel)
    offs = np.concatenate([[0], np.cumsum(numel)[:-1]]).astype(np.int64)
    arenas = [torch.empty(total, dtype=torch.bfloat16, device="cuda").normal_(0.0, w.std) for _ in range(w.P)]
    plan = mcr.mcr_fuse_plan_create(tuned_ctx, numel, w.bucket_elems, mcr.BF16)
    try:
        bn, tb, to = mcr.mcr_fuse_plan_info(plan, n_t)
        assert len(bn) == 73
        mcr.mcr_fuse_plan_bind(tuned_ctx, plan, [arenas[p].data_ptr() + int(offs[i]) * 2 for p in range(w.P) for i in range(n_t)], w.P)
        rng = np.random.Generator(np.random.Philox(key=77))
        # windows: every small tensor near its start, and places inside the big ones
        wins = []
        for i in list(range(0, n_t, 7)) + [numel.index(max(numel))]:
            n = numel[i]
            ww = min(W, n)
            for st in {0, n - ww, int(rng.integers(0, n - ww + 1))}:
                wins.append((i, st, ww))
        before = {k: [_host(arenas[p], int(offs[k[0]]) + k[1], k[2], mcr.BF16) for p in range(w.P)] for k in wins}
        # fuse of two buckets (checked before anything is reduced)
        flats = [torch.zeros(max(bn), dtype=torch.bfloat16, device="cuda") for _ in range(w.P)]
        for k in (tb[numel.index(max(numel))], 5):
            mcr.mcr_fuse(tuned_ctx, plan, k, flats, w.P)
            gu.sync()
            for i in [j for j in range(n_t) if tb[j] == k][:4]:
                ww = min(W, numel[i])
                gu.assert_bits_equal(_host(flats[3], to[i], ww, mcr.BF16), _host(arenas[3], int(offs[i]), ww, mcr.BF16), f"fuse t={i}")
        mcr.mcr_allreduce_multi(tuned_ctx, plan, -1, mcr.AVG)
        gu.sync()
        for k in wins:
            exp = before[k]
            oracle.allreduce(exp, oracle.BF16, oracle.AVG)
            for p in (0, w.P - 1):
                gu.assert_bits_equal(_host(arenas[p], int(offs[k[0]]) + k[1], k[2], mcr.BF16), exp[p], f"allreduce_multi t={k[0]} at {k[1]}")
        for p in range(1, w.P):
            assert torch.equal(arenas[p].view(torch.int16), arenas[0].view(torch.int16))
    finally:
        mcr.mcr_fuse_plan_destroy(plan)


@pytest.mark.parametrize("dtype", [mcr.F16, mcr.I32])
def test_f16_i32_reductions_sampled(tuned_ctx, dtype):
    """64 MiB per rank of fp16 / int32 through MCR_AUTO (their tables are borrowed from bf16 / fp32):
    reduce_scatter, then all_reduce in place."""
    M = 64 << 20
    n = M // gu.EB[dtype]
    b = n // P
    rng = np.random.Generator(np.random.Philox(key=M + 10 * dtype))
    g = torch.Generator(device="cuda")
    ins = []
    for p in range(P):
        g.manual_seed(2900 + p)
        if dtype == mcr.F16:
            ins.append(torch.empty(n, dtype=torch.float16, device="cuda").uniform_(-4.0, 4.0, generator=g))
        else:
            ins.append(torch.randint(-2**31, 2**31 - 1, (n,), dtype=torch.int32, device="cuda", generator=g))
    host = lambda t, s: t[s:s + W].cpu().numpy().copy()
    op = mcr.AVG if dtype == mcr.F16 else mcr.SUM
    outs = [torch.zeros(b, dtype=ins[0].dtype, device="cuda") for _ in range(P)]
    mcr.mcr_reduce_scatter(tuned_ctx, outs, ins, n, dtype, op, P)
    gu.sync()
    for r in (0, P - 1):
        for st in _starts(b, rng)[::2]:
            win = [host(ins[p], r * b + st) for p in range(P)]
            oracle.allreduce(win, dtype, op)
            gu.assert_bits_equal(host(outs[r], st), win[0], f"reduce_scatter dt={dtype} r={r} at {st}")
    starts = _starts(n, rng)
    before = {st: [host(ins[p], st) for p in range(P)] for st in starts}
    mcr.mcr_allreduce(tuned_ctx, ins, n, dtype, op, P)
    gu.sync()
    for st in starts:
        exp = before[st]
        oracle.allreduce(exp, dtype, op)
        gu.assert_bits_equal(host(ins[P - 1], st), exp[0], f"allreduce dt={dtype} at {st}")
    view = torch.int16 if dtype == mcr.F16 else torch.int32
    for r in range(1, P):
        assert torch.equal(ins[r].view(view), ins[0].view(view))


def test_alltoallv_displacements_sampled(tuned_ctx):
    """P=8, rows of 4 KiB, about 1.5 GiB moved with caller-chosen displacements: every block lands at
    its own offset (blocks in reverse sender order with gaps), checked on windows of rows."""
    dtype, re = mcr.BF16, 2048
    rng = np.random.Generator(np.random.Philox(key=777))
    C = rng.integers(2000, 9000, size=(P, P)).astype(np.int64)
    C[1, 2] = 0
    SD = np.zeros((P, P), dtype=np.int64)
    RD = np.zeros((P, P), dtype=np.int64)
    for p in range(P):
        at = 3
        for r in rng.permutation(P):
            SD[p, r] = at
            at += int(C[p, r]) + 5
    in_rows = int((SD + C).max()) + 1
    for r in range(P):
        at = 1
        for p in reversed(range(P)):
            RD[r, p] = at
            at += int(C[p, r]) + 7
    out_rows = int(max(RD[r, p] + C[p, r] for r in range(P) for p in range(P))) + 2
    ins = [_fill(in_rows * re, dtype, 3000 + p) for p in range(P)]
    outs = [torch.zeros(out_rows * re, dtype=torch.bfloat16, device="cuda") for _ in range(P)]
    mcr.mcr_alltoallv_displs(tuned_ctx, outs, ins, C.reshape(-1), SD.reshape(-1), RD.reshape(-1), in_rows, out_rows, re, dtype, P)
    gu.sync()
    rows_of = lambda t, row, k: t[row * re:(row + k) * re].view(torch.int16).cpu().numpy()
    for r in (0, 3, P - 1):
        for p in (0, 2, P - 1):
            c = int(C[p, r])
            if c == 0:
                continue
            for k0 in sorted({0, c - 2, c // 2, int(rng.integers(0, c - 2))}):
                got = rows_of(outs[r], int(RD[r, p]) + k0, 2)
                exp = rows_of(ins[p], int(SD[p, r]) + k0, 2)
                assert np.array_equal(got, exp), f"alltoallv_displs r={r} p={p} row {k0}"
            # the gap rows around the block are untouched
            assert (rows_of(outs[r], int(RD[r, p]) + c, 1) == 0).all()
            assert (rows_of(outs[r], int(RD[r, p]) - 1, 1) == 0).all()
