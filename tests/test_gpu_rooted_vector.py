"""GPU parity of the rooted and vector collectives (reduce, bcast, gather(v), scatter(v),
all_gatherv) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
from paper_2303_08374_amd import inputs, mcr
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
DTYPES = [mcr.F32, mcr.BF16]


def _bufs(P, n, dtype, seed):
    return inputs.rank_buffers(P, n, seed, "normal", bf16=(dtype == mcr.BF16))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("P", [1, 2, 5, 8, 16])
def test_reduce_to_root(dtype, P):
    for count in (1, 7, 4096, 13319):
        host = _bufs(P, count, dtype, 1400 + P)
        for root in sorted({0, P - 1, P // 2}):
            for op in (mcr.SUM, mcr.AVG):
                exp = [h.copy() for h in host]
                oracle.reduce(exp, dtype, op, root)
                for variant in (mcr.AUTO, 0, 1, 6, 9):
                    dev = [gu.to_dev(h) for h in host]
                    mcr.mcr_reduce(gu.ctx(), dev, count, dtype, op, root, P, variant)
                    gu.sync()
                    for r in range(P):
                        gu.assert_reduced_equal(gu.to_host(dev[r], gu.NPDT[dtype]), exp[r], dtype,
                                                f"reduce dt={dtype} P={P} n={count} root={root} op={op} v={variant} r={r}")


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("P", [1, 3, 8, 16])
def test_bcast(dtype, P):
    for count in (1, 5, 8, 4104, 70000):
        host = _bufs(P, count, dtype, 1500 + P)
        vec_ok = count % (4 if dtype == mcr.F32 else 8) == 0
        for root in sorted({0, P - 1}):
            exp = [h.copy() for h in host]
            oracle.bcast(exp, dtype, root)
            for variant in [mcr.AUTO, 0] + ([1, 4, 12] if vec_ok else []):
                dev = [gu.to_dev(h) for h in host]
                mcr.mcr_bcast(gu.ctx(), dev, count, dtype, root, P, variant)
                gu.sync()
                for r in range(P):
                    gu.assert_bits_equal(gu.to_host(dev[r], gu.NPDT[dtype]), exp[r], f"bcast P={P} n={count} root={root} v={variant}")


def test_long_shared_segments_take_the_super_chunk_order():
    """A segment that one sender hands to several receivers and that is longer than 16 MiB is copied
    super-chunk by super-chunk: bcast and all_gatherv (packed and with displacements), with a ragged
    last tile, a short sender beside the long ones and an empty one."""
    P, dtype, W = 4, mcr.F32, 4
    n = (40 << 20) // 4 + 4 * 77                           # 40 MiB + a ragged tail: three super-chunks
    host = _bufs(P, n, dtype, 1550)
    for root in (0, 2):
        exp = [h.copy() for h in host]
        oracle.bcast(exp, dtype, root)
        dev = [gu.to_dev(h) for h in host]
        mcr.mcr_bcast(gu.ctx(), dev, n, dtype, root, P)
        gu.sync()
        for r in range(P):
            gu.assert_bits_equal(gu.to_host(dev[r], np.float32), exp[r], f"long bcast root={root} r={r}")
    counts = [(18 << 20) // 4 + W * 3, 0, W * 1001, (33 << 20) // 4 + W * 250]
    total = sum(counts)
    ins = [inputs.uniform_pm1(c, 1551, p) for p, c in enumerate(counts)]
    d_ins = [gu.to_dev(x) if x.size else gu.dev_empty(8, dtype, 0) for x in ins]
    ag_exp = oracle.allgatherv(ins, counts, dtype)
    d_ag = [gu.dev_empty(total + 8, dtype, 0) for _ in range(P)]
    mcr.mcr_allgatherv(gu.ctx(), d_ag, d_ins, counts, dtype, P)
    gu.sync()
    for r in range(P):
        a = gu.to_host(d_ag[r], np.float32)
        gu.assert_bits_equal(a[:total], ag_exp[r], f"long allgatherv r={r}")
        assert (a[total:] == 0).all()
    displs = [W * 5, 0, counts[0] + W * 9, counts[0] + counts[2] + W * 40]
    extent = displs[3] + counts[3] + W * 2
    agd_exp = [np.zeros(extent, dtype=np.float32) for _ in range(P)]
    oracle.allgatherv_displs(agd_exp, ins, counts, displs, dtype)
    d_agd = [gu.dev_empty(extent, dtype, 0) for _ in range(P)]
    mcr.mcr_allgatherv_displs(gu.ctx(), d_agd, extent, d_ins, counts, displs, dtype, P)
    gu.sync()
    for r in range(P):
        gu.assert_bits_equal(gu.to_host(d_agd[r], np.float32), agd_exp[r], f"long allgatherv_displs r={r}")


def _count_sets(P, W, rng):
    yield [W * int(c) for c in rng.integers(0, 600, size=P)]               # 128-bit friendly, some may be 0
    yield [int(c) for c in rng.integers(0, 50, size=P)]                    # arbitrary: element path
    yield [0] * P
    yield [W * 1000] * P                                                   # equal counts (gather / scatter)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("P", [1, 2, 7, 16])
def test_gatherv_scatterv_allgatherv(dtype, P):
    W = 4 if dtype == mcr.F32 else 8
    rng = np.random.Generator(np.random.Philox(key=1600 + P))
    bf = dtype == mcr.BF16
    for counts in _count_sets(P, W, rng):
        total = sum(counts)
        vec_ok = all(c % W == 0 for c in counts)
        ins = [inputs.uniform_pm1(c, 1601, p, bf16=bf) for p, c in enumerate(counts)]
        g_exp = oracle.gatherv(ins, counts, dtype)
        ag_exp = oracle.allgatherv(ins, counts, dtype)
        d_ins = [gu.to_dev(x) if x.size else gu.dev_empty(8, dtype, 0) for x in ins]
        for variant in [mcr.AUTO, 0] + ([1, 5, 9] if vec_ok else []):
            d_g = gu.dev_empty(total + 8, dtype, 0)
            mcr.mcr_gatherv(gu.ctx(), d_g, d_ins, counts, dtype, P, variant)
            d_ag = [gu.dev_empty(total + 8, dtype, 0) for _ in range(P)]
            mcr.mcr_allgatherv(gu.ctx(), d_ag, d_ins, counts, dtype, P, variant)
            d_sc = [gu.dev_empty(c + 8, dtype, 0) for c in counts]
            mcr.mcr_scatterv(gu.ctx(), d_sc, d_g, counts, dtype, P, variant)
            gu.sync()
            got = gu.to_host(d_g, gu.NPDT[dtype])
            gu.assert_bits_equal(got[:total], g_exp, f"gatherv P={P} v={variant}")
            assert (got[total:] == 0).all()                                  # nothing past the payload is written
            for r in range(P):
                a = gu.to_host(d_ag[r], gu.NPDT[dtype])
                gu.assert_bits_equal(a[:total], ag_exp[r], f"allgatherv P={P} v={variant} r={r}")
                assert (a[total:] == 0).all()
                s = gu.to_host(d_sc[r], gu.NPDT[dtype])
                gu.assert_bits_equal(s[:counts[r]], ins[r], f"scatterv(gatherv) P={P} v={variant} r={r}")
                assert (s[counts[r]:] == 0).all()
        if not vec_ok:
            with pytest.raises(mcr.McrError) as e:
                mcr.mcr_gatherv(gu.ctx(), gu.dev_empty(total + 8, dtype, 0), d_ins, counts, dtype, P, 1)
            assert e.value.status == mcr.EVARIANT


def test_gather_scatter_equal_counts():
    P, n, dtype = 8, 4096, mcr.F32
    ins = _bufs(P, n, dtype, 1700)
    d_out = gu.dev_empty(P * n, dtype, 0)
    mcr.mcr_gather(gu.ctx(), d_out, [gu.to_dev(x) for x in ins], n, dtype, P)
    d_back = [gu.dev_empty(n, dtype, 0) for _ in range(P)]
    mcr.mcr_scatter(gu.ctx(), d_back, d_out, n, dtype, P)
    gu.sync()
    gu.assert_bits_equal(gu.to_host(d_out, np.float32), oracle.allgather(ins, dtype)[0], "gather = a row of all_gather")
    sc_exp = oracle.scatterv(np.concatenate(ins), [n] * P, dtype)
    for r in range(P):
        gu.assert_bits_equal(gu.to_host(d_back[r], np.float32), sc_exp[r], "scatter")


# ------------------------------------------------- displacements chosen by the caller
def _scattered_displs(counts, W, rng, vec):
    """Blocks in a shuffled order with gaps; offsets multiples of W when `vec`."""
    order = rng.permutation(len(counts))
    displs = [0] * len(counts)
    at = int(rng.integers(0, 3)) * (W if vec else 1)
    for p in order:
        displs[p] = at
        gap = int(rng.integers(0, 5))
        at += counts[p] + (gap * W if vec else gap)
    return displs, at + 8


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("P", [1, 2, 5, 16])
def test_vector_collectives_with_displacements(dtype, P):
    W = 4 if dtype == mcr.F32 else 8
    npdt = gu.NPDT[dtype]
    rng = np.random.Generator(np.random.Philox(key=1800 + P))
    bf = dtype == mcr.BF16
    for vec in (True, False):
        counts = [int(c) * (W if vec else 1) for c in rng.integers(0, 40 if vec else 50, size=P)]
        counts[P // 2] = 0
        if P == 16 and vec:
            counts[3] = 70000 * W                                                   # several tiles and a tail in one pair
        displs, extent = _scattered_displs(counts, W, rng, vec)
        ins = [inputs.uniform_pm1(c, 1801, p, bf16=bf) for p, c in enumerate(counts)]
        d_ins = [gu.to_dev(x) if x.size else gu.dev_empty(8, dtype, 0) for x in ins]
        g_exp = np.full(extent, 0, dtype=npdt)
        oracle.gatherv_displs(g_exp, ins, counts, displs, dtype)
        ag_exp = [np.full(extent, 0, dtype=npdt) for _ in range(P)]
        oracle.allgatherv_displs(ag_exp, ins, counts, displs, dtype)
        root = inputs.uniform_pm1(extent, 1802, 0, bf16=bf)
        sc_exp = oracle.scatterv_displs(root, counts, displs, dtype)
        d_root = gu.to_dev(root)
        for variant in [mcr.AUTO, 0] + ([1, 5, 9] if vec else []):
            d_g = gu.dev_empty(extent, dtype, 0)
            mcr.mcr_gatherv_displs(gu.ctx(), d_g, extent, d_ins, counts, displs, dtype, P, variant)
            d_ag = [gu.dev_empty(extent, dtype, 0) for _ in range(P)]
            mcr.mcr_allgatherv_displs(gu.ctx(), d_ag, extent, d_ins, counts, displs, dtype, P, variant)
            d_sc = [gu.dev_empty(c + 8, dtype, 0) for c in counts]
            mcr.mcr_scatterv_displs(gu.ctx(), d_sc, d_root, extent, counts, displs, dtype, P, variant)
            gu.sync()
            gu.assert_bits_equal(gu.to_host(d_g, npdt), g_exp, f"gatherv_displs P={P} v={variant}")     # gaps stay 0
            for r in range(P):
                gu.assert_bits_equal(gu.to_host(d_ag[r], npdt), ag_exp[r], f"allgatherv_displs P={P} v={variant} r={r}")
                s = gu.to_host(d_sc[r], npdt)
                gu.assert_bits_equal(s[:counts[r]], sc_exp[r], f"scatterv_displs P={P} v={variant} r={r}")
                assert (s[counts[r]:] == 0).all()


@pytest.mark.parametrize("dtype,row_elems", [(mcr.F32, 4), (mcr.BF16, 8), (mcr.F32, 3), (mcr.BF16, 5), (mcr.BF16, 2048)])
@pytest.mark.parametrize("P", [1, 3, 8, 16])
def test_alltoallv_with_displacements(dtype, row_elems, P):
    npdt = gu.NPDT[dtype]
    rng = np.random.Generator(np.random.Philox(key=1900 + P + row_elems))
    bf = dtype == mcr.BF16
    C = rng.integers(0, 9, size=(P, P)).astype(np.int64)
    C[0, P - 1] = 0
    if row_elems == 2048:
        C[P - 1, 0] = 300                                                          # 1.2 MB in one pair
    # send side: blocks of a sender in shuffled order with gaps; receive side likewise
    SD = np.zeros((P, P), dtype=np.int64)
    RD = np.zeros((P, P), dtype=np.int64)
    in_rows = out_rows = 0
    for p in range(P):
        at = int(rng.integers(0, 3))
        for r in rng.permutation(P):
            SD[p, r] = at
            at += int(C[p, r]) + int(rng.integers(0, 3))
        in_rows = max(in_rows, at)
    for r in range(P):
        at = int(rng.integers(0, 3))
        for p in rng.permutation(P):
            RD[r, p] = at
            at += int(C[p, r]) + int(rng.integers(0, 3))
        out_rows = max(out_rows, at)
    in_rows, out_rows = in_rows + 1, out_rows + 1
    ins = [inputs.uniform_pm1(in_rows * row_elems, 1901, p, bf16=bf) for p in range(P)]
    exp = [np.zeros(out_rows * row_elems, dtype=npdt) for _ in range(P)]
    oracle.alltoallv_displs(exp, ins, C, SD, RD, row_elems, dtype)
    d_ins = [gu.to_dev(x) for x in ins]
    vec_ok = (row_elems * gu.EB[dtype]) % 16 == 0
    for variant in [mcr.AUTO, 0] + ([1, 6, 11] if vec_ok else []):
        d_out = [gu.dev_empty(out_rows * row_elems, dtype, 0) for _ in range(P)]
        mcr.mcr_alltoallv_displs(gu.ctx(), d_out, d_ins, C.reshape(-1), SD.reshape(-1), RD.reshape(-1), in_rows, out_rows,
                                 row_elems, dtype, P, variant)
        gu.sync()
        for r in range(P):
            gu.assert_bits_equal(gu.to_host(d_out[r], npdt), exp[r], f"alltoallv_displs P={P} v={variant} r={r}")
