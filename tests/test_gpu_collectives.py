"""GPU parity of the four collectives against the CPU oracle, element by element, through the
C ABI.  Sizes span several workgroup tiles plus a ragged tail; every kernel variant is run."""
import numpy as np
import pytest
import torch

import oracle
from paper_2303_08374_amd import inputs, mcr
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

DTYPES = [mcr.F32, mcr.BF16]


def _make(P, n, dtype, seed, dist="normal"):
    return inputs.rank_buffers(P, n, seed, dist, bf16=(dtype == mcr.BF16))


# ------------------------------------------------------------------ all_reduce
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("P", [1, 2, 3, 4, 8, 16])
def test_allreduce_all_variants(dtype, P):
    for count in (1, 5, 1000, 13319, 70001):
        host = _make(P, count, dtype, seed=100 + P)
        for op in (mcr.SUM, mcr.AVG):
            exp = [h.copy() for h in host]
            oracle.allreduce(exp, dtype, op)
            for variant in [mcr.AUTO] + gu.ALL_VARIANTS + gu.REDUCE_EXTRA:
                dev = [gu.to_dev(h) for h in host]
                mcr.mcr_allreduce(gu.ctx(), dev, count, dtype, op, P, variant)
                gu.sync()
                for r in range(P):
                    gu.assert_reduced_equal(gu.to_host(dev[r], gu.NPDT[dtype]), exp[r], dtype,
                                            f"allreduce dt={dtype} P={P} n={count} op={op} v={variant} r={r}")


def test_allreduce_config1_full_size():
    """P=4, 2^20 fp32 N(0,1), rank order 0..3, written to all four buffers."""
    w = inputs.AllreduceSmall()
    host = w.buffers()
    exp = [h.copy() for h in host]
    oracle.allreduce(exp, oracle.F32, oracle.SUM)
    for variant in [mcr.AUTO] + gu.ALL_VARIANTS + gu.REDUCE_EXTRA:
        dev = [gu.to_dev(h) for h in host]
        mcr.mcr_allreduce(gu.ctx(), dev, w.n, mcr.F32, mcr.SUM, w.P, variant)
        gu.sync()
        for r in range(w.P):
            gu.assert_bits_equal(gu.to_host(dev[r], np.float32), exp[r], f"cfg1 v={variant} r={r}")


@pytest.mark.parametrize("dtype,P", [(mcr.F32, 3), (mcr.BF16, 8), (mcr.F32, 16)])
def test_persistent_reductions_over_several_rounds(dtype, P):
    """The persistent variants on a message long enough that every workgroup walks more than one
    round and the last ones end in a ragged tail: all_reduce (AVG), reduce to a root, reduce_scatter."""
    W = 4 if dtype == mcr.F32 else 8
    round_vecs = 8 * 1024 * 256                                      # one round of every workgroup of a 256-unit grid
    b = (round_vecs * W * 5 // 4) // P // W * W + W                  # per-rank slice of reduce_scatter: whole vectors
    n = P * b
    host = _make(P, n + 3, dtype, seed=300 + P, dist="uniform")     # all_reduce takes 3 more elements: a ragged end
    exp_ar = [h.copy() for h in host]
    oracle.allreduce(exp_ar, dtype, mcr.AVG)
    exp_red = [h.copy() for h in host]
    oracle.reduce(exp_red, dtype, mcr.SUM, 1)
    exp_rs = oracle.reduce_scatter([h[:n] for h in host], dtype, mcr.SUM)
    for variant in gu.REDUCE_LONG:
        dev = [gu.to_dev(h) for h in host]
        mcr.mcr_allreduce(gu.ctx(), dev, n + 3, dtype, mcr.AVG, P, variant)
        d_red = [gu.to_dev(h) for h in host]
        mcr.mcr_reduce(gu.ctx(), d_red, n + 3, dtype, mcr.SUM, 1, P, variant)
        d_in = [gu.to_dev(h[:n]) for h in host]
        d_rs = [gu.dev_empty(b, dtype, 0) for _ in range(P)]
        mcr.mcr_reduce_scatter(gu.ctx(), d_rs, d_in, n, dtype, mcr.SUM, P, variant)
        gu.sync()
        for r in range(P):
            gu.assert_reduced_equal(gu.to_host(dev[r], gu.NPDT[dtype]), exp_ar[r], dtype, f"persistent allreduce v={variant} r={r}")
            gu.assert_reduced_equal(gu.to_host(d_red[r], gu.NPDT[dtype]), exp_red[r], dtype, f"persistent reduce v={variant} r={r}")
            gu.assert_reduced_equal(gu.to_host(d_rs[r], gu.NPDT[dtype]), exp_rs[r], dtype, f"persistent reduce_scatter v={variant} r={r}")


@pytest.mark.parametrize("dtype", DTYPES)
def test_allreduce_special_values(dtype):
    """+-0, infinities, NaN, largest finite, subnormals: bit-equal, NaN stays NaN."""
    pats = np.array([0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x7FC00000, 0x7F7FFFFF, 0x00000001,
                     0x00010000, 0x80010000, 0x3F800000, 0xBF800000, 0x33800000, 0x007F0000, 0x7F7F0000], dtype=np.uint32)
    P = 3
    n = len(pats) ** 2
    a = np.repeat(pats, len(pats)).view(np.float32)
    b = np.tile(pats, len(pats)).view(np.float32)
    c = np.full(n, -0.0, dtype=np.float32)
    host = [a, b, c]
    if dtype == mcr.BF16:
        host = [inputs.f32_bits_to_bf16_trunc(h) for h in host]
    host = [np.ascontiguousarray(h) for h in host]
    exp = [h.copy() for h in host]
    with np.errstate(all="ignore"):
        oracle.allreduce(exp, dtype, oracle.SUM)
    for variant in (0, 1, 3):
        dev = [gu.to_dev(h) for h in host]
        mcr.mcr_allreduce(gu.ctx(), dev, n, dtype, mcr.SUM, P, variant)
        gu.sync()
        for r in range(P):
            gu.assert_reduced_equal(gu.to_host(dev[r], gu.NPDT[dtype]), exp[r], dtype, f"special v={variant}")


@pytest.mark.parametrize("dtype", DTYPES)
def test_allreduce_closed_form_any_association(dtype):
    P, n = 8, 50000
    i = np.arange(n)
    mod = 251 if dtype == mcr.F32 else 7
    vals = [((p + 1) * (i % mod)).astype(np.float32) for p in range(P)]
    host = vals if dtype == mcr.F32 else [inputs.f32_bits_to_bf16_trunc(v) for v in vals]
    dev = [gu.to_dev(h) for h in host]
    mcr.mcr_allreduce(gu.ctx(), dev, n, dtype, mcr.SUM, P, mcr.AUTO)
    gu.sync()
    got = gu.to_host(dev[5], gu.NPDT[dtype])
    got = got if dtype == mcr.F32 else inputs.bf16_bits_to_f32(got)
    assert np.array_equal(got, (36 * (i % mod)).astype(np.float32))


@pytest.mark.parametrize("dtype", DTYPES)
def test_allreduce_misaligned_buffers(dtype):
    """Buffers that are only element-aligned.  Misaligned by the same amount on every rank (the same
    view of a tensor): the 128-bit variants still apply, with the elements in front of the first
    16-byte boundary and behind the last whole vector reduced one by one.  Misaligned by different
    amounts: AUTO falls back to the element kernel and an explicit 128-bit variant is refused.
    Nothing outside the views is written."""
    P = 4
    npdt = gu.NPDT[dtype]
    W = 4 if dtype == mcr.F32 else 8
    pad = 16
    for skip in (1, 3, W - 1):
        for n in (1, W - 2, 4097, 70001):
            host = _make(P, pad + n + pad, dtype, seed=7 + skip)
            for op in (mcr.SUM, mcr.AVG):
                exp = [h[skip:skip + n].copy() for h in host]
                oracle.allreduce(exp, dtype, op)
                for variant in (mcr.AUTO, 0, 3, 5, 12):
                    dev = [gu.to_dev(h) for h in host]
                    views = [d[skip:skip + n] for d in dev]
                    if variant > 0 and n < W - skip:           # the message ends before the first 16-byte boundary
                        with pytest.raises(mcr.McrError) as e:
                            mcr.mcr_allreduce(gu.ctx(), views, n, dtype, op, P, variant)
                        assert e.value.status == mcr.EVARIANT
                        continue
                    mcr.mcr_allreduce(gu.ctx(), views, n, dtype, op, P, variant)
                    gu.sync()
                    for r in range(P):
                        got = gu.to_host(dev[r], npdt)
                        gu.assert_reduced_equal(got[skip:skip + n], exp[r], dtype, f"misaligned skip={skip} n={n} op={op} v={variant}")
                        gu.assert_bits_equal(got[:skip], host[r][:skip], "in front of the view")
                        gu.assert_bits_equal(got[skip + n:], host[r][skip + n:], "behind the view")
            # rooted: only the root's view changes
            exp = [h[skip:skip + n].copy() for h in host]
            oracle.reduce(exp, dtype, mcr.SUM, 2)
            dev = [gu.to_dev(h) for h in host]
            mcr.mcr_reduce(gu.ctx(), [d[skip:skip + n] for d in dev], n, dtype, mcr.SUM, 2, P, 6 if n >= W - skip else mcr.AUTO)
            gu.sync()
            for r in range(P):
                got = gu.to_host(dev[r], npdt)
                gu.assert_reduced_equal(got[skip:skip + n], exp[r], dtype, f"misaligned reduce skip={skip} n={n} r={r}")
                gu.assert_bits_equal(got[:skip], host[r][:skip], "in front of the view")
                gu.assert_bits_equal(got[skip + n:], host[r][skip + n:], "behind the view")
    # different misalignments
    n = 4097
    host = _make(P, pad + n + pad, dtype, seed=11)
    skips = [1, 2, 1, 0]
    exp = [h[k:k + n].copy() for h, k in zip(host, skips)]
    oracle.allreduce(exp, dtype, mcr.SUM)
    dev = [gu.to_dev(h) for h in host]
    views = [d[k:k + n] for d, k in zip(dev, skips)]
    with pytest.raises(mcr.McrError) as e:
        mcr.mcr_allreduce(gu.ctx(), views, n, dtype, mcr.SUM, P, 3)
    assert e.value.status == mcr.EVARIANT
    mcr.mcr_allreduce(gu.ctx(), views, n, dtype, mcr.SUM, P, mcr.AUTO)
    gu.sync()
    for r, k in enumerate(skips):
        got = gu.to_host(dev[r], npdt)
        gu.assert_reduced_equal(got[k:k + n], exp[r], dtype, "different misalignments")
        gu.assert_bits_equal(got[:k], host[r][:k], "in front of the view")
        gu.assert_bits_equal(got[k + n:], host[r][k + n:], "behind the view")


def test_allreduce_empty_is_a_no_op():
    dev = [gu.dev_empty(4, mcr.F32, 1.0) for _ in range(2)]
    mcr.mcr_allreduce(gu.ctx(), dev, 0, mcr.F32, mcr.SUM, 2, mcr.AUTO)
    gu.sync()
    assert (dev[0].cpu().numpy() == 1.0).all()


def test_allreduce_on_side_stream():
    P, n = 4, 100000
    host = _make(P, n, mcr.F32, seed=9)
    exp = [h.copy() for h in host]
    oracle.allreduce(exp, oracle.F32, oracle.SUM)
    dev = [gu.to_dev(h) for h in host]
    gu.sync()
    s = torch.cuda.Stream()
    mcr.mcr_allreduce(gu.ctx(), dev, n, mcr.F32, mcr.SUM, P, mcr.AUTO, stream=s)
    ev = torch.cuda.Event()
    ev.record(s)                     # the caller's work handle
    ev.synchronize()
    gu.assert_bits_equal(gu.to_host(dev[2], np.float32), exp[2], "side stream")


# --------------------------------------------------- reduce_scatter / all_gather / all_to_all
def _variants_for(vec_ok, extra=()):
    return [mcr.AUTO] + (gu.ALL_VARIANTS + list(extra) if vec_ok else [0])


def test_variant_lists_match_the_library():
    for op in range(10):
        names = mcr.mcr_get_variants(gu.ctx(), op)
        extra = {mcr.OP_ALLGATHER: gu.ALLGATHER_EXTRA, mcr.OP_ALLREDUCE: gu.REDUCE_EXTRA, mcr.OP_REDUCE_SCATTER: gu.REDUCE_EXTRA,
                 mcr.OP_ALLTOALL: gu.ALLTOALL_EXTRA}
        want = len(gu.ALL_VARIANTS) + len(extra.get(op, []))
        assert len(names) == want, (op, names)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("P", [1, 2, 3, 8, 16])
def test_reduce_scatter(dtype, P):
    W = 4 if dtype == mcr.F32 else 8
    for b in (1, 5, 8, 1032, 9 * 1024 + 8):
        n = P * b
        host = _make(P, n, dtype, seed=200 + P, dist="uniform")
        for op in (mcr.SUM, mcr.AVG):
            exp = oracle.reduce_scatter(host, dtype, op)
            for variant in _variants_for(b % W == 0, gu.REDUCE_EXTRA):
                dev_in = [gu.to_dev(h) for h in host]
                dev_out = [gu.dev_empty(b, dtype, 0) for _ in range(P)]
                mcr.mcr_reduce_scatter(gu.ctx(), dev_out, dev_in, n, dtype, op, P, variant)
                gu.sync()
                for r in range(P):
                    gu.assert_reduced_equal(gu.to_host(dev_out[r], gu.NPDT[dtype]), exp[r], dtype,
                                            f"reduce_scatter dt={dtype} P={P} b={b} op={op} v={variant} r={r}")
            if b % W != 0:
                with pytest.raises(mcr.McrError) as e:
                    mcr.mcr_reduce_scatter(gu.ctx(), dev_out, dev_in, n, dtype, op, P, 1)
                assert e.value.status == mcr.EVARIANT


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("P", [1, 2, 5, 8, 16])
def test_allgather(dtype, P):
    W = 4 if dtype == mcr.F32 else 8
    for m in (1, 7, 8, 1032, 9 * 1024 + 8):
        host = _make(P, m, dtype, seed=300 + P, dist="uniform")
        exp = oracle.allgather(host, dtype)
        for variant in _variants_for(m % W == 0, gu.ALLGATHER_EXTRA):
            dev_in = [gu.to_dev(h) for h in host]
            dev_out = [gu.dev_empty(P * m, dtype, 0) for _ in range(P)]
            mcr.mcr_allgather(gu.ctx(), dev_out, dev_in, m, dtype, P, variant)
            gu.sync()
            for r in range(P):
                gu.assert_bits_equal(gu.to_host(dev_out[r], gu.NPDT[dtype]), exp[r],
                                     f"allgather dt={dtype} P={P} m={m} v={variant} r={r}")


def test_allgather_superchunk_spans_several_superchunks():
    """5 MiB + a ragged tail per rank: two 4 MiB super-chunks, the second partial."""
    P, dtype = 4, mcr.F32
    m = (5 << 20) // 4 + 1028
    host = _make(P, m, dtype, seed=333, dist="uniform")
    exp = oracle.allgather(host, dtype)
    for variant in gu.ALLGATHER_EXTRA:
        dev_out = [gu.dev_empty(P * m, dtype, 0) for _ in range(P)]
        mcr.mcr_allgather(gu.ctx(), dev_out, [gu.to_dev(h) for h in host], m, dtype, P, variant)
        gu.sync()
        for r in range(P):
            gu.assert_bits_equal(gu.to_host(dev_out[r], np.float32), exp[r], f"superchunk v={variant} r={r}")


def test_allgather_preserves_nan_payloads():
    pats = np.array([0x7FC01234, 0x80000000, 0x7F800001, 0x00000001] * 4, dtype=np.uint32).view(np.float32)
    host = [pats, pats[::-1].copy()]
    exp = oracle.allgather(host, oracle.F32)
    for variant in (0, 1):
        dev_out = [gu.dev_empty(2 * pats.size, mcr.F32, 0) for _ in range(2)]
        mcr.mcr_allgather(gu.ctx(), dev_out, [gu.to_dev(h) for h in host], pats.size, mcr.F32, 2, variant)
        gu.sync()
        gu.assert_bits_equal(gu.to_host(dev_out[1], np.float32), exp[1], "nan payload")


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("P", [1, 2, 3, 8, 16])
def test_alltoall(dtype, P):
    W = 4 if dtype == mcr.F32 else 8
    for b in (1, 3, 8, 1032, 5 * 1024 + 16):
        n = P * b
        host = _make(P, n, dtype, seed=400 + P, dist="uniform")
        exp = oracle.alltoall(host, dtype)
        for variant in _variants_for(b % W == 0, gu.ALLTOALL_EXTRA):
            dev_in = [gu.to_dev(h) for h in host]
            dev_out = [gu.dev_empty(n, dtype, 0) for _ in range(P)]
            mcr.mcr_alltoall(gu.ctx(), dev_out, dev_in, n, dtype, P, variant)
            gu.sync()
            for r in range(P):
                gu.assert_bits_equal(gu.to_host(dev_out[r], gu.NPDT[dtype]), exp[r],
                                     f"alltoall dt={dtype} P={P} b={b} v={variant} r={r}")


def test_rs_then_ag_equals_allreduce_on_gpu():
    P, b, dtype = 8, 4096, mcr.BF16
    n = P * b
    host = _make(P, n, dtype, seed=55)
    dev_in = [gu.to_dev(h) for h in host]
    rs = [gu.dev_empty(b, dtype) for _ in range(P)]
    ag = [gu.dev_empty(n, dtype) for _ in range(P)]
    mcr.mcr_reduce_scatter(gu.ctx(), rs, dev_in, n, dtype, mcr.SUM, P)
    mcr.mcr_allgather(gu.ctx(), ag, rs, b, dtype, P)
    mcr.mcr_allreduce(gu.ctx(), dev_in, n, dtype, mcr.SUM, P)
    gu.sync()
    for r in range(P):
        assert torch.equal(ag[r], dev_in[r])


# -------------------------------------------------------------------- all_to_allv
@pytest.mark.parametrize("dtype,w", [(mcr.F32, 1), (mcr.F32, 4), (mcr.BF16, 3), (mcr.BF16, 2048)])
@pytest.mark.parametrize("P", [1, 3, 16])
def test_alltoallv_transposed_matrix(dtype, w, P):
    """MCR_SPLITS_TRANSPOSED: the way back.  Host and device matrices, every variant, against the
    oracle's own loop nest for the way back; and forward then back through the library returns every
    sent row to where it was."""
    S = _splits(P, 40 if w < 1000 else 9, seed=P * 1000 + w)
    in_rows = int(S.sum(axis=0).max()) + 3                            # a rank sends back what its column says it got
    out_rows = int(S.sum(axis=1).max()) + 2
    host = [inputs.uniform_pm1(in_rows * w, 600 + w, p, bf16=(dtype == mcr.BF16)) for p in range(P)]
    sentinel = np.full(out_rows * w, 0x5A5A if dtype == mcr.BF16 else -123.0, dtype=gu.NPDT[dtype])
    exp = [sentinel.copy() for _ in range(P)]
    oracle.alltoallv(host, S, w, dtype, exp, transposed=True)
    vec_ok = (w * gu.EB[dtype]) % 16 == 0
    dS = torch.from_numpy(S).cuda()
    for variant in _variants_for(vec_ok):
        for flags in (mcr.SPLITS_TRANSPOSED, mcr.SPLITS_TRANSPOSED | mcr.SPLITS_ON_DEVICE):
            dev_in = [gu.to_dev(h) for h in host]
            dev_out = [gu.to_dev(sentinel) for _ in range(P)]
            mcr.mcr_alltoallv(gu.ctx(), dev_out, dev_in, dS if flags & mcr.SPLITS_ON_DEVICE else S, flags, in_rows, out_rows, w,
                              dtype, P, variant)
            gu.sync()
            for r in range(P):
                gu.assert_bits_equal(gu.to_host(dev_out[r], gu.NPDT[dtype]), exp[r],
                                     f"alltoallv transposed dt={dtype} w={w} P={P} v={variant} flags={flags} r={r}")
    # there and back again on the device: rows [0, sum_r S[p][r]) of every rank come home
    there = [gu.dev_empty(in_rows * w, dtype, 0) for _ in range(P)]
    src = [inputs.uniform_pm1(out_rows * w, 700 + w, p, bf16=(dtype == mcr.BF16)) for p in range(P)]
    home = [gu.dev_empty(out_rows * w, dtype, 0) for _ in range(P)]
    mcr.mcr_alltoallv(gu.ctx(), there, [gu.to_dev(h) for h in src], dS, mcr.SPLITS_ON_DEVICE, out_rows, in_rows, w, dtype, P)
    mcr.mcr_alltoallv(gu.ctx(), home, there, dS, mcr.SPLITS_ON_DEVICE | mcr.SPLITS_TRANSPOSED, in_rows, out_rows, w, dtype, P)
    gu.sync()
    for p in range(P):
        sent = int(S[p].sum()) * w
        gu.assert_bits_equal(gu.to_host(home[p], gu.NPDT[dtype])[:sent], src[p][:sent], f"there and back, rank {p}")
    with pytest.raises(mcr.McrError) as e:
        mcr.mcr_alltoallv(gu.ctx(), home, there, dS, 4, in_rows, out_rows, w, dtype, P)
    assert e.value.status == mcr.EINVAL


def _splits(P, max_rows, seed, zero_frac=0.2):
    g = np.random.Generator(np.random.Philox(key=seed))
    S = g.integers(0, max_rows + 1, size=(P, P), dtype=np.int64)
    S[g.random((P, P)) < zero_frac] = 0
    return S


@pytest.mark.parametrize("dtype,w", [(mcr.F32, 1), (mcr.F32, 4), (mcr.F32, 128), (mcr.BF16, 3), (mcr.BF16, 8), (mcr.BF16, 2048), (mcr.F32, 12)])
@pytest.mark.parametrize("P", [1, 2, 5, 16])
def test_alltoallv_host_and_device_splits(dtype, w, P):
    S = _splits(P, 40 if w < 1000 else 9, seed=P * 100 + w)
    in_rows = int(S.sum(axis=1).max()) + 3
    out_rows = int(S.sum(axis=0).max()) + 2
    host = [inputs.uniform_pm1(in_rows * w, 500 + w, p, bf16=(dtype == mcr.BF16)) for p in range(P)]
    sentinel = np.full(out_rows * w, 0x5A5A if dtype == mcr.BF16 else -123.0, dtype=gu.NPDT[dtype])
    exp = [sentinel.copy() for _ in range(P)]
    oracle.alltoallv(host, S, w, dtype, exp)
    vec_ok = (w * gu.EB[dtype]) % 16 == 0
    dS = torch.from_numpy(S).cuda()
    for variant in _variants_for(vec_ok):
        for on_device in (False, True):
            dev_in = [gu.to_dev(h) for h in host]
            dev_out = [gu.to_dev(sentinel) for _ in range(P)]
            mcr.mcr_alltoallv(gu.ctx(), dev_out, dev_in, dS if on_device else S, on_device, in_rows, out_rows, w,
                              dtype, P, variant)
            gu.sync()
            for r in range(P):
                gu.assert_bits_equal(gu.to_host(dev_out[r], gu.NPDT[dtype]), exp[r],
                                     f"alltoallv dt={dtype} w={w} P={P} v={variant} dev={on_device} r={r}")


def test_alltoallv_skewed_large():
    """One destination gets ten times the rows of another; several tiles per pair."""
    P, w, dtype = 8, 256, mcr.BF16
    S = np.zeros((P, P), dtype=np.int64)
    for p in range(P):
        S[p] = [700, 350, 200, 120, 90, 70, 70, 0]
    S[3, 0] = 0
    in_rows, out_rows = int(S.sum(axis=1).max()), int(S.sum(axis=0).max())
    host = [inputs.normal(in_rows * w, 600, p, bf16=True) for p in range(P)]
    exp = [np.zeros(out_rows * w, dtype=np.uint16) for _ in range(P)]
    oracle.alltoallv(host, S, w, dtype, exp)
    for variant in (mcr.AUTO, 3, 6, 12):
        dev_out = [gu.dev_empty(out_rows * w, dtype, 0) for _ in range(P)]
        mcr.mcr_alltoallv(gu.ctx(), dev_out, [gu.to_dev(h) for h in host], torch.from_numpy(S).cuda(), True, in_rows,
                          out_rows, w, dtype, P, variant)
        gu.sync()
        for r in range(P):
            gu.assert_bits_equal(gu.to_host(dev_out[r], np.uint16), exp[r], f"skew v={variant} r={r}")


def test_alltoallv_equal_split_default_and_involution():
    P, rows, w, dtype = 4, 64, 32, mcr.F32
    host = [inputs.normal(rows * w, 700, p) for p in range(P)]
    exp = oracle.alltoall(host, dtype)
    dev_in = [gu.to_dev(h) for h in host]
    dev_mid = [gu.dev_empty(rows * w, dtype, 0) for _ in range(P)]
    dev_back = [gu.dev_empty(rows * w, dtype, 0) for _ in range(P)]
    mcr.mcr_alltoallv(gu.ctx(), dev_mid, dev_in, None, False, rows, rows, w, dtype, P)
    mcr.mcr_alltoallv(gu.ctx(), dev_back, dev_mid, None, False, rows, rows, w, dtype, P)
    gu.sync()
    for r in range(P):
        gu.assert_bits_equal(gu.to_host(dev_mid[r], np.float32), exp[r], "equal split")
        gu.assert_bits_equal(gu.to_host(dev_back[r], np.float32), host[r], "involution")


def test_alltoallv_device_splits_out_of_bounds_are_skipped():
    """A device-resident split matrix is untrusted: rows that would leave the declared
    buffers are skipped by the kernel's own bounds checks, everything else is copied."""
    P, w, dtype = 2, 4, mcr.F32
    in_rows, out_rows = 4, 5
    S = np.array([[2, 9], [-3, 4]], dtype=np.int64)        # row 0 claims 11 rows of a 4-row buffer
    host = [np.arange(in_rows * w, dtype=np.float32) + 100 * p for p in range(P)]
    dev_out = [gu.dev_empty(out_rows * w, dtype, -1.0) for _ in range(P)]
    mcr.mcr_alltoallv(gu.ctx(), dev_out, [gu.to_dev(h) for h in host], torch.from_numpy(S).cuda(), True, in_rows,
                      out_rows, w, dtype, P, 1)
    gu.sync()
    # effective matrix after clamping to in_rows and dropping rows past the buffers:
    # S' = [[2,4],[0,4]]; rank 0 sends rows 0,1 -> rank 0 and rows 2,3 (of the claimed 4) -> rank 1
    o0 = gu.to_host(dev_out[0], np.float32).reshape(out_rows, w)
    o1 = gu.to_host(dev_out[1], np.float32).reshape(out_rows, w)
    assert np.array_equal(o0[:2], host[0].reshape(in_rows, w)[:2]) and (o0[2:] == -1).all()
    assert np.array_equal(o1[:2], host[0].reshape(in_rows, w)[2:4])
    # rank 1's four rows land after rank 0's claimed four; only one fits in the 5-row buffer
    assert np.array_equal(o1[4], host[1].reshape(in_rows, w)[0]) and (o1[2:4] == -1).all()


# ------------------------------------------------------------------ other ReduceOps
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("op", [mcr.MAX, mcr.MIN, mcr.PROD])
def test_max_min_prod(dtype, op):
    """all_reduce, reduce_scatter, reduce and the fused multi-tensor all_reduce with the other
    ReduceOps; NaNs, infinities and signed zeros sprinkled into the inputs."""
    P, b = 5, 2056
    n = P * b
    host = _make(P, n, dtype, seed=900 + op, dist="uniform")
    specials = np.array([0x7FC00000, 0x7F800000, 0xFF800000, 0x00000000, 0x80000000], dtype=np.uint32).view(np.float32)
    sp = specials if dtype == mcr.F32 else inputs.f32_bits_to_bf16_trunc(specials)
    g = np.random.Generator(np.random.Philox(key=901))
    for p in range(P):
        idx = g.integers(0, n, size=40)
        host[p][idx] = sp[g.integers(0, len(sp), size=40)]
    with np.errstate(all="ignore"):
        exp_ar = [h.copy() for h in host]
        oracle.allreduce(exp_ar, dtype, op)
        exp_rs = oracle.reduce_scatter(host, dtype, op)
        exp_red = [h.copy() for h in host]
        oracle.reduce(exp_red, dtype, op, 2)
    for variant in (mcr.AUTO, 0, 2, 6, 13, 14):
        dev = [gu.to_dev(h) for h in host]
        mcr.mcr_allreduce(gu.ctx(), dev, n, dtype, op, P, variant)
        d_in = [gu.to_dev(h) for h in host]
        d_rs = [gu.dev_empty(b, dtype, 0) for _ in range(P)]
        mcr.mcr_reduce_scatter(gu.ctx(), d_rs, d_in, n, dtype, op, P, variant)
        d_red = [gu.to_dev(h) for h in host]
        mcr.mcr_reduce(gu.ctx(), d_red, n, dtype, op, 2, P, variant)
        gu.sync()
        for r in range(P):
            gu.assert_reduced_equal(gu.to_host(dev[r], gu.NPDT[dtype]), exp_ar[r], dtype, f"allreduce op={op} v={variant}")
            gu.assert_reduced_equal(gu.to_host(d_rs[r], gu.NPDT[dtype]), exp_rs[r], dtype, f"reduce_scatter op={op} v={variant}")
            gu.assert_reduced_equal(gu.to_host(d_red[r], gu.NPDT[dtype]), exp_red[r], dtype, f"reduce op={op} v={variant}")
    # fused multi-tensor path
    numel = [100, 4096, 37, 9000]
    plan = mcr.mcr_fuse_plan_create(gu.ctx(), numel, 1 << 30, dtype)
    try:
        th = [[inputs.uniform_pm1(m, 902, p, i, bf16=(dtype == mcr.BF16)) for i, m in enumerate(numel)] for p in range(P)]
        td = [[gu.to_dev(t) for t in th[p]] for p in range(P)]
        mcr.mcr_fuse_plan_bind(gu.ctx(), plan, [t for p in range(P) for t in td[p]], P)
        mcr.mcr_allreduce_multi(gu.ctx(), plan, -1, op)
        gu.sync()
        for i in range(len(numel)):
            e = [th[p][i].copy() for p in range(P)]
            oracle.allreduce(e, dtype, op)
            for p in range(P):
                gu.assert_reduced_equal(gu.to_host(td[p][i], gu.NPDT[dtype]), e[p], dtype, f"multi op={op} t={i}")
    finally:
        mcr.mcr_fuse_plan_destroy(plan)
