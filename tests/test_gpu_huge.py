"""Buffers past 4 GiB per rank: every element and byte offset in the kernels must be 64-bit clean.
Windows of the outputs are checked against the oracle run on the downloaded inputs of the window
(as in test_gpu_full_size.py); the windows sit at the far end, beyond 2^32 bytes and beyond 2^31
elements, and at the start."""
import numpy as np
import pytest
import torch

import oracle
from paper_2303_08374_amd import mcr
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

W = 1536


def _fill(n, dtype, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    td = torch.float32 if dtype == mcr.F32 else torch.bfloat16
    t = torch.empty(n, dtype=td, device="cuda")
    step = 1 << 28
    for i in range(0, n, step):
        t[i:i + step].uniform_(-1.0, 1.0, generator=g)
    return t


def _host(t, s, w, dtype):
    a = t[s:s + w]
    if dtype == mcr.BF16:
        return a.view(torch.int16).cpu().numpy().view(np.uint16).copy()
    return a.cpu().numpy().copy()


def _windows(n, extra=()):
    cand = [0, n - W, n - W - 4099, (1 << 31) - W // 2, (1 << 31) + 77, (1 << 30) - 5] + list(extra)
    return sorted({min(max(c, 0), n - W) for c in cand})


def test_allreduce_and_reduce_scatter_past_2_31_elements():
    """bf16, P=2, 2^31 + 8200 elements per rank (4 GiB + 16 KiB): vector body and a ragged tail."""
    P, dtype = 2, mcr.BF16
    n = (1 << 31) + 8200 + 2                      # divisible by P; not by 8: the last elements take the scalar tail
    ins = [_fill(n, dtype, 3300 + p) for p in range(P)]
    b = n // P
    outs = [torch.zeros(b, dtype=torch.bfloat16, device="cuda") for _ in range(P)]
    mcr.mcr_reduce_scatter(gu.ctx(), outs, ins, n, dtype, mcr.SUM, P)
    gu.sync()
    for r in range(P):
        for st in _windows(b):
            win = [_host(ins[p], r * b + st, W, dtype) for p in range(P)]
            oracle.allreduce(win, dtype, oracle.SUM)
            gu.assert_bits_equal(_host(outs[r], st, W, dtype), win[0], f"reduce_scatter r={r} at {st}")
    del outs
    starts = _windows(n)
    before = {st: [_host(ins[p], st, W, dtype) for p in range(P)] for st in starts}
    mcr.mcr_allreduce(gu.ctx(), ins, n, dtype, mcr.AVG, P)
    gu.sync()
    for st in starts:
        exp = before[st]
        oracle.allreduce(exp, dtype, oracle.AVG)
        for r in range(P):
            gu.assert_bits_equal(_host(ins[r], st, W, dtype), exp[r], f"allreduce r={r} at {st}")


def test_allgather_and_alltoall_past_4_GiB_offsets():
    """fp32, P=3: 1.5 GiB + per rank in, all_gather outputs of 4.5 GiB each; all_to_all of the same inputs."""
    P, dtype = 3, mcr.F32
    n = 3 * ((1 << 27) + 1028)                    # elements per rank, divisible by P and by 4
    ins = [_fill(n, dtype, 3400 + p) for p in range(P)]
    outs = [torch.zeros(P * n, dtype=torch.float32, device="cuda") for _ in range(P)]
    for variant in (mcr.AUTO, 14):                # the table's pick and the 8 MiB super-chunk form
        for o in outs:
            o.zero_()
        mcr.mcr_allgather(gu.ctx(), outs, ins, n, dtype, P, variant)
        gu.sync()
        for r in (0, P - 1):
            for p in range(P):
                for st in _windows(n)[::2]:
                    gu.assert_bits_equal(_host(outs[r], p * n + st, W, dtype), _host(ins[p], st, W, dtype),
                                         f"allgather v={variant} r={r} p={p} at {st}")
    del outs
    b = n // P
    outs = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(P)]
    mcr.mcr_alltoall(gu.ctx(), outs, ins, n, dtype, P)
    gu.sync()
    for r in range(P):
        for p in range(P):
            for st in _windows(b)[::2]:
                gu.assert_bits_equal(_host(outs[r], p * b + st, W, dtype), _host(ins[p], r * b + st, W, dtype),
                                     f"alltoall r={r} p={p} at {st}")


def test_rows_past_4_GiB():
    """One rank, 2^19 + 5 rows of 8 KiB (4 GiB + 40 KiB): pack by a far-reaching permutation, all_to_allv with
    displacements of the packed buffer onto itself shifted by one row, unpack with the inverse."""
    P, dtype, H = 1, mcr.BF16, 4096
    T = (1 << 19) + 5
    src = [_fill(T * H, dtype, 3500)]
    # token t -> slot (t * 13 + 3) mod T: a permutation since gcd(13, T) = 1
    assert np.gcd(13, T) == 1
    slot_h = ((np.arange(T, dtype=np.int64) * 13 + 3) % T).astype(np.int32)
    slot = [torch.from_numpy(slot_h).cuda()]
    packed = [torch.zeros(T * H, dtype=torch.bfloat16, device="cuda")]
    mcr.mcr_pack(gu.ctx(), packed, src, slot, T, T, H, dtype, P)
    back = [torch.ones(T * H, dtype=torch.bfloat16, device="cuda")]
    mcr.mcr_unpack(gu.ctx(), back, packed, slot, None, T, T, H, dtype, P)
    shifted = [torch.zeros((T + 1) * H, dtype=torch.bfloat16, device="cuda")]
    mcr.mcr_alltoallv_displs(gu.ctx(), shifted, packed, [T], [0], [1], T, T + 1, H, dtype, P)
    gu.sync()
    rows = lambda t, row: t[row * H:(row + 1) * H].view(torch.int16).cpu().numpy()
    for t in (0, 1, T - 1, T - 2, T // 2, (1 << 19) - 1, 74898, 299593):
        assert np.array_equal(rows(packed[0], int(slot_h[t])), rows(src[0], t)), f"pack row {t}"
        assert np.array_equal(rows(back[0], t), rows(src[0], t)), f"unpack row {t}"
    for row in (0, T - 1, T // 3, (1 << 19) + 1):
        assert np.array_equal(rows(shifted[0], row + 1), rows(packed[0], row)), f"alltoallv_displs row {row}"
    assert (rows(shifted[0], 0) == 0).all()
