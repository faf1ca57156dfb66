"""Helpers for the GPU parity tests: host numpy <-> device torch buffers (torch is used for
device memory only), a shared library context, bitwise comparison."""
import numpy as np
import torch

import oracle
from paper_2303_08374_amd import mcr

_ctx = None


def ctx():
    global _ctx
    if _ctx is None:
        _ctx = mcr.mcr_init(0)
    return _ctx


def to_dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def to_host(t: torch.Tensor, like: np.dtype) -> np.ndarray:
    a = t.cpu().numpy()
    if np.dtype(like) == np.uint16:
        a = a.view(np.uint16)
    return a


def dev_empty(n: int, dtype: int, fill=None) -> torch.Tensor:
    td = {mcr.F32: torch.float32, mcr.BF16: torch.int16, mcr.F16: torch.float16, mcr.I32: torch.int32}[dtype]
    t = torch.empty(n, dtype=td, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def sync():
    torch.cuda.synchronize()


def assert_bits_equal(got: np.ndarray, exp: np.ndarray, what=""):
    g = np.ascontiguousarray(got).view(np.uint8)
    e = np.ascontiguousarray(exp).view(np.uint8)
    assert g.shape == e.shape, (what, g.shape, e.shape)
    if not np.array_equal(g, e):
        es = exp.dtype.itemsize
        bad = np.nonzero((g.reshape(-1, es) != e.reshape(-1, es)).any(axis=1))[0]
        raise AssertionError(f"{what}: {bad.size} of {exp.size} elements differ, first at {bad[:5].tolist()}: "
                             f"got {got.reshape(-1)[bad[:5]]} expected {exp.reshape(-1)[bad[:5]]}")


def assert_reduced_equal(got: np.ndarray, exp: np.ndarray, dtype: int, what=""):
    """Reduced outputs: bit-equal except that a NaN only has to be a NaN."""
    if dtype == mcr.I32:
        return assert_bits_equal(got, exp, what)
    if dtype in (mcr.F32, mcr.F16):
        gn, en = np.isnan(got), np.isnan(exp)
    else:
        isnan = lambda h: ((h & 0x7F80) == 0x7F80) & ((h & 0x7F) != 0)
        gn, en = isnan(got), isnan(exp)
    assert np.array_equal(gn, en), f"{what}: NaN positions differ"
    assert_bits_equal(np.where(gn, 0, got).astype(got.dtype), np.where(en, 0, exp).astype(exp.dtype), what)


VEC_VARIANTS = list(range(1, 13))          # every 128-bit launch shape
ALL_VARIANTS = [0] + VEC_VARIANTS
ALLGATHER_EXTRA = [13, 14, 15, 16]         # super-chunk forms of all_gather
REDUCE_EXTRA = list(range(13, 35))         # persistent form, one-wavefront workgroups, XCD-unit forms
# for the tests on long messages: the persistent and one-wavefront forms and XCD-unit forms of every shape, from the
# smallest to the largest unit (the unit is a run-time argument of one kernel per shape)
REDUCE_LONG = [13, 14, 15, 19, 22, 26, 29, 30, 33, 34]
ALLTOALL_EXTRA = [13, 14, 15]              # flat, one-wavefront and LDS-staged forms of all_to_all_single of all_reduce / reduce / reduce_scatter
NPDT = {mcr.F32: np.float32, mcr.BF16: np.uint16, mcr.F16: np.float16, mcr.I32: np.int32}
EB = {mcr.F32: 4, mcr.BF16: 2, mcr.F16: 2, mcr.I32: 4}
assert (oracle.F32, oracle.BF16, oracle.F16, oracle.I32, oracle.SUM, oracle.AVG) == (mcr.F32, mcr.BF16, mcr.F16, mcr.I32, mcr.SUM, mcr.AVG)
