"""ctypes front end of the CPU oracle (``mcr_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's
CPU-baseline leg call this; the GPU library never does, and nothing here
imports the GPU package.  All arrays are numpy, host resident; bf16 travels
as ``uint16`` bit patterns.

Argument marshalling only -- every loop of the operations lives in the C++
file, which cites the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

F32 = 0
BF16 = 1
F16 = 2          # IEEE binary16, carried as numpy float16
I32 = 3
SUM = 0
AVG = 1
MAX = 2
MIN = 3
PROD = 4

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mcr_oracle.cpp")
_LIB = os.path.join(_HERE, "libmcr_oracle.so")

CXXFLAGS = ["-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
            "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (about a second); returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["g++", *CXXFLAGS, "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_f32_to_bf16.restype = ctypes.c_uint16
        _lib.orc_f32_to_bf16.argtypes = [ctypes.c_float]
        _lib.orc_bf16_to_f32.restype = ctypes.c_float
        _lib.orc_bf16_to_f32.argtypes = [ctypes.c_uint16]
    return _lib


def np_dtype(dtype: int):
    return {F32: np.float32, BF16: np.uint16, F16: np.float16, I32: np.int32}[dtype]


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what} rejected its arguments (rc={rc})")


def _ptrs(arrs: Sequence[np.ndarray]):
    for a in arrs:
        assert a.flags["C_CONTIGUOUS"], "oracle arrays must be contiguous"
    return (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


# ---- bf16 -------------------------------------------------------------------
def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().orc_f32_to_bf16_array(_p(x), _p(out), ctypes.c_size_t(x.size))
    return out


def bf16_to_f32(h: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    lib().orc_bf16_to_f32_array(_p(h), _p(out), ctypes.c_size_t(h.size))
    return out


# ---- fp16 (bit patterns in, bit patterns out, so that NaN payloads can be looked at) ----
def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().orc_f32_to_f16_array(_p(x), _p(out), ctypes.c_size_t(x.size))
    return out


def f16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    lib().orc_f16_to_f32_array(_p(h), _p(out), ctypes.c_size_t(h.size))
    return out


# ---- collectives ------------------------------------------------------------
def allreduce(bufs: List[np.ndarray], dtype: int, op: int = SUM) -> None:
    """In place on every array of ``bufs`` (one per rank)."""
    n = bufs[0].size
    assert all(b.size == n and b.dtype == np_dtype(dtype) for b in bufs)
    _check(lib().orc_allreduce(_ptrs(bufs), ctypes.c_size_t(n), dtype, op, len(bufs)), "allreduce")


def allreduce_ref64(bufs: List[np.ndarray], dtype: int, op: int = SUM):
    """(binary64 sum, binary64 sum of magnitudes) per element."""
    n = bufs[0].size
    out = np.empty(n, dtype=np.float64)
    mag = np.empty(n, dtype=np.float64)
    _check(lib().orc_allreduce_ref64(_ptrs(bufs), ctypes.c_size_t(n), dtype, op, len(bufs),
                                     _p(out), _p(mag)), "allreduce_ref64")
    return out, mag


def reduce(bufs: List[np.ndarray], dtype: int, op: int, root: int) -> None:
    """In place on ``bufs[root]`` only."""
    n = bufs[0].size
    _check(lib().orc_reduce(_ptrs(bufs), ctypes.c_size_t(n), dtype, op, len(bufs), root), "reduce")


def bcast(bufs: List[np.ndarray], dtype: int, root: int) -> None:
    n = bufs[0].size
    _check(lib().orc_bcast(_ptrs(bufs), ctypes.c_size_t(n), dtype, len(bufs), root), "bcast")


def gatherv(ins: List[np.ndarray], counts: Sequence[int], dtype: int) -> np.ndarray:
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    out = np.zeros(int(c.sum()), dtype=np_dtype(dtype))
    _check(lib().orc_gatherv(_p(out), _ptrs(ins), _p(c), dtype, len(ins)), "gatherv")
    return out


def scatterv(root_in: np.ndarray, counts: Sequence[int], dtype: int) -> List[np.ndarray]:
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    outs = [np.zeros(int(n), dtype=np_dtype(dtype)) for n in c]
    _check(lib().orc_scatterv(_ptrs(outs), _p(root_in), _p(c), dtype, len(outs)), "scatterv")
    return outs


def allgatherv(ins: List[np.ndarray], counts: Sequence[int], dtype: int) -> List[np.ndarray]:
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    outs = [np.zeros(int(c.sum()), dtype=np_dtype(dtype)) for _ in ins]
    _check(lib().orc_allgatherv(_ptrs(outs), _ptrs(ins), _p(c), dtype, len(ins)), "allgatherv")
    return outs


def gatherv_displs(out: np.ndarray, ins: List[np.ndarray], counts: Sequence[int], displs: Sequence[int], dtype: int) -> None:
    """Writes into ``out`` (kept elsewhere): out[displs[p] + j] = ins[p][j]."""
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    d = np.ascontiguousarray(displs, dtype=np.uint64)
    assert all(int(d[p] + c[p]) <= out.size and ins[p].size >= int(c[p]) for p in range(len(ins)))
    _check(lib().orc_gatherv_displs(_p(out), _ptrs(ins), _p(c), _p(d), dtype, len(ins)), "gatherv_displs")


def scatterv_displs(root_in: np.ndarray, counts: Sequence[int], displs: Sequence[int], dtype: int) -> List[np.ndarray]:
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    d = np.ascontiguousarray(displs, dtype=np.uint64)
    assert all(int(d[r] + c[r]) <= root_in.size for r in range(c.size))
    outs = [np.zeros(int(n), dtype=np_dtype(dtype)) for n in c]
    _check(lib().orc_scatterv_displs(_ptrs(outs), _p(root_in), _p(c), _p(d), dtype, len(outs)), "scatterv_displs")
    return outs


def allgatherv_displs(outs: List[np.ndarray], ins: List[np.ndarray], counts: Sequence[int], displs: Sequence[int],
                      dtype: int) -> None:
    c = np.ascontiguousarray(counts, dtype=np.uint64)
    d = np.ascontiguousarray(displs, dtype=np.uint64)
    assert all(int(d[p] + c[p]) <= o.size for o in outs for p in range(len(ins)))
    _check(lib().orc_allgatherv_displs(_ptrs(outs), _ptrs(ins), _p(c), _p(d), dtype, len(ins)), "allgatherv_displs")


def alltoallv_displs(outs: List[np.ndarray], ins: List[np.ndarray], counts: np.ndarray, sdispls: np.ndarray,
                     rdispls: np.ndarray, row_elems: int, dtype: int) -> None:
    """counts[p, r] rows from row sdispls[p, r] of ins[p] to row rdispls[r, p] of outs[r]."""
    P = len(ins)
    C = np.ascontiguousarray(counts, dtype=np.int64)
    SD = np.ascontiguousarray(sdispls, dtype=np.int64)
    RD = np.ascontiguousarray(rdispls, dtype=np.int64)
    assert C.shape == SD.shape == RD.shape == (P, P)
    for p in range(P):
        for r in range(P):
            assert (SD[p, r] + C[p, r]) * row_elems <= ins[p].size and (RD[r, p] + C[p, r]) * row_elems <= outs[r].size
    _check(lib().orc_alltoallv_displs(_ptrs(outs), _ptrs(ins), _p(C), _p(SD), _p(RD), ctypes.c_size_t(row_elems), dtype, P),
           "alltoallv_displs")


def reduce_scatter(ins: List[np.ndarray], dtype: int, op: int = SUM) -> List[np.ndarray]:
    P = len(ins)
    n = ins[0].size
    if n % P:
        raise ValueError("count not divisible by P")
    outs = [np.zeros(n // P, dtype=np_dtype(dtype)) for _ in range(P)]
    _check(lib().orc_reduce_scatter(_ptrs(outs), _ptrs(ins), ctypes.c_size_t(n), dtype, op, P),
           "reduce_scatter")
    return outs


def allgather(ins: List[np.ndarray], dtype: int) -> List[np.ndarray]:
    P = len(ins)
    m = ins[0].size
    outs = [np.zeros(P * m, dtype=np_dtype(dtype)) for _ in range(P)]
    _check(lib().orc_allgather(_ptrs(outs), _ptrs(ins), ctypes.c_size_t(m), dtype, P), "allgather")
    return outs


def alltoall(ins: List[np.ndarray], dtype: int) -> List[np.ndarray]:
    P = len(ins)
    n = ins[0].size
    if n % P:
        raise ValueError("count not divisible by P")
    outs = [np.zeros(n, dtype=np_dtype(dtype)) for _ in range(P)]
    _check(lib().orc_alltoall(_ptrs(outs), _ptrs(ins), ctypes.c_size_t(n), dtype, P), "alltoall")
    return outs


def alltoallv(ins: List[np.ndarray], S: np.ndarray, row_elems: int, dtype: int,
              outs: Optional[List[np.ndarray]] = None, transposed: bool = False) -> List[np.ndarray]:
    """``S[p, r]`` rows go from rank p to rank r (``transposed``: the way back, ``S[p, r]`` rows go
    from rank r to rank p).  ``outs`` (if given) keeps its rows beyond the received ones; otherwise
    exact-size outputs are made."""
    P = len(ins)
    S = np.ascontiguousarray(S, dtype=np.int64)
    assert S.shape == (P, P)
    sent = S.sum(axis=0) if transposed else S.sum(axis=1)
    received = S.sum(axis=1) if transposed else S.sum(axis=0)
    if outs is None:
        outs = [np.zeros(int(received[r]) * row_elems, dtype=np_dtype(dtype)) for r in range(P)]
    for p in range(P):
        assert ins[p].size >= int(sent[p]) * row_elems
    for r in range(P):
        assert outs[r].size >= int(received[r]) * row_elems
    fn = lib().orc_alltoallv_transposed if transposed else lib().orc_alltoallv
    _check(fn(_ptrs(outs), _ptrs(ins), _p(S), ctypes.c_size_t(row_elems), dtype, P), "alltoallv")
    return outs


# ---- MoE --------------------------------------------------------------------
def moe_route(ids: np.ndarray, E: int, P: int, C: int):
    """One rank: returns (slot[T] int32, counts[E] int32, srow[P] int64)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T = ids.size
    slot = np.empty(T, dtype=np.int32)
    counts = np.empty(E, dtype=np.int32)
    srow = np.empty(P, dtype=np.int64)
    _check(lib().orc_moe_route(_p(ids), T, E, P, C, _p(slot), _p(counts), _p(srow)), "moe_route")
    return slot, counts, srow


def moe_expert_layout(counts: np.ndarray):
    """counts [P, E] int32 -> (block_first [P, E], expert_first [E], expert_rows [E]) int64."""
    counts = np.ascontiguousarray(counts, dtype=np.int32)
    P, E = counts.shape
    bf = np.zeros((P, E), dtype=np.int64)
    ef = np.zeros(E, dtype=np.int64)
    er = np.zeros(E, dtype=np.int64)
    _check(lib().orc_moe_expert_layout(_p(counts), E, P, _p(bf), _p(ef), _p(er)), "moe_expert_layout")
    return bf, ef, er


def _i32_ptrs(arrs):
    keep = [np.ascontiguousarray(a, dtype=np.int32) for a in arrs]
    return keep, _ptrs(keep)


def moe_dispatch_by_expert(recv: List[np.ndarray], toks: List[np.ndarray], ids, slots, counts: np.ndarray, row_elems: int,
                           dtype: int, K: int = 1) -> None:
    """ids, slots: per rank K*T entries, choice-major (entry k*T + t = choice k of token t)."""
    counts = np.ascontiguousarray(counts, dtype=np.int32)
    P, E = counts.shape
    k1, pi = _i32_ptrs(ids)
    k2, ps = _i32_ptrs(slots)
    assert k1[0].size % K == 0
    _check(lib().orc_moe_dispatch_by_expert(_ptrs(recv), _ptrs(toks), pi, ps, _p(counts), ctypes.c_int64(k1[0].size // K), K,
                                            E, P, ctypes.c_size_t(row_elems), dtype), "moe_dispatch_by_expert")


def moe_combine_by_expert(expert_out: List[np.ndarray], ids, slots, gates, counts: np.ndarray, row_elems: int,
                          dtype: int, K: int = 1) -> List[np.ndarray]:
    counts = np.ascontiguousarray(counts, dtype=np.int32)
    P, E = counts.shape
    k1, pi = _i32_ptrs(ids)
    k2, ps = _i32_ptrs(slots)
    assert k1[0].size % K == 0
    T = k1[0].size // K
    outs = [np.empty(T * row_elems, dtype=np_dtype(dtype)) for _ in range(P)]
    if gates is None:
        pg = None
    else:
        kg = [np.ascontiguousarray(g, dtype=np.float32) for g in gates]
        pg = _ptrs(kg)
    _check(lib().orc_moe_combine_by_expert(_ptrs(outs), _ptrs(expert_out), pi, ps, pg, _p(counts), ctypes.c_int64(T), K, E, P,
                                           ctypes.c_size_t(row_elems), dtype), "moe_combine_by_expert")
    return outs


def pack(tok: np.ndarray, slot: np.ndarray, row_elems: int, dtype: int, out: np.ndarray) -> np.ndarray:
    slot = np.ascontiguousarray(slot, dtype=np.int32)
    _check(lib().orc_pack(_p(out), _p(tok), _p(slot), ctypes.c_int64(slot.size),
                          ctypes.c_size_t(row_elems), dtype), "pack")
    return out


def unpack(packed: np.ndarray, slot: np.ndarray, gate: Optional[np.ndarray], row_elems: int,
           dtype: int) -> np.ndarray:
    slot = np.ascontiguousarray(slot, dtype=np.int32)
    if gate is not None:
        gate = np.ascontiguousarray(gate, dtype=np.float32)
        assert gate.size == slot.size
    out = np.empty(slot.size * row_elems, dtype=np_dtype(dtype))
    _check(lib().orc_unpack(_p(out), _p(packed), _p(slot), _p(gate), ctypes.c_int64(slot.size),
                            ctypes.c_size_t(row_elems), dtype), "unpack")
    return out


# ---- DLRM -------------------------------------------------------------------
def dlrm_forward(src: List[np.ndarray], n_tables: int, batch: int, dim: int, dtype: int) -> List[np.ndarray]:
    P = len(src)
    outs = [np.zeros((batch // P) * n_tables * dim, dtype=np_dtype(dtype)) for _ in range(P)]
    _check(lib().orc_dlrm_forward(_ptrs(outs), _ptrs(src), n_tables, ctypes.c_int64(batch),
                                  ctypes.c_size_t(dim), dtype, P), "dlrm_forward")
    return outs


def dlrm_backward(grad_out: List[np.ndarray], n_tables: int, batch: int, dim: int, dtype: int) -> List[np.ndarray]:
    P = len(grad_out)
    n_local = [len(range(p, n_tables, P)) for p in range(P)]
    gsrc = [np.zeros(n_local[p] * batch * dim, dtype=np_dtype(dtype)) for p in range(P)]
    _check(lib().orc_dlrm_backward(_ptrs(gsrc), _ptrs(grad_out), n_tables, ctypes.c_int64(batch),
                                   ctypes.c_size_t(dim), dtype, P), "dlrm_backward")
    return gsrc


# ---- tensor fusion ----------------------------------------------------------
def fuse_plan(numel: Sequence[int], B: int):
    """Returns (tensor_bucket[int32], tensor_offset[uint64], bucket_numel[uint64])."""
    numel = np.ascontiguousarray(numel, dtype=np.uint64)
    n = numel.size
    tb = np.zeros(max(n, 1), dtype=np.int32)
    to = np.zeros(max(n, 1), dtype=np.uint64)
    bn = np.zeros(max(n, 1), dtype=np.uint64)
    nb = ctypes.c_int32(0)
    _check(lib().orc_fuse_plan(_p(numel), n, ctypes.c_uint64(B), _p(tb), _p(to), ctypes.byref(nb), _p(bn)),
           "fuse_plan")
    return tb[:n].copy(), to[:n].copy(), bn[:nb.value].copy()


def fuse(tensors: List[np.ndarray], offsets: Sequence[int], total: int, dtype: int) -> np.ndarray:
    flat = np.zeros(total, dtype=np_dtype(dtype))
    numel = np.array([t.size for t in tensors], dtype=np.uint64)
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    _check(lib().orc_fuse(_p(flat), _ptrs(tensors), _p(numel), _p(off), len(tensors), dtype), "fuse")
    return flat


def unfuse(flat: np.ndarray, numel: Sequence[int], offsets: Sequence[int], dtype: int) -> List[np.ndarray]:
    tensors = [np.zeros(int(n), dtype=np_dtype(dtype)) for n in numel]
    nn = np.ascontiguousarray(numel, dtype=np.uint64)
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    _check(lib().orc_unfuse(_ptrs(tensors), _p(flat), _p(nn), _p(off), len(tensors), dtype), "unfuse")
    return tensors


# ---- tuning table -----------------------------------------------------------
def tune_lookup(sizes: Sequence[int], choice: Sequence[int], nbytes: int) -> int:
    s = np.ascontiguousarray(sizes, dtype=np.uint64)
    c = np.ascontiguousarray(choice, dtype=np.int32)
    return int(lib().orc_tune_lookup(_p(s), _p(c), int(s.size), ctypes.c_uint64(nbytes)))
