"""Thin ctypes binding of libmcr.so (see include/mcr.h for the contract of every call).

Argument marshalling only: each function has the name and argument order of its C
entry point, turns torch tensors into device addresses, passes torch's current HIP
stream unless told otherwise, and raises :class:`McrError` on a non-zero status.
There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Union

F32, BF16, F16, I32 = 0, 1, 2, 3
SUM, AVG, MAX, MIN, PROD = 0, 1, 2, 3, 4
AUTO = -1
MAX_RANKS = 16
MAX_EXPERTS = 512
MAX_TOPK = 4

OP_ALLREDUCE, OP_REDUCE_SCATTER, OP_ALLGATHER, OP_ALLTOALL, OP_ALLTOALLV = 0, 1, 2, 3, 4
OP_PACK, OP_UNPACK, OP_FUSE, OP_UNFUSE, OP_ALLREDUCE_MULTI, OP_MOE_ROUTE = 5, 6, 7, 8, 9, 10
OP_MOE_DISPATCH, OP_MOE_COMBINE, OP_DLRM_SHUFFLE = 11, 12, 13
OP_MOE_DISPATCH_BY_EXPERT, OP_MOE_COMBINE_BY_EXPERT = 14, 15
OP_NAMES = ["allreduce", "reduce_scatter", "allgather", "alltoall", "alltoallv", "pack", "unpack",
            "fuse", "unfuse", "allreduce_multi", "moe_route", "moe_dispatch", "moe_combine", "dlrm_shuffle",
            "moe_dispatch_by_expert", "moe_combine_by_expert"]

OK, EINVAL, EDTYPE, EOP, EVARIANT, ESPLIT, EHIP, ENOMEM, EIO, ESTATE, ELIMIT = 0, -1, -2, -3, -4, -5, -6, -7, -8, -9, -10
ROUTE_SCRATCH_BYTES = 1 << 20

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmcr.so")

Ptr = Union[int, "torch.Tensor"]  # noqa: F821


class McrError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} ({status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Opens libmcr.so; raises if it has not been built (python -m paper_2303_08374_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2303_08374_amd.build`; "
                              "there is no fallback path")
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.mcr_strerror.restype = ctypes.c_char_p
        _lib.mcr_strerror.argtypes = [ctypes.c_int]
    return _lib


def strerror(status: int) -> str:
    return lib().mcr_strerror(status).decode()


mcr_strerror = strerror


def _addr(x) -> int:
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _ptr_array(xs: Optional[Sequence[Ptr]], need: int = 0):
    """Host array of device addresses.  The library reads `need` entries (one per rank), so a
    shorter list is refused here: it would make the library read past the array."""
    if xs is None:
        return None
    if len(xs) < need:
        raise ValueError(f"a list of {len(xs)} device pointers was given where the call reads {need}")
    return (ctypes.c_void_p * len(xs))(*[_addr(x) for x in xs])


_raw_stream = None


def _current_stream_handle() -> int:
    """The calling thread's current torch stream as a raw handle.  torch's own accessor for the raw
    handle costs 0.1 us where building a torch.cuda.Stream object costs 3 us, which is a third of what
    a small collective takes from Python."""
    global _raw_stream
    import torch
    if _raw_stream is None:
        fast = getattr(torch._C, "_cuda_getCurrentRawStream", None)
        _raw_stream = (lambda: fast(torch.cuda.current_device())) if fast else (lambda: torch.cuda.current_stream().cuda_stream)
    return _raw_stream()


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        return ctypes.c_void_p(_current_stream_handle())
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise McrError(rc, what)


_sz = ctypes.c_size_t


# ---- lifecycle -----------------------------------------------------------------------------
SHIPPED_TABLE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tuning", "mi355x.tbl")


def mcr_init(device: int = 0) -> ctypes.c_void_p:
    ctx = ctypes.c_void_p()
    _check(lib().mcr_init(ctypes.byref(ctx), device), "mcr_init")
    return ctx


def mcr_finalize(ctx) -> None:
    _check(lib().mcr_finalize(ctx), "mcr_finalize")


def mcr_synchronize(ctx, stream=None) -> None:
    _check(lib().mcr_synchronize(ctx, _stream(stream)), "mcr_synchronize")


def mcr_get_variants(ctx, op_id: int) -> List[str]:
    n = ctypes.c_int(64)
    names = (ctypes.c_char_p * 64)()
    _check(lib().mcr_get_variants(ctx, op_id, names, ctypes.byref(n)), "mcr_get_variants")
    return [names[i].decode() for i in range(n.value)]


# ---- collectives ---------------------------------------------------------------------------
def mcr_allreduce(ctx, bufs: Sequence[Ptr], count: int, dtype: int, op: int, P: int, variant: int = AUTO,
                  stream=None) -> None:
    _check(lib().mcr_allreduce(ctx, _ptr_array(bufs, P), _sz(count), dtype, op, P, variant, _stream(stream)),
           "mcr_allreduce")


def mcr_reduce_scatter(ctx, out: Sequence[Ptr], inp: Sequence[Ptr], count: int, dtype: int, op: int, P: int,
                       variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_reduce_scatter(ctx, _ptr_array(out, P), _ptr_array(inp, P), _sz(count), dtype, op, P, variant,
                                    _stream(stream)), "mcr_reduce_scatter")


def mcr_allgather(ctx, out: Sequence[Ptr], inp: Sequence[Ptr], count: int, dtype: int, P: int,
                  variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_allgather(ctx, _ptr_array(out, P), _ptr_array(inp, P), _sz(count), dtype, P, variant,
                               _stream(stream)), "mcr_allgather")


def mcr_alltoall(ctx, out: Sequence[Ptr], inp: Sequence[Ptr], count: int, dtype: int, P: int,
                 variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_alltoall(ctx, _ptr_array(out, P), _ptr_array(inp, P), _sz(count), dtype, P, variant,
                              _stream(stream)), "mcr_alltoall")


SPLITS_ON_DEVICE, SPLITS_TRANSPOSED = 1, 2


def mcr_alltoallv(ctx, out: Sequence[Ptr], inp: Sequence[Ptr], splits, splits_flags: int, in_rows: int,
                  out_rows: int, row_elems: int, dtype: int, P: int, variant: int = AUTO, stream=None) -> None:
    """``splits``: None (equal split), a device tensor / address (SPLITS_ON_DEVICE in splits_flags;
    True and False still mean "on device" and "on the host"), or a host sequence of P*P integers,
    row-major.  SPLITS_TRANSPOSED: the matrix is read transposed (the way back)."""
    keep = None
    splits_flags = int(splits_flags)
    if splits is None:
        sp = ctypes.c_void_p(0)
    elif splits_flags & SPLITS_ON_DEVICE:
        sp = ctypes.c_void_p(_addr(splits))
    else:
        flat = [int(v) for row in splits for v in (row if hasattr(row, "__len__") else [row])]
        keep = (ctypes.c_int64 * len(flat))(*flat)
        sp = ctypes.cast(keep, ctypes.c_void_p)
    _check(lib().mcr_alltoallv(ctx, _ptr_array(out, P), _ptr_array(inp, P), sp, splits_flags,
                               _sz(in_rows), _sz(out_rows), _sz(row_elems), dtype, P, variant, _stream(stream)),
           "mcr_alltoallv")


# ---- rooted and vector collectives ---------------------------------------------------------
def _counts(counts: Sequence[int]):
    return (ctypes.c_size_t * len(counts))(*[int(c) for c in counts])


def mcr_reduce(ctx, bufs: Sequence[Ptr], count: int, dtype: int, op: int, root: int, P: int, variant: int = AUTO,
               stream=None) -> None:
    _check(lib().mcr_reduce(ctx, _ptr_array(bufs, P), _sz(count), dtype, op, root, P, variant, _stream(stream)), "mcr_reduce")


def mcr_bcast(ctx, bufs: Sequence[Ptr], count: int, dtype: int, root: int, P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_bcast(ctx, _ptr_array(bufs, P), _sz(count), dtype, root, P, variant, _stream(stream)), "mcr_bcast")


def mcr_gather(ctx, out: Ptr, inp: Sequence[Ptr], count: int, dtype: int, P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_gather(ctx, ctypes.c_void_p(_addr(out)), _ptr_array(inp, P), _sz(count), dtype, P, variant,
                            _stream(stream)), "mcr_gather")


def mcr_gatherv(ctx, out: Ptr, inp: Sequence[Ptr], counts: Sequence[int], dtype: int, P: int, variant: int = AUTO,
                stream=None) -> None:
    _check(lib().mcr_gatherv(ctx, ctypes.c_void_p(_addr(out)), _ptr_array(inp, P), _counts(counts), dtype, P, variant,
                             _stream(stream)), "mcr_gatherv")


def mcr_scatter(ctx, out: Sequence[Ptr], inp: Ptr, count: int, dtype: int, P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_scatter(ctx, _ptr_array(out, P), ctypes.c_void_p(_addr(inp)), _sz(count), dtype, P, variant,
                             _stream(stream)), "mcr_scatter")


def mcr_scatterv(ctx, out: Sequence[Ptr], inp: Ptr, counts: Sequence[int], dtype: int, P: int, variant: int = AUTO,
                 stream=None) -> None:
    _check(lib().mcr_scatterv(ctx, _ptr_array(out, P), ctypes.c_void_p(_addr(inp)), _counts(counts), dtype, P, variant,
                              _stream(stream)), "mcr_scatterv")


def mcr_allgatherv(ctx, out: Sequence[Ptr], inp: Sequence[Ptr], counts: Sequence[int], dtype: int, P: int,
                   variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_allgatherv(ctx, _ptr_array(out, P), _ptr_array(inp, P), _counts(counts), dtype, P, variant,
                                _stream(stream)), "mcr_allgatherv")


# ---- MoE -----------------------------------------------------------------------------------
def mcr_moe_route(ctx, expert_ids: Sequence[Ptr], T: int, E: int, P: int, capacity: int, slot: Sequence[Ptr],
                  counts: Sequence[Ptr], splits: Ptr, stream=None) -> None:
    _check(lib().mcr_moe_route(ctx, _ptr_array(expert_ids, P), T, E, P, capacity, _ptr_array(slot, P), _ptr_array(counts, P),
                               ctypes.c_void_p(_addr(splits)), _stream(stream)), "mcr_moe_route")


def mcr_moe_route_workspace_bytes(T: int, E: int, P: int) -> int:
    fn = lib().mcr_moe_route_workspace_bytes
    fn.restype = ctypes.c_size_t
    return int(fn(T, E, P))


def mcr_moe_route_ws(ctx, expert_ids: Sequence[Ptr], T: int, E: int, P: int, capacity: int, slot: Sequence[Ptr],
                     counts: Sequence[Ptr], splits: Ptr, workspace: Optional[Ptr], workspace_bytes: int, stream=None) -> None:
    ws = ctypes.c_void_p(_addr(workspace)) if workspace is not None else ctypes.c_void_p(0)
    _check(lib().mcr_moe_route_ws(ctx, _ptr_array(expert_ids, P), T, E, P, capacity, _ptr_array(slot, P), _ptr_array(counts, P),
                                  ctypes.c_void_p(_addr(splits)), ws, _sz(workspace_bytes), _stream(stream)), "mcr_moe_route_ws")


def mcr_moe_route_static(ctx, expert_ids: Sequence[Ptr], T: int, E: int, P: int, capacity: int, slot: Sequence[Ptr],
                         counts: Sequence[Ptr], splits: Ptr, stream=None) -> None:
    _check(lib().mcr_moe_route_static(ctx, _ptr_array(expert_ids, P), T, E, P, capacity, _ptr_array(slot, P), _ptr_array(counts, P),
                                      ctypes.c_void_p(_addr(splits)), _stream(stream)), "mcr_moe_route_static")


def mcr_pack(ctx, out: Sequence[Ptr], inp: Sequence[Ptr], slot: Sequence[Ptr], T: int, out_rows: int, row_elems: int,
             dtype: int, P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_pack(ctx, _ptr_array(out, P), _ptr_array(inp, P), _ptr_array(slot, P), _sz(T), _sz(out_rows),
                          _sz(row_elems), dtype, P, variant, _stream(stream)), "mcr_pack")


def mcr_unpack(ctx, out: Sequence[Ptr], inp: Sequence[Ptr], slot: Sequence[Ptr], gate: Optional[Sequence[Ptr]], T: int,
               in_rows: int, row_elems: int, dtype: int, P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_unpack(ctx, _ptr_array(out, P), _ptr_array(inp, P), _ptr_array(slot, P), _ptr_array(gate, P), _sz(T),
                            _sz(in_rows), _sz(row_elems), dtype, P, variant, _stream(stream)), "mcr_unpack")


def _i64_array(xs):
    flat = [int(x) for x in xs]
    return (ctypes.c_int64 * max(len(flat), 1))(*flat)


def mcr_alltoallv_displs(ctx, out: Sequence[Ptr], inp: Sequence[Ptr], counts, sdispls, rdispls, in_rows: int, out_rows: int,
                         row_elems: int, dtype: int, P: int, variant: int = AUTO, stream=None) -> None:
    """counts, sdispls, rdispls: P*P integers each, row-major ([p][r], [p][r], [r][p])."""
    _check(lib().mcr_alltoallv_displs(ctx, _ptr_array(out, P), _ptr_array(inp, P), _i64_array(counts), _i64_array(sdispls),
                                      _i64_array(rdispls), _sz(in_rows), _sz(out_rows), _sz(row_elems), dtype, P, variant,
                                      _stream(stream)), "mcr_alltoallv_displs")


def mcr_gatherv_displs(ctx, out: Ptr, out_elems: int, inp: Sequence[Ptr], counts: Sequence[int], displs: Sequence[int],
                       dtype: int, P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_gatherv_displs(ctx, ctypes.c_void_p(_addr(out)), _sz(out_elems), _ptr_array(inp, P), _counts(counts),
                                    _counts(displs), dtype, P, variant, _stream(stream)), "mcr_gatherv_displs")


def mcr_scatterv_displs(ctx, out: Sequence[Ptr], inp: Ptr, in_elems: int, counts: Sequence[int], displs: Sequence[int],
                        dtype: int, P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_scatterv_displs(ctx, _ptr_array(out, P), ctypes.c_void_p(_addr(inp)), _sz(in_elems), _counts(counts),
                                     _counts(displs), dtype, P, variant, _stream(stream)), "mcr_scatterv_displs")


def mcr_allgatherv_displs(ctx, out: Sequence[Ptr], out_elems: int, inp: Sequence[Ptr], counts: Sequence[int],
                          displs: Sequence[int], dtype: int, P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_allgatherv_displs(ctx, _ptr_array(out, P), _sz(out_elems), _ptr_array(inp, P), _counts(counts),
                                       _counts(displs), dtype, P, variant, _stream(stream)), "mcr_allgatherv_displs")


# ---- fused pipelines -----------------------------------------------------------------------
def mcr_moe_dispatch(ctx, recv: Sequence[Ptr], tokens: Sequence[Ptr], slot: Sequence[Ptr], splits: Ptr, T: int,
                     recv_rows: int, row_elems: int, dtype: int, P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_moe_dispatch(ctx, _ptr_array(recv, P), _ptr_array(tokens, P), _ptr_array(slot, P),
                                  ctypes.c_void_p(_addr(splits)), _sz(T), _sz(recv_rows), _sz(row_elems), dtype, P,
                                  variant, _stream(stream)), "mcr_moe_dispatch")


def mcr_moe_combine(ctx, out: Sequence[Ptr], expert_out: Sequence[Ptr], slot: Sequence[Ptr],
                    gate: Optional[Sequence[Ptr]], splits: Ptr, T: int, recv_rows: int, row_elems: int, dtype: int,
                    P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_moe_combine(ctx, _ptr_array(out, P), _ptr_array(expert_out, P), _ptr_array(slot, P), _ptr_array(gate, P),
                                 ctypes.c_void_p(_addr(splits)), _sz(T), _sz(recv_rows), _sz(row_elems), dtype, P,
                                 variant, _stream(stream)), "mcr_moe_combine")


def mcr_moe_expert_layout(ctx, counts: Sequence[Ptr], E: int, P: int, row_table: Ptr, expert_first: Ptr, expert_rows: Ptr,
                          stream=None) -> None:
    _check(lib().mcr_moe_expert_layout(ctx, _ptr_array(counts, P), E, P, ctypes.c_void_p(_addr(row_table)),
                                       ctypes.c_void_p(_addr(expert_first)), ctypes.c_void_p(_addr(expert_rows)),
                                       _stream(stream)), "mcr_moe_expert_layout")


def mcr_moe_source_layout(ctx, counts: Sequence[Ptr], E: int, P: int, row_table: Ptr, stream=None) -> None:
    _check(lib().mcr_moe_source_layout(ctx, _ptr_array(counts, P), E, P, ctypes.c_void_p(_addr(row_table)), _stream(stream)),
           "mcr_moe_source_layout")


def mcr_moe_dispatch_by_expert(ctx, recv: Sequence[Ptr], tokens: Sequence[Ptr], expert_ids: Sequence[Ptr], slot: Sequence[Ptr],
                               row_table: Ptr, T: int, K: int, E: int, recv_rows: int, row_elems: int, dtype: int, P: int,
                               variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_moe_dispatch_by_expert(ctx, _ptr_array(recv, P), _ptr_array(tokens, P), _ptr_array(expert_ids, P), _ptr_array(slot, P),
                                            ctypes.c_void_p(_addr(row_table)), _sz(T), K, E, _sz(recv_rows), _sz(row_elems),
                                            dtype, P, variant, _stream(stream)), "mcr_moe_dispatch_by_expert")


def mcr_moe_combine_by_expert(ctx, out: Sequence[Ptr], expert_out: Sequence[Ptr], expert_ids: Sequence[Ptr],
                              slot: Sequence[Ptr], gate: Optional[Sequence[Ptr]], row_table: Ptr, T: int, K: int, E: int,
                              recv_rows: int, row_elems: int, dtype: int, P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_moe_combine_by_expert(ctx, _ptr_array(out, P), _ptr_array(expert_out, P), _ptr_array(expert_ids, P),
                                           _ptr_array(slot, P), _ptr_array(gate, P), ctypes.c_void_p(_addr(row_table)), _sz(T), K, E,
                                           _sz(recv_rows), _sz(row_elems), dtype, P, variant, _stream(stream)),
           "mcr_moe_combine_by_expert")


def mcr_dlrm_shuffle(ctx, out: Sequence[Ptr], inp: Sequence[Ptr], n_tables: int, batch: int, dim: int, dtype: int,
                     P: int, backward: bool = False, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_dlrm_shuffle(ctx, _ptr_array(out, P), _ptr_array(inp, P), n_tables, _sz(batch), _sz(dim), dtype, P,
                                  int(bool(backward)), variant, _stream(stream)), "mcr_dlrm_shuffle")


# ---- tensor fusion -------------------------------------------------------------------------
_plan_tensors = {}          # plan handle -> its number of tensors (what mcr_fuse_plan_bind reads per rank)


def mcr_fuse_plan_create(ctx, numel: Sequence[int], bucket_elems: int, dtype: int) -> ctypes.c_void_p:
    arr = (ctypes.c_size_t * max(len(numel), 1))(*[int(n) for n in numel])
    plan = ctypes.c_void_p()
    _check(lib().mcr_fuse_plan_create(ctx, arr, len(numel), _sz(bucket_elems), dtype, ctypes.byref(plan)),
           "mcr_fuse_plan_create")
    _plan_tensors[plan.value] = len(numel)
    return plan


def mcr_fuse_plan_info(plan, n_tensors: int):
    """Returns (bucket_numel, tensor_bucket, tensor_offset) as Python lists."""
    nb = ctypes.c_int(0)
    _check(lib().mcr_fuse_plan_info(plan, ctypes.byref(nb), None, None, None), "mcr_fuse_plan_info")
    bn = (ctypes.c_size_t * max(nb.value, 1))()
    tb = (ctypes.c_int * max(n_tensors, 1))()
    to = (ctypes.c_size_t * max(n_tensors, 1))()
    _check(lib().mcr_fuse_plan_info(plan, ctypes.byref(nb), bn, tb, to), "mcr_fuse_plan_info")
    return list(bn[:nb.value]), list(tb[:n_tensors]), list(to[:n_tensors])


def mcr_fuse_plan_bind(ctx, plan, tensors: Sequence[Ptr], P: int) -> None:
    """``tensors``: P*n_tensors entries, rank-major."""
    n_tensors = _plan_tensors.get(getattr(plan, "value", plan), 0)
    _check(lib().mcr_fuse_plan_bind(ctx, plan, _ptr_array(tensors, max(P, 0) * n_tensors), P), "mcr_fuse_plan_bind")


def mcr_fuse(ctx, plan, bucket: int, flat: Sequence[Ptr], P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_fuse(ctx, plan, bucket, _ptr_array(flat, P), P, variant, _stream(stream)), "mcr_fuse")


def mcr_unfuse(ctx, plan, bucket: int, flat: Sequence[Ptr], P: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_unfuse(ctx, plan, bucket, _ptr_array(flat, P), P, variant, _stream(stream)), "mcr_unfuse")


def mcr_allreduce_multi(ctx, plan, bucket: int, op: int, variant: int = AUTO, stream=None) -> None:
    _check(lib().mcr_allreduce_multi(ctx, plan, bucket, op, variant, _stream(stream)), "mcr_allreduce_multi")


def mcr_fuse_plan_destroy(plan) -> None:
    _plan_tensors.pop(getattr(plan, "value", plan), None)
    _check(lib().mcr_fuse_plan_destroy(plan), "mcr_fuse_plan_destroy")


# ---- diagnostic ----------------------------------------------------------------------------
def mcr_dispatch_overhead(ctx, out: Sequence[Ptr], inp: Sequence[Ptr], count: int, dtype: int, P: int, iters: int,
                          stream=None):
    """Microseconds per op: (through MCR_AUTO, as bare kernel launches, host cost per MCR_AUTO call,
    host cost per bare launch, CPU cost of the dispatch layer alone)."""
    a, d, ha, hd, do = (ctypes.c_double(0) for _ in range(5))
    _check(lib().mcr_dispatch_overhead(ctx, _ptr_array(out, P), _ptr_array(inp, P), _sz(count), dtype, P, iters,
                                       _stream(stream), ctypes.byref(a), ctypes.byref(d), ctypes.byref(ha),
                                       ctypes.byref(hd), ctypes.byref(do)), "mcr_dispatch_overhead")
    return a.value, d.value, ha.value, hd.value, do.value


# ---- tuning table --------------------------------------------------------------------------
def mcr_tune_set(ctx, op_id: int, dtype: int, P: int, nbytes: int, variant: int) -> None:
    _check(lib().mcr_tune_set(ctx, op_id, dtype, P, _sz(nbytes), variant), "mcr_tune_set")


def mcr_tune_get(ctx, op_id: int, dtype: int, P: int, nbytes: int) -> int:
    v = ctypes.c_int(-1)
    _check(lib().mcr_tune_get(ctx, op_id, dtype, P, _sz(nbytes), ctypes.byref(v)), "mcr_tune_get")
    return v.value


def mcr_auto_variant(ctx, op_id: int, dtype: int, P: int, nbytes: int, vec_ok: bool = True) -> int:
    v = ctypes.c_int(-1)
    _check(lib().mcr_auto_variant(ctx, op_id, dtype, P, _sz(nbytes), int(vec_ok), ctypes.byref(v)), "mcr_auto_variant")
    return v.value


def mcr_tune_clear(ctx) -> None:
    _check(lib().mcr_tune_clear(ctx), "mcr_tune_clear")


def mcr_tune_count(ctx) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().mcr_tune_count(ctx, ctypes.byref(n)), "mcr_tune_count")
    return n.value


def mcr_tune_save(ctx, path: str) -> None:
    _check(lib().mcr_tune_save(ctx, path.encode()), "mcr_tune_save")


def mcr_tune_load(ctx, path: str) -> None:
    _check(lib().mcr_tune_load(ctx, path.encode()), "mcr_tune_load")
