"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host logic (argument validation, tuning table, bucket plan) behaves as the header
says.  A host-only context (MCR_NO_DEVICE) is used, so no kernel is ever launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2303_08374_amd import inputs, mcr
from tests import golden_io as gio

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mcr.h")


@pytest.fixture(scope="module")
def ctx():
    c = mcr.mcr_init(-1)
    yield c
    mcr.mcr_finalize(c)


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mcr_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 25 and "mcr_allreduce" in names and "mcr_alltoallv" in names
    lib = mcr.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/mcr.h but not exported by libmcr.so"


def test_binding_has_the_same_names():
    for n in declared_symbols():
        assert hasattr(mcr, n), f"the Python binding lacks {n}"


def test_strerror_and_variants(ctx):
    assert mcr.strerror(0) == "ok"
    for code in range(-10, 0):
        assert mcr.strerror(code) not in ("ok", "unknown status")
    for op in range(10):
        v = mcr.mcr_get_variants(ctx, op)
        assert v[0] == "scalar" and len(v) == len(set(v)) == {mcr.OP_ALLGATHER: 17, mcr.OP_ALLREDUCE: 35, mcr.OP_REDUCE_SCATTER: 35, mcr.OP_ALLTOALL: 16}.get(op, 13)
    assert mcr.mcr_get_variants(ctx, mcr.OP_MOE_ROUTE) == ["wave_ballot"]
    with pytest.raises(mcr.McrError) as e:
        mcr.mcr_get_variants(ctx, 99)
    assert e.value.status == mcr.EOP


def _status(fn, *a, **k):
    try:
        fn(*a, **k)
    except mcr.McrError as e:
        return e.status
    return 0


A16 = [0x10000 * (i + 1) for i in range(16)]       # fake, 16-byte aligned device addresses (never dereferenced)


def test_binding_refuses_pointer_lists_shorter_than_the_library_reads(ctx):
    """The library reads P entries of every per-rank pointer array (P * n_tensors for a plan's
    tensors); the binding refuses a shorter list instead of letting it read past the end."""
    S = mcr
    with pytest.raises(ValueError):
        S.mcr_allreduce(ctx, A16[:3], 1024, S.F32, S.SUM, 4, S.AUTO, 0)
    with pytest.raises(ValueError):
        S.mcr_reduce_scatter(ctx, A16[:8], A16[:7], 1024, S.F32, S.SUM, 8, S.AUTO, 0)
    with pytest.raises(ValueError):
        S.mcr_alltoallv(ctx, A16[:2], A16[:1], None, 0, 8, 8, 4, S.F32, 2, S.AUTO, 0)
    with pytest.raises(ValueError):
        S.mcr_unpack(ctx, A16[:2], A16[:2], A16[:2], A16[:1], 8, 8, 4, S.F32, 2, S.AUTO, 0)
    plan = S.mcr_fuse_plan_create(ctx, [10, 20, 30], 100, S.F32)
    try:
        with pytest.raises(ValueError):
            S.mcr_fuse_plan_bind(ctx, plan, A16[:5], 2)               # 2 ranks x 3 tensors = 6 pointers
        assert _status(S.mcr_fuse_plan_bind, ctx, plan, A16[:6], 2) == S.ESTATE
    finally:
        S.mcr_fuse_plan_destroy(plan)


def test_static_scratch_routing_refuses_what_does_not_fit(ctx):
    """mcr_moe_route_static: a routing whose chunk counters exceed the static array is refused with
    MCR_ELIMIT before anything else happens; one that fits passes validation (and then stops at the
    host-only context)."""
    S = mcr
    assert S.mcr_moe_route_workspace_bytes(2048 * 40, 512, 16) > S.ROUTE_SCRATCH_BYTES
    assert _status(S.mcr_moe_route_static, ctx, A16, 2048 * 40, 512, 16, 8, A16, A16, A16[0], 0) == S.ELIMIT
    assert 0 < S.mcr_moe_route_workspace_bytes(40000, 64, 16) <= S.ROUTE_SCRATCH_BYTES
    assert _status(S.mcr_moe_route_static, ctx, A16, 40000, 64, 16, 8, A16, A16, A16[0], 0) == S.ESTATE
    assert _status(S.mcr_moe_route_static, ctx, A16, 40000, 64, 16, 8, A16, A16, A16[0] + 4, 0) == S.EINVAL   # splits not 8-byte aligned
    assert _status(S.mcr_moe_route_static, ctx, A16, 40000, 60, 16, 8, A16, A16, A16[0], 0) == S.EINVAL       # P does not divide E


def test_validation_errors(ctx):
    S = mcr
    # a fully valid call passes validation and then stops at the host-only context
    assert _status(S.mcr_allreduce, ctx, A16[:4], 1024, S.F32, S.SUM, 4, S.AUTO, 0) == S.ESTATE
    assert _status(S.mcr_allreduce, ctx, A16[:4], 1024, 7, S.SUM, 4, S.AUTO, 0) == S.EDTYPE
    assert _status(S.mcr_allreduce, ctx, A16[:4], 1024, S.F32, 9, 4, S.AUTO, 0) == S.EOP
    assert _status(S.mcr_allreduce, ctx, A16[:4], 1024, S.F32, S.PROD, 4, S.AUTO, 0) == S.ESTATE
    assert _status(S.mcr_allreduce, ctx, A16[:4], 1024, S.F32, S.SUM, 0, S.AUTO, 0) == S.EINVAL
    assert _status(S.mcr_allreduce, ctx, A16[:4] + A16, 1024, S.F32, S.SUM, 17, S.AUTO, 0) == S.EINVAL
    assert _status(S.mcr_allreduce, ctx, [A16[0], 0], 1024, S.F32, S.SUM, 2, S.AUTO, 0) == S.EINVAL      # null rank buffer
    assert _status(S.mcr_allreduce, ctx, [A16[0], A16[1] + 2], 8, S.F32, S.SUM, 2, S.AUTO, 0) == S.EINVAL  # not element aligned
    assert _status(S.mcr_allreduce, ctx, A16[:2], 8, S.F32, S.SUM, 2, 99, 0) == S.EVARIANT
    assert _status(S.mcr_allreduce, ctx, [A16[0], A16[1] + 4], 8, S.F32, S.SUM, 2, 3, 0) == S.EVARIANT    # vector variant, misaligned
    assert _status(S.mcr_allreduce, ctx, [A16[0], A16[1] + 4], 8, S.F32, S.SUM, 2, S.AUTO, 0) == S.ESTATE  # AUTO falls back
    # misaligned by the same amount on every rank: the 128-bit variants apply once the message reaches the boundary
    assert _status(S.mcr_allreduce, ctx, [A16[0] + 4, A16[1] + 4], 8, S.F32, S.SUM, 2, 3, 0) == S.ESTATE
    assert _status(S.mcr_allreduce, ctx, [A16[0] + 4, A16[1] + 4], 3, S.F32, S.SUM, 2, 3, 0) == S.ESTATE   # 3 elements reach it
    assert _status(S.mcr_allreduce, ctx, [A16[0] + 4, A16[1] + 4], 2, S.F32, S.SUM, 2, 3, 0) == S.EVARIANT  # 2 do not
    assert _status(S.mcr_allreduce, ctx, [A16[0] + 4, A16[1] + 8], 8, S.F32, S.SUM, 2, 3, 0) == S.EVARIANT  # different amounts
    assert _status(S.mcr_allreduce, ctx, [A16[0] + 2, A16[1] + 2], 64, S.BF16, S.AVG, 2, 6, 0) == S.ESTATE
    assert _status(S.mcr_reduce, ctx, [A16[0] + 12, A16[1] + 12], 64, S.F32, S.MAX, 1, 2, 9, 0) == S.ESTATE
    # count must divide by P
    assert _status(S.mcr_reduce_scatter, ctx, A16[:3], A16[3:6], 10, S.F32, S.SUM, 3, S.AUTO, 0) == S.EINVAL
    assert _status(S.mcr_alltoall, ctx, A16[:3], A16[3:6], 10, S.BF16, 3, S.AUTO, 0) == S.EINVAL
    assert _status(S.mcr_reduce_scatter, ctx, A16[:3], A16[3:6], 12, S.F32, S.SUM, 3, S.AUTO, 0) == S.ESTATE
    # slices of 1 element cannot use a 128-bit variant
    assert _status(S.mcr_reduce_scatter, ctx, A16[:3], A16[3:6], 3, S.F32, S.SUM, 3, 1, 0) == S.EVARIANT
    assert _status(S.mcr_allgather, ctx, A16[:2], A16[2:4], 3, S.BF16, 2, 2, 0) == S.EVARIANT
    # alltoallv: negative split, row/column sums against the declared rows, equal split divisibility
    assert _status(S.mcr_alltoallv, ctx, A16[:2], A16[2:4], [[1, -1], [0, 0]], False, 8, 8, 4, S.F32, 2, S.AUTO, 0) == S.EINVAL
    assert _status(S.mcr_alltoallv, ctx, A16[:2], A16[2:4], [[5, 4], [0, 0]], False, 8, 8, 4, S.F32, 2, S.AUTO, 0) == S.ESPLIT
    assert _status(S.mcr_alltoallv, ctx, A16[:2], A16[2:4], [[5, 0], [4, 0]], False, 8, 8, 4, S.F32, 2, S.AUTO, 0) == S.ESPLIT
    assert _status(S.mcr_alltoallv, ctx, A16[:2], A16[2:4], [[5, 3], [3, 5]], False, 8, 8, 4, S.F32, 2, S.AUTO, 0) == S.ESTATE
    assert _status(S.mcr_alltoallv, ctx, A16[:2], A16[2:4], None, False, 7, 8, 4, S.F32, 2, S.AUTO, 0) == S.EINVAL
    # the matrix read transposed: rank 0 sends column 0 (9 rows of its 8: refused), receives row 0
    T = S.SPLITS_TRANSPOSED
    assert _status(S.mcr_alltoallv, ctx, A16[:2], A16[2:4], [[5, 0], [4, 0]], T, 8, 9, 4, S.F32, 2, S.AUTO, 0) == S.ESPLIT
    assert _status(S.mcr_alltoallv, ctx, A16[:2], A16[2:4], [[5, 0], [4, 0]], T, 9, 8, 4, S.F32, 2, S.AUTO, 0) == S.ESTATE
    assert _status(S.mcr_alltoallv, ctx, A16[:2], A16[2:4], [[5, 0], [4, 0]], 0, 9, 8, 4, S.F32, 2, S.AUTO, 0) == S.ESPLIT
    assert _status(S.mcr_alltoallv, ctx, A16[:2], A16[2:4], [[1, 1], [1, 1]], 4, 8, 8, 4, S.F32, 2, S.AUTO, 0) == S.EINVAL    # unknown flag bit
    assert _status(S.mcr_alltoallv, ctx, A16[:2], A16[2:4], [[1, 1], [1, 1]], False, 8, 8, 3, S.BF16, 2, 3, 0) == S.EVARIANT
    # rooted and vector collectives
    assert _status(S.mcr_reduce, ctx, A16[:4], 64, S.F32, S.SUM, 4, 4, S.AUTO, 0) == S.EINVAL                 # root out of range
    assert _status(S.mcr_reduce, ctx, A16[:4], 64, S.F32, S.SUM, 3, 4, S.AUTO, 0) == S.ESTATE
    assert _status(S.mcr_bcast, ctx, A16[:4], 64, S.BF16, -1, 4, S.AUTO, 0) == S.EINVAL
    assert _status(S.mcr_bcast, ctx, A16[:4], 7, S.BF16, 0, 4, 1, 0) == S.EVARIANT                            # 7 bf16 is not a multiple of 16 bytes
    assert _status(S.mcr_gatherv, ctx, A16[0], A16[1:3], [8, 8], S.F32, 2, S.AUTO, 0) == S.ESTATE
    assert _status(S.mcr_gatherv, ctx, A16[0], [A16[1], 0], [8, 8], S.F32, 2, S.AUTO, 0) == S.EINVAL            # null sender with a non-zero count
    assert _status(S.mcr_gatherv, ctx, A16[0], [A16[1], 0], [8, 0], S.F32, 2, S.AUTO, 0) == S.ESTATE            # ... but fine with count 0
    assert _status(S.mcr_scatterv, ctx, A16[1:3], 0, [8, 8], S.F32, 2, S.AUTO, 0) == S.EINVAL
    assert _status(S.mcr_allgatherv, ctx, A16[:2], A16[2:4], [3, 8], S.F32, 2, 2, 0) == S.EVARIANT
    assert _status(S.mcr_allgatherv, ctx, A16[:2], A16[2:4], [0, 0], S.F32, 2, S.AUTO, 0) == 0                   # nothing to move
    assert S.mcr_moe_route_workspace_bytes(2048, 64, 16) == 0 and S.mcr_moe_route_workspace_bytes(16384, 64, 16) == 16 * 8 * 64 * 4
    assert S.mcr_moe_route_workspace_bytes(1 << 30, 512, 16) == 16 * 64 * 512 * 4                              # never more than 64 chunks
    assert _status(S.mcr_moe_route_ws, ctx, A16[:2], 8192, 4, 2, 10, A16[2:4], A16[4:6], A16[6], A16[7], 64, 0) == S.EINVAL   # workspace too small
    assert _status(S.mcr_moe_route_ws, ctx, A16[:2], 8192, 4, 2, 10, A16[2:4], A16[4:6], A16[6], A16[7], 128, 0) == S.ESTATE
    assert _status(S.mcr_moe_route_ws, ctx, A16[:2], 8192, 4, 2, 10, A16[2:4], A16[4:6], A16[6], None, 0, 0) == S.ESTATE      # no workspace: the plain call
    # displacements chosen by the caller: extents, overlaps, alignment of the vector path
    C, SD, RD = [1, 2, 2, 1], [4, 1, 3, 0], [3, 0, 2, 5]
    assert _status(S.mcr_alltoallv_displs, ctx, A16[:2], A16[2:4], C, SD, RD, 6, 6, 4, S.F32, 2, S.AUTO, 0) == S.ESTATE
    assert _status(S.mcr_alltoallv_displs, ctx, A16[:2], A16[2:4], C, SD, RD, 4, 6, 4, S.F32, 2, S.AUTO, 0) == S.ESPLIT     # 4+1 > 4 send rows
    assert _status(S.mcr_alltoallv_displs, ctx, A16[:2], A16[2:4], C, SD, RD, 6, 5, 4, S.F32, 2, S.AUTO, 0) == S.ESPLIT     # 5+1 > 5 receive rows
    assert _status(S.mcr_alltoallv_displs, ctx, A16[:2], A16[2:4], C, SD, [1, 0, 2, 5], 6, 6, 4, S.F32, 2, S.AUTO, 0) == S.EINVAL   # blocks overlap at rank 0
    assert _status(S.mcr_alltoallv_displs, ctx, A16[:2], A16[2:4], C, [4, -1, 3, 0], RD, 6, 6, 4, S.F32, 2, S.AUTO, 0) == S.EINVAL
    assert _status(S.mcr_alltoallv_displs, ctx, A16[:2], A16[2:4], C, SD, RD, 6, 6, 3, S.F32, 2, 1, 0) == S.EVARIANT         # 12-byte rows, vector variant
    assert _status(S.mcr_gatherv_displs, ctx, A16[0], 20, A16[1:3], [8, 8], [12, 0], S.F32, 2, S.AUTO, 0) == S.ESTATE
    assert _status(S.mcr_gatherv_displs, ctx, A16[0], 19, A16[1:3], [8, 8], [12, 0], S.F32, 2, S.AUTO, 0) == S.ESPLIT
    assert _status(S.mcr_gatherv_displs, ctx, A16[0], 20, A16[1:3], [8, 8], [7, 0], S.F32, 2, S.AUTO, 0) == S.EINVAL          # overlap
    assert _status(S.mcr_gatherv_displs, ctx, A16[0], 20, A16[1:3], [8, 8], [10, 0], S.F32, 2, 1, 0) == S.EVARIANT             # offset 10 floats is not 16-byte aligned
    assert _status(S.mcr_scatterv_displs, ctx, A16[1:3], A16[0], 16, [8, 8], [8, 0], S.F32, 2, S.AUTO, 0) == S.ESTATE
    assert _status(S.mcr_scatterv_displs, ctx, A16[1:3], A16[0], 16, [8, 8], [4, 0], S.F32, 2, S.AUTO, 0) == S.ESTATE          # source blocks may overlap
    assert _status(S.mcr_scatterv_displs, ctx, A16[1:3], A16[0], 15, [8, 8], [8, 0], S.F32, 2, S.AUTO, 0) == S.ESPLIT
    assert _status(S.mcr_allgatherv_displs, ctx, A16[:2], 32, A16[2:4], [8, 4], [20, 0], S.F32, 2, S.AUTO, 0) == S.ESTATE
    assert _status(S.mcr_allgatherv_displs, ctx, A16[:2], 27, A16[2:4], [8, 4], [20, 0], S.F32, 2, S.AUTO, 0) == S.ESPLIT
    assert _status(S.mcr_allgatherv_displs, ctx, A16[:2], 32, A16[2:4], [0, 0], [20, 0], S.F32, 2, S.AUTO, 0) == 0
    # MoE routing
    assert _status(S.mcr_moe_route, ctx, A16[:4], 64, 6, 4, 10, A16[4:8], A16[8:12], A16[12], 0) == S.EINVAL    # P does not divide E
    assert _status(S.mcr_moe_route, ctx, A16[:2], 64, 1024, 2, 10, A16[2:4], A16[4:6], A16[6], 0) == S.EINVAL  # too many experts
    assert _status(S.mcr_moe_route, ctx, A16[:2], -1, 4, 2, 10, A16[2:4], A16[4:6], A16[6], 0) == S.EINVAL
    assert _status(S.mcr_moe_route, ctx, A16[:2], 64, 4, 2, 10, A16[2:4], A16[4:6], A16[6], 0) == S.ESTATE
    # pack / unpack
    assert _status(S.mcr_pack, ctx, A16[:1], A16[1:2], [0], 8, 8, 4, S.F32, 1, S.AUTO, 0) == S.EINVAL           # null slot
    assert _status(S.mcr_unpack, ctx, A16[:1], A16[1:2], A16[2:3], None, 8, 8, 3, S.F32, 1, 1, 0) == S.EVARIANT
    assert _status(S.mcr_unpack, ctx, A16[:1], A16[1:2], A16[2:3], A16[3:4], 8, 8, 4, S.F32, 1, S.AUTO, 0) == S.ESTATE


def test_null_context_is_rejected():
    assert _status(mcr.mcr_allreduce, None, A16[:2], 8, mcr.F32, mcr.SUM, 2, mcr.AUTO, 0) == mcr.EINVAL
    assert _status(mcr.mcr_tune_set, None, 0, 0, 8, 4096, 1) == mcr.EINVAL


# ------------------------------------------------------------------- tuning table
def test_tuning_table_reproduces_table2(ctx, tmp_path):
    """Table II of the paper as a fixture: three 'backends' stand for three variants."""
    mcr.mcr_tune_clear(ctx)
    rows = [s.split() for s in gio.lines("table2_allgather.txt")]
    backend_to_variant = {"MVAPICH2-GDR": 1, "NCCL": 3, "SCCL": 14}
    for size, backend in reversed(rows):                       # insertion order must not matter
        mcr.mcr_tune_set(ctx, mcr.OP_ALLGATHER, mcr.F32, 8, int(size), backend_to_variant[backend])
    sizes = [int(r[0]) for r in rows]
    choice = [backend_to_variant[r[1]] for r in rows]
    for probe in [1, 255, 256, 257, 2048, 4095, 4096, 4097, 8192, 16383, 16384, 32768, 1 << 30]:
        assert mcr.mcr_tune_get(ctx, mcr.OP_ALLGATHER, mcr.F32, 8, probe) == oracle.tune_lookup(sizes, choice, probe)
    assert mcr.mcr_tune_get(ctx, mcr.OP_ALLGATHER, mcr.F32, 8, 4095) == 1
    assert mcr.mcr_tune_get(ctx, mcr.OP_ALLGATHER, mcr.F32, 8, 4096) == 3
    assert mcr.mcr_tune_get(ctx, mcr.OP_ALLGATHER, mcr.F32, 8, 100) == 1          # below the first row
    assert mcr.mcr_tune_get(ctx, mcr.OP_ALLGATHER, mcr.F32, 8, 1 << 40) == 14     # above the last row
    # other keys have no table
    assert _status(mcr.mcr_tune_get, ctx, mcr.OP_ALLGATHER, mcr.BF16, 8, 4096) == mcr.EVARIANT
    assert _status(mcr.mcr_tune_get, ctx, mcr.OP_ALLGATHER, mcr.F32, 4, 4096) == mcr.EVARIANT
    # entry count = collectives x scales x message sizes
    assert mcr.mcr_tune_count(ctx) == 1 * 1 * 8
    mcr.mcr_tune_set(ctx, mcr.OP_ALLGATHER, mcr.F32, 8, 4096, 2)                  # overwrite, no new row
    assert mcr.mcr_tune_count(ctx) == 8 and mcr.mcr_tune_get(ctx, mcr.OP_ALLGATHER, mcr.F32, 8, 5000) == 2
    for P in (2, 4):
        for size in sizes:
            mcr.mcr_tune_set(ctx, mcr.OP_ALLREDUCE, mcr.BF16, P, size, 4)
    assert mcr.mcr_tune_count(ctx) == 8 + 1 * 2 * 8
    # every element type and the last op of the enumeration have a name in the file
    mcr.mcr_tune_set(ctx, mcr.OP_REDUCE_SCATTER, mcr.F16, 8, 1 << 20, 5)
    mcr.mcr_tune_set(ctx, mcr.OP_MOE_COMBINE_BY_EXPERT, mcr.I32, 16, 1 << 26, 7)
    # save / load round trip
    path = str(tmp_path / "table.txt")
    mcr.mcr_tune_save(ctx, path)
    text = open(path).read()
    assert "reduce_scatter f16 8 1048576 v2nt" in text and "moe_combine_by_expert i32 16 67108864 v1ln" in text
    other = mcr.mcr_init(-1)
    try:
        mcr.mcr_tune_load(other, path)
        assert mcr.mcr_tune_count(other) == 26
        assert mcr.mcr_tune_get(other, mcr.OP_REDUCE_SCATTER, mcr.F16, 8, 1 << 21) == 5
        assert mcr.mcr_tune_get(other, mcr.OP_MOE_COMBINE_BY_EXPERT, mcr.I32, 16, 1 << 27) == 7
        mcr.mcr_tune_clear(ctx)
        mcr.mcr_tune_load(ctx, path)
        assert mcr.mcr_tune_count(ctx) == 26
        for probe in [1, 300, 4096, 9000, 1 << 20]:
            assert mcr.mcr_tune_get(other, mcr.OP_ALLGATHER, mcr.F32, 8, probe) == mcr.mcr_tune_get(ctx, mcr.OP_ALLGATHER, mcr.F32, 8, probe)
            assert mcr.mcr_tune_get(other, mcr.OP_ALLREDUCE, mcr.BF16, 4, probe) == 4
    finally:
        mcr.mcr_finalize(other)
    # a malformed file changes nothing
    bad = tmp_path / "bad.txt"
    bad.write_text("allgather f32 8 4096 v4\nallgather f32 8 oops v4\n")
    assert _status(mcr.mcr_tune_load, ctx, str(bad)) == mcr.EIO
    assert mcr.mcr_tune_count(ctx) == 26
    assert _status(mcr.mcr_tune_load, ctx, str(tmp_path / "missing.txt")) == mcr.EIO
    assert _status(mcr.mcr_tune_set, ctx, 0, 0, 8, 4096, 99) == mcr.EVARIANT
    assert _status(mcr.mcr_tune_set, ctx, 99, 0, 8, 4096, 1) == mcr.EOP
    mcr.mcr_tune_clear(ctx)
    assert mcr.mcr_tune_count(ctx) == 0


def test_auto_falls_back_to_the_nearest_scale(ctx):
    """A table exists for P=8 only: mcr_tune_get reports nothing for other rank counts, MCR_AUTO borrows
    the closest scale's table, and with no table at all takes the built-in default."""
    mcr.mcr_tune_clear(ctx)
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.F32, 4, 64 << 20) == 3            # default: v4 above 1 MiB
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.F32, 4, 4096) == 1                # default: v1 below
    mcr.mcr_tune_set(ctx, mcr.OP_ALLTOALL, mcr.F32, 8, 4096, 2)
    mcr.mcr_tune_set(ctx, mcr.OP_ALLTOALL, mcr.F32, 8, 1 << 20, 4)
    mcr.mcr_tune_set(ctx, mcr.OP_ALLTOALL, mcr.F32, 2, 4096, 7)
    assert _status(mcr.mcr_tune_get, ctx, mcr.OP_ALLTOALL, mcr.F32, 4, 4096) == mcr.EVARIANT
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.F32, 8, 64 << 20) == 4
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.F32, 16, 64 << 20) == 4           # nearest scale is 8
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.F32, 6, 8192) == 2                # 6 is closer to 8 than to 2
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.F32, 3, 8192) == 7                # 3 is closer to 2
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.BF16, 8, 8192) == 1               # other dtype: no table, default
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.F32, 8, 8192, False) == 0         # shape rules the vectors out
    # an element type without a table borrows the tuned type of the same size
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.I32, 8, 64 << 20) == 4             # int32 from fp32
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.F16, 8, 8192) == 1                # fp16 from bf16, which has none: default
    mcr.mcr_tune_set(ctx, mcr.OP_ALLTOALL, mcr.BF16, 8, 4096, 9)
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.F16, 4, 8192) == 9                # ... now it has, at the nearest scale
    mcr.mcr_tune_set(ctx, mcr.OP_ALLTOALL, mcr.F16, 8, 4096, 5)
    assert mcr.mcr_auto_variant(ctx, mcr.OP_ALLTOALL, mcr.F16, 8, 8192) == 5                # its own table wins
    mcr.mcr_tune_clear(ctx)


def test_shipped_tuning_table_is_well_formed(ctx):
    """The table measured on MI355X that ships with the package loads, and holds a row for
    every (op, dtype, size) cell of the sweep at P=8."""
    path = os.path.join(ROOT, "paper_2303_08374_amd", "tuning", "mi355x.tbl")
    if not os.path.exists(path):
        pytest.skip("no shipped table yet")
    mcr.mcr_tune_clear(ctx)
    mcr.mcr_tune_load(ctx, path)
    n_ops, n_dtypes, n_sizes = len(inputs.SWEEP_OPS), len(inputs.SWEEP_DTYPES), len(inputs.SWEEP_BYTES)
    assert mcr.mcr_tune_count(ctx) >= n_ops * n_dtypes * n_sizes
    for op in range(4):
        for dt in (mcr.F32, mcr.BF16):
            for b in inputs.SWEEP_BYTES:
                assert 0 <= mcr.mcr_tune_get(ctx, op, dt, inputs.SWEEP_P, b) < len(mcr.mcr_get_variants(ctx, op))
    mcr.mcr_tune_clear(ctx)


# ---------------------------------------------------------------------- bucket plan
def test_fuse_plan_matches_oracle_and_fixture(ctx):
    g = gio.keyed_ints("fuse_plan_case.txt")
    plan = mcr.mcr_fuse_plan_create(ctx, g["numel"], g["B"][0], mcr.BF16)
    bn, tb, to = mcr.mcr_fuse_plan_info(plan, len(g["numel"]))
    mcr.mcr_fuse_plan_destroy(plan)
    assert bn == g["bucket_numel"] and tb == g["tensor_bucket"] and to == g["tensor_offset"]
    w = inputs.GradBucketWorkload()
    rng = np.random.Generator(np.random.Philox(key=3))
    cases = [(w.numel(), w.bucket_elems), (w.numel()[::-1], w.bucket_elems), ([], 10), ([5], 5), ([6], 5),
             ([0, 0, 3, 0], 2)]
    cases += [(rng.integers(1, 50, size=40).tolist(), int(B)) for B in (1, 7, 49, 50, 1000)]
    for numel, B in cases:
        plan = mcr.mcr_fuse_plan_create(ctx, numel, B, mcr.F32)
        bn, tb, to = mcr.mcr_fuse_plan_info(plan, len(numel))
        otb, oto, obn = oracle.fuse_plan(numel, B)
        assert bn == obn.tolist() and tb == otb.tolist() and to == oto.tolist(), (numel[:8], B)
        # a host-only context cannot bind or launch
        assert _status(mcr.mcr_fuse_plan_bind, ctx, plan, [A16[0]] * max(len(numel), 1), 1) in (mcr.ESTATE, mcr.EINVAL)
        assert _status(mcr.mcr_allreduce_multi, ctx, plan, -1, mcr.SUM, mcr.AUTO, 0) == mcr.ESTATE
        mcr.mcr_fuse_plan_destroy(plan)
    assert _status(mcr.mcr_fuse_plan_create, ctx, [1, 2], 0, mcr.F32) == mcr.EINVAL
    assert _status(mcr.mcr_fuse_plan_create, ctx, [1, 2], 4, 5) == mcr.EDTYPE
