// C ABI: argument validation, variant selection (explicit or from the static
// tuning table, the paper's "auto" backend of Sec. IV-A / IV-E), fusion plans,
// and the tuning table itself.  No kernel lives here.
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <type_traits>

#include "mcr_internal.hpp"

namespace mcr {

const char* const kStreamVariantNames[AG_COUNT] = {"scalar", "v1", "v2", "v4", "v1nt", "v2nt", "v4nt", "v1ln", "v2ln", "v4ln",
                                                   "v1sn", "v2sn", "v4sn", "sc4", "sc8", "sc16", "sc16x"};

const char* const kReduceVariantNames[RV_XUNIT0 - SV_COUNT] = {"pk8", "w64"};
const char* const kAlltoallVariantNames[A2A_COUNT - SV_COUNT] = {"flat", "w64", "lds"};

namespace {

const char* const kOpNames[MCR_OP_COUNT] = {"allreduce", "reduce_scatter", "allgather", "alltoall",
                                            "alltoallv", "pack", "unpack", "fuse",
                                            "unfuse", "allreduce_multi", "moe_route", "moe_dispatch",
                                            "moe_combine", "dlrm_shuffle", "moe_dispatch_by_expert",
                                            "moe_combine_by_expert"};
const char* const kDtypeNames[4] = {"f32", "bf16", "f16", "i32"};
const char* const kRouteVariantNames[1] = {"wave_ballot"};

bool valid_dtype(int d) { return d >= MCR_F32 && d <= MCR_I32; }
bool valid_redop(int o) { return o >= MCR_SUM && o <= MCR_PROD; }
// integers have no average
bool redop_fits(int o, int dtype) { return !(dtype == MCR_I32 && o == MCR_AVG); }
bool valid_P(int P) { return P >= 1 && P <= MCR_MAX_RANKS; }
bool is_reduction(int op) { return op == MCR_OP_ALLREDUCE || op == MCR_OP_REDUCE_SCATTER; }
int n_variants(int op) {
  return op == MCR_OP_MOE_ROUTE ? 1 : op == MCR_OP_ALLGATHER ? AG_COUNT : is_reduction(op) ? RV_COUNT
         : op == MCR_OP_ALLTOALL ? A2A_COUNT : SV_COUNT;
}
// Name of variant `i` of `op`: the ids from SV_COUNT on belong to one op each (super-chunk forms of
// all_gather, persistent forms of the reductions).
const char* variant_name(int op, int i) {
  if (op == MCR_OP_MOE_ROUTE) return kRouteVariantNames[i];
  if (is_reduction(op) && i >= RV_XUNIT0) return kReduceUnitVariants[i - RV_XUNIT0].name;
  if (is_reduction(op) && i >= SV_COUNT) return kReduceVariantNames[i - SV_COUNT];
  if (op == MCR_OP_ALLTOALL && i >= SV_COUNT) return kAlltoallVariantNames[i - SV_COUNT];
  return kStreamVariantNames[i];
}

bool elem_aligned(const void* p, int dtype) {
  return (reinterpret_cast<uintptr_t>(p) & (elem_bytes(dtype) - 1)) == 0;
}

// Copies a host array of P device pointers into a kernel-argument table.
// Returns false on a null entry (when `need`), or one not aligned to the element.
template <class Tab, class Ptr>
bool fill_tab(Tab& tab, Ptr const* arr, int P, int dtype_for_align, bool need, bool* all16) {
  for (int i = 0; i < MCR_MAX_RANKS; ++i) tab.p[i] = nullptr;
  if (!arr) return false;
  for (int p = 0; p < P; ++p) {
    if (need && arr[p] == nullptr) return false;
    if (dtype_for_align >= 0 && !elem_aligned(arr[p], dtype_for_align)) return false;
    if (all16 && !aligned16(arr[p])) *all16 = false;
    typedef typename std::remove_reference<decltype(tab.p[0])>::type Slot;
    tab.p[p] = (Slot)arr[p];
  }
  return true;
}

// Table lookup: floor-to-row rule.  Returns -1 when there is no table for the key.  With
// nearest_scale, a missing table for this rank count is replaced by the one for the closest rank
// count of the same op and dtype (the paper notes that trends carry over between similar scales);
// MCR_AUTO uses that, mcr_tune_get reports the table as it is.
int table_lookup(mcr_ctx* ctx, int op, int dtype, int P, size_t bytes, bool nearest_scale) {
  std::lock_guard<std::mutex> lock(ctx->mu);
  auto it = ctx->tables.find(TuneKey{op, dtype, P});
  if ((it == ctx->tables.end() || it->second.empty()) && nearest_scale) {
    int best_gap = 1 << 30;
    for (auto jt = ctx->tables.begin(); jt != ctx->tables.end(); ++jt) {
      if (jt->first.op != op || jt->first.dtype != dtype || jt->second.empty()) continue;
      const int gap = jt->first.P > P ? jt->first.P - P : P - jt->first.P;
      if (gap < best_gap) { best_gap = gap; it = jt; }
    }
  }
  if (it == ctx->tables.end() || it->second.empty()) return -1;
  const auto& rows = it->second;
  int pick = rows.front().second;
  for (const auto& row : rows) {
    if (row.first <= bytes) pick = row.second; else break;
  }
  return pick;
}

// Built-in choice when the table has nothing: a plain 16-byte-per-thread launch for
// small messages (least latency), four vectors per thread for large ones.
int default_variant(size_t bytes) { return bytes >= (size_t(1) << 20) ? SV_V4 : SV_V1; }

// Resolves `variant` for a streaming op.  vec_ok: the shape and alignment allow
// the 128-bit variants.
int resolve_variant(mcr_ctx* ctx, int op, int dtype, int P, size_t bytes, bool vec_ok, int variant, int* out) {
  if (variant == MCR_AUTO) {
    if (!vec_ok) { *out = SV_SCALAR; return MCR_OK; }
    int v = table_lookup(ctx, op, dtype, P, bytes, true);
    // an element type with no table of its own borrows the one of the tuned type of the same size
    // (the traffic is the same): fp16 from bf16, int32 from fp32
    if (v < 0 && dtype == MCR_F16) v = table_lookup(ctx, op, MCR_BF16, P, bytes, true);
    if (v < 0 && dtype == MCR_I32) v = table_lookup(ctx, op, MCR_F32, P, bytes, true);
    if (v < 0 || v >= n_variants(op)) v = default_variant(bytes);
    *out = v;
    return MCR_OK;
  }
  if (variant < 0 || variant >= n_variants(op)) return MCR_EVARIANT;
  if (variant != SV_SCALAR && !vec_ok) return MCR_EVARIANT;
  *out = variant;
  return MCR_OK;
}

// Makes the context's device current for the rest of the calling scope and puts the caller's
// device back when the scope ends, so a call never changes the calling thread's current device.
// A host-only context (device < 0) validates, plans and tunes but never launches: MCR_ESTATE.
class DeviceScope {
 public:
  explicit DeviceScope(const mcr_ctx* ctx) {
    if (ctx->device < 0) { status_ = MCR_ESTATE; return; }
    if (hipGetDevice(&previous_) != hipSuccess) { status_ = MCR_EHIP; return; }
    if (previous_ != ctx->device) {
      if (hipSetDevice(ctx->device) != hipSuccess) { status_ = MCR_EHIP; return; }
      restore_ = true;
    }
  }
  ~DeviceScope() {
    if (restore_) (void)hipSetDevice(previous_);
  }
  DeviceScope(const DeviceScope&) = delete;
  DeviceScope& operator=(const DeviceScope&) = delete;
  int status() const { return status_; }

 private:
  int previous_ = 0;
  int status_ = MCR_OK;
  bool restore_ = false;
};

// Everything mcr_alltoall does before it launches: argument checks, the rank pointer tables,
// the launch-shape choice.
int prepare_alltoall(mcr_ctx* ctx, void* const* out, const void* const* in, size_t count, mcr_dtype dtype, int P,
                     int variant, PtrTab* to, CPtrTab* ti, int* v) {
  if (!ctx || !out || !in || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (count % static_cast<size_t>(P) != 0) return MCR_EINVAL;
  bool all16 = true;
  if (!fill_tab(*to, out, P, dtype, count > 0, &all16) || !fill_tab(*ti, in, P, dtype, count > 0, &all16)) return MCR_EINVAL;
  const bool vec_ok = all16 && ((count / P) % per_vec(dtype) == 0);
  return resolve_variant(ctx, MCR_OP_ALLTOALL, dtype, P, count * elem_bytes(dtype), vec_ok, variant, v);
}

// Common tail of the vector collectives: counts[i] elements per block; the split matrix is built by
// `fill(S, rows)` from counts expressed in rows of `row_elems` elements (one 128-bit vector when
// every count and pointer allows it, else one element).
template <class Fill>
int vector_collective(mcr_ctx* ctx, const PtrTab& to, const CPtrTab& ti, bool all16, const size_t* counts, int n_counts,
                      mcr_dtype dtype, int P, int same_src, int variant, void* stream, Fill fill) {
  const size_t W = per_vec(dtype);
  bool vec_ok = all16;
  size_t total = 0, biggest = 0;
  for (int i = 0; i < n_counts; ++i) {
    if (counts[i] % W != 0) vec_ok = false;
    total += counts[i];
    if (counts[i] > biggest) biggest = counts[i];
  }
  int v;
  int rc = resolve_variant(ctx, MCR_OP_ALLTOALLV, dtype, P, biggest * elem_bytes(dtype), vec_ok, variant, &v);
  if (rc != MCR_OK) return rc;
  if (total == 0) return MCR_OK;
  const size_t row_elems = (v == SV_SCALAR) ? 1 : W;
  int64_t S[MCR_MAX_RANKS * MCR_MAX_RANKS];
  for (int i = 0; i < P * P; ++i) S[i] = 0;
  fill(S, row_elems);
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  // every buffer is bounded by the whole payload: the split matrix is ours, so the bounds never bind
  const size_t rows = total / row_elems;
  return launch_alltoallv(ctx, to, ti, S, nullptr, rows, rows, row_elems * elem_bytes(dtype),
                          static_cast<int>(elem_bytes(dtype)), P, same_src, false, v, static_cast<hipStream_t>(stream));
}

// Pairs with caller-chosen offsets, in elements: pair i = p*P + r copies cnt[i] elements from
// offset sd[i] of in[p] to offset rd[i] of out[r].  src_elems[p] / dst_elems[r] are the extents the
// caller vouches for; a pair outside them, or two pairs that overlap in one destination, is an
// error (the result would depend on the order of the copies).
int pair_collective(mcr_ctx* ctx, const PtrTab& to, const CPtrTab& ti, bool all16, const uint64_t* cnt, const uint64_t* sd,
                    const uint64_t* rd, const uint64_t* src_elems, const uint64_t* dst_elems, mcr_dtype dtype, int P,
                    int variant, void* stream) {
  const uint64_t W = per_vec(dtype);
  bool vec_ok = all16;
  uint64_t total = 0, biggest = 0;
  for (int p = 0; p < P; ++p) {
    for (int r = 0; r < P; ++r) {
      const int i = p * P + r;
      if (cnt[i] == 0) continue;
      if (sd[i] > src_elems[p] || cnt[i] > src_elems[p] - sd[i]) return MCR_ESPLIT;
      if (rd[i] > dst_elems[r] || cnt[i] > dst_elems[r] - rd[i]) return MCR_ESPLIT;
      if (!to.p[r] || !ti.p[p]) return MCR_EINVAL;
      if (cnt[i] % W || sd[i] % W || rd[i] % W) vec_ok = false;
      total += cnt[i];
      if (cnt[i] > biggest) biggest = cnt[i];
      for (int q = 0; q < p; ++q) {                                   // overlap with an earlier sender's block at r
        const int k = q * P + r;
        if (cnt[k] && rd[i] < rd[k] + cnt[k] && rd[k] < rd[i] + cnt[i]) return MCR_EINVAL;
      }
    }
  }
  int v;
  int rc = resolve_variant(ctx, MCR_OP_ALLTOALLV, dtype, P, biggest * elem_bytes(dtype), vec_ok, variant, &v);
  if (rc != MCR_OK) return rc;
  if (total == 0) return MCR_OK;
  const uint64_t unit = (v == SV_SCALAR) ? 1 : W;
  uint32_t c32[MCR_MAX_RANKS * MCR_MAX_RANKS], s32[MCR_MAX_RANKS * MCR_MAX_RANKS], r32[MCR_MAX_RANKS * MCR_MAX_RANKS];
  for (int i = 0; i < P * P; ++i) {
    const uint64_t c = cnt[i] / unit, s = cnt[i] ? sd[i] / unit : 0, d = cnt[i] ? rd[i] / unit : 0;
    if (c > 0xffffffffull || s > 0xffffffffull || d > 0xffffffffull) return MCR_EINVAL;
    c32[i] = static_cast<uint32_t>(c);
    s32[i] = static_cast<uint32_t>(s);
    r32[i] = static_cast<uint32_t>(d);
  }
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_alltoallv_pairs(ctx, to, ti, c32, s32, r32, static_cast<int>(elem_bytes(dtype)), P, v,
                                static_cast<hipStream_t>(stream));
}

// Buffers that all miss 16-byte alignment by the same amount (the same view of a tensor on every
// rank): the number of elements in front of the next 16-byte boundary, and the table advanced to
// that boundary.  0 and an untouched table when the buffers are aligned, differ from each other,
// or the message ends before the boundary.
unsigned peel_common_head(PtrTab& tab, int P, int dtype, size_t count) {
  const uintptr_t miss = reinterpret_cast<uintptr_t>(tab.p[0]) & 15u;
  if (miss == 0) return 0;
  for (int p = 1; p < P; ++p)
    if ((reinterpret_cast<uintptr_t>(tab.p[p]) & 15u) != miss) return 0;
  const size_t skip = 16 - miss;                               // a whole number of elements: every pointer is element-aligned
  const size_t head = skip / elem_bytes(dtype);
  if (head > count) return 0;
  for (int p = 0; p < P; ++p) tab.p[p] = static_cast<char*>(tab.p[p]) + skip;
  return static_cast<unsigned>(head);
}

// all_reduce and reduce: variant and head for the buffers in `tab` (advanced past the head when
// the 128-bit path is taken on misaligned buffers).
int plan_allreduce(mcr_ctx* ctx, PtrTab& tab, bool all16, size_t count, mcr_dtype dtype, int P, int variant, int* v,
                   unsigned* head) {
  *head = 0;
  PtrTab advanced = tab;
  unsigned h = 0;
  if (!all16 && count > 0) h = peel_common_head(advanced, P, dtype, count);
  const int rc = resolve_variant(ctx, MCR_OP_ALLREDUCE, dtype, P, count * elem_bytes(dtype), all16 || h > 0, variant, v);
  if (rc != MCR_OK) return rc;
  if (*v != SV_SCALAR && h > 0) {
    tab = advanced;
    *head = h;
  }
  return MCR_OK;
}

}  // namespace
}  // namespace mcr

using namespace mcr;

extern "C" {

const char* mcr_strerror(int status) {
  switch (status) {
    case MCR_OK: return "ok";
    case MCR_EINVAL: return "invalid argument";
    case MCR_EDTYPE: return "unknown dtype";
    case MCR_EOP: return "unknown op";
    case MCR_EVARIANT: return "unknown or inapplicable variant";
    case MCR_ESPLIT: return "split matrix exceeds the declared buffer rows";
    case MCR_EHIP: return "HIP runtime error";
    case MCR_ENOMEM: return "out of host memory";
    case MCR_EIO: return "tuning table file error";
    case MCR_ESTATE: return "call not valid in this state";
    case MCR_ELIMIT: return "problem exceeds the static scratch array";
  }
  return "unknown status";
}

int mcr_init(mcr_ctx** out, int device) {
  if (!out || device < MCR_NO_DEVICE) return MCR_EINVAL;
  mcr_ctx* ctx = new (std::nothrow) mcr_ctx;
  if (!ctx) return MCR_ENOMEM;
  ctx->device = device;
  if (device != MCR_NO_DEVICE) {
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess) { delete ctx; return MCR_EHIP; }
    if (device >= count) { delete ctx; return MCR_EINVAL; }
    DeviceScope on_device(ctx);                          // the caller's current device is put back on return
    int rc = on_device.status();
    // the static scratch array of mcr_moe_route_static: its address on this device, looked up
    // here so that the entry point itself does nothing but launch
    int32_t* unused = nullptr;
    if (rc == MCR_OK) rc = route_scratch_address(device, &unused);
    if (rc == MCR_OK && hipMalloc(reinterpret_cast<void**>(&ctx->pair_ring), kPairRingSlots * sizeof(PairSlot)) != hipSuccess) {
      ctx->pair_ring = nullptr;
      rc = MCR_EHIP;
    }
    if (rc != MCR_OK) { delete ctx; return rc; }
    int n_cu = 0;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && n_cu > 0) ctx->n_cu = n_cu;
  }
  const char* path = std::getenv("MCR_TUNING_TABLE");
  if (path && *path) (void)mcr_tune_load(ctx, path);   // an unreadable file leaves the table empty
  *out = ctx;
  return MCR_OK;
}

int mcr_finalize(mcr_ctx* ctx) {
  if (!ctx) return MCR_EINVAL;
  if (ctx->pair_ring) {
    DeviceScope on_device(ctx);
    (void)hipFree(ctx->pair_ring);
  }
  delete ctx;
  return MCR_OK;
}

int mcr_synchronize(mcr_ctx* ctx, void* stream) {
  if (!ctx) return MCR_EINVAL;
  return hip_status(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
}

int mcr_get_variants(mcr_ctx* ctx, int op_id, const char** names, int* n) {
  if (!ctx || !n) return MCR_EINVAL;
  if (op_id < 0 || op_id >= MCR_OP_COUNT) return MCR_EOP;
  const int have = n_variants(op_id);
  const int cap = *n;
  if (names) {
    for (int i = 0; i < have && i < cap; ++i)
      names[i] = variant_name(op_id, i);
  }
  *n = have;
  return MCR_OK;
}

// ---- collectives ----------------------------------------------------------------
int mcr_allreduce(mcr_ctx* ctx, void* const* bufs, size_t count, mcr_dtype dtype, mcr_redop op, int P,
                  int variant, void* stream) {
  if (!ctx || !bufs || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (!valid_redop(op) || !redop_fits(op, dtype)) return MCR_EOP;
  PtrTab tab;
  bool all16 = true;
  if (!fill_tab(tab, bufs, P, dtype, count > 0, &all16)) return MCR_EINVAL;
  int v;
  unsigned head;
  int rc = plan_allreduce(ctx, tab, all16, count, dtype, P, variant, &v, &head);
  if (rc != MCR_OK) return rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_allreduce(ctx, tab, count, head, dtype, op, P, -1, v, static_cast<hipStream_t>(stream));
}

int mcr_reduce_scatter(mcr_ctx* ctx, void* const* out, const void* const* in, size_t count, mcr_dtype dtype,
                       mcr_redop op, int P, int variant, void* stream) {
  if (!ctx || !out || !in || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (!valid_redop(op) || !redop_fits(op, dtype)) return MCR_EOP;
  if (count % static_cast<size_t>(P) != 0) return MCR_EINVAL;
  PtrTab to;
  CPtrTab ti;
  bool all16 = true;
  if (!fill_tab(to, out, P, dtype, count > 0, &all16) || !fill_tab(ti, in, P, dtype, count > 0, &all16)) return MCR_EINVAL;
  const bool vec_ok = all16 && ((count / P) % per_vec(dtype) == 0);
  int v;
  int rc = resolve_variant(ctx, MCR_OP_REDUCE_SCATTER, dtype, P, count * elem_bytes(dtype), vec_ok, variant, &v);
  if (rc != MCR_OK) return rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_reduce_scatter(ctx, to, ti, count, dtype, op, P, v, static_cast<hipStream_t>(stream));
}

int mcr_allgather(mcr_ctx* ctx, void* const* out, const void* const* in, size_t count, mcr_dtype dtype, int P,
                  int variant, void* stream) {
  if (!ctx || !out || !in || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  PtrTab to;
  CPtrTab ti;
  bool all16 = true;
  if (!fill_tab(to, out, P, dtype, count > 0, &all16) || !fill_tab(ti, in, P, dtype, count > 0, &all16)) return MCR_EINVAL;
  const bool vec_ok = all16 && (count % per_vec(dtype) == 0);
  int v;
  int rc = resolve_variant(ctx, MCR_OP_ALLGATHER, dtype, P, count * elem_bytes(dtype), vec_ok, variant, &v);
  if (rc != MCR_OK) return rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_allgather(ctx, to, ti, count, dtype, P, v, static_cast<hipStream_t>(stream));
}

int mcr_alltoall(mcr_ctx* ctx, void* const* out, const void* const* in, size_t count, mcr_dtype dtype, int P,
                 int variant, void* stream) {
  PtrTab to;
  CPtrTab ti;
  int v;
  int rc = prepare_alltoall(ctx, out, in, count, dtype, P, variant, &to, &ti, &v);
  if (rc != MCR_OK) return rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_alltoall(ctx, to, ti, count, dtype, P, v, static_cast<hipStream_t>(stream));
}

int mcr_alltoallv(mcr_ctx* ctx, void* const* out, const void* const* in, const int64_t* splits,
                  int splits_flags, size_t in_rows, size_t out_rows, size_t row_elems, mcr_dtype dtype, int P,
                  int variant, void* stream) {
  if (!ctx || !out || !in || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (splits_flags & ~(MCR_SPLITS_ON_DEVICE | MCR_SPLITS_TRANSPOSED)) return MCR_EINVAL;
  const bool transposed = splits && (splits_flags & MCR_SPLITS_TRANSPOSED);
  const size_t row_bytes = row_elems * elem_bytes(dtype);
  int64_t local[MCR_MAX_RANKS * MCR_MAX_RANKS];                       // equal split, or a host matrix transposed
  const int64_t* host = nullptr;
  const int64_t* dev = nullptr;
  if (!splits) {
    if (in_rows % static_cast<size_t>(P) != 0 || out_rows < in_rows) return MCR_EINVAL;
    for (int i = 0; i < P * P; ++i) local[i] = static_cast<int64_t>(in_rows / P);
    host = local;
  } else if (splits_flags & MCR_SPLITS_ON_DEVICE) {
    dev = splits;
  } else {
    host = splits;
    if (transposed) {
      for (int p = 0; p < P; ++p)
        for (int r = 0; r < P; ++r) local[p * P + r] = splits[r * P + p];
      host = local;
    }
    for (int i = 0; i < P * P; ++i)
      if (host[i] < 0) return MCR_EINVAL;
    for (int p = 0; p < P; ++p) {
      uint64_t rs = 0, cs = 0;
      for (int q = 0; q < P; ++q) {
        rs += static_cast<uint64_t>(host[p * P + q]);
        cs += static_cast<uint64_t>(host[q * P + p]);
      }
      if (rs > in_rows || cs > out_rows) return MCR_ESPLIT;
    }
  }
  const bool any = in_rows > 0 && out_rows > 0 && row_elems > 0;
  PtrTab to;
  CPtrTab ti;
  bool all16 = true;
  if (!fill_tab(to, out, P, dtype, any, &all16) || !fill_tab(ti, in, P, dtype, any, &all16)) return MCR_EINVAL;
  if (!any) return MCR_OK;
  const bool vec_ok = all16 && (row_bytes % 16 == 0);
  int v;
  int rc = resolve_variant(ctx, MCR_OP_ALLTOALLV, dtype, P, in_rows * row_bytes, vec_ok, variant, &v);
  if (rc != MCR_OK) return rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_alltoallv(ctx, to, ti, host, dev, in_rows, out_rows, row_bytes, static_cast<int>(elem_bytes(dtype)), P,
                          0, dev && transposed, v, static_cast<hipStream_t>(stream));
}

// ---- rooted and vector collectives (API listing: reduce, bcast, gather(v), scatter(v),
// all_gatherv).  reduce is the all_reduce kernel storing to the root only; the others are
// all_to_allv with a split matrix that has one column (gather), one row (scatter) or constant
// rows and a common source block (all_gatherv, bcast). ---------------------------------------
int mcr_reduce(mcr_ctx* ctx, void* const* bufs, size_t count, mcr_dtype dtype, mcr_redop op, int root, int P,
               int variant, void* stream) {
  if (!ctx || !bufs || !valid_P(P) || root < 0 || root >= P) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (!valid_redop(op) || !redop_fits(op, dtype)) return MCR_EOP;
  PtrTab tab;
  bool all16 = true;
  if (!fill_tab(tab, bufs, P, dtype, count > 0, &all16)) return MCR_EINVAL;
  int v;
  unsigned head;
  int rc = plan_allreduce(ctx, tab, all16, count, dtype, P, variant, &v, &head);
  if (rc != MCR_OK) return rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_allreduce(ctx, tab, count, head, dtype, op, P, root, v, static_cast<hipStream_t>(stream));
}

int mcr_bcast(mcr_ctx* ctx, void* const* bufs, size_t count, mcr_dtype dtype, int root, int P, int variant,
              void* stream) {
  if (!ctx || !bufs || !valid_P(P) || root < 0 || root >= P) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  PtrTab to;
  CPtrTab ti;
  bool all16 = true;
  if (!fill_tab(to, bufs, P, dtype, count > 0, &all16) || !fill_tab(ti, bufs, P, dtype, count > 0, nullptr)) return MCR_EINVAL;
  const size_t counts[1] = {count};
  return vector_collective(ctx, to, ti, all16, counts, 1, dtype, P, 1, variant, stream, [&](int64_t* S, size_t re) {
    for (int r = 0; r < P; ++r)
      if (r != root) S[root * P + r] = static_cast<int64_t>(count / re);
  });
}

int mcr_gatherv(mcr_ctx* ctx, void* out, const void* const* in, const size_t* counts, mcr_dtype dtype, int P,
                int variant, void* stream) {
  if (!ctx || !in || !counts || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  size_t total = 0;
  for (int p = 0; p < P; ++p) total += counts[p];
  if (total > 0 && (!out || !elem_aligned(out, dtype))) return MCR_EINVAL;
  PtrTab to;
  CPtrTab ti;
  bool all16 = aligned16(out);
  for (int i = 0; i < MCR_MAX_RANKS; ++i) { to.p[i] = nullptr; ti.p[i] = nullptr; }
  to.p[0] = out;                                        // the root is "receiver 0" of the split matrix
  for (int p = 0; p < P; ++p) {
    if (counts[p] > 0 && (!in[p] || !elem_aligned(in[p], dtype))) return MCR_EINVAL;
    if (counts[p] > 0 && !aligned16(in[p])) all16 = false;
    ti.p[p] = in[p];
  }
  return vector_collective(ctx, to, ti, all16, counts, P, dtype, P, 0, variant, stream, [&](int64_t* S, size_t re) {
    for (int p = 0; p < P; ++p) S[p * P + 0] = static_cast<int64_t>(counts[p] / re);
  });
}

int mcr_gather(mcr_ctx* ctx, void* out, const void* const* in, size_t count, mcr_dtype dtype, int P, int variant,
               void* stream) {
  if (!valid_P(P)) return MCR_EINVAL;
  size_t counts[MCR_MAX_RANKS];
  for (int p = 0; p < P; ++p) counts[p] = count;
  return mcr_gatherv(ctx, out, in, counts, dtype, P, variant, stream);
}

int mcr_scatterv(mcr_ctx* ctx, void* const* out, const void* in, const size_t* counts, mcr_dtype dtype, int P,
                 int variant, void* stream) {
  if (!ctx || !out || !counts || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  size_t total = 0;
  for (int p = 0; p < P; ++p) total += counts[p];
  if (total > 0 && (!in || !elem_aligned(in, dtype))) return MCR_EINVAL;
  PtrTab to;
  CPtrTab ti;
  bool all16 = aligned16(in);
  for (int i = 0; i < MCR_MAX_RANKS; ++i) { to.p[i] = nullptr; ti.p[i] = nullptr; }
  ti.p[0] = in;                                         // the root is "sender 0" of the split matrix
  for (int r = 0; r < P; ++r) {
    if (counts[r] > 0 && (!out[r] || !elem_aligned(out[r], dtype))) return MCR_EINVAL;
    if (counts[r] > 0 && !aligned16(out[r])) all16 = false;
    to.p[r] = out[r];
  }
  return vector_collective(ctx, to, ti, all16, counts, P, dtype, P, 0, variant, stream, [&](int64_t* S, size_t re) {
    for (int r = 0; r < P; ++r) S[0 * P + r] = static_cast<int64_t>(counts[r] / re);
  });
}

int mcr_scatter(mcr_ctx* ctx, void* const* out, const void* in, size_t count, mcr_dtype dtype, int P, int variant,
                void* stream) {
  if (!valid_P(P)) return MCR_EINVAL;
  size_t counts[MCR_MAX_RANKS];
  for (int p = 0; p < P; ++p) counts[p] = count;
  return mcr_scatterv(ctx, out, in, counts, dtype, P, variant, stream);
}

int mcr_allgatherv(mcr_ctx* ctx, void* const* out, const void* const* in, const size_t* counts, mcr_dtype dtype,
                   int P, int variant, void* stream) {
  if (!ctx || !out || !in || !counts || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  size_t total = 0;
  for (int p = 0; p < P; ++p) total += counts[p];
  PtrTab to;
  CPtrTab ti;
  bool all16 = true;
  if (!fill_tab(to, out, P, dtype, total > 0, &all16)) return MCR_EINVAL;
  for (int i = 0; i < MCR_MAX_RANKS; ++i) ti.p[i] = nullptr;
  for (int p = 0; p < P; ++p) {
    if (counts[p] > 0 && (!in[p] || !elem_aligned(in[p], dtype))) return MCR_EINVAL;
    if (counts[p] > 0 && !aligned16(in[p])) all16 = false;
    ti.p[p] = in[p];
  }
  return vector_collective(ctx, to, ti, all16, counts, P, dtype, P, 1, variant, stream, [&](int64_t* S, size_t re) {
    for (int p = 0; p < P; ++p)
      for (int r = 0; r < P; ++r) S[p * P + r] = static_cast<int64_t>(counts[p] / re);
  });
}

// ---- the vector collectives with displacements chosen by the caller ---------------------
int mcr_alltoallv_displs(mcr_ctx* ctx, void* const* out, const void* const* in, const int64_t* counts,
                         const int64_t* sdispls, const int64_t* rdispls, size_t in_rows, size_t out_rows, size_t row_elems,
                         mcr_dtype dtype, int P, int variant, void* stream) {
  if (!ctx || !out || !in || !counts || !sdispls || !rdispls || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (row_elems > (size_t(1) << 28) || in_rows > (size_t(1) << 40) || out_rows > (size_t(1) << 40)) return MCR_EINVAL;
  uint64_t cnt[MCR_MAX_RANKS * MCR_MAX_RANKS], sd[MCR_MAX_RANKS * MCR_MAX_RANKS], rd[MCR_MAX_RANKS * MCR_MAX_RANKS];
  uint64_t src_e[MCR_MAX_RANKS], dst_e[MCR_MAX_RANKS];
  bool any = false;
  for (int p = 0; p < P; ++p) {
    for (int r = 0; r < P; ++r) {
      const int i = p * P + r;
      if (counts[i] < 0 || sdispls[i] < 0 || rdispls[r * P + p] < 0) return MCR_EINVAL;
      if (static_cast<uint64_t>(counts[i]) > in_rows || static_cast<uint64_t>(sdispls[i]) > in_rows ||
          static_cast<uint64_t>(rdispls[r * P + p]) > out_rows)
        return MCR_ESPLIT;
      cnt[i] = static_cast<uint64_t>(counts[i]) * row_elems;
      sd[i] = static_cast<uint64_t>(sdispls[i]) * row_elems;
      rd[i] = static_cast<uint64_t>(rdispls[r * P + p]) * row_elems;
      any = any || cnt[i] > 0;
    }
    src_e[p] = static_cast<uint64_t>(in_rows) * row_elems;
    dst_e[p] = static_cast<uint64_t>(out_rows) * row_elems;
  }
  PtrTab to;
  CPtrTab ti;
  bool all16 = true;
  if (!fill_tab(to, out, P, dtype, any, &all16) || !fill_tab(ti, in, P, dtype, any, &all16)) return MCR_EINVAL;
  return pair_collective(ctx, to, ti, all16, cnt, sd, rd, src_e, dst_e, dtype, P, variant, stream);
}

int mcr_gatherv_displs(mcr_ctx* ctx, void* out, size_t out_elems, const void* const* in, const size_t* counts,
                       const size_t* displs, mcr_dtype dtype, int P, int variant, void* stream) {
  if (!ctx || !in || !counts || !displs || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  uint64_t cnt[MCR_MAX_RANKS * MCR_MAX_RANKS] = {0}, sd[MCR_MAX_RANKS * MCR_MAX_RANKS] = {0}, rd[MCR_MAX_RANKS * MCR_MAX_RANKS] = {0};
  uint64_t src_e[MCR_MAX_RANKS], dst_e[MCR_MAX_RANKS];
  PtrTab to;
  CPtrTab ti;
  bool all16 = aligned16(out);
  for (int i = 0; i < MCR_MAX_RANKS; ++i) { to.p[i] = nullptr; ti.p[i] = nullptr; }
  if (out && !elem_aligned(out, dtype)) return MCR_EINVAL;
  to.p[0] = out;                                        // the root is "receiver 0"
  for (int p = 0; p < P; ++p) {
    if (counts[p] > 0 && (!in[p] || !elem_aligned(in[p], dtype))) return MCR_EINVAL;
    if (counts[p] > 0 && !aligned16(in[p])) all16 = false;
    ti.p[p] = in[p];
    cnt[p * P + 0] = counts[p];
    rd[p * P + 0] = displs[p];
    src_e[p] = counts[p];
    dst_e[p] = p == 0 ? out_elems : 0;
  }
  return pair_collective(ctx, to, ti, all16, cnt, sd, rd, src_e, dst_e, dtype, P, variant, stream);
}

int mcr_scatterv_displs(mcr_ctx* ctx, void* const* out, const void* in, size_t in_elems, const size_t* counts,
                        const size_t* displs, mcr_dtype dtype, int P, int variant, void* stream) {
  if (!ctx || !out || !counts || !displs || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  uint64_t cnt[MCR_MAX_RANKS * MCR_MAX_RANKS] = {0}, sd[MCR_MAX_RANKS * MCR_MAX_RANKS] = {0}, rd[MCR_MAX_RANKS * MCR_MAX_RANKS] = {0};
  uint64_t src_e[MCR_MAX_RANKS], dst_e[MCR_MAX_RANKS];
  PtrTab to;
  CPtrTab ti;
  bool all16 = aligned16(in);
  for (int i = 0; i < MCR_MAX_RANKS; ++i) { to.p[i] = nullptr; ti.p[i] = nullptr; }
  if (in && !elem_aligned(in, dtype)) return MCR_EINVAL;
  ti.p[0] = in;                                         // the root is "sender 0"
  for (int r = 0; r < P; ++r) {
    if (counts[r] > 0 && (!out[r] || !elem_aligned(out[r], dtype))) return MCR_EINVAL;
    if (counts[r] > 0 && !aligned16(out[r])) all16 = false;
    to.p[r] = out[r];
    cnt[0 * P + r] = counts[r];
    sd[0 * P + r] = displs[r];
    dst_e[r] = counts[r];
    src_e[r] = r == 0 ? in_elems : 0;
  }
  return pair_collective(ctx, to, ti, all16, cnt, sd, rd, src_e, dst_e, dtype, P, variant, stream);
}

int mcr_allgatherv_displs(mcr_ctx* ctx, void* const* out, size_t out_elems, const void* const* in, const size_t* counts,
                          const size_t* displs, mcr_dtype dtype, int P, int variant, void* stream) {
  if (!ctx || !out || !in || !counts || !displs || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  uint64_t cnt[MCR_MAX_RANKS * MCR_MAX_RANKS] = {0}, sd[MCR_MAX_RANKS * MCR_MAX_RANKS] = {0}, rd[MCR_MAX_RANKS * MCR_MAX_RANKS] = {0};
  uint64_t src_e[MCR_MAX_RANKS], dst_e[MCR_MAX_RANKS];
  size_t total = 0;
  for (int p = 0; p < P; ++p) total += counts[p];
  PtrTab to;
  CPtrTab ti;
  bool all16 = true;
  if (!fill_tab(to, out, P, dtype, total > 0, &all16)) return MCR_EINVAL;
  for (int i = 0; i < MCR_MAX_RANKS; ++i) ti.p[i] = nullptr;
  for (int p = 0; p < P; ++p) {
    if (counts[p] > 0 && (!in[p] || !elem_aligned(in[p], dtype))) return MCR_EINVAL;
    if (counts[p] > 0 && !aligned16(in[p])) all16 = false;
    ti.p[p] = in[p];
    src_e[p] = counts[p];
    dst_e[p] = out_elems;
    for (int r = 0; r < P; ++r) {
      cnt[p * P + r] = counts[p];
      rd[p * P + r] = displs[p];
    }
  }
  return pair_collective(ctx, to, ti, all16, cnt, sd, rd, src_e, dst_e, dtype, P, variant, stream);
}

// ---- MoE ------------------------------------------------------------------------
int mcr_moe_route(mcr_ctx* ctx, const int32_t* const* expert_ids, int T, int E, int P, int capacity,
                  int32_t* const* slot, int32_t* const* counts, int64_t* splits, void* stream) {
  if (!ctx || !expert_ids || !slot || !counts || !splits || !valid_P(P)) return MCR_EINVAL;
  if (T < 0 || E < 1 || E > MCR_MAX_EXPERTS || capacity < 0 || E % P != 0) return MCR_EINVAL;
  if (reinterpret_cast<uintptr_t>(splits) & 7u) return MCR_EINVAL;
  CPtrTab ti;
  PtrTab ts, tc;
  // dtype code MCR_F32 stands for "4-byte aligned" here
  if (!fill_tab(ti, expert_ids, P, MCR_F32, T > 0, nullptr) || !fill_tab(ts, slot, P, MCR_F32, T > 0, nullptr) ||
      !fill_tab(tc, counts, P, MCR_F32, true, nullptr))
    return MCR_EINVAL;
  int rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_moe_route(ctx, ti, T, E, P, capacity, ts, tc, splits, static_cast<hipStream_t>(stream));
}

size_t mcr_moe_route_workspace_bytes(int T, int E, int P) {
  if (T < 0 || E < 1 || E > MCR_MAX_EXPERTS || !valid_P(P)) return 0;
  int chunk_steps;
  const int chunks = route_chunks(T, &chunk_steps);
  if (chunks < 2) return 0;
  return static_cast<size_t>(P) * chunks * E * sizeof(int32_t);
}

int mcr_moe_route_ws(mcr_ctx* ctx, const int32_t* const* expert_ids, int T, int E, int P, int capacity,
                     int32_t* const* slot, int32_t* const* counts, int64_t* splits, void* workspace, size_t workspace_bytes,
                     void* stream) {
  const size_t need = mcr_moe_route_workspace_bytes(T, E, P);
  if (need == 0 || !workspace) return mcr_moe_route(ctx, expert_ids, T, E, P, capacity, slot, counts, splits, stream);
  if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 3u)) return MCR_EINVAL;
  if (!ctx || !expert_ids || !slot || !counts || !splits || !valid_P(P)) return MCR_EINVAL;
  if (T < 0 || E < 1 || E > MCR_MAX_EXPERTS || capacity < 0 || E % P != 0) return MCR_EINVAL;
  if (reinterpret_cast<uintptr_t>(splits) & 7u) return MCR_EINVAL;
  CPtrTab ti;
  PtrTab ts, tc;
  if (!fill_tab(ti, expert_ids, P, MCR_F32, T > 0, nullptr) || !fill_tab(ts, slot, P, MCR_F32, T > 0, nullptr) ||
      !fill_tab(tc, counts, P, MCR_F32, true, nullptr))
    return MCR_EINVAL;
  int rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_moe_route_chunked(ctx, ti, T, E, P, capacity, ts, tc, splits, static_cast<int32_t*>(workspace),
                                  static_cast<hipStream_t>(stream));
}

int mcr_moe_route_static(mcr_ctx* ctx, const int32_t* const* expert_ids, int T, int E, int P, int capacity,
                         int32_t* const* slot, int32_t* const* counts, int64_t* splits, void* stream) {
  if (!ctx || !expert_ids || !slot || !counts || !splits || !valid_P(P)) return MCR_EINVAL;
  if (T < 0 || E < 1 || E > MCR_MAX_EXPERTS || capacity < 0 || E % P != 0) return MCR_EINVAL;
  if (reinterpret_cast<uintptr_t>(splits) & 7u) return MCR_EINVAL;
  const size_t need = mcr_moe_route_workspace_bytes(T, E, P);
  if (need > MCR_ROUTE_SCRATCH_BYTES) return MCR_ELIMIT;
  if (need == 0) return mcr_moe_route(ctx, expert_ids, T, E, P, capacity, slot, counts, splits, stream);
  CPtrTab ti;
  PtrTab ts, tc;
  if (!fill_tab(ti, expert_ids, P, MCR_F32, T > 0, nullptr) || !fill_tab(ts, slot, P, MCR_F32, T > 0, nullptr) ||
      !fill_tab(tc, counts, P, MCR_F32, true, nullptr))
    return MCR_EINVAL;
  int rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  int32_t* counters = nullptr;                 // this device's copy of the static array
  if ((rc = route_scratch_address(ctx->device, &counters)) != MCR_OK) return rc;
  return launch_moe_route_chunked(ctx, ti, T, E, P, capacity, ts, tc, splits, counters, static_cast<hipStream_t>(stream));
}

int mcr_pack(mcr_ctx* ctx, void* const* out, const void* const* in, const int32_t* const* slot, size_t T,
             size_t out_rows, size_t row_elems, mcr_dtype dtype, int P, int variant, void* stream) {
  if (!ctx || !out || !in || !slot || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (row_elems > (size_t(1) << 28)) return MCR_EINVAL;
  const bool any = T > 0 && row_elems > 0;
  PtrTab to;
  CPtrTab ti, tsl;
  bool all16 = true;
  if (!fill_tab(to, out, P, dtype, any && out_rows > 0, &all16) || !fill_tab(ti, in, P, dtype, any, &all16) ||
      !fill_tab(tsl, slot, P, MCR_F32, any, nullptr))
    return MCR_EINVAL;
  const size_t row_bytes = row_elems * elem_bytes(dtype);
  const bool vec_ok = all16 && (row_bytes % 16 == 0);
  int v;
  int rc = resolve_variant(ctx, MCR_OP_PACK, dtype, P, T * row_bytes, vec_ok, variant, &v);
  if (rc != MCR_OK) return rc;
  if (!any || out_rows == 0) return MCR_OK;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_pack(ctx, to, ti, tsl, T, out_rows, row_bytes, static_cast<int>(elem_bytes(dtype)), P, v,
                     static_cast<hipStream_t>(stream));
}

int mcr_unpack(mcr_ctx* ctx, void* const* out, const void* const* in, const int32_t* const* slot,
               const float* const* gate, size_t T, size_t in_rows, size_t row_elems, mcr_dtype dtype, int P,
               int variant, void* stream) {
  if (!ctx || !out || !in || !slot || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (row_elems > (size_t(1) << 28)) return MCR_EINVAL;
  const bool any = T > 0 && row_elems > 0;
  PtrTab to;
  CPtrTab ti, tsl, tg;
  bool all16 = true;
  if (!fill_tab(to, out, P, dtype, any, &all16) || !fill_tab(ti, in, P, dtype, any && in_rows > 0, &all16) ||
      !fill_tab(tsl, slot, P, MCR_F32, any, nullptr))
    return MCR_EINVAL;
  if (gate && dtype == MCR_I32) return MCR_EDTYPE;                    // a weight cannot scale integers
  if (gate && !fill_tab(tg, gate, P, MCR_F32, any, nullptr)) return MCR_EINVAL;
  const size_t row_bytes = row_elems * elem_bytes(dtype);
  const bool vec_ok = all16 && (row_bytes % 16 == 0);
  int v;
  int rc = resolve_variant(ctx, MCR_OP_UNPACK, dtype, P, T * row_bytes, vec_ok, variant, &v);
  if (rc != MCR_OK) return rc;
  if (!any) return MCR_OK;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_unpack(ctx, to, ti, tsl, gate ? &tg : nullptr, T, in_rows, row_elems, dtype, P, v,
                       static_cast<hipStream_t>(stream));
}

// ---- fused pipelines ---------------------------------------------------------------
int mcr_moe_dispatch(mcr_ctx* ctx, void* const* recv, const void* const* tokens, const int32_t* const* slot,
                     const int64_t* splits, size_t T, size_t recv_rows, size_t row_elems, mcr_dtype dtype, int P,
                     int variant, void* stream) {
  if (!ctx || !recv || !tokens || !slot || !splits || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (row_elems > (size_t(1) << 28) || T > 0x7fffffffull || (reinterpret_cast<uintptr_t>(splits) & 7u)) return MCR_EINVAL;
  const bool any = T > 0 && row_elems > 0 && recv_rows > 0;
  PtrTab to;
  CPtrTab ti, tsl;
  bool all16 = true;
  if (!fill_tab(to, recv, P, dtype, any, &all16) || !fill_tab(ti, tokens, P, dtype, any, &all16) ||
      !fill_tab(tsl, slot, P, MCR_F32, any, nullptr))
    return MCR_EINVAL;
  const size_t row_bytes = row_elems * elem_bytes(dtype);
  int v;
  int rc = resolve_variant(ctx, MCR_OP_MOE_DISPATCH, dtype, P, T * row_bytes, all16 && row_bytes % 16 == 0, variant, &v);
  if (rc != MCR_OK) return rc;
  if (!any) return MCR_OK;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_moe_dispatch(ctx, to, ti, tsl, splits, T, recv_rows, row_bytes, static_cast<int>(elem_bytes(dtype)), P, v,
                             static_cast<hipStream_t>(stream));
}

int mcr_moe_combine(mcr_ctx* ctx, void* const* out, const void* const* expert_out, const int32_t* const* slot,
                    const float* const* gate, const int64_t* splits, size_t T, size_t recv_rows, size_t row_elems,
                    mcr_dtype dtype, int P, int variant, void* stream) {
  if (!ctx || !out || !expert_out || !slot || !splits || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (row_elems > (size_t(1) << 28) || T > 0x7fffffffull || (reinterpret_cast<uintptr_t>(splits) & 7u)) return MCR_EINVAL;
  const bool any = T > 0 && row_elems > 0;
  PtrTab to;
  CPtrTab ti, tsl, tg;
  bool all16 = true;
  if (!fill_tab(to, out, P, dtype, any, &all16) || !fill_tab(ti, expert_out, P, dtype, any && recv_rows > 0, &all16) ||
      !fill_tab(tsl, slot, P, MCR_F32, any, nullptr))
    return MCR_EINVAL;
  if (gate && dtype == MCR_I32) return MCR_EDTYPE;                    // a weight cannot scale integers
  if (gate && !fill_tab(tg, gate, P, MCR_F32, any, nullptr)) return MCR_EINVAL;
  const size_t row_bytes = row_elems * elem_bytes(dtype);
  int v;
  int rc = resolve_variant(ctx, MCR_OP_MOE_COMBINE, dtype, P, T * row_bytes, all16 && row_bytes % 16 == 0, variant, &v);
  if (rc != MCR_OK) return rc;
  if (!any) return MCR_OK;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_moe_combine(ctx, to, ti, tsl, gate ? &tg : nullptr, splits, T, recv_rows, row_elems, dtype, P, v,
                            static_cast<hipStream_t>(stream));
}

int mcr_moe_expert_layout(mcr_ctx* ctx, const int32_t* const* counts, int E, int P, int64_t* row_table,
                          int64_t* expert_first, int64_t* expert_rows, void* stream) {
  if (!ctx || !counts || !row_table || !expert_first || !expert_rows || !valid_P(P)) return MCR_EINVAL;
  if (E < 1 || E > MCR_MAX_EXPERTS || E % P != 0) return MCR_EINVAL;
  if ((reinterpret_cast<uintptr_t>(row_table) | reinterpret_cast<uintptr_t>(expert_first) |
       reinterpret_cast<uintptr_t>(expert_rows)) & 7u)
    return MCR_EINVAL;
  CPtrTab tc;
  if (!fill_tab(tc, counts, P, MCR_F32, true, nullptr)) return MCR_EINVAL;
  int rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_moe_expert_layout(ctx, tc, E, P, row_table, expert_first, expert_rows, static_cast<hipStream_t>(stream));
}

int mcr_moe_source_layout(mcr_ctx* ctx, const int32_t* const* counts, int E, int P, int64_t* row_table, void* stream) {
  if (!ctx || !counts || !row_table || !valid_P(P)) return MCR_EINVAL;
  if (E < 1 || E > MCR_MAX_EXPERTS || E % P != 0) return MCR_EINVAL;
  if (reinterpret_cast<uintptr_t>(row_table) & 7u) return MCR_EINVAL;
  CPtrTab tc;
  if (!fill_tab(tc, counts, P, MCR_F32, true, nullptr)) return MCR_EINVAL;
  int rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_moe_source_layout(ctx, tc, E, P, row_table, static_cast<hipStream_t>(stream));
}

int mcr_moe_dispatch_by_expert(mcr_ctx* ctx, void* const* recv, const void* const* tokens, const int32_t* const* expert_ids,
                               const int32_t* const* slot, const int64_t* row_table, size_t T, int K, int E,
                               size_t recv_rows, size_t row_elems, mcr_dtype dtype, int P, int variant, void* stream) {
  if (!ctx || !recv || !tokens || !expert_ids || !slot || !row_table || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (E < 1 || E > MCR_MAX_EXPERTS || E % P != 0 || K < 1 || K > MCR_MAX_TOPK) return MCR_EINVAL;
  if (row_elems > (size_t(1) << 28) || T > 0x7fffffffull / static_cast<size_t>(K) ||
      (reinterpret_cast<uintptr_t>(row_table) & 7u))
    return MCR_EINVAL;
  const bool any = T > 0 && row_elems > 0 && recv_rows > 0;
  PtrTab to;
  CPtrTab ti, tid, tsl;
  bool all16 = true;
  if (!fill_tab(to, recv, P, dtype, any, &all16) || !fill_tab(ti, tokens, P, dtype, any, &all16) ||
      !fill_tab(tid, expert_ids, P, MCR_F32, any, nullptr) || !fill_tab(tsl, slot, P, MCR_F32, any, nullptr))
    return MCR_EINVAL;
  const size_t row_bytes = row_elems * elem_bytes(dtype);
  int v;
  int rc = resolve_variant(ctx, MCR_OP_MOE_DISPATCH_BY_EXPERT, dtype, P, T * row_bytes, all16 && row_bytes % 16 == 0, variant, &v);
  if (rc != MCR_OK) return rc;
  if (!any) return MCR_OK;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_moe_dispatch_by_expert(ctx, to, ti, tid, tsl, row_table, E, T, K, recv_rows, row_bytes,
                                       static_cast<int>(elem_bytes(dtype)), P, v, static_cast<hipStream_t>(stream));
}

int mcr_moe_combine_by_expert(mcr_ctx* ctx, void* const* out, const void* const* expert_out, const int32_t* const* expert_ids,
                              const int32_t* const* slot, const float* const* gate, const int64_t* row_table, size_t T, int K,
                              int E, size_t recv_rows, size_t row_elems, mcr_dtype dtype, int P, int variant, void* stream) {
  if (!ctx || !out || !expert_out || !expert_ids || !slot || !row_table || !valid_P(P)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (dtype == MCR_I32 && K > 1) return MCR_EDTYPE;                   // the weighted sum is a floating-point one
  if (E < 1 || E > MCR_MAX_EXPERTS || E % P != 0 || K < 1 || K > MCR_MAX_TOPK) return MCR_EINVAL;
  if (row_elems > (size_t(1) << 28) || T > 0x7fffffffull / static_cast<size_t>(K) ||
      (reinterpret_cast<uintptr_t>(row_table) & 7u))
    return MCR_EINVAL;
  const bool any = T > 0 && row_elems > 0;
  PtrTab to;
  CPtrTab ti, tid, tsl, tg;
  bool all16 = true;
  if (!fill_tab(to, out, P, dtype, any, &all16) || !fill_tab(ti, expert_out, P, dtype, any && recv_rows > 0, &all16) ||
      !fill_tab(tid, expert_ids, P, MCR_F32, any, nullptr) || !fill_tab(tsl, slot, P, MCR_F32, any, nullptr))
    return MCR_EINVAL;
  if (gate && dtype == MCR_I32) return MCR_EDTYPE;                    // a weight cannot scale integers
  if (gate && !fill_tab(tg, gate, P, MCR_F32, any, nullptr)) return MCR_EINVAL;
  const size_t row_bytes = row_elems * elem_bytes(dtype);
  int v;
  int rc = resolve_variant(ctx, MCR_OP_MOE_COMBINE_BY_EXPERT, dtype, P, T * row_bytes, all16 && row_bytes % 16 == 0, variant, &v);
  if (rc != MCR_OK) return rc;
  if (!any) return MCR_OK;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_moe_combine_by_expert(ctx, to, ti, tid, tsl, gate ? &tg : nullptr, row_table, E, T, K, recv_rows, row_elems, dtype,
                                      P, v, static_cast<hipStream_t>(stream));
}

int mcr_dlrm_shuffle(mcr_ctx* ctx, void* const* out, const void* const* in, int n_tables, size_t batch, size_t dim,
                     mcr_dtype dtype, int P, int backward, int variant, void* stream) {
  if (!ctx || !out || !in || !valid_P(P) || n_tables < 0) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (batch % static_cast<size_t>(P) != 0 || dim > (size_t(1) << 28)) return MCR_EINVAL;
  const bool any = n_tables > 0 && batch > 0 && dim > 0;
  // a rank that owns no table (n_tables < P) has an empty table-major buffer and may pass NULL
  PtrTab to;
  CPtrTab ti;
  bool all16 = true;
  for (int i = 0; i < MCR_MAX_RANKS; ++i) { to.p[i] = nullptr; ti.p[i] = nullptr; }
  for (int p = 0; p < P; ++p) {
    const bool owns = p < n_tables;
    const bool need_out = any && (backward ? owns : true);
    const bool need_in = any && (backward ? true : owns);
    if ((need_out && !out[p]) || (need_in && !in[p])) return MCR_EINVAL;
    if (!elem_aligned(out[p], dtype) || !elem_aligned(in[p], dtype)) return MCR_EINVAL;
    if ((need_out && !aligned16(out[p])) || (need_in && !aligned16(in[p]))) all16 = false;
    to.p[p] = out[p];
    ti.p[p] = in[p];
  }
  const size_t row_bytes = dim * elem_bytes(dtype);
  int v;
  int rc = resolve_variant(ctx, MCR_OP_DLRM_SHUFFLE, dtype, P, (batch / P) * n_tables * row_bytes,
                           all16 && row_bytes % 16 == 0, variant, &v);
  if (rc != MCR_OK) return rc;
  if (!any) return MCR_OK;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_dlrm_shuffle(ctx, to, ti, n_tables, batch, row_bytes, static_cast<int>(elem_bytes(dtype)), P, backward != 0,
                             v, static_cast<hipStream_t>(stream));
}

// ---- tensor fusion ---------------------------------------------------------------
static void plan_free_device(mcr_fuse_plan* plan) {
  if (plan->d_numel) (void)hipFree(plan->d_numel);
  if (plan->d_offset) (void)hipFree(plan->d_offset);
  if (plan->d_chunk_start) (void)hipFree(plan->d_chunk_start);
  if (plan->d_chunk_tensor) (void)hipFree(plan->d_chunk_tensor);
  if (plan->d_ptrs) (void)hipFree(plan->d_ptrs);
  plan->d_numel = plan->d_offset = nullptr;
  plan->d_chunk_start = plan->d_chunk_tensor = nullptr;
  plan->d_ptrs = nullptr;
}

int mcr_fuse_plan_create(mcr_ctx* ctx, const size_t* numel, int n_tensors, size_t bucket_elems, mcr_dtype dtype,
                         mcr_fuse_plan** out) {
  if (!ctx || !out || n_tensors < 0 || bucket_elems == 0 || (n_tensors > 0 && !numel)) return MCR_EINVAL;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  mcr_fuse_plan* plan = new (std::nothrow) mcr_fuse_plan;
  if (!plan) return MCR_ENOMEM;
  plan->ctx = ctx;
  plan->dtype = dtype;
  plan->n_tensors = n_tensors;
  plan->bucket_elems = bucket_elems;
  plan->numel.assign(numel, numel + n_tensors);
  plan->offset.resize(n_tensors);
  plan->tensor_bucket.resize(n_tensors);
  plan->bucket_first.push_back(0);
  // greedy, order preserving: a tensor that does not fit closes the open bucket; an
  // oversize tensor sits alone
  size_t fill = 0;
  int count_in_open = 0;
  for (int i = 0; i < n_tensors; ++i) {
    const size_t n = plan->numel[i];
    const bool oversize = n > bucket_elems;
    if (count_in_open > 0 && (oversize || fill + n > bucket_elems)) {
      plan->bucket_numel.push_back(fill);
      plan->bucket_first.push_back(i);
      fill = 0;
      count_in_open = 0;
    }
    plan->tensor_bucket[i] = static_cast<int>(plan->bucket_numel.size());
    plan->offset[i] = fill;
    fill += n;
    ++count_in_open;
    if (oversize) {
      plan->bucket_numel.push_back(fill);
      plan->bucket_first.push_back(i + 1);
      fill = 0;
      count_in_open = 0;
    }
  }
  if (count_in_open > 0) {
    plan->bucket_numel.push_back(fill);
    plan->bucket_first.push_back(n_tensors);
  }
  plan->n_buckets = static_cast<int>(plan->bucket_numel.size());
  // chunk tables
  const size_t ce = kChunkBytes / elem_bytes(dtype);
  plan->chunk_start.resize(n_tensors + 1);
  std::vector<uint32_t> chunk_tensor;
  uint64_t chunks = 0;
  for (int i = 0; i < n_tensors; ++i) {
    plan->chunk_start[i] = static_cast<uint32_t>(chunks);
    const uint64_t nc = (plan->numel[i] + ce - 1) / ce;
    chunks += nc;
    if (chunks > 0x7fffffffull) { delete plan; return MCR_EINVAL; }
    chunk_tensor.insert(chunk_tensor.end(), nc, static_cast<uint32_t>(i));
  }
  plan->chunk_start[n_tensors] = static_cast<uint32_t>(chunks);
  if (ctx->device < 0) {   // host-only context: the plan can be inspected, not launched
    *out = plan;
    return MCR_OK;
  }
  DeviceScope on_device(ctx);
  if (on_device.status() != MCR_OK) { delete plan; return MCR_EHIP; }
  std::vector<uint64_t> h_numel(plan->numel.begin(), plan->numel.end());
  std::vector<uint64_t> h_off(plan->offset.begin(), plan->offset.end());
  bool ok = true;
  auto up = [&](auto** dptr, const void* src, size_t bytes) {
    if (!ok) return;
    if (hipMalloc(reinterpret_cast<void**>(dptr), bytes ? bytes : 16) != hipSuccess) { ok = false; return; }
    if (bytes && hipMemcpy(*dptr, src, bytes, hipMemcpyHostToDevice) != hipSuccess) ok = false;
  };
  up(&plan->d_numel, h_numel.data(), h_numel.size() * 8);
  up(&plan->d_offset, h_off.data(), h_off.size() * 8);
  up(&plan->d_chunk_start, plan->chunk_start.data(), plan->chunk_start.size() * 4);
  up(&plan->d_chunk_tensor, chunk_tensor.data(), chunk_tensor.size() * 4);
  if (!ok) {
    plan_free_device(plan);
    delete plan;
    return MCR_EHIP;
  }
  *out = plan;
  return MCR_OK;
}

int mcr_fuse_plan_info(const mcr_fuse_plan* plan, int* n_buckets, size_t* bucket_numel, int* tensor_bucket,
                       size_t* tensor_offset) {
  if (!plan) return MCR_EINVAL;
  if (n_buckets) *n_buckets = plan->n_buckets;
  if (bucket_numel) std::copy(plan->bucket_numel.begin(), plan->bucket_numel.end(), bucket_numel);
  if (tensor_bucket) std::copy(plan->tensor_bucket.begin(), plan->tensor_bucket.end(), tensor_bucket);
  if (tensor_offset) std::copy(plan->offset.begin(), plan->offset.end(), tensor_offset);
  return MCR_OK;
}

int mcr_fuse_plan_bind(mcr_ctx* ctx, mcr_fuse_plan* plan, void* const* tensors, int P) {
  if (!ctx || !plan || plan->ctx != ctx || !valid_P(P)) return MCR_EINVAL;
  const size_t n = static_cast<size_t>(plan->n_tensors);
  if (n > 0 && !tensors) return MCR_EINVAL;
  for (size_t k = 0; k < n * P; ++k) {
    const size_t i = k % n;
    if (plan->numel[i] > 0 && (tensors[k] == nullptr || !elem_aligned(tensors[k], plan->dtype))) return MCR_EINVAL;
  }
  int rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  if (P > plan->alloc_P) {
    if (plan->d_ptrs) (void)hipFree(plan->d_ptrs);
    plan->d_ptrs = nullptr;
    plan->alloc_P = 0;
    if (hipMalloc(reinterpret_cast<void**>(&plan->d_ptrs), std::max<size_t>(n * P * sizeof(void*), 16)) != hipSuccess)
      return MCR_EHIP;
    plan->alloc_P = P;
  }
  if (n > 0 && hipMemcpy(plan->d_ptrs, tensors, n * P * sizeof(void*), hipMemcpyHostToDevice) != hipSuccess)
    return MCR_EHIP;
  plan->bound_P = P;
  return MCR_OK;
}

static int fuse_common(mcr_ctx* ctx, const mcr_fuse_plan* plan, int bucket, void* const* flat, int P, int variant,
                       void* stream, bool unfuse) {
  if (!ctx || !plan || plan->ctx != ctx || !flat || !valid_P(P)) return MCR_EINVAL;
  if (bucket < 0 || bucket >= plan->n_buckets) return MCR_EINVAL;
  if (plan->bound_P == 0 || plan->bound_P != P) return MCR_ESTATE;
  PtrTab tf;
  if (!fill_tab(tf, flat, P, plan->dtype, plan->bucket_numel[bucket] > 0, nullptr)) return MCR_EINVAL;
  int v;
  int rc = resolve_variant(ctx, unfuse ? MCR_OP_UNFUSE : MCR_OP_FUSE, plan->dtype, P,
                           plan->bucket_numel[bucket] * elem_bytes(plan->dtype), true, variant, &v);
  if (rc != MCR_OK) return rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_fuse(ctx, plan, bucket, tf, unfuse, v, static_cast<hipStream_t>(stream));
}

int mcr_fuse(mcr_ctx* ctx, const mcr_fuse_plan* plan, int bucket, void* const* flat, int P, int variant,
             void* stream) {
  return fuse_common(ctx, plan, bucket, flat, P, variant, stream, false);
}

int mcr_unfuse(mcr_ctx* ctx, const mcr_fuse_plan* plan, int bucket, const void* const* flat, int P, int variant,
               void* stream) {
  return fuse_common(ctx, plan, bucket, const_cast<void* const*>(flat), P, variant, stream, true);
}

int mcr_allreduce_multi(mcr_ctx* ctx, const mcr_fuse_plan* plan, int bucket, mcr_redop op, int variant,
                        void* stream) {
  if (!ctx || !plan || plan->ctx != ctx) return MCR_EINVAL;
  if (bucket < -1 || bucket >= plan->n_buckets) return MCR_EINVAL;
  if (!valid_redop(op) || !redop_fits(op, plan->dtype)) return MCR_EOP;
  if (plan->bound_P == 0) return MCR_ESTATE;
  const int t0 = bucket < 0 ? 0 : plan->bucket_first[bucket];
  const int t1 = bucket < 0 ? plan->n_tensors : plan->bucket_first[bucket + 1];
  size_t elems = 0;
  for (int i = t0; i < t1; ++i) elems += plan->numel[i];
  int v;
  int rc = resolve_variant(ctx, MCR_OP_ALLREDUCE_MULTI, plan->dtype, plan->bound_P, elems * elem_bytes(plan->dtype),
                           true, variant, &v);
  if (rc != MCR_OK) return rc;
  DeviceScope on_device(ctx);
  if ((rc = on_device.status()) != MCR_OK) return rc;
  return launch_allreduce_multi(ctx, plan, t0, t1, op, v, static_cast<hipStream_t>(stream));
}

int mcr_fuse_plan_destroy(mcr_fuse_plan* plan) {
  if (!plan) return MCR_EINVAL;
  if (plan->ctx && plan->ctx->device >= 0) (void)hipSetDevice(plan->ctx->device);
  plan_free_device(plan);
  delete plan;
  return MCR_OK;
}

// ---- dispatch overhead (paper Sec. V-B: the runtime's overhead over a C-level benchmark) ------
int mcr_dispatch_overhead(mcr_ctx* ctx, void* const* out, const void* const* in, size_t count, mcr_dtype dtype, int P,
                          int iters, void* stream, double* us_auto, double* us_direct, double* host_us_auto,
                          double* host_us_direct, double* dispatch_only_us) {
  if (!ctx || !us_auto || !us_direct || iters < 1) return MCR_EINVAL;
  DeviceScope on_device(ctx);                              // the bare launches below need it too
  if (on_device.status() != MCR_OK) return on_device.status();
  hipStream_t st = static_cast<hipStream_t>(stream);
  // the full entry point once: validates everything and warms the kernel up
  int rc = mcr_alltoall(ctx, out, in, count, dtype, P, MCR_AUTO, stream);
  if (rc != MCR_OK) return rc;
  PtrTab to;
  CPtrTab ti;
  int v;
  rc = prepare_alltoall(ctx, out, in, count, dtype, P, MCR_AUTO, &to, &ti, &v);
  if (rc != MCR_OK) return rc;
  if (hipStreamSynchronize(st) != hipSuccess) return MCR_EHIP;
  typedef std::chrono::steady_clock clk;
  auto us = [](clk::time_point a, clk::time_point b, int n) {
    return std::chrono::duration<double, std::micro>(b - a).count() / n;
  };
  double best_auto = 1e30, best_direct = 1e30, host_auto = 1e30, host_direct = 1e30;
  // one timed loop of `iters` calls: through the entry point (table lookup and checks) or bare launches
  auto timed_loop = [&](bool through_entry, double* total_us, double* enqueue_us) -> int {
    auto a = clk::now();
    for (int i = 0; i < iters; ++i) {
      const int r = through_entry ? mcr_alltoall(ctx, out, in, count, dtype, P, MCR_AUTO, stream)
                                  : launch_alltoall(ctx, to, ti, count, dtype, P, v, st);
      if (r != MCR_OK) return r;
    }
    auto b = clk::now();                                         // everything enqueued
    if (hipStreamSynchronize(st) != hipSuccess) return MCR_EHIP;
    auto c = clk::now();
    *total_us = std::min(*total_us, us(a, c, iters));
    *enqueue_us = std::min(*enqueue_us, us(a, b, iters));
    return MCR_OK;
  };
  // the two loops swap places every round, so that neither always runs in the other's wake
  for (int round = 0; round < 4; ++round) {
    const bool entry_first = (round % 2) == 0;
    if ((rc = timed_loop(entry_first, entry_first ? &best_auto : &best_direct, entry_first ? &host_auto : &host_direct)) != MCR_OK)
      return rc;
    if ((rc = timed_loop(!entry_first, entry_first ? &best_direct : &best_auto, entry_first ? &host_direct : &host_auto)) != MCR_OK)
      return rc;
  }
  if (dispatch_only_us) {
    // the dispatch layer by itself: no launch, no GPU, so nothing but the CPU work is in it
    const int n = iters * 20;
    double best = 1e30;
    int sink = 0;
    for (int round = 0; round < 4; ++round) {
      auto a = clk::now();
      for (int i = 0; i < n; ++i) {
        PtrTab t2;
        CPtrTab s2;
        int v2 = 0;
        sink += prepare_alltoall(ctx, out, in, count, dtype, P, MCR_AUTO, &t2, &s2, &v2) + v2 +
                static_cast<int>(reinterpret_cast<uintptr_t>(t2.p[0]) & 1u);
      }
      auto b = clk::now();
      best = std::min(best, us(a, b, n));
    }
    if (sink == -12345) return MCR_ESTATE;          // keeps the loop's results alive
    *dispatch_only_us = best;
  }
  *us_auto = best_auto;
  *us_direct = best_direct;
  if (host_us_auto) *host_us_auto = host_auto;
  if (host_us_direct) *host_us_direct = host_direct;
  return MCR_OK;
}

// ---- tuning table -----------------------------------------------------------------
int mcr_tune_set(mcr_ctx* ctx, int op_id, mcr_dtype dtype, int P, size_t bytes, int variant) {
  if (!ctx || !valid_P(P)) return MCR_EINVAL;
  if (op_id < 0 || op_id >= MCR_OP_COUNT) return MCR_EOP;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (variant < 0 || variant >= n_variants(op_id)) return MCR_EVARIANT;
  std::lock_guard<std::mutex> lock(ctx->mu);
  auto& rows = ctx->tables[TuneKey{op_id, dtype, P}];
  auto it = std::lower_bound(rows.begin(), rows.end(), bytes,
                             [](const std::pair<size_t, int>& r, size_t b) { return r.first < b; });
  if (it != rows.end() && it->first == bytes) it->second = variant;
  else rows.insert(it, std::make_pair(bytes, variant));
  return MCR_OK;
}

int mcr_tune_get(mcr_ctx* ctx, int op_id, mcr_dtype dtype, int P, size_t bytes, int* variant) {
  if (!ctx || !variant || !valid_P(P)) return MCR_EINVAL;
  if (op_id < 0 || op_id >= MCR_OP_COUNT) return MCR_EOP;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  const int v = table_lookup(ctx, op_id, dtype, P, bytes, false);
  if (v < 0) return MCR_EVARIANT;
  *variant = v;
  return MCR_OK;
}

int mcr_auto_variant(mcr_ctx* ctx, int op_id, mcr_dtype dtype, int P, size_t bytes, int vec_ok, int* variant) {
  if (!ctx || !variant || !valid_P(P)) return MCR_EINVAL;
  if (op_id < 0 || op_id >= MCR_OP_COUNT) return MCR_EOP;
  if (!valid_dtype(dtype)) return MCR_EDTYPE;
  if (op_id == MCR_OP_MOE_ROUTE) { *variant = 0; return MCR_OK; }
  return resolve_variant(ctx, op_id, dtype, P, bytes, vec_ok != 0, MCR_AUTO, variant);
}

int mcr_tune_clear(mcr_ctx* ctx) {
  if (!ctx) return MCR_EINVAL;
  std::lock_guard<std::mutex> lock(ctx->mu);
  ctx->tables.clear();
  return MCR_OK;
}

int mcr_tune_count(mcr_ctx* ctx, size_t* n_rows) {
  if (!ctx || !n_rows) return MCR_EINVAL;
  std::lock_guard<std::mutex> lock(ctx->mu);
  size_t n = 0;
  for (const auto& kv : ctx->tables) n += kv.second.size();
  *n_rows = n;
  return MCR_OK;
}

int mcr_tune_save(mcr_ctx* ctx, const char* path) {
  if (!ctx || !path) return MCR_EINVAL;
  std::FILE* f = std::fopen(path, "w");
  if (!f) return MCR_EIO;
  std::lock_guard<std::mutex> lock(ctx->mu);
  std::fprintf(f, "# op dtype P bytes variant\n");
  for (const auto& kv : ctx->tables) {
    for (const auto& row : kv.second) {
      const char* vname = variant_name(kv.first.op, row.second);
      std::fprintf(f, "%s %s %d %zu %s\n", kOpNames[kv.first.op], kDtypeNames[kv.first.dtype], kv.first.P, row.first, vname);
    }
  }
  const bool bad = std::ferror(f) != 0;
  if (std::fclose(f) != 0 || bad) return MCR_EIO;
  return MCR_OK;
}

int mcr_tune_load(mcr_ctx* ctx, const char* path) {
  if (!ctx || !path) return MCR_EINVAL;
  std::FILE* f = std::fopen(path, "r");
  if (!f) return MCR_EIO;
  // parse everything first; the table changes only if the whole file is good
  struct Row { int op, dtype, P; size_t bytes; int variant; };
  std::vector<Row> parsed;
  char line[512];
  bool ok = true;
  while (ok && std::fgets(line, sizeof line, f)) {
    char* s = line;
    while (*s == ' ' || *s == '\t') ++s;
    if (*s == '#' || *s == '\n' || *s == '\r' || *s == 0) continue;
    char op[64], dt[16], var[32];
    int P;
    unsigned long long bytes;
    if (std::sscanf(s, "%63s %15s %d %llu %31s", op, dt, &P, &bytes, var) != 5) { ok = false; break; }
    Row r{-1, -1, P, static_cast<size_t>(bytes), -1};
    for (int i = 0; i < MCR_OP_COUNT; ++i) if (!std::strcmp(op, kOpNames[i])) r.op = i;
    for (int i = 0; i < 4; ++i) if (!std::strcmp(dt, kDtypeNames[i])) r.dtype = i;
    if (r.op >= 0) {
      for (int i = 0; i < n_variants(r.op); ++i) {
        const char* vname = variant_name(r.op, i);
        if (!std::strcmp(var, vname)) r.variant = i;
      }
    }
    if (r.op < 0 || r.dtype < 0 || r.variant < 0 || !valid_P(P)) ok = false;
    else parsed.push_back(r);
  }
  std::fclose(f);
  if (!ok) return MCR_EIO;
  for (const Row& r : parsed) {
    const int rc = mcr_tune_set(ctx, r.op, static_cast<mcr_dtype>(r.dtype), r.P, r.bytes, r.variant);
    if (rc != MCR_OK) return rc;
  }
  return MCR_OK;
}

}  // extern "C"
