// Host-side internals: context, variant ids, launcher prototypes.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <atomic>
#include <cstdint>
#include <map>
#include <mutex>
#include <string>
#include <tuple>
#include <vector>

#include "../../include/mcr.h"
#include "mcr_device.hpp"

namespace mcr {

// Launch shapes of the streaming kernels, shared by every op but moe_route.
// "scalar" moves one element per thread and accepts any alignment; "vN" moves N
// 128-bit vectors per thread, a workgroup of 256 threads covering N*256
// consecutive vectors.  The suffix is the cache hint: "nt" = nontemporal loads
// and stores, "ln" = nontemporal loads only, "sn" = nontemporal stores only.
enum StreamVariant {
  SV_SCALAR = 0,
  SV_V1 = 1, SV_V2 = 2, SV_V4 = 3,
  SV_V1NT = 4, SV_V2NT = 5, SV_V4NT = 6,
  SV_V1LN = 7, SV_V2LN = 8, SV_V4LN = 9,
  SV_V1SN = 10, SV_V2SN = 11, SV_V4SN = 12,
  SV_COUNT = 13
};
// all_gather only: "scN" walks the message in super-chunks of N MiB per source and
// copies each super-chunk to one destination after the other, so that at any
// moment the chip streams from one source region into one destination region.  "sc16x" is "sc16"
// with the tiles of a super-chunk renumbered so that each of the 8 XCDs works through contiguous
// units of 512 KiB.
enum AllgatherVariant { AG_SC4 = 13, AG_SC8 = 14, AG_SC16 = 15, AG_SC16X = 16, AG_COUNT = 17 };
// all_reduce, reduce and reduce_scatter only: the persistent form "pk8", one workgroup of 1024
// threads per compute unit walking a contiguous run of the message in rounds of 8 steps of one
// vector per thread.  SUM / AVG on fp32 and bf16; other ReduceOps and element types run "v4nt" in
// its place.
enum ReduceVariant { SV_PK8 = 13, SV_W64 = 14, RV_XUNIT0 = 15, RV_COUNT = 35 };
// Ids from RV_XUNIT0 on: a launch shape of the list above with its tiles dealt to the 8 XCDs in
// contiguous units ("<shape>.x<unit in KiB>": every XCD works through `unit` bytes of each rank
// buffer at a stretch instead of every eighth tile).  Which (shape, unit) wins depends on the size
// and on the distance between the rank buffers; the unit is a kernel argument, so the 20 of them
// cost no code.
struct ReduceUnitVariant {
  int shape;            // SV_V1NT, SV_V2NT, SV_V4NT or SV_W64
  unsigned unit_kib;
  const char* name;
};
constexpr ReduceUnitVariant kReduceUnitVariants[RV_COUNT - RV_XUNIT0] = {
    {SV_V1NT, 128, "v1nt.x128"}, {SV_V1NT, 256, "v1nt.x256"}, {SV_V1NT, 512, "v1nt.x512"}, {SV_V1NT, 1024, "v1nt.x1024"}, {SV_V1NT, 2048, "v1nt.x2048"},
    {SV_V2NT, 128, "v2nt.x128"}, {SV_V2NT, 256, "v2nt.x256"}, {SV_V2NT, 512, "v2nt.x512"}, {SV_V2NT, 1024, "v2nt.x1024"}, {SV_V2NT, 2048, "v2nt.x2048"},
    {SV_V4NT, 128, "v4nt.x128"}, {SV_V4NT, 256, "v4nt.x256"}, {SV_V4NT, 512, "v4nt.x512"}, {SV_V4NT, 1024, "v4nt.x1024"}, {SV_V4NT, 2048, "v4nt.x2048"},
    {SV_W64, 128, "w64.x128"}, {SV_W64, 256, "w64.x256"}, {SV_W64, 512, "w64.x512"}, {SV_W64, 1024, "w64.x1024"}, {SV_W64, 2048, "w64.x2048"}};
// "w64" (the reductions and all_to_all_single): workgroups of one wavefront, two vectors per thread
// (one for all_to_all), nontemporal: four times as many, smaller workgroups as "v2nt" for the
// messages of a few MiB whose kernels last a few microseconds.
// all_to_all_single only: "flat" numbers the threads along the output of a destination (thread i
// writes vector i of out[r] and fetches it from the block it belongs to), so that blocks shorter
// than a workgroup do not leave lanes idle; "lds" is "flat" with four vectors per thread staged
// through LDS between a read phase and a write phase of the workgroup.
enum AlltoallVariant { A2A_FLAT = 13, A2A_W64 = 14, A2A_LDS = 15, A2A_COUNT = 16 };
extern const char* const kAlltoallVariantNames[A2A_COUNT - SV_COUNT];
extern const char* const kStreamVariantNames[AG_COUNT];
extern const char* const kReduceVariantNames[RV_XUNIT0 - SV_COUNT];

struct TuneKey {
  int op, dtype, P;
  bool operator<(const TuneKey& o) const {
    return std::tie(op, dtype, P) < std::tie(o.op, o.dtype, o.P);
  }
};

}  // namespace mcr

// Slots of the context's ring of displacement tables (mcr::PairSlot, 4 KiB each): a fused MoE
// call takes the next one, so that many calls may be in flight on different streams before two of
// them share a slot.
constexpr unsigned kPairRingSlots = 64;

struct mcr_ctx {
  int device = 0;
  int n_cu = 256;                                                     // compute units of the device
  mcr::PairSlot* pair_ring = nullptr;                                 // device memory, kPairRingSlots entries, from mcr_init
  std::atomic<unsigned> pair_next{0};
  std::mutex mu;                                                      // guards `tables`
  std::map<mcr::TuneKey, std::vector<std::pair<size_t, int>>> tables; // sorted by bytes
};

struct mcr_fuse_plan {
  mcr_ctx* ctx = nullptr;
  int dtype = 0;
  int n_tensors = 0;
  int n_buckets = 0;
  size_t bucket_elems = 0;
  std::vector<size_t> numel, offset;        // per tensor; offset inside its bucket
  std::vector<int> tensor_bucket;
  std::vector<size_t> bucket_numel;
  std::vector<int> bucket_first;            // n_buckets+1: first tensor of each bucket
  std::vector<uint32_t> chunk_start;        // n_tensors+1: prefix of per-tensor chunk counts
  // device mirrors
  uint64_t* d_numel = nullptr;              // n_tensors
  uint64_t* d_offset = nullptr;             // n_tensors
  uint32_t* d_chunk_start = nullptr;        // n_tensors+1
  uint32_t* d_chunk_tensor = nullptr;       // per chunk: the tensor it belongs to
  void** d_ptrs = nullptr;                  // bound_P * n_tensors, rank-major
  int bound_P = 0;
  int alloc_P = 0;
};

namespace mcr {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elem_bytes(int dtype) { return (dtype == MCR_F32 || dtype == MCR_I32) ? 4 : 2; }
inline int per_vec(int dtype) { return (dtype == MCR_F32 || dtype == MCR_I32) ? 4 : 8; }

// Elements one workgroup covers per tensor chunk in the multi-tensor kernels
// (fuse / unfuse / allreduce_multi): 256 threads x kChunkVecs vectors of 16 bytes.
constexpr int kChunkVecs = 4;    // 2 measured slower for fuse and unfuse, no faster for the multi-tensor all_reduce
constexpr uint32_t kChunkBytes = 256 * kChunkVecs * 16;

// Every launcher returns MCR_OK or MCR_EHIP and assumes validated arguments.
int launch_allreduce(mcr_ctx*, const PtrTab& bufs, size_t count, unsigned head, int dtype, int op, int P, int root,
                     int variant, hipStream_t);
int launch_reduce_scatter(mcr_ctx*, const PtrTab& out, const CPtrTab& in, size_t count, int dtype, int op, int P, int variant, hipStream_t);
int launch_allgather(mcr_ctx*, const PtrTab& out, const CPtrTab& in, size_t count, int dtype, int P, int variant, hipStream_t);
int launch_alltoall(mcr_ctx*, const PtrTab& out, const CPtrTab& in, size_t count, int dtype, int P, int variant, hipStream_t);
int launch_alltoallv(mcr_ctx*, const PtrTab& out, const CPtrTab& in, const int64_t* host_splits, const int64_t* dev_splits,
                     size_t in_rows, size_t out_rows, size_t row_bytes, int elem_b, int P, int same_src, bool dev_transposed,
                     int variant, hipStream_t);
int launch_alltoallv_pairs(mcr_ctx*, const PtrTab& out, const CPtrTab& in, const uint32_t* cnt, const uint32_t* sd,
                           const uint32_t* rd, int elem_b, int P, int variant, hipStream_t);
int launch_moe_route(mcr_ctx*, const CPtrTab& ids, int T, int E, int P, int capacity, const PtrTab& slot, const PtrTab& counts,
                     int64_t* splits, hipStream_t);
int route_chunks(int T, int* chunk_steps);
int launch_moe_route_chunked(mcr_ctx*, const CPtrTab& ids, int T, int E, int P, int capacity, const PtrTab& slot,
                             const PtrTab& counts, int64_t* splits, int32_t* workspace, hipStream_t);
int route_scratch_address(int device, int32_t** out);
int launch_pack(mcr_ctx*, const PtrTab& out, const CPtrTab& in, const CPtrTab& slot, size_t T, size_t out_rows, size_t row_bytes,
                int elem_b, int P, int variant, hipStream_t);
int launch_unpack(mcr_ctx*, const PtrTab& out, const CPtrTab& in, const CPtrTab& slot, const CPtrTab* gate, size_t T,
                  size_t in_rows, size_t row_elems, int dtype, int P, int variant, hipStream_t);
int launch_fuse(mcr_ctx*, const mcr_fuse_plan*, int bucket, const PtrTab& flat, bool unfuse, int variant, hipStream_t);
int launch_allreduce_multi(mcr_ctx*, const mcr_fuse_plan*, int t0, int t1, int op, int variant, hipStream_t);
int launch_moe_dispatch(mcr_ctx*, const PtrTab& recv, const CPtrTab& tok, const CPtrTab& slot, const int64_t* splits, size_t T,
                        size_t recv_rows, size_t row_bytes, int elem_b, int P, int variant, hipStream_t);
int launch_moe_combine(mcr_ctx*, const PtrTab& out, const CPtrTab& expert_out, const CPtrTab& slot, const CPtrTab* gate,
                       const int64_t* splits, size_t T, size_t recv_rows, size_t row_elems, int dtype, int P, int variant,
                       hipStream_t);
int launch_moe_expert_layout(mcr_ctx*, const CPtrTab& counts, int E, int P, int64_t* row_table, int64_t* expert_first,
                             int64_t* expert_rows, hipStream_t);
int launch_moe_source_layout(mcr_ctx*, const CPtrTab& counts, int E, int P, int64_t* row_table, hipStream_t);
int launch_moe_dispatch_by_expert(mcr_ctx*, const PtrTab& recv, const CPtrTab& tok, const CPtrTab& ids, const CPtrTab& slot,
                                  const int64_t* row_table, int E, size_t T, int K, size_t recv_rows, size_t row_bytes,
                                  int elem_b, int P, int variant, hipStream_t);
int launch_moe_combine_by_expert(mcr_ctx*, const PtrTab& out, const CPtrTab& expert_out, const CPtrTab& ids,
                                 const CPtrTab& slot, const CPtrTab* gate, const int64_t* row_table, int E, size_t T, int K,
                                 size_t recv_rows, size_t row_elems, int dtype, int P, int variant, hipStream_t);
int launch_dlrm_shuffle(mcr_ctx*, const PtrTab& dst, const CPtrTab& src, int n_tables, size_t batch, size_t row_bytes,
                        int elem_b, int P, bool backward, int variant, hipStream_t);

inline int hip_status(hipError_t e) { return e == hipSuccess ? MCR_OK : MCR_EHIP; }
inline int launch_status() { return hip_status(hipGetLastError()); }

}  // namespace mcr
