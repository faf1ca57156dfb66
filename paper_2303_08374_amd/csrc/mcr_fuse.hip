// Tensor fusion (paper Sec. IV-D): bucket plan, flatten / unflatten of a
// bucket, and the fused small-message path that all-reduces every tensor of a
// bucket where it lies in a single launch.
//
// Work is dealt out by bytes, not by tensor: every tensor is cut into chunks of
// 16 KiB (256 threads x 4 vectors of 16 bytes) and a device table maps each
// chunk to its tensor, so a 4 KiB LayerNorm gradient and a 200 MiB embedding
// gradient in one bucket load the workgroups evenly.
#include "mcr_dispatch.hpp"

namespace mcr {
namespace {

struct PlanDev {
  const uint64_t* numel;
  const uint64_t* offset;
  const uint32_t* chunk_start;
  const uint32_t* chunk_tensor;
  void* const* ptrs;   // bound_P * n_tensors, rank-major
  int n_tensors;
};

// UNFUSE = false: flat[off + j] = tensor[j];  true: tensor[j] = flat[off + j].  blockIdx.y = rank.
template <int EB, bool UNFUSE, bool NTL, bool NTS, bool FORCE_SCALAR>
__global__ void __launch_bounds__(kBlock)
fuse_kernel(PlanDev d, PtrTab flat, uint32_t first_chunk) {
  const uint32_t c = first_chunk + blockIdx.x;
  const uint32_t i = d.chunk_tensor[c];
  const unsigned rank = blockIdx.y;
  constexpr uint64_t CE = kChunkBytes / EB;
  const uint64_t e0 = static_cast<uint64_t>(c - d.chunk_start[i]) * CE;
  const uint64_t n = d.numel[i];
  const uint64_t ne = (n - e0 < CE) ? (n - e0) : CE;
  char* tp = static_cast<char*>(d.ptrs[static_cast<size_t>(rank) * d.n_tensors + i]) + e0 * EB;
  char* fp = static_cast<char*>(flat.p[rank]) + (d.offset[i] + e0) * EB;
  const char* src = UNFUSE ? fp : tp;
  char* dst = UNFUSE ? tp : fp;
  const bool vec_ok = !FORCE_SCALAR &&
      (((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) == 0);
  uint64_t done = 0;
  if (vec_ok) {
    constexpr int W = 16 / EB;
    const uint32_t nv = static_cast<uint32_t>(ne / W);
    u32x4 v[kChunkVecs];
#pragma unroll
    for (int u = 0; u < kChunkVecs; ++u) {
      const uint32_t idx = u * kBlock + threadIdx.x;
      if (idx < nv) v[u] = load16<NTL>(src, idx);
    }
#pragma unroll
    for (int u = 0; u < kChunkVecs; ++u) {
      const uint32_t idx = u * kBlock + threadIdx.x;
      if (idx < nv) store16<NTS>(dst, idx, v[u]);
    }
    done = static_cast<uint64_t>(nv) * W;
  }
  typedef typename std::conditional<EB == 4, uint32_t, uint16_t>::type S;
  for (uint64_t e = done + threadIdx.x; e < ne; e += kBlock)
    reinterpret_cast<S*>(dst)[e] = reinterpret_cast<const S*>(src)[e];
}

// All-reduce of one chunk of one tensor across the bound ranks, in place.
template <int DT, int P, bool NTL, bool NTS, bool FORCE_SCALAR, bool GENERIC>
__global__ void __launch_bounds__(kBlock)
allreduce_multi_kernel(PlanDev d, uint32_t first_chunk, float scale, int op, uint32_t unit_shift) {
  using E = Elem<DT>;
  constexpr int W = E::kPerVec;
  constexpr uint64_t CE = kChunkBytes / E::kBytes;
  const uint32_t c = first_chunk + xcd_unit_tile(blockIdx.x, unit_shift);
  const uint32_t i = d.chunk_tensor[c];
  const uint64_t e0 = static_cast<uint64_t>(c - d.chunk_start[i]) * CE;
  const uint64_t n = d.numel[i];
  const uint64_t ne = (n - e0 < CE) ? (n - e0) : CE;
  char* base[P];
  uintptr_t all = 0;
#pragma unroll
  for (int p = 0; p < P; ++p) {
    base[p] = static_cast<char*>(d.ptrs[static_cast<size_t>(p) * d.n_tensors + i]) + e0 * E::kBytes;
    all |= reinterpret_cast<uintptr_t>(base[p]);
  }
  uint64_t done = 0;
  if (!FORCE_SCALAR && (all & 15u) == 0) {
    const uint32_t nv = static_cast<uint32_t>(ne / W);
    u32x4 v[kChunkVecs][P];
#pragma unroll
    for (int p = 0; p < P; ++p) {            // rank-major issue order, as in all_reduce
#pragma unroll
      for (int u = 0; u < kChunkVecs; ++u) {
        const uint32_t idx = u * kBlock + threadIdx.x;
        if (idx < nv) v[u][p] = load16<NTL>(base[p], idx);
      }
    }
    u32x4 y[kChunkVecs];
#pragma unroll
    for (int u = 0; u < kChunkVecs; ++u) {
      const uint32_t idx = u * kBlock + threadIdx.x;
      if (idx < nv) {
        typename E::acc_t acc[W];
        E::widen(v[u][0], acc);
#pragma unroll
        for (int p = 1; p < P; ++p) {
          typename E::acc_t x[W];
          E::widen(v[u][p], x);
#pragma unroll
          for (int k = 0; k < W; ++k) acc[k] = GENERIC ? combine(acc[k], x[k], op) : plain_sum(acc[k], x[k]);
        }
        if (op == MCR_AVG) {
#pragma unroll
          for (int k = 0; k < W; ++k) acc[k] = avg_step(acc[k], scale);
        }
        y[u] = E::narrow(acc);
      }
    }
#pragma unroll
    for (int p = 0; p < P; ++p) {
#pragma unroll
      for (int u = 0; u < kChunkVecs; ++u) {
        const uint32_t idx = u * kBlock + threadIdx.x;
        if (idx < nv) store16<NTS>(base[p], idx, y[u]);
      }
    }
    done = static_cast<uint64_t>(nv) * W;
  }
  for (uint64_t e = done + threadIdx.x; e < ne; e += kBlock) {
    typename E::acc_t acc = E::load1(base[0], e);
#pragma unroll
    for (int p = 1; p < P; ++p) acc = GENERIC ? combine(acc, E::load1(base[p], e), op) : plain_sum(acc, E::load1(base[p], e));
    if (op == MCR_AVG) acc = avg_step(acc, scale);
#pragma unroll
    for (int p = 0; p < P; ++p) E::store1(base[p], e, acc);
  }
}

inline PlanDev plan_dev(const mcr_fuse_plan* plan) {
  PlanDev d;
  d.numel = plan->d_numel;
  d.offset = plan->d_offset;
  d.chunk_start = plan->d_chunk_start;
  d.chunk_tensor = plan->d_chunk_tensor;
  d.ptrs = plan->d_ptrs;
  d.n_tensors = plan->n_tensors;
  return d;
}

}  // namespace

int launch_fuse(mcr_ctx*, const mcr_fuse_plan* plan, int bucket, const PtrTab& flat, bool unfuse, int variant,
                hipStream_t stream) {
  const int t0 = plan->bucket_first[bucket], t1 = plan->bucket_first[bucket + 1];
  const uint32_t c0 = plan->chunk_start[t0], c1 = plan->chunk_start[t1];
  if (c1 == c0) return MCR_OK;
  const PlanDev d = plan_dev(plan);
  const dim3 grid(c1 - c0, plan->bound_P);
  auto go = [&](auto eb, auto un, auto ntl, auto nts, auto fs) {
    hipLaunchKernelGGL((fuse_kernel<decltype(eb)::value, decltype(un)::value, decltype(ntl)::value, decltype(nts)::value,
                                    decltype(fs)::value>),
                       grid, dim3(kBlock), 0, stream, d, flat, c0);
    return launch_status();
  };
  auto by_shape = [&](auto eb, auto un) {
    if (variant == SV_SCALAR) return go(eb, un, Bool<false>{}, Bool<false>{}, Bool<true>{});
    return dispatch_hint(variant, [&](auto ntl, auto nts) { return go(eb, un, ntl, nts, Bool<false>{}); });
  };
  if (elem_bytes(plan->dtype) == 4) return unfuse ? by_shape(Int<4>{}, Bool<true>{}) : by_shape(Int<4>{}, Bool<false>{});
  return unfuse ? by_shape(Int<2>{}, Bool<true>{}) : by_shape(Int<2>{}, Bool<false>{});
}

// Chunks per XCD unit of the multi-tensor all_reduce, as a shift: consecutive chunks are consecutive
// memory inside a tensor, and 64 of them (1 MiB of every rank's tensor) per XCD at a stretch take
// the 292-tensor gradient list in 7.65 ms instead of 7.98 (units of 256 KiB to 2 MiB alike).
constexpr uint32_t kMultiUnitShift = 6;

int launch_allreduce_multi(mcr_ctx*, const mcr_fuse_plan* plan, int t0, int t1, int op, int variant,
                           hipStream_t stream) {
  const uint32_t c0 = plan->chunk_start[t0], c1 = plan->chunk_start[t1];
  if (c1 == c0) return MCR_OK;
  const PlanDev d = plan_dev(plan);
  const int P = plan->bound_P;
  const float scale = 1.0f / static_cast<float>(P);
  return dispatch_dtype(plan->dtype, [&](auto dt) {
    return dispatch_ranks(P, [&](auto pp) {
      constexpr int DT = decltype(dt)::value;
      constexpr int kP = decltype(pp)::value;
      if (op > MCR_AVG || !all_shapes(DT)) {      // the other ReduceOps and element types: one nontemporal shape, or the element path
        if (variant == SV_SCALAR)
          hipLaunchKernelGGL((allreduce_multi_kernel<DT, kP, false, false, true, true>), dim3(c1 - c0), dim3(kBlock), 0, stream, d, c0, scale, op, 0u);
        else
          hipLaunchKernelGGL((allreduce_multi_kernel<DT, kP, true, true, false, true>), dim3(c1 - c0), dim3(kBlock), 0, stream, d, c0, scale, op, 0u);
        return launch_status();
      }
      if constexpr (all_shapes(DT)) {
        if (variant == SV_SCALAR) {
          hipLaunchKernelGGL((allreduce_multi_kernel<DT, kP, false, false, true, false>), dim3(c1 - c0), dim3(kBlock), 0, stream, d, c0, scale, op, 0u);
          return launch_status();
        }
        // plain or fully nontemporal: the ids with one-sided hints run the nontemporal kernel, as in the reductions
        if (variant == SV_V1 || variant == SV_V2 || variant == SV_V4)
          hipLaunchKernelGGL((allreduce_multi_kernel<DT, kP, false, false, false, false>), dim3(c1 - c0), dim3(kBlock), 0, stream, d, c0,
                             scale, op, kMultiUnitShift);
        else
          hipLaunchKernelGGL((allreduce_multi_kernel<DT, kP, true, true, false, false>), dim3(c1 - c0), dim3(kBlock), 0, stream, d, c0,
                             scale, op, kMultiUnitShift);
        return launch_status();
      } else {
        return static_cast<int>(MCR_EVARIANT);          // not reached: taken by the branch above
      }
    });
  });
}

}  // namespace mcr
