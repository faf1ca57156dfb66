// Kernels and per-element-type launcher of all_reduce over P rank buffers in one GPU's
// memory (API listing of the paper).
//
// A streaming sum: every element index is read from all P buffers with 128-bit
// loads, summed in rank order in binary32, optionally scaled by 1/P, rounded
// once, and written back to all P buffers with 128-bit stores.  The thread that
// reads an index is the only one that writes it, so in place has no race.
// reduce (rooted) is the same kernel with the stores to all but the root's
// buffer switched off (root >= 0).
// Buffers that are not 16-byte aligned but all misaligned by the same amount (the same view of
// a tensor on every rank) still take the 128-bit path: the pointers handed to the kernel are
// advanced to the next 16-byte boundary and the `head` elements in front of them are reduced
// one by one, like the elements past the last whole vector.
// Bound by HBM bandwidth: (P-1) adds per 2*P*s bytes.
#pragma once
#include "mcr_reduce_tile.hpp"

namespace mcr {
namespace {

// The elements that are not part of a whole vector, reduced one by one by workgroup 0: those past
// the last whole vector, and the `head` (< elements per vector) ones in front of the first.
template <int DT, int P>
__device__ __forceinline__ void allreduce_edges(const PtrTab& bufs, const CPtrTab& in, size_t nvec, size_t count, float scale,
                                                int op, int root, unsigned head) {
  using E = Elem<DT>;
  const size_t done = nvec * E::kPerVec;
  if (blockIdx.x == 0 && done + threadIdx.x < count) {
    const size_t i = done + threadIdx.x;
    const typename E::acc_t y = reduce_scalar<DT>(in, i, P, scale, op);
#pragma unroll
    for (int p = 0; p < P; ++p)
      if (root < 0 || root == p) E::store1(bufs.p[p], i, y);
  }
  if (blockIdx.x == 0 && threadIdx.x < head) {
    CPtrTab front;
#pragma unroll
    for (int p = 0; p < P; ++p) front.p[p] = static_cast<const char*>(in.p[p]) - static_cast<size_t>(head) * E::kBytes;
    const typename E::acc_t y = reduce_scalar<DT>(front, threadIdx.x, P, scale, op);
#pragma unroll
    for (int p = 0; p < P; ++p)
      if (root < 0 || root == p) E::store1(const_cast<void*>(front.p[p]), threadIdx.x, y);
  }
}

template <int DT, int P, int U, bool NTL, bool NTS, bool GENERIC, int BS = kBlock>
__global__ void __launch_bounds__(BS)
allreduce_vec(PtrTab bufs, size_t nvec, size_t count, float scale, int op, int root, unsigned head, unsigned unit_shift) {
  constexpr size_t kTile = static_cast<size_t>(U) * BS;
  CPtrTab in;
#pragma unroll
  for (int p = 0; p < P; ++p) in.p[p] = bufs.p[p];
  const size_t tile = static_cast<size_t>(xcd_unit_tile(blockIdx.x, unit_shift)) * kTile;
  if (tile < nvec) {
    u32x4 out[U];
    const bool full = tile + kTile <= nvec;
    if (full) reduce_tile<DT, P, U, NTL, true, GENERIC, BS>(in, 0, tile, nvec, scale, op, out);
    else reduce_tile<DT, P, U, NTL, false, GENERIC, BS>(in, 0, tile, nvec, scale, op, out);
#pragma unroll
    for (int p = 0; p < P; ++p) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const size_t idx = tile + static_cast<size_t>(u) * BS + threadIdx.x;
        if ((full || idx < nvec) && (root < 0 || root == p)) store16<NTS>(bufs.p[p], idx, out[u]);
      }
    }
  }
  allreduce_edges<DT, P>(bufs, in, nvec, count, scale, op, root, head);
}

// The persistent form (see reduce_persistent).
template <int DT, int P, int U, int K>
__global__ void __launch_bounds__(kPersistBlock)
allreduce_persist(PtrTab bufs, size_t nvec, size_t count, float scale, int op, int root, unsigned head) {
  CPtrTab in;
#pragma unroll
  for (int p = 0; p < P; ++p) in.p[p] = bufs.p[p];
  reduce_persistent<DT, P, U, K, false, false>(bufs, in, nvec, scale, op, root);
  allreduce_edges<DT, P>(bufs, in, nvec, count, scale, op, root, head);
}

// Element path (buffers with different alignments, any count).  Still 16 bytes per access, at
// whatever address the elements fall on; kScalarUnroll vectors per thread, the loads of all P
// ranks of all of them issued before the first is used; the count mod (elements per vector)
// elements behind the last whole vector are reduced one by one by workgroup 0.
template <int DT, int P>
__global__ void __launch_bounds__(kBlock)
allreduce_scalar(PtrTab bufs, size_t count, float scale, int op, int root) {
  using E = Elem<DT>;
  constexpr int U = kScalarUnroll;
  constexpr int W = E::kPerVec;
  const size_t nvec = count / W;
  const size_t step = static_cast<size_t>(gridDim.x) * kBlock * U;
  for (size_t i0 = static_cast<size_t>(blockIdx.x) * kBlock * U + threadIdx.x; i0 < nvec; i0 += step) {
    u32x4 v[U][P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const size_t i = i0 + static_cast<size_t>(u) * kBlock;
        if (i < nvec) v[u][p] = load16_unaligned(bufs.p[p], i * 16);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t i = i0 + static_cast<size_t>(u) * kBlock;
      if (i >= nvec) continue;
      typename E::acc_t acc[W];
      E::widen(v[u][0], acc);
#pragma unroll
      for (int p = 1; p < P; ++p) {
        typename E::acc_t x[W];
        E::widen(v[u][p], x);
#pragma unroll
        for (int k = 0; k < W; ++k) acc[k] = combine(acc[k], x[k], op);
      }
      if (op == MCR_AVG) {
#pragma unroll
        for (int k = 0; k < W; ++k) acc[k] = avg_step(acc[k], scale);
      }
      const u32x4 y = E::narrow(acc);
#pragma unroll
      for (int p = 0; p < P; ++p)
        if (root < 0 || root == p) store16_unaligned(bufs.p[p], i * 16, y);
    }
  }
  const size_t i = nvec * W + threadIdx.x;
  if (blockIdx.x == 0 && i < count) {
    typename E::acc_t acc = E::load1(bufs.p[0], i);
#pragma unroll
    for (int p = 1; p < P; ++p) acc = combine(acc, E::load1(bufs.p[p], i), op);
    if (op == MCR_AVG) acc = avg_step(acc, scale);
#pragma unroll
    for (int p = 0; p < P; ++p)
      if (root < 0 || root == p) E::store1(bufs.p[p], i, acc);
  }
}

}  // namespace

// One element type's launches.  Each element type is instantiated in a translation unit of its
// own, which keeps the compile time of the reductions (16 rank counts x launch shapes) spread
// over the build's workers.
template <int DT>
int launch_allreduce_dt(const PtrTab& bufs, size_t count, unsigned head, int op, int P, int root, int variant, int n_cu,
                        hipStream_t stream) {
  const float scale = 1.0f / static_cast<float>(P);
  unsigned unit_kib = 0;
  if (variant >= RV_XUNIT0) {
    unit_kib = kReduceUnitVariants[variant - RV_XUNIT0].unit_kib;
    variant = kReduceUnitVariants[variant - RV_XUNIT0].shape;
  }
  if (variant == SV_SCALAR) {
    return dispatch_ranks(P, [&](auto pp) {
      hipLaunchKernelGGL((allreduce_scalar<DT, decltype(pp)::value>), dim3(scalar_grid(count / Elem<DT>::kPerVec, kScalarUnroll)), dim3(kBlock), 0,
                         stream, bufs, count, scale, op, root);
      return launch_status();
    });
  }
  // bufs point at the first whole vector: `head` elements lie in front of it, count - head from it on
  count -= head;
  const size_t nvec = count / Elem<DT>::kPerVec;
  if (variant == SV_PK8) {
    if (op > MCR_AVG || !all_shapes(DT)) {
      variant = SV_V4NT;                                  // the shape that stands in for the persistent one
    } else {
      const unsigned g = persistent_grid(n_cu, 1);
      return dispatch_ranks(P, [&](auto pp) {
        constexpr int kP = decltype(pp)::value;
        if constexpr (all_shapes(DT)) {
          hipLaunchKernelGGL((allreduce_persist<DT, kP, kPersistU, kPersistK>), dim3(g), dim3(kPersistBlock), 0, stream, bufs, nvec,
                             count, scale, op, root, head);
          return launch_status();
        } else {
          return static_cast<int>(MCR_EVARIANT);          // not reached: ruled out above
        }
      });
    }
  }
  if (variant == SV_W64) {
    if (op > MCR_AVG || !all_shapes(DT)) {
      variant = SV_V2NT;                                  // the shape that stands in for it
    } else {
      const size_t per = 2 * kWave;
      const unsigned g = static_cast<unsigned>(nvec ? (nvec + per - 1) / per : 1);
      return dispatch_ranks(P, [&](auto pp) {
        constexpr int kP = decltype(pp)::value;
        if constexpr (all_shapes(DT)) {
          hipLaunchKernelGGL((allreduce_vec<DT, kP, 2, true, true, false, kWave>), dim3(g), dim3(kWave), 0, stream, bufs, nvec, count,
                             scale, op, root, head, unit_kib ? xcd_unit_shift(unit_kib, per) : 0u);
          return launch_status();
        } else {
          return static_cast<int>(MCR_EVARIANT);          // not reached: ruled out above
        }
      });
    }
  }
  const unsigned gx = grid_x(nvec, variant);
  return dispatch_ranks(P, [&](auto pp) {
    constexpr int kP = decltype(pp)::value;
    if (op > MCR_AVG || !all_shapes(DT)) {
      hipLaunchKernelGGL((allreduce_vec<DT, kP, kGenericUnroll, true, true, true>), dim3(grid_x(nvec, kGenericShape)), dim3(kBlock), 0,
                         stream, bufs, nvec, count, scale, op, root, head, 0u);
      return launch_status();
    }
    if constexpr (all_shapes(DT)) {
      return dispatch_reduce_shape(variant, [&](auto uu, auto nt) {
        constexpr int U = decltype(uu)::value;
        hipLaunchKernelGGL((allreduce_vec<DT, kP, U, decltype(nt)::value, decltype(nt)::value, false>),
                           dim3(gx), dim3(kBlock), 0, stream, bufs, nvec, count, scale, op, root, head,
                           unit_kib ? xcd_unit_shift(unit_kib, static_cast<size_t>(U) * kBlock) : 0u);
        return launch_status();
      });
    } else {
      return static_cast<int>(MCR_EVARIANT);          // not reached: taken by the branch above
    }
  });
}

}  // namespace mcr
