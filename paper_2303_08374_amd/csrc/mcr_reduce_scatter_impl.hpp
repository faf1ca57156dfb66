// Kernels and per-element-type launcher of reduce_scatter over P rank buffers in one GPU's
// memory (API listing of the paper; it has no root): rank r receives slice r of the
// rank-order sum.
// P reads and one 1/P-size write per element: the most read-heavy of the four
// collectives.  Bound by HBM bandwidth.
#pragma once
#include "mcr_reduce_tile.hpp"

namespace mcr {
namespace {

// blockIdx.y = destination rank r; slice r of every input is bvec vectors long.
template <int DT, int P, int U, bool NTL, bool NTS, bool GENERIC, int BS = kBlock>
__global__ void __launch_bounds__(BS)
reduce_scatter_vec(PtrTab out, CPtrTab in, size_t bvec, float scale, int op, unsigned unit_shift) {
  constexpr size_t kTile = static_cast<size_t>(U) * BS;
  const unsigned r = blockIdx.y;
  void* dst = out.p[r];
  const size_t off = static_cast<size_t>(r) * bvec;
  const size_t tile = static_cast<size_t>(xcd_unit_tile(blockIdx.x, unit_shift)) * kTile;
  if (tile >= bvec) return;
  u32x4 res[U];
  const bool full = tile + kTile <= bvec;
  if (full) reduce_tile<DT, P, U, NTL, true, GENERIC, BS>(in, off, tile, bvec, scale, op, res);
  else reduce_tile<DT, P, U, NTL, false, GENERIC, BS>(in, off, tile, bvec, scale, op, res);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t idx = tile + static_cast<size_t>(u) * BS + threadIdx.x;
    if (full || idx < bvec) store16<NTS>(dst, idx, res[u]);
  }
}

// The persistent form (see reduce_persistent): grid (workgroups per slice, P).
template <int DT, int P, int U, int K>
__global__ void __launch_bounds__(kPersistBlock)
reduce_scatter_persist(PtrTab out, CPtrTab in, size_t bvec, float scale, int op) {
  reduce_persistent<DT, P, U, K, true, false>(out, in, bvec, scale, op, -1);
}

// Element path (any alignment, any slice length): 16 bytes per access at element-aligned
// addresses, kScalarUnroll vectors per thread with all P x kScalarUnroll loads in flight together;
// the elements behind a slice's last whole vector one by one (see all_reduce's element path).
template <int DT, int P>
__global__ void __launch_bounds__(kBlock)
reduce_scatter_scalar(PtrTab out, CPtrTab in, size_t b, float scale, int op) {
  using E = Elem<DT>;
  constexpr int U = kScalarUnroll;
  constexpr int W = E::kPerVec;
  const unsigned r = blockIdx.y;
  void* dst = out.p[r];
  const size_t off_bytes = static_cast<size_t>(r) * b * E::kBytes;
  const size_t nvec = b / W;
  const size_t step = static_cast<size_t>(gridDim.x) * kBlock * U;
  for (size_t j0 = static_cast<size_t>(blockIdx.x) * kBlock * U + threadIdx.x; j0 < nvec; j0 += step) {
    u32x4 v[U][P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const size_t j = j0 + static_cast<size_t>(u) * kBlock;
        if (j < nvec) v[u][p] = load16_unaligned(in.p[p], off_bytes + j * 16);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t j = j0 + static_cast<size_t>(u) * kBlock;
      if (j >= nvec) continue;
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
      store16_unaligned(dst, j * 16, E::narrow(acc));
    }
  }
  const size_t j = nvec * W + threadIdx.x;
  if (blockIdx.x == 0 && j < b) {
    const size_t i = static_cast<size_t>(r) * b + j;
    typename E::acc_t acc = E::load1(in.p[0], i);
#pragma unroll
    for (int p = 1; p < P; ++p) acc = combine(acc, E::load1(in.p[p], i), op);
    if (op == MCR_AVG) acc = avg_step(acc, scale);
    E::store1(dst, j, acc);
  }
}

}  // namespace

// One element type's launches (instantiated in a translation unit of its own, as for all_reduce).
template <int DT>
int launch_reduce_scatter_dt(const PtrTab& out, const CPtrTab& in, size_t count, int op, int P, int variant, int n_cu,
                             hipStream_t stream) {
  const float scale = 1.0f / static_cast<float>(P);
  const size_t b = count / static_cast<size_t>(P);
  unsigned unit_kib = 0;
  if (variant >= RV_XUNIT0) {
    unit_kib = kReduceUnitVariants[variant - RV_XUNIT0].unit_kib;
    variant = kReduceUnitVariants[variant - RV_XUNIT0].shape;
  }
  if (variant == SV_SCALAR) {
    return dispatch_ranks(P, [&](auto pp) {
      hipLaunchKernelGGL((reduce_scatter_scalar<DT, decltype(pp)::value>), dim3(scalar_grid(b / Elem<DT>::kPerVec, kScalarUnroll), P), dim3(kBlock),
                         0, stream, out, in, b, scale, op);
      return launch_status();
    });
  }
  const size_t bvec = b / Elem<DT>::kPerVec;
  if (variant == SV_PK8) {
    if (op > MCR_AVG || !all_shapes(DT)) {
      variant = SV_V4NT;                                  // the shape that stands in for the persistent one
    } else {
      const dim3 grid(persistent_grid(n_cu, P), P);
      return dispatch_ranks(P, [&](auto pp) {
        constexpr int kP = decltype(pp)::value;
        if constexpr (all_shapes(DT)) {
          hipLaunchKernelGGL((reduce_scatter_persist<DT, kP, kPersistU, kPersistK>), grid, dim3(kPersistBlock), 0, stream, out, in,
                             bvec, scale, op);
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
      const dim3 grid(static_cast<unsigned>(bvec ? (bvec + per - 1) / per : 1), P);
      return dispatch_ranks(P, [&](auto pp) {
        constexpr int kP = decltype(pp)::value;
        if constexpr (all_shapes(DT)) {
          hipLaunchKernelGGL((reduce_scatter_vec<DT, kP, 2, true, true, false, kWave>), grid, dim3(kWave), 0, stream, out, in, bvec,
                             scale, op, unit_kib ? xcd_unit_shift(unit_kib, per) : 0u);
          return launch_status();
        } else {
          return static_cast<int>(MCR_EVARIANT);          // not reached: ruled out above
        }
      });
    }
  }
  const unsigned gx = grid_x(bvec, variant);
  return dispatch_ranks(P, [&](auto pp) {
    constexpr int kP = decltype(pp)::value;
    if (op > MCR_AVG || !all_shapes(DT)) {
      hipLaunchKernelGGL((reduce_scatter_vec<DT, kP, kGenericUnroll, true, true, true>), dim3(grid_x(bvec, kGenericShape), P), dim3(kBlock),
                         0, stream, out, in, bvec, scale, op, 0u);
      return launch_status();
    }
    if constexpr (all_shapes(DT)) {
      return dispatch_reduce_shape(variant, [&](auto uu, auto nt) {
        constexpr int U = decltype(uu)::value;
        hipLaunchKernelGGL((reduce_scatter_vec<DT, kP, U, decltype(nt)::value, decltype(nt)::value, false>),
                           dim3(gx, P), dim3(kBlock), 0, stream, out, in, bvec, scale, op,
                           unit_kib ? xcd_unit_shift(unit_kib, static_cast<size_t>(U) * kBlock) : 0u);
        return launch_status();
      });
    } else {
      return static_cast<int>(MCR_EVARIANT);          // not reached: taken by the branch above
    }
  });
}

}  // namespace mcr
