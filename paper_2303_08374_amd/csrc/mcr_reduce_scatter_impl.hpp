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
template <int DT, int P, int U, bool NTL, bool NTS, bool GENERIC>
__global__ void __launch_bounds__(kBlock)
reduce_scatter_vec(PtrTab out, CPtrTab in, size_t bvec, float scale, int op) {
  constexpr size_t kTile = static_cast<size_t>(U) * kBlock;
  const unsigned r = blockIdx.y;
  void* dst = out.p[r];
  const size_t off = static_cast<size_t>(r) * bvec;
  const size_t tile = static_cast<size_t>(blockIdx.x) * kTile;
  if (tile >= bvec) return;
  u32x4 res[U];
  const bool full = tile + kTile <= bvec;
  if (full) reduce_tile<DT, P, U, NTL, true, GENERIC>(in, off, tile, bvec, scale, op, res);
  else reduce_tile<DT, P, U, NTL, false, GENERIC>(in, off, tile, bvec, scale, op, res);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
    if (full || idx < bvec) store16<NTS>(dst, idx, res[u]);
  }
}

// Element path: kScalarUnroll elements per thread, all P x kScalarUnroll loads in flight together.
template <int DT, int P>
__global__ void __launch_bounds__(kBlock)
reduce_scatter_scalar(PtrTab out, CPtrTab in, size_t b, float scale, int op) {
  using E = Elem<DT>;
  constexpr int U = kScalarUnroll;
  const unsigned r = blockIdx.y;
  void* dst = out.p[r];
  const size_t off = static_cast<size_t>(r) * b;
  const size_t step = static_cast<size_t>(gridDim.x) * kBlock * U;
  for (size_t j0 = static_cast<size_t>(blockIdx.x) * kBlock * U + threadIdx.x; j0 < b; j0 += step) {
    typename E::acc_t x[U][P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const size_t j = j0 + static_cast<size_t>(u) * kBlock;
        if (j < b) x[u][p] = E::load1(in.p[p], off + j);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t j = j0 + static_cast<size_t>(u) * kBlock;
      if (j >= b) continue;
      typename E::acc_t acc = x[u][0];
#pragma unroll
      for (int p = 1; p < P; ++p) acc = combine(acc, x[u][p], op);
      if (op == MCR_AVG) acc = avg_step(acc, scale);
      E::store1(dst, j, acc);
    }
  }
}

}  // namespace

// One element type's launches (instantiated in a translation unit of its own, as for all_reduce).
template <int DT>
int launch_reduce_scatter_dt(const PtrTab& out, const CPtrTab& in, size_t count, int op, int P, int variant,
                             hipStream_t stream) {
  const float scale = 1.0f / static_cast<float>(P);
  const size_t b = count / static_cast<size_t>(P);
  if (variant == SV_SCALAR) {
    return dispatch_ranks(P, [&](auto pp) {
      hipLaunchKernelGGL((reduce_scatter_scalar<DT, decltype(pp)::value>), dim3(scalar_grid(b, kScalarUnroll), P), dim3(kBlock),
                         0, stream, out, in, b, scale, op);
      return launch_status();
    });
  }
  const size_t bvec = b / Elem<DT>::kPerVec;
  const unsigned gx = grid_x(bvec, variant);
  return dispatch_ranks(P, [&](auto pp) {
    constexpr int kP = decltype(pp)::value;
    if (op > MCR_AVG || !all_shapes(DT)) {
      return dispatch_unroll(variant, [&](auto uu) {
        hipLaunchKernelGGL((reduce_scatter_vec<DT, kP, decltype(uu)::value, true, true, true>), dim3(gx, P), dim3(kBlock), 0,
                           stream, out, in, bvec, scale, op);
        return launch_status();
      });
    }
    if constexpr (all_shapes(DT)) {
      return dispatch_shape(variant, [&](auto uu, auto ntl, auto nts) {
        constexpr int U = decltype(uu)::value;
        hipLaunchKernelGGL((reduce_scatter_vec<DT, kP, U, decltype(ntl)::value, decltype(nts)::value, false>),
                           dim3(gx, P), dim3(kBlock), 0, stream, out, in, bvec, scale, op);
        return launch_status();
      });
    } else {
      return static_cast<int>(MCR_EVARIANT);          // not reached: taken by the branch above
    }
  });
}

}  // namespace mcr
