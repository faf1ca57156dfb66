// all_reduce and reduce_scatter over P rank buffers in one GPU's memory
// (API listing of the paper: all_reduce, reduce_scatter).
//
// Both are streaming sums: every element index is read from all P buffers with
// 128-bit loads, summed left to right in rank order in binary32 starting from
// rank 0's value, optionally scaled by 1/P, rounded once, and written with
// 128-bit stores (to all P buffers for all_reduce, to the owning rank's slice
// for reduce_scatter).  A thread that reads an index is the only one that
// writes it, so the in-place all_reduce has no race.  Bound by HBM bandwidth:
// (P-1) adds per 2*P*s bytes.
#include "mcr_dispatch.hpp"

namespace mcr {
namespace {

// Sum of one tile: U vectors per thread, a workgroup covering U*256 consecutive
// vectors starting at `tile`.  All U*P loads are issued before the first add.
template <int DT, int P, int U, bool NT, bool FULL>
__device__ __forceinline__ void reduce_tile(const CPtrTab& in, size_t in_vec_off, size_t tile,
                                            size_t nvec, float scale, bool do_scale,
                                            u32x4 (&out)[U]) {
  using E = Elem<DT>;
  constexpr int W = E::kPerVec;
  u32x4 v[U][P];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
    if (FULL || idx < nvec) {
#pragma unroll
      for (int p = 0; p < P; ++p) v[u][p] = load16<NT>(in.p[p], in_vec_off + idx);
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
    if (FULL || idx < nvec) {
      float acc[W];
      E::widen(v[u][0], acc);
#pragma unroll
      for (int p = 1; p < P; ++p) {
        float x[W];
        E::widen(v[u][p], x);
#pragma unroll
        for (int k = 0; k < W; ++k) acc[k] = acc[k] + x[k];
      }
      if (do_scale) {
#pragma unroll
        for (int k = 0; k < W; ++k) acc[k] = acc[k] * scale;
      }
      out[u] = E::narrow(acc);
    }
  }
}

template <int DT>
__device__ __forceinline__ float reduce_scalar(const CPtrTab& in, size_t i, int P, float scale,
                                               bool do_scale) {
  using E = Elem<DT>;
  float acc = E::load1(in.p[0], i);
  for (int p = 1; p < P; ++p) acc = acc + E::load1(in.p[p], i);
  if (do_scale) acc = acc * scale;
  return acc;
}

// ---- all_reduce ---------------------------------------------------------------
template <int DT, int P, int U, bool NT, bool PERSIST>
__global__ void __launch_bounds__(kBlock)
allreduce_vec(PtrTab bufs, size_t nvec, size_t count, float scale, int do_scale) {
  using E = Elem<DT>;
  constexpr size_t kTile = static_cast<size_t>(U) * kBlock;
  CPtrTab in;
#pragma unroll
  for (int p = 0; p < P; ++p) in.p[p] = bufs.p[p];
  size_t tile = static_cast<size_t>(blockIdx.x) * kTile;
  const size_t step = static_cast<size_t>(gridDim.x) * kTile;
  while (tile < nvec) {
    u32x4 out[U];
    const bool full = tile + kTile <= nvec;
    if (full) reduce_tile<DT, P, U, NT, true>(in, 0, tile, nvec, scale, do_scale != 0, out);
    else reduce_tile<DT, P, U, NT, false>(in, 0, tile, nvec, scale, do_scale != 0, out);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
      if (full || idx < nvec) {
#pragma unroll
        for (int p = 0; p < P; ++p) store16<NT>(bufs.p[p], idx, out[u]);
      }
    }
    if (!PERSIST) break;
    tile += step;
  }
  // elements past the last whole vector
  const size_t done = nvec * E::kPerVec;
  if (blockIdx.x == 0 && done + threadIdx.x < count) {
    const size_t i = done + threadIdx.x;
    const float y = reduce_scalar<DT>(in, i, P, scale, do_scale != 0);
#pragma unroll
    for (int p = 0; p < P; ++p) E::store1(bufs.p[p], i, y);
  }
}

template <int DT>
__global__ void __launch_bounds__(kBlock)
allreduce_scalar(PtrTab bufs, size_t count, int P, float scale, int do_scale) {
  using E = Elem<DT>;
  CPtrTab in;
  for (int p = 0; p < MCR_MAX_RANKS; ++p) in.p[p] = bufs.p[p];
  const size_t step = static_cast<size_t>(gridDim.x) * kBlock;
  for (size_t i = static_cast<size_t>(blockIdx.x) * kBlock + threadIdx.x; i < count; i += step) {
    const float y = reduce_scalar<DT>(in, i, P, scale, do_scale != 0);
    for (int p = 0; p < P; ++p) E::store1(bufs.p[p], i, y);
  }
}

// ---- reduce_scatter -----------------------------------------------------------
// blockIdx.y = destination rank r; slice r of every input is bvec vectors long.
template <int DT, int P, int U, bool NT, bool PERSIST>
__global__ void __launch_bounds__(kBlock)
reduce_scatter_vec(PtrTab out, CPtrTab in, size_t bvec, float scale, int do_scale) {
  constexpr size_t kTile = static_cast<size_t>(U) * kBlock;
  const unsigned r = blockIdx.y;
  void* dst = out.p[r];
  const size_t off = static_cast<size_t>(r) * bvec;
  size_t tile = static_cast<size_t>(blockIdx.x) * kTile;
  const size_t step = static_cast<size_t>(gridDim.x) * kTile;
  while (tile < bvec) {
    u32x4 res[U];
    const bool full = tile + kTile <= bvec;
    if (full) reduce_tile<DT, P, U, NT, true>(in, off, tile, bvec, scale, do_scale != 0, res);
    else reduce_tile<DT, P, U, NT, false>(in, off, tile, bvec, scale, do_scale != 0, res);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
      if (full || idx < bvec) store16<NT>(dst, idx, res[u]);
    }
    if (!PERSIST) break;
    tile += step;
  }
}

template <int DT>
__global__ void __launch_bounds__(kBlock)
reduce_scatter_scalar(PtrTab out, CPtrTab in, size_t b, int P, float scale, int do_scale) {
  using E = Elem<DT>;
  const unsigned r = blockIdx.y;
  void* dst = out.p[r];
  const size_t step = static_cast<size_t>(gridDim.x) * kBlock;
  for (size_t j = static_cast<size_t>(blockIdx.x) * kBlock + threadIdx.x; j < b; j += step) {
    const float y = reduce_scalar<DT>(in, static_cast<size_t>(r) * b + j, P, scale, do_scale != 0);
    E::store1(dst, j, y);
  }
}

inline unsigned scalar_grid(size_t n) {
  size_t blocks = (n + kBlock - 1) / kBlock;
  if (blocks == 0) blocks = 1;
  if (blocks > (1u << 20)) blocks = 1u << 20;   // grid-stride beyond that
  return static_cast<unsigned>(blocks);
}

}  // namespace

int launch_allreduce(mcr_ctx* ctx, const PtrTab& bufs, size_t count, int dtype, int op, int P,
                     int variant, hipStream_t stream) {
  if (count == 0) return MCR_OK;
  const float scale = 1.0f / static_cast<float>(P);
  const int do_scale = (op == MCR_AVG) ? 1 : 0;
  if (variant == SV_SCALAR) {
    return dispatch_dtype(dtype, [&](auto dt) {
      constexpr int DT = decltype(dt)::value;
      hipLaunchKernelGGL((allreduce_scalar<DT>), dim3(scalar_grid(count)), dim3(kBlock), 0, stream,
                         bufs, count, P, scale, do_scale);
      return launch_status();
    });
  }
  const size_t nvec = count / per_vec(dtype);
  const unsigned gx = grid_x(ctx, nvec, variant, 1);
  return dispatch_dtype(dtype, [&](auto dt) {
    return dispatch_ranks(P, [&](auto pp) {
      return dispatch_shape(variant, [&](auto uu, auto nt, auto ps) {
        constexpr int DT = decltype(dt)::value;
        constexpr int kP = decltype(pp)::value;
        constexpr int U = decltype(uu)::value;
        hipLaunchKernelGGL((allreduce_vec<DT, kP, U, decltype(nt)::value, decltype(ps)::value>),
                           dim3(gx), dim3(kBlock), 0, stream, bufs, nvec, count, scale, do_scale);
        return launch_status();
      });
    });
  });
}

int launch_reduce_scatter(mcr_ctx* ctx, const PtrTab& out, const CPtrTab& in, size_t count, int dtype,
                          int op, int P, int variant, hipStream_t stream) {
  if (count == 0) return MCR_OK;
  const float scale = 1.0f / static_cast<float>(P);
  const int do_scale = (op == MCR_AVG) ? 1 : 0;
  const size_t b = count / static_cast<size_t>(P);
  if (variant == SV_SCALAR) {
    return dispatch_dtype(dtype, [&](auto dt) {
      constexpr int DT = decltype(dt)::value;
      hipLaunchKernelGGL((reduce_scatter_scalar<DT>), dim3(scalar_grid(b), P), dim3(kBlock), 0, stream,
                         out, in, b, P, scale, do_scale);
      return launch_status();
    });
  }
  const size_t bvec = b / per_vec(dtype);
  const unsigned gx = grid_x(ctx, bvec, variant, P);
  return dispatch_dtype(dtype, [&](auto dt) {
    return dispatch_ranks(P, [&](auto pp) {
      return dispatch_shape(variant, [&](auto uu, auto nt, auto ps) {
        constexpr int DT = decltype(dt)::value;
        constexpr int kP = decltype(pp)::value;
        constexpr int U = decltype(uu)::value;
        hipLaunchKernelGGL((reduce_scatter_vec<DT, kP, U, decltype(nt)::value, decltype(ps)::value>),
                           dim3(gx, P), dim3(kBlock), 0, stream, out, in, bvec, scale, do_scale);
        return launch_status();
      });
    });
  });
}

}  // namespace mcr
