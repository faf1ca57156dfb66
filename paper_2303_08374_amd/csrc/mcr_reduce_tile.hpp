// The streaming sum shared by all_reduce and reduce_scatter: one tile of U*256
// consecutive 128-bit vectors, read from all P rank buffers and summed left to
// right in rank order in binary32, starting from rank 0's value (or combined with
// max / min / product, the other ReduceOps).
#pragma once
#include "mcr_dispatch.hpp"

namespace mcr {

// All U*P loads are issued before the first add, stream by stream (rank-major):
// a wavefront then asks each rank buffer for U pieces in a row, which the memory
// system serves better than a round-robin over the P buffers.
// GENERIC = false is the sum (SUM / AVG), the hot path; GENERIC = true switches on the run-time
// ReduceOp (MAX / MIN / PROD) and is compiled for fewer launch shapes.
// BS = threads of the workgroup (the stride between a thread's U vectors).
template <int DT, int P, int U, bool NTL, bool FULL, bool GENERIC, int BS = kBlock>
__device__ __forceinline__ void reduce_tile(const CPtrTab& in, size_t in_vec_off, size_t tile,
                                            size_t nvec, float scale, int op,
                                            u32x4 (&out)[U]) {
  using E = Elem<DT>;
  constexpr int W = E::kPerVec;
  u32x4 v[U][P];
#pragma unroll
  for (int p = 0; p < P; ++p) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t idx = tile + static_cast<size_t>(u) * BS + threadIdx.x;
      if (FULL || idx < nvec) v[u][p] = load16<NTL>(in.p[p], in_vec_off + idx);
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t idx = tile + static_cast<size_t>(u) * BS + threadIdx.x;
    if (FULL || idx < nvec) {
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
      out[u] = E::narrow(acc);
    }
  }
}

template <int DT>
__device__ __forceinline__ typename Elem<DT>::acc_t reduce_scalar(const CPtrTab& in, size_t i, int P, float scale,
                                                                   int op) {
  using E = Elem<DT>;
  typename E::acc_t acc = E::load1(in.p[0], i);
  for (int p = 1; p < P; ++p) acc = combine(acc, E::load1(in.p[p], i), op);
  if (op == MCR_AVG) acc = avg_step(acc, scale);
  return acc;
}


// ---- the persistent form ------------------------------------------------------------------------
// One workgroup of kPersistBlock threads per compute unit, each walking a contiguous run of the
// message in rounds: K steps of U vectors per thread are read from all P buffers and reduced into
// registers, then the K*U results are stored in one go.  Every compute unit then streams long
// contiguous runs and alternates between reading and writing them; for long messages this shape
// is on a par with the one-shot grids of small workgroups and ahead of them for some sizes
// (reduce_scatter of 32 MiB per rank at 8 ranks: 50 against 51-52 us); which one runs is the
// tuning table's choice.
// SLICED (reduce_scatter): blockIdx.y = destination rank, nvec = vectors per slice, the slice's
// results go to dst.p[blockIdx.y] from vector 0 on.  Otherwise (all_reduce / reduce): nvec = whole
// message, results go to vector idx of every dst.p[p] (of dst.p[root] when root >= 0).
constexpr int kPersistBlock = 1024;

template <int DT, int P, int U, int K, bool SLICED, bool GENERIC>
__device__ __forceinline__ void reduce_persistent(const PtrTab& dst, const CPtrTab& in, size_t nvec, float scale, int op,
                                                  int root) {
  constexpr int BS = kPersistBlock;
  constexpr size_t kStep = static_cast<size_t>(U) * BS;               // vectors per step of the workgroup
  const unsigned slice = SLICED ? blockIdx.y : 0;
  const size_t off = SLICED ? static_cast<size_t>(slice) * nvec : 0;
  const size_t steps = (nvec + kStep - 1) / kStep;
  const size_t per = (steps + gridDim.x - 1) / gridDim.x;             // steps per workgroup, contiguous
  const size_t s_begin = static_cast<size_t>(blockIdx.x) * per;
  const size_t s_end = (s_begin + per < steps) ? s_begin + per : steps;
  for (size_t s0 = s_begin; s0 < s_end; s0 += K) {
    u32x4 y[K][U];
    const bool full = s0 + K <= s_end && (s0 + K) * kStep <= nvec;    // uniform over the workgroup
    if (full) {
#pragma unroll
      for (int k = 0; k < K; ++k) reduce_tile<DT, P, U, true, true, GENERIC, BS>(in, off, (s0 + k) * kStep, nvec, scale, op, y[k]);
    } else {
#pragma unroll
      for (int k = 0; k < K; ++k)
        if (s0 + k < s_end) reduce_tile<DT, P, U, true, false, GENERIC, BS>(in, off, (s0 + k) * kStep, nvec, scale, op, y[k]);
    }
    if constexpr (SLICED) {
#pragma unroll
      for (int k = 0; k < K; ++k) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const size_t idx = (s0 + k) * kStep + static_cast<size_t>(u) * BS + threadIdx.x;
          if (full || (s0 + k < s_end && idx < nvec)) store16<true>(dst.p[slice], idx, y[k][u]);
        }
      }
    } else {
#pragma unroll
      for (int p = 0; p < P; ++p) {
        if (root >= 0 && root != p) continue;
#pragma unroll
        for (int k = 0; k < K; ++k) {
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const size_t idx = (s0 + k) * kStep + static_cast<size_t>(u) * BS + threadIdx.x;
            if (full || (s0 + k < s_end && idx < nvec)) store16<true>(dst.p[p], idx, y[k][u]);
          }
        }
      }
    }
  }
}

// Vectors per thread and step (U) and steps per round (K) of the persistent variant: the registers it
// needs (4 * U * (P + K) for loads and results) fit, next to the addressing, in the 128 a thread of
// a 1024-thread workgroup has, for every rank count.
constexpr int kPersistU = 1;
constexpr int kPersistK = 8;
inline unsigned persistent_grid(int n_cu, int slices) {
  int g = n_cu / slices;
  return static_cast<unsigned>(g < 1 ? 1 : g);
}

// log2 of the tiles per unit for units of `unit_kib` KiB and tiles of `tile_vecs` 16-byte vectors.
inline unsigned xcd_unit_shift(unsigned unit_kib, size_t tile_vecs) {
  const size_t tiles = (static_cast<size_t>(unit_kib) << 10) / (tile_vecs * 16);
  unsigned shift = 0;
  while ((size_t(2) << shift) <= tiles) ++shift;
  return shift;
}

// The one launch shape the generic-op kernels (MAX, MIN, PROD; fp16 and int32) are compiled for: two
// vectors per thread, nontemporal loads and stores, whatever vector variant was asked for.
constexpr int kGenericUnroll = 2;
constexpr int kGenericShape = SV_V2NT;

// 16-byte pieces each thread of an element-path reduction kernel works on at a time.
constexpr int kScalarUnroll = 2;

inline unsigned scalar_grid(size_t n, int per_thread = 1) {
  const size_t per_block = static_cast<size_t>(kBlock) * per_thread;
  size_t blocks = (n + per_block - 1) / per_block;
  if (blocks == 0) blocks = 1;
  if (blocks > (1u << 20)) blocks = 1u << 20;   // grid-stride beyond that
  return static_cast<unsigned>(blocks);
}

}  // namespace mcr
