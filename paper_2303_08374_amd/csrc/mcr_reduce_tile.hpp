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
template <int DT, int P, int U, bool NTL, bool FULL, bool GENERIC>
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
      const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
      if (FULL || idx < nvec) v[u][p] = load16<NTL>(in.p[p], in_vec_off + idx);
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
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


// The launch shapes the generic-op kernels are compiled for: the variant's unroll, nontemporal
// loads and stores.  f(Int<U>)
template <class F>
inline int dispatch_unroll(int variant, F&& f) {
  switch (shape_unroll(variant)) {
    case 2: return f(Int<2>{});
    case 4: return f(Int<4>{});
  }
  return f(Int<1>{});
}

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
