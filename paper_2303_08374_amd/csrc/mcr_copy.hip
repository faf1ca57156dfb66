// all_gather, all_to_all_single (equal split) and all_to_allv over P rank
// buffers in one GPU's memory (API listing of the paper).  Pure bit copies:
// each source vector is read once with a 128-bit load and stored once
// (P times for all_gather).  Bound by HBM bandwidth.
#include "mcr_dispatch.hpp"

namespace mcr {
namespace {

template <int BYTES> struct Unit;
template <> struct Unit<16> { typedef u32x4 type; };
template <> struct Unit<4> { typedef uint32_t type; };
template <> struct Unit<2> { typedef uint16_t type; };

template <bool NT, class T>
__device__ __forceinline__ T load_unit(const void* base, size_t i) {
  const T* p = reinterpret_cast<const T*>(base) + i;
  if constexpr (NT) return __builtin_nontemporal_load(p);
  return *p;
}
template <bool NT, class T>
__device__ __forceinline__ void store_unit(void* base, size_t i, T v) {
  T* p = reinterpret_cast<T*>(base) + i;
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// ---- all_gather -----------------------------------------------------------------
// Classic form.  blockIdx.y = source rank p; its m units land at offset p*m of every
// output: one load, P stores per thread.
template <int UB, int P, int U, bool NTL, bool NTS>
__global__ void __launch_bounds__(kBlock)
allgather_kernel(PtrTab out, CPtrTab in, size_t m) {
  typedef typename Unit<UB>::type T;
  constexpr size_t kTile = static_cast<size_t>(U) * kBlock;
  const unsigned p = blockIdx.y;
  const void* src = in.p[p];
  const size_t off = static_cast<size_t>(p) * m;
  const size_t step = static_cast<size_t>(gridDim.x) * kTile;
  for (size_t tile = static_cast<size_t>(blockIdx.x) * kTile; tile < m; tile += step) {
    T v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
      if (idx < m) v[u] = load_unit<NTL, T>(src, idx);
    }
#pragma unroll
    for (int r = 0; r < P; ++r) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
        if (idx < m) store_unit<NTS, T>(out.p[r], off + idx, v[u]);
      }
    }
  }
}

// Super-chunk form.  P simultaneous write streams cost the memory system more than
// one, so the message of each source is cut into super-chunks of `bpc` workgroup
// tiles, and the workgroups are numbered [source p (y)] [super-chunk] [destination
// r] [tile]: in dispatch order the chip copies one super-chunk to destination 0,
// then the same super-chunk to destination 1, ...  Re-reads of the super-chunk are
// served by the last-level cache (plain loads); the stores are nontemporal so they
// do not push it out.  HBM traffic stays at one read and P writes per unit.
__global__ void __launch_bounds__(kBlock)
allgather_superchunk_kernel(PtrTab out, CPtrTab in, size_t mvec, unsigned bpc, unsigned P) {
  const unsigned p = blockIdx.y;
  const unsigned per_sc = P * bpc;
  const size_t sc = blockIdx.x / per_sc;
  const unsigned rem = blockIdx.x - static_cast<unsigned>(sc * per_sc);
  const unsigned r = rem / bpc, j = rem - r * bpc;
  const size_t idx = (sc * bpc + j) * static_cast<size_t>(kBlock) + threadIdx.x;
  if (idx >= mvec) return;
  const u32x4 v = load16<false>(in.p[p], idx);
  store16<true>(out.p[r], static_cast<size_t>(p) * mvec + idx, v);
}

// ---- all_to_all_single, equal split ---------------------------------------------
// blockIdx.y = source p, blockIdx.z = destination r; block (p -> r) is b units.  In
// dispatch order (x, then y, then z) each output buffer is written front to back
// while the reads hop between sources: writes are the side that is sensitive to
// many interleaved streams.
template <int UB, int U, bool NTL, bool NTS>
__global__ void __launch_bounds__(kBlock)
alltoall_kernel(PtrTab out, CPtrTab in, size_t b) {
  typedef typename Unit<UB>::type T;
  constexpr size_t kTile = static_cast<size_t>(U) * kBlock;
  const unsigned p = blockIdx.y, r = blockIdx.z;
  const void* src = in.p[p];
  void* dst = out.p[r];
  const size_t soff = static_cast<size_t>(r) * b, doff = static_cast<size_t>(p) * b;
  const size_t step = static_cast<size_t>(gridDim.x) * kTile;
  for (size_t tile = static_cast<size_t>(blockIdx.x) * kTile; tile < b; tile += step) {
    T v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
      if (idx < b) v[u] = load_unit<NTL, T>(src, soff + idx);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
      if (idx < b) store_unit<NTS, T>(dst, doff + idx, v[u]);
    }
  }
}

// ---- all_to_allv -----------------------------------------------------------------
// All rows of all senders form one flat sequence in send order (sender p, then
// destination r, then row k); pair i = p*P + r owns rows [rowstart[i],
// rowstart[i+1]).  Work is dealt out over that flat sequence in units, so the
// load per workgroup is even no matter how skewed the split matrix is.  Every
// workgroup rebuilds the displacement tables in LDS from the P*P split matrix
// (host matrix passed by value, or device matrix read here: no host sync).
struct SplitArg {
  int64_t s[MCR_MAX_RANKS * MCR_MAX_RANKS];
};

struct A2AVTables {
  int64_t S[MCR_MAX_RANKS * MCR_MAX_RANKS];
  int64_t rowstart[MCR_MAX_RANKS * MCR_MAX_RANKS + 1];
  int64_t rdispl[MCR_MAX_RANKS * MCR_MAX_RANKS];
  int64_t rowsum[MCR_MAX_RANKS];
  int64_t sendbase[MCR_MAX_RANKS];
  const void* in[MCR_MAX_RANKS];
  void* out[MCR_MAX_RANKS];
};

template <bool DEV>
__device__ __forceinline__ void build_tables(A2AVTables& t, const SplitArg& hs, const int64_t* ds,
                                             const PtrTab& out, const CPtrTab& in, int P,
                                             uint64_t in_rows) {
  const int tid = threadIdx.x;
  const int PP = P * P;
  if (tid < PP) {
    // a device matrix is untrusted: negative -> 0, and no pair can carry more rows than a
    // send buffer holds, which also bounds the loop below
    int64_t s = DEV ? ds[tid] : hs.s[tid];
    if (s < 0) s = 0;
    if (static_cast<uint64_t>(s) > in_rows) s = static_cast<int64_t>(in_rows);
    t.S[tid] = s;
  }
  if (tid < P) {
    t.in[tid] = in.p[tid];
    t.out[tid] = out.p[tid];
  }
  __syncthreads();
  if (tid < P) {
    int64_t a = 0;
    for (int r = 0; r < P; ++r) a += t.S[tid * P + r];
    t.rowsum[tid] = a;
  }
  __syncthreads();
  if (tid < P) {
    int64_t a = 0;
    for (int q = 0; q < tid; ++q) a += t.rowsum[q];
    t.sendbase[tid] = a;
  }
  __syncthreads();
  if (tid < PP) {
    const int p = tid / P, r = tid % P;
    int64_t sd = 0, rd = 0;
    for (int q = 0; q < r; ++q) sd += t.S[p * P + q];
    for (int q = 0; q < p; ++q) rd += t.S[q * P + r];
    t.rowstart[tid] = t.sendbase[p] + sd;
    t.rdispl[tid] = rd;
    if (tid == PP - 1) t.rowstart[PP] = t.sendbase[p] + sd + t.S[tid];
  }
  __syncthreads();
}

// upr = units per row; shift >= 0 when upr is a power of two.
template <int UB, int U, bool NTL, bool NTS, bool DEV>
__global__ void __launch_bounds__(kBlock)
alltoallv_kernel(PtrTab out, CPtrTab in, SplitArg hs, const int64_t* ds, int P, uint32_t upr,
                 int shift, uint64_t in_rows, uint64_t out_rows) {
  typedef typename Unit<UB>::type T;
  __shared__ A2AVTables t;
  build_tables<DEV>(t, hs, ds, out, in, P, in_rows);
  const int PP = P * P;
  const uint64_t total = static_cast<uint64_t>(t.rowstart[PP]) * upr;
  constexpr uint64_t kTile = static_cast<uint64_t>(U) * kBlock;
  const uint64_t step = static_cast<uint64_t>(gridDim.x) * kTile;
  for (uint64_t tile = static_cast<uint64_t>(blockIdx.x) * kTile; tile < total; tile += step) {
    T v[U];
    void* dptr[U];
    uint64_t didx[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t idx = tile + static_cast<uint64_t>(u) * kBlock + threadIdx.x;
      ok[u] = idx < total;
      if (ok[u]) {
        uint64_t g, c;
        if (shift >= 0) {
          g = idx >> shift;
          c = idx & (upr - 1u);
        } else {
          g = idx / upr;
          c = idx - g * upr;
        }
        // last pair whose first row is <= g
        int lo = 0, hi = PP;   // invariant: rowstart[lo] <= g < rowstart[hi]
        while (hi - lo > 1) {
          const int mid = (lo + hi) >> 1;
          if (static_cast<uint64_t>(t.rowstart[mid]) <= g) lo = mid; else hi = mid;
        }
        const int p = lo / P, r = lo - p * P;
        const uint64_t srow = g - static_cast<uint64_t>(t.sendbase[p]);
        const uint64_t drow = static_cast<uint64_t>(t.rdispl[lo]) + (g - static_cast<uint64_t>(t.rowstart[lo]));
        ok[u] = srow < in_rows && drow < out_rows;
        if (ok[u]) {
          v[u] = load_unit<NTL, T>(t.in[p], srow * upr + c);
          dptr[u] = t.out[r];
          didx[u] = drow * upr + c;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (ok[u]) store_unit<NTS, T>(dptr[u], didx[u], v[u]);
    }
  }
}

inline int log2_exact(uint64_t x) {
  if (x == 0 || (x & (x - 1))) return -1;
  int s = 0;
  while ((x >> s) != 1) ++s;
  return s;
}

inline unsigned capped_blocks(size_t units, size_t per_block, size_t cap) {
  size_t blocks = (units + per_block - 1) / per_block;
  if (blocks == 0) blocks = 1;
  if (cap && blocks > cap) blocks = cap;
  return static_cast<unsigned>(blocks);
}

}  // namespace

int launch_allgather(mcr_ctx*, const PtrTab& out, const CPtrTab& in, size_t count, int dtype, int P,
                     int variant, hipStream_t stream) {
  if (count == 0) return MCR_OK;
  if (variant == SV_SCALAR) {
    const unsigned gx = capped_blocks(count, kBlock, 1u << 20);
    return dispatch_ranks(P, [&](auto pp) {
      constexpr int kP = decltype(pp)::value;
      if (dtype == MCR_F32)
        hipLaunchKernelGGL((allgather_kernel<4, kP, 1, false, false>), dim3(gx, P), dim3(kBlock), 0, stream, out, in, count);
      else
        hipLaunchKernelGGL((allgather_kernel<2, kP, 1, false, false>), dim3(gx, P), dim3(kBlock), 0, stream, out, in, count);
      return launch_status();
    });
  }
  const size_t mvec = count / per_vec(dtype);
  if (variant >= AG_SC4 && variant <= AG_SC16) {
    const size_t sc_bytes = (variant == AG_SC4 ? 4u : variant == AG_SC8 ? 8u : 16u) << 20;
    const size_t nblk = (mvec + kBlock - 1) / kBlock;                    // tiles of 4 KiB per source
    size_t bpc = sc_bytes / (kBlock * 16);
    if (bpc > nblk) bpc = nblk;
    const size_t nsc = (nblk + bpc - 1) / bpc;
    const size_t gx = nsc * bpc * static_cast<size_t>(P);
    if (gx > 0x7fffffffull) return MCR_EVARIANT;
    hipLaunchKernelGGL(allgather_superchunk_kernel, dim3(static_cast<unsigned>(gx), P), dim3(kBlock), 0, stream, out, in,
                       mvec, static_cast<unsigned>(bpc), static_cast<unsigned>(P));
    return launch_status();
  }
  const unsigned gx = grid_x(mvec, variant);
  return dispatch_ranks(P, [&](auto pp) {
    return dispatch_shape(variant, [&](auto uu, auto ntl, auto nts) {
      constexpr int kP = decltype(pp)::value;
      constexpr int U = decltype(uu)::value;
      hipLaunchKernelGGL((allgather_kernel<16, kP, U, decltype(ntl)::value, decltype(nts)::value>),
                         dim3(gx, P), dim3(kBlock), 0, stream, out, in, mvec);
      return launch_status();
    });
  });
}

int launch_alltoall(mcr_ctx*, const PtrTab& out, const CPtrTab& in, size_t count, int dtype, int P,
                    int variant, hipStream_t stream) {
  if (count == 0) return MCR_OK;
  const size_t b = count / static_cast<size_t>(P);
  if (variant == SV_SCALAR) {
    const unsigned gx = capped_blocks(b, kBlock, 1u << 16);
    if (dtype == MCR_F32)
      hipLaunchKernelGGL((alltoall_kernel<4, 1, false, false>), dim3(gx, P, P), dim3(kBlock), 0, stream, out, in, b);
    else
      hipLaunchKernelGGL((alltoall_kernel<2, 1, false, false>), dim3(gx, P, P), dim3(kBlock), 0, stream, out, in, b);
    return launch_status();
  }
  const size_t bvec = b / per_vec(dtype);
  const unsigned gx = grid_x(bvec, variant);
  return dispatch_shape(variant, [&](auto uu, auto ntl, auto nts) {
    constexpr int U = decltype(uu)::value;
    hipLaunchKernelGGL((alltoall_kernel<16, U, decltype(ntl)::value, decltype(nts)::value>),
                       dim3(gx, P, P), dim3(kBlock), 0, stream, out, in, bvec);
    return launch_status();
  });
}

int launch_alltoallv(mcr_ctx* ctx, const PtrTab& out, const CPtrTab& in, const int64_t* host_splits,
                     const int64_t* dev_splits, size_t in_rows, size_t out_rows, size_t row_bytes,
                     int elem_b, int P, int variant, hipStream_t stream) {
  SplitArg hs;
  uint64_t total_rows = 0;
  for (int i = 0; i < MCR_MAX_RANKS * MCR_MAX_RANKS; ++i) hs.s[i] = 0;
  if (host_splits) {
    for (int i = 0; i < P * P; ++i) {
      hs.s[i] = host_splits[i];
      total_rows += static_cast<uint64_t>(host_splits[i]);
    }
  } else {
    total_rows = static_cast<uint64_t>(P) * in_rows;   // upper bound; the kernel knows the real total
  }
  if (total_rows == 0 || row_bytes == 0) return MCR_OK;
  const bool dev = host_splits == nullptr;

  auto go = [&](auto ub, auto uu, auto ntl, auto nts, size_t cap) {
    constexpr int UB = decltype(ub)::value;
    constexpr int U = decltype(uu)::value;
    constexpr bool NTL = decltype(ntl)::value;
    constexpr bool NTS = decltype(nts)::value;
    const uint64_t upr = row_bytes / UB;
    const unsigned gx = capped_blocks(total_rows * upr, static_cast<size_t>(U) * kBlock, cap);
    const int shift = log2_exact(upr);
    if (dev)
      hipLaunchKernelGGL((alltoallv_kernel<UB, U, NTL, NTS, true>), dim3(gx), dim3(kBlock), 0, stream, out, in, hs,
                         dev_splits, P, static_cast<uint32_t>(upr), shift, static_cast<uint64_t>(in_rows),
                         static_cast<uint64_t>(out_rows));
    else
      hipLaunchKernelGGL((alltoallv_kernel<UB, U, NTL, NTS, false>), dim3(gx), dim3(kBlock), 0, stream, out, in, hs,
                         dev_splits, P, static_cast<uint32_t>(upr), shift, static_cast<uint64_t>(in_rows),
                         static_cast<uint64_t>(out_rows));
    return launch_status();
  };
  if (variant == SV_SCALAR) {
    const size_t cap = static_cast<size_t>(ctx->num_cus) * 32;
    if (elem_b == 4) return go(Int<4>{}, Int<1>{}, Bool<false>{}, Bool<false>{}, cap);
    return go(Int<2>{}, Int<1>{}, Bool<false>{}, Bool<false>{}, cap);
  }
  return dispatch_shape(variant, [&](auto uu, auto ntl, auto nts) { return go(Int<16>{}, uu, ntl, nts, size_t(1) << 30); });
}

}  // namespace mcr
