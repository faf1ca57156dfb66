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

// One linear copy of n units of UB bytes from src to dst, shared by the workgroups along x
// (blockIdx.x strides over tiles).  UB = 16: aligned 128-bit accesses, U per thread in flight.
// UB < 16 is the element path (addresses aligned to the element only, any length): still 16 bytes
// per access, at whatever address the element falls on -- the hardware serves unaligned global
// accesses, and 64 lanes x 2 bytes per instruction is what made this path 2-3 times slower than
// the aligned one -- with the nontemporal hint both ways (what the tuning suite picks for the
// aligned copies from a few MiB up), and the n mod (16 / UB) elements behind the last whole 16
// bytes one by one.
template <int UB, int U>
__device__ constexpr uint64_t run_tile_units() {
  return static_cast<uint64_t>(U) * kBlock * (16 / UB);
}
template <int UB, int U, bool NTL, bool NTS>
__device__ __forceinline__ void copy_run(const typename Unit<UB>::type* src, typename Unit<UB>::type* dst, uint64_t n) {
  constexpr uint64_t kTile = static_cast<uint64_t>(U) * kBlock;          // 16-byte pieces per tile
  if constexpr (UB == 16) {
    const uint64_t step = static_cast<uint64_t>(gridDim.x) * kTile;
    for (uint64_t tile = static_cast<uint64_t>(blockIdx.x) * kTile; tile < n; tile += step) {
      u32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint64_t idx = tile + static_cast<uint64_t>(u) * kBlock + threadIdx.x;
        if (idx < n) v[u] = load_unit<NTL, u32x4>(src, idx);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint64_t idx = tile + static_cast<uint64_t>(u) * kBlock + threadIdx.x;
        if (idx < n) store_unit<NTS, u32x4>(dst, idx, v[u]);
      }
    }
  } else {
    constexpr uint64_t kPer = 16 / UB;
    const uint64_t nv = n / kPer;
    const char* s = reinterpret_cast<const char*>(src);
    char* d = reinterpret_cast<char*>(dst);
    const uint64_t step = static_cast<uint64_t>(gridDim.x) * kTile;
    for (uint64_t tile = static_cast<uint64_t>(blockIdx.x) * kTile; tile < nv; tile += step) {
      u32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint64_t idx = tile + static_cast<uint64_t>(u) * kBlock + threadIdx.x;
        if (idx < nv) v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_elem_aligned*>(s + 16 * idx));
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint64_t idx = tile + static_cast<uint64_t>(u) * kBlock + threadIdx.x;
        if (idx < nv) __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4_elem_aligned*>(d + 16 * idx));
      }
    }
    const uint64_t e = nv * kPer + threadIdx.x;
    if (blockIdx.x == 0 && e < n) dst[e] = src[e];
  }
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
  if constexpr (UB == 2) {
    // element path on 2-byte elements: 16 bytes per access at element-aligned addresses (see
    // copy_run), then the m mod 8 elements behind the last whole 16 bytes.  (4-byte elements are
    // faster one element per lane here: 805 against 899 us for 64 MiB per rank.)
    constexpr size_t kPer = 16 / UB;
    const size_t nv = m / kPer;
    for (size_t tile = static_cast<size_t>(blockIdx.x) * kTile; tile < nv; tile += step) {
      u32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
        if (idx < nv) v[u] = load16_unaligned(src, idx * 16);
      }
#pragma unroll
      for (int r = 0; r < P; ++r) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const size_t idx = tile + static_cast<size_t>(u) * kBlock + threadIdx.x;
          if (idx < nv) store16_unaligned(out.p[r], off * UB + idx * 16, v[u]);
        }
      }
    }
    const size_t e = nv * kPer + threadIdx.x;
    if (blockIdx.x == 0 && e < m) {
      const T x = static_cast<const T*>(src)[e];
#pragma unroll
      for (int r = 0; r < P; ++r) static_cast<T*>(out.p[r])[off + e] = x;
    }
    return;
  }
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
allgather_superchunk_kernel(PtrTab out, CPtrTab in, size_t mvec, unsigned bpc, unsigned P, unsigned unit_shift) {
  const unsigned p = blockIdx.y;
  const unsigned per_sc = P * bpc;
  const size_t sc = blockIdx.x / per_sc;
  const unsigned rem = blockIdx.x - static_cast<unsigned>(sc * per_sc);
  const unsigned r = rem / bpc;
  unsigned j = rem - r * bpc;
  // "sc16x": the workgroups of one XCD cover contiguous units of 1 << unit_shift tiles instead of every
  // eighth tile.  Still the same XCD for a tile whatever the destination (bpc is a multiple of the
  // group of 8 units), so the re-reads find it in that XCD's L2.
  if (unit_shift) j = xcd_unit_renumber(j, unit_shift);
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
  const unsigned p = blockIdx.y, r = blockIdx.z;
  copy_run<UB, U, NTL, NTS>(static_cast<const T*>(in.p[p]) + static_cast<size_t>(r) * b,
                            static_cast<T*>(out.p[r]) + static_cast<size_t>(p) * b, b);
}

// "flat": blockIdx.y = destination r; the threads are numbered along out[r], U vectors each, and
// every vector is fetched from the block of the source it belongs to (p = index / b).  A block
// shorter than a workgroup then costs no idle lanes, and out[r] is written front to back.
// BS = threads per workgroup.  LDS: the U vectors of every thread go through LDS between the
// workgroup's loads and its stores (a read phase and a write phase per workgroup).
template <int BS, int U, bool LDS>
__global__ void __launch_bounds__(BS)
alltoall_flat_kernel(PtrTab out, CPtrTab in, uint32_t b, uint32_t P) {
  __shared__ u32x4 stage[LDS ? U * BS : 1];
  const unsigned r = blockIdx.y;
  const uint64_t n = static_cast<uint64_t>(b) * P;                       // vectors of one output
  const uint64_t first = static_cast<uint64_t>(blockIdx.x) * (U * BS) + threadIdx.x;
  u32x4 v[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint64_t i = first + static_cast<uint64_t>(u) * BS;
    if (i < n) {
      const uint32_t p = static_cast<uint32_t>(i / b);
      const uint64_t k = i - static_cast<uint64_t>(p) * b;
      v[u] = load16<true>(in.p[p], static_cast<uint64_t>(r) * b + k);
    }
  }
  if constexpr (LDS) {
#pragma unroll
    for (int u = 0; u < U; ++u) stage[u * BS + threadIdx.x] = v[u];
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = stage[u * BS + threadIdx.x];
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint64_t i = first + static_cast<uint64_t>(u) * BS;
    if (i < n) store16<true>(out.p[r], i, v[u]);
  }
}

// ---- all_to_allv -----------------------------------------------------------------
// blockIdx.y = sender p, blockIdx.z = receiver r, blockIdx.x = tile of the pair's
// rows.  With packed displacements the rows of one pair are contiguous on both
// sides, so a pair is a plain linear copy of S[p][r]*upr units from
//   in[p]  + sdispl[p][r]*upr    (sdispl = sum of row p of S left of r)
// to out[r] + rdispl[r][p]*upr   (rdispl = sum of column r of S above p),
// A host matrix is turned into a table of pair lengths and displacements on the
// host (alltoallv_pairs_kernel below).  For a matrix in device memory (no host
// sync) every workgroup derives its two displacements itself from at most
// 2*(P-1) entries of S: no table, no search, no division per thread.
// In dispatch order the chip walks one pair after the other: one read stream
// and one write stream at a time.  Skew costs nothing but workgroups that find
// their tile beyond the pair's end and leave at once; pairs longer than the
// grid are covered by striding.  gather(v), scatter(v), all_gatherv and bcast
// are this kernel with a one-column, one-row or row-constant split matrix.
struct SplitArg {
  int64_t s[MCR_MAX_RANKS * MCR_MAX_RANKS];
};

// A split entry as the kernel uses it: a device matrix is untrusted, so negative
// counts as 0 and nothing exceeds the rows a send buffer holds.
__device__ __forceinline__ uint64_t clamp_split(int64_t s, uint64_t in_rows) {
  if (s < 0) return 0;
  return static_cast<uint64_t>(s) > in_rows ? in_rows : static_cast<uint64_t>(s);
}

// `tr` (device matrix only): the matrix is read transposed, entry (p, r) is ds[r * P + p].
template <int UB, int U, bool NTL, bool NTS, bool DEV>
__global__ void __launch_bounds__(kBlock)
alltoallv_kernel(PtrTab out, CPtrTab in, SplitArg hs, const int64_t* ds, int P, uint64_t upr,
                 uint64_t in_rows, uint64_t out_rows, int same_src, int tr) {
  typedef typename Unit<UB>::type T;
  constexpr uint64_t kTile = run_tile_units<UB, U>();
  const int p = blockIdx.y, r = blockIdx.z;
  const int64_t* S = DEV ? ds : hs.s;
  // strides of the sender and the receiver index in the matrix as stored
  const int sp = (DEV && tr) ? 1 : P, sr = (DEV && tr) ? P : 1;
  uint64_t rows, sdispl = 0, rdispl = 0;
  if constexpr (DEV) {
    // One memory round trip for everything the workgroup needs from the matrix: lane q of every
    // wavefront loads the q-th entry of row p and of column r, both loads go out together; the
    // pair's own length is lane r's row entry, the two displacements are the sums over the lanes
    // below r (row) and below p (column), added up by a butterfly over the 16 lanes.  (A loop of
    // uniform loads costs one round trip per entry, up to 2 * (P - 1) of them in a row.)
    // same_src: every receiver gets the sender's rows from row 0 on (all_gatherv, bcast)
    const int lane = static_cast<int>(__lane_id());
    uint64_t row_e = 0, col_e = 0;
    if (lane < P) {
      row_e = clamp_split(ds[p * sp + lane * sr], in_rows);
      col_e = clamp_split(ds[lane * sp + r * sr], in_rows);
    }
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<uint32_t>(row_e), r);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<uint32_t>(row_e >> 32), r);
    rows = (static_cast<uint64_t>(hi) << 32) | lo;
    if (static_cast<uint64_t>(blockIdx.x) * kTile >= rows * upr) return;    // the common early exit
    uint64_t a = (!same_src && lane < r) ? row_e : 0, b = lane < p ? col_e : 0;
#pragma unroll
    for (int d = MCR_MAX_RANKS / 2; d >= 1; d >>= 1) {
      a += __shfl_xor(static_cast<unsigned long long>(a), d);
      b += __shfl_xor(static_cast<unsigned long long>(b), d);
    }
    sdispl = (static_cast<uint64_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32))) << 32) |
             __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
    rdispl = (static_cast<uint64_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b >> 32))) << 32) |
             __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b));
  } else {
    // a host matrix normally goes through the pair-table kernel; this is the fallback for pairs too
    // long for its 32-bit offsets
    rows = clamp_split(S[p * P + r], in_rows);
    if (static_cast<uint64_t>(blockIdx.x) * kTile >= rows * upr) return;
    if (!same_src)
      for (int q = 0; q < r; ++q) sdispl += clamp_split(S[p * P + q], in_rows);
    for (int q = 0; q < p; ++q) rdispl += clamp_split(S[q * P + r], in_rows);
  }
  // rows that would leave either buffer are not copied
  if (sdispl >= in_rows || rdispl >= out_rows) return;
  if (rows > in_rows - sdispl) rows = in_rows - sdispl;
  if (rows > out_rows - rdispl) rows = out_rows - rdispl;
  copy_run<UB, U, NTL, NTS>(static_cast<const T*>(in.p[p]) + sdispl * upr, static_cast<T*>(out.p[r]) + rdispl * upr,
                            rows * upr);
}

// all_to_allv with displacements chosen by the caller: the host has checked every pair against
// the buffer extents and passes, per (sender p, receiver r), the pair's length and its two
// offsets in units of UB bytes.  Same grid and copy loop as above.
struct PairArg {
  uint32_t cnt[MCR_MAX_RANKS * MCR_MAX_RANKS];
  uint32_t sd[MCR_MAX_RANKS * MCR_MAX_RANKS];   // offset in in[p]
  uint32_t rd[MCR_MAX_RANKS * MCR_MAX_RANKS];   // offset in out[r], also indexed [p*P + r]
};

template <int UB, int U, bool NTL, bool NTS>
__global__ void __launch_bounds__(kBlock)
alltoallv_pairs_kernel(PtrTab out, CPtrTab in, PairArg a, int P) {
  typedef typename Unit<UB>::type T;
  constexpr uint64_t kTile = run_tile_units<UB, U>();
  const int p = blockIdx.y, r = blockIdx.z;
  const int i = p * P + r;
  const uint64_t n = a.cnt[i];
  if (static_cast<uint64_t>(blockIdx.x) * kTile >= n) return;
  copy_run<UB, U, NTL, NTS>(static_cast<const T*>(in.p[p]) + a.sd[i], static_cast<T*>(out.p[r]) + a.rd[i], n);
}

// Every sender hands the *same* segment to all of its receivers (bcast, all_gatherv): pair by pair,
// each receiver's copy of a segment longer than the caches keep would fetch it from memory again, and
// with loads that bypass the cache a short one too.  Super-chunk order as in all_gather: workgroups numbered
// [sender slot (y)] [super-chunk] [receiver] [tile], plain loads so that the re-reads of a
// super-chunk hit the cache, nontemporal stores so that they do not push it out.  The host resolves
// every address and lists, per sender that sends anything, its receivers without gaps, so that the
// grid holds no sender plane and no receiver plane that has nothing to do (a bcast to 7 of 8 ranks
// with an idle plane for the root itself: 6.09 against 6.22 TB/s at 256 MiB).
struct SharedSegments {
  const u32x4* src[MCR_MAX_RANKS];                       // by sender slot: start of the segment
  u32x4* dst[MCR_MAX_RANKS * MCR_MAX_RANKS];             // [slot * MCR_MAX_RANKS + k]: the sender's k-th receiver, null behind the last
  uint32_t cnt[MCR_MAX_RANKS];                           // by sender slot: 16-byte units of the segment
};

__global__ void __launch_bounds__(kBlock)
alltoallv_pairs_superchunk_kernel(SharedSegments a, unsigned bpc, unsigned R, unsigned unit_shift) {
  const unsigned y = blockIdx.y;
  const unsigned per_sc = R * bpc;                       // R: the most receivers any sender has
  const size_t sc = blockIdx.x / per_sc;
  const unsigned rem = blockIdx.x - static_cast<unsigned>(sc * per_sc);
  const unsigned r = rem / bpc;
  unsigned j = rem - r * bpc;
  if (unit_shift) j = xcd_unit_renumber(j, unit_shift);   // contiguous units per XCD, as in all_gather's "sc16x"
  const u32x4* src = a.src[y];
  u32x4* dst = a.dst[y * MCR_MAX_RANKS + r];
  const size_t idx = (sc * bpc + j) * static_cast<size_t>(kBlock) + threadIdx.x;
  if (idx >= a.cnt[y] || !dst) return;
  store16<true>(dst, idx, load16<false>(src, idx));
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
    // one piece (a 4-byte element, or 16 bytes of 2-byte elements) per thread: with P stores behind
    // every load, more per thread are slower here
    const unsigned gx = capped_blocks(elem_bytes(dtype) == 4 ? count : count / 8, kBlock, 1u << 20);
    return dispatch_ranks(P, [&](auto pp) {
      constexpr int kP = decltype(pp)::value;
      if (elem_bytes(dtype) == 4)
        hipLaunchKernelGGL((allgather_kernel<4, kP, 1, false, false>), dim3(gx, P), dim3(kBlock), 0, stream, out, in, count);
      else
        hipLaunchKernelGGL((allgather_kernel<2, kP, 1, false, false>), dim3(gx, P), dim3(kBlock), 0, stream, out, in, count);
      return launch_status();
    });
  }
  const size_t mvec = count / per_vec(dtype);
  if (variant >= AG_SC4 && variant <= AG_SC16X) {
    const size_t sc_bytes = (variant == AG_SC4 ? 4u : variant == AG_SC8 ? 8u : 16u) << 20;
    const size_t nblk = (mvec + kBlock - 1) / kBlock;                    // tiles of 4 KiB per source
    size_t bpc = sc_bytes / (kBlock * 16);
    if (bpc > nblk) bpc = nblk;
    const size_t nsc = (nblk + bpc - 1) / bpc;
    const size_t gx = nsc * bpc * static_cast<size_t>(P);
    if (gx > 0x7fffffffull) return MCR_EVARIANT;
    // "sc16x": units of 512 KiB per XCD (2.92 against 3.01 ms at 256 MiB per rank, P=8; units of 64 or
    // 128 KiB are a third slower, 1 MiB the same); needs super-chunks made of whole groups
    unsigned unit_shift = variant == AG_SC16X ? 7u : 0u;
    if (bpc % (8u << unit_shift) != 0) unit_shift = 0;
    hipLaunchKernelGGL(allgather_superchunk_kernel, dim3(static_cast<unsigned>(gx), P), dim3(kBlock), 0, stream, out, in,
                       mvec, static_cast<unsigned>(bpc), static_cast<unsigned>(P), unit_shift);
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
    const unsigned gx = capped_blocks(b, kBlock * (16 / elem_bytes(dtype)), 1u << 16);   // tiles of 256 16-byte pieces
    if (elem_bytes(dtype) == 4)
      hipLaunchKernelGGL((alltoall_kernel<4, 1, false, false>), dim3(gx, P, P), dim3(kBlock), 0, stream, out, in, b);
    else
      hipLaunchKernelGGL((alltoall_kernel<2, 1, false, false>), dim3(gx, P, P), dim3(kBlock), 0, stream, out, in, b);
    return launch_status();
  }
  const size_t bvec = b / per_vec(dtype);
  // blocks too long for the 32-bit arithmetic of the flat forms run "v1nt" in their place
  if ((variant == A2A_FLAT || variant == A2A_W64 || variant == A2A_LDS) && bvec * static_cast<size_t>(P) > (size_t(1) << 36))
    variant = SV_V1NT;
  if (variant == A2A_FLAT || variant == A2A_W64 || variant == A2A_LDS) {
    const uint64_t n = static_cast<uint64_t>(bvec) * P;
    const uint32_t b32 = static_cast<uint32_t>(bvec), P32 = static_cast<uint32_t>(P);
    if (variant == A2A_FLAT)
      hipLaunchKernelGGL((alltoall_flat_kernel<kBlock, 1, false>), dim3(static_cast<unsigned>((n + kBlock - 1) / kBlock), P), dim3(kBlock), 0,
                         stream, out, in, b32, P32);
    else if (variant == A2A_W64)
      hipLaunchKernelGGL((alltoall_flat_kernel<kWave, 1, false>), dim3(static_cast<unsigned>((n + kWave - 1) / kWave), P), dim3(kWave), 0,
                         stream, out, in, b32, P32);
    else
      hipLaunchKernelGGL((alltoall_flat_kernel<kBlock, 4, true>), dim3(static_cast<unsigned>((n + 4 * kBlock - 1) / (4 * kBlock)), P),
                         dim3(kBlock), 0, stream, out, in, b32, P32);
    return launch_status();
  }
  const unsigned gx = grid_x(bvec, variant);
  return dispatch_shape(variant, [&](auto uu, auto ntl, auto nts) {
    constexpr int U = decltype(uu)::value;
    hipLaunchKernelGGL((alltoall_kernel<16, U, decltype(ntl)::value, decltype(nts)::value>),
                       dim3(gx, P, P), dim3(kBlock), 0, stream, out, in, bvec);
    return launch_status();
  });
}

int launch_alltoallv(mcr_ctx*, const PtrTab& out, const CPtrTab& in, const int64_t* host_splits,
                     const int64_t* dev_splits, size_t in_rows, size_t out_rows, size_t row_bytes,
                     int elem_b, int P, int same_src, bool dev_transposed, int variant, hipStream_t stream) {
  const int tr = dev_transposed ? 1 : 0;
  SplitArg hs;
  for (int i = 0; i < MCR_MAX_RANKS * MCR_MAX_RANKS; ++i) hs.s[i] = 0;
  // rows of the longest pair: exact for a host matrix, the buffer bound for a device one
  uint64_t max_pair = 0;
  if (host_splits) {
    for (int i = 0; i < P * P; ++i) {
      hs.s[i] = host_splits[i];
      if (static_cast<uint64_t>(host_splits[i]) > max_pair) max_pair = static_cast<uint64_t>(host_splits[i]);
    }
  } else {
    max_pair = in_rows < out_rows ? in_rows : out_rows;
  }
  if (max_pair == 0 || row_bytes == 0) return MCR_OK;
  const bool dev = host_splits == nullptr;
  if (!dev) {
    // a host matrix: the displacements are worked out here and handed to the pair-table kernel,
    // so that no workgroup computes a prefix sum; rows that would leave either buffer are clipped
    const uint64_t upr = row_bytes / (variant == SV_SCALAR ? static_cast<size_t>(elem_b) : 16);
    uint32_t cnt[MCR_MAX_RANKS * MCR_MAX_RANKS], sd[MCR_MAX_RANKS * MCR_MAX_RANKS], rd[MCR_MAX_RANKS * MCR_MAX_RANKS];
    bool fits = true;
    uint64_t col[MCR_MAX_RANKS] = {0};
    for (int p = 0; p < P && fits; ++p) {
      uint64_t run = 0;
      for (int r = 0; r < P; ++r) {
        const int i = p * P + r;
        uint64_t rows = static_cast<uint64_t>(host_splits[i]);
        const uint64_t from = same_src ? 0 : run, to = col[r];
        run += rows;
        col[r] += rows;
        if (from >= in_rows || to >= out_rows) rows = 0;
        if (rows > in_rows - from) rows = in_rows - from;
        if (rows > out_rows - to) rows = out_rows - to;
        const uint64_t c = rows * upr, s = rows ? from * upr : 0, d = rows ? to * upr : 0;
        if (c > 0xffffffffull || s > 0xffffffffull || d > 0xffffffffull) { fits = false; break; }
        cnt[i] = static_cast<uint32_t>(c);
        sd[i] = static_cast<uint32_t>(s);
        rd[i] = static_cast<uint32_t>(d);
      }
    }
    if (fits) return launch_alltoallv_pairs(nullptr, out, in, cnt, sd, rd, elem_b, P, variant, stream);
  }

  auto go = [&](auto ub, auto uu, auto ntl, auto nts) {
    constexpr int UB = decltype(ub)::value;
    constexpr int U = decltype(uu)::value;
    constexpr bool NTL = decltype(ntl)::value;
    constexpr bool NTS = decltype(nts)::value;
    const uint64_t upr = row_bytes / UB;
    // a device matrix usually fills a fraction of the bound: cap the tiles per pair, longer pairs stride
    const unsigned gx = capped_blocks(max_pair * upr, static_cast<size_t>(U) * kBlock * (16 / UB), dev ? 256 : 65535 * 16);
    if (dev)
      hipLaunchKernelGGL((alltoallv_kernel<UB, U, NTL, NTS, true>), dim3(gx, P, P), dim3(kBlock), 0, stream, out, in,
                         hs, dev_splits, P, upr, static_cast<uint64_t>(in_rows), static_cast<uint64_t>(out_rows), same_src, tr);
    else
      hipLaunchKernelGGL((alltoallv_kernel<UB, U, NTL, NTS, false>), dim3(gx, P, P), dim3(kBlock), 0, stream, out, in,
                         hs, dev_splits, P, upr, static_cast<uint64_t>(in_rows), static_cast<uint64_t>(out_rows), same_src, tr);
    return launch_status();
  };
  if (variant == SV_SCALAR) {
    if (elem_b == 4) return go(Int<4>{}, Int<4>{}, Bool<false>{}, Bool<false>{});
    return go(Int<2>{}, Int<4>{}, Bool<false>{}, Bool<false>{});
  }
  return dispatch_shape(variant, [&](auto uu, auto ntl, auto nts) { return go(Int<16>{}, uu, ntl, nts); });
}

// cnt / sd / rd: P*P entries each, [p*P + r], in units of 16 bytes (vector variants) or of one
// element (SV_SCALAR); the caller has checked them against the buffers.
int launch_alltoallv_pairs(mcr_ctx*, const PtrTab& out, const CPtrTab& in, const uint32_t* cnt, const uint32_t* sd,
                           const uint32_t* rd, int elem_b, int P, int variant, hipStream_t stream) {
  PairArg a;
  uint32_t longest = 0;
  for (int i = 0; i < MCR_MAX_RANKS * MCR_MAX_RANKS; ++i) {
    const bool live = i < P * P;
    a.cnt[i] = live ? cnt[i] : 0;
    a.sd[i] = live ? sd[i] : 0;
    a.rd[i] = live ? rd[i] : 0;
    if (a.cnt[i] > longest) longest = a.cnt[i];
  }
  if (longest == 0) return MCR_OK;
  // One segment per sender, sent to two receivers or more: super-chunk order, so that the segment
  // is fetched from memory once (the variant's hints and unroll do not apply to it).  A segment
  // of up to 16 MiB is one super-chunk.
  constexpr uint32_t kSuperChunkVecs = (16u << 20) / 16;
  if (variant != SV_SCALAR) {
    SharedSegments seg;
    for (int q = 0; q < MCR_MAX_RANKS; ++q) { seg.src[q] = nullptr; seg.cnt[q] = 0; }
    for (int q = 0; q < MCR_MAX_RANKS * MCR_MAX_RANKS; ++q) seg.dst[q] = nullptr;
    unsigned n_senders = 0, most = 0;
    bool shared = true, fanout = false;
    for (int p = 0; p < P && shared; ++p) {
      int first = -1, live = 0;
      for (int r = 0; r < P; ++r) {
        const int i = p * P + r;
        if (a.cnt[i] == 0) continue;
        if (first < 0) first = i;
        else if (a.cnt[i] != a.cnt[first] || a.sd[i] != a.sd[first]) shared = false;
        seg.dst[n_senders * MCR_MAX_RANKS + live] = static_cast<u32x4*>(out.p[r]) + a.rd[i];
        ++live;
      }
      if (live > 0) {
        seg.src[n_senders] = static_cast<const u32x4*>(in.p[p]) + a.sd[first];
        seg.cnt[n_senders] = a.cnt[first];
        ++n_senders;
      }
      if (live > 1) fanout = true;
      if (static_cast<unsigned>(live) > most) most = static_cast<unsigned>(live);
    }
    if (shared && fanout) {
      const size_t nblk = (static_cast<size_t>(longest) + kBlock - 1) / kBlock;
      // tiles per super-chunk: a multiple of the 8 XCDs, so that every receiver's copy of a tile runs
      // on the XCD whose L2 holds it
      size_t bpc = (nblk + 7) / 8 * 8;
      if (bpc > kSuperChunkVecs / kBlock) bpc = kSuperChunkVecs / kBlock;
      const size_t nsc = (nblk + bpc - 1) / bpc;
      const size_t gx = nsc * bpc * static_cast<size_t>(most);
      if (gx <= 0x7fffffffull) {
        const unsigned unit_shift = bpc % (8u << 7) == 0 ? 7u : 0u;
        hipLaunchKernelGGL(alltoallv_pairs_superchunk_kernel, dim3(static_cast<unsigned>(gx), n_senders), dim3(kBlock), 0,
                           stream, seg, static_cast<unsigned>(bpc), most, unit_shift);
        return launch_status();
      }
    }
  }
  // The grid's sender and receiver planes: only ranks that send, and only ranks that receive,
  // anything at all (gather has one receiver, scatter one sender: with all P x P planes 7 of 8
  // workgroups would find an empty pair, and an idle workgroup is not free: it waits for its
  // pair's length before it can leave).  The tables are repacked accordingly here on the host.
  int sl[MCR_MAX_RANKS], rl[MCR_MAX_RANKS], ns = 0, nr = 0;
  for (int q = 0; q < P; ++q) {
    bool sends = false, receives = false;
    for (int k = 0; k < P; ++k) {
      sends = sends || a.cnt[q * P + k] != 0;
      receives = receives || a.cnt[k * P + q] != 0;
    }
    if (sends) sl[ns++] = q;
    if (receives) rl[nr++] = q;
  }
  PairArg c;
  PtrTab out_c;
  CPtrTab in_c;
  for (int i = 0; i < MCR_MAX_RANKS * MCR_MAX_RANKS; ++i) c.cnt[i] = c.sd[i] = c.rd[i] = 0;
  for (int q = 0; q < MCR_MAX_RANKS; ++q) {
    in_c.p[q] = q < ns ? in.p[sl[q]] : nullptr;
    out_c.p[q] = q < nr ? out.p[rl[q]] : nullptr;
  }
  for (int y = 0; y < ns; ++y)
    for (int z = 0; z < nr; ++z) {
      const int from = sl[y] * P + rl[z], to = y * P + z;
      c.cnt[to] = a.cnt[from];
      c.sd[to] = a.sd[from];
      c.rd[to] = a.rd[from];
    }
  auto go = [&](auto ub, auto uu, auto ntl, auto nts) {
    constexpr int UB = decltype(ub)::value;
    constexpr int U = decltype(uu)::value;
    const unsigned gx = capped_blocks(longest, static_cast<size_t>(U) * kBlock * (16 / UB), 65535 * 16);
    hipLaunchKernelGGL((alltoallv_pairs_kernel<UB, U, decltype(ntl)::value, decltype(nts)::value>), dim3(gx, ns, nr),
                       dim3(kBlock), 0, stream, out_c, in_c, c, P);
    return launch_status();
  };
  if (variant == SV_SCALAR) {
    if (elem_b == 4) return go(Int<4>{}, Int<4>{}, Bool<false>{}, Bool<false>{});
    return go(Int<2>{}, Int<4>{}, Bool<false>{}, Bool<false>{});
  }
  return dispatch_shape(variant, [&](auto uu, auto ntl, auto nts) { return go(Int<16>{}, uu, ntl, nts); });
}

}  // namespace mcr
