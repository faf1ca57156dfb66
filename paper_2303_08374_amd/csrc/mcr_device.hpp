// Device-side helpers shared by the gfx950 kernels: 128-bit access types, bf16
// widening / rounding, the rank pointer table.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mcr.h"

namespace mcr {

constexpr int kBlock = 256;   // 4 wavefronts of 64 lanes
constexpr int kWave = 64;
// Row gathers behind a lookup (unpack, combine) on rows wider than half a workgroup: workgroup size
// and 16-byte units each thread keeps in flight.
constexpr int kRowGatherBlock = 128;
constexpr int kRowGatherVecs = 2;
// The fused dispatch that finds a row's place from the split matrix, one row per workgroup.  Every
// wavefront of a workgroup walks the whole lookup chain on the scalar unit, and with a chain as long
// as this kernel's (and half of the workgroups carrying a dropped token and nothing else) that, not
// the memory system, is what the rate hangs on: one wavefront per row runs it once per row
// (187 against 220 us on the MoE workload).  The kernels with a short chain (pack, the table-driven
// dispatch) are faster with a whole workgroup of 256 threads per row.
constexpr int kPairScatterBlock = 64;
constexpr int kPairScatterVecs = 4;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Rank pointer table, passed by value as a kernel argument (16 x 8 bytes).
struct PtrTab {
  void* p[MCR_MAX_RANKS];
};
struct CPtrTab {
  const void* p[MCR_MAX_RANKS];
};

// Displacements of an all_to_allv with packed blocks, worked out once per call from a split matrix
// in device memory for the kernels that place single rows (the fused MoE dispatch / combine).  For
// sender p, with sd[r] = rows it packs before its block for receiver r and rd[r] = first row of its
// block in receiver r's buffer:
//   start[p][r] = min(sd[r], 2^31 - 1) for r < P, the largest int32 for P <= r < 16, and
//   start[p][16] = min(all the rows p sends, 2^31 - 1): a slot is below 2^31 - 1, so the receiver of
//                  a slot is found with 32-bit compares and no bound on r;
//   delta[p][r] = rd[r] - sd[r]: slot s of sender p lands in row s + delta[p][r] of receiver r.
// Workgroups are dealt to the 8 XCDs in turn.  Index `i` renumbered within its group of
// 8 << unit_shift so that the eight residues mod 8 (the XCDs) each cover a contiguous unit of
// 1 << unit_shift indices: a bijection of every whole group onto itself.
__device__ __forceinline__ unsigned xcd_unit_renumber(unsigned i, unsigned unit_shift) {
  const unsigned span = 8u << unit_shift;
  const unsigned within = i & (span - 1);
  return (i - within) + ((within & 7u) << unit_shift) + (within >> 3);
}
// The tile of workgroup `bx` of a one-dimensional walk: with unit_shift != 0 the tiles of every whole
// group of 8 << unit_shift workgroups are renumbered in XCD units (a partial group at the end of the
// grid keeps its numbering).
__device__ __forceinline__ unsigned xcd_unit_tile(unsigned bx, unsigned unit_shift) {
  if (unit_shift && (bx | ((8u << unit_shift) - 1)) < gridDim.x) return xcd_unit_renumber(bx, unit_shift);
  return bx;
}
struct PairSlot {
  int32_t start[MCR_MAX_RANKS][32];
  int64_t delta[MCR_MAX_RANKS][MCR_MAX_RANKS];
};

// 128-bit global access.  NT = nontemporal (streaming) hint.
template <bool NT>
__device__ __forceinline__ u32x4 load16(const void* base, size_t vec_index) {
  const u32x4* p = reinterpret_cast<const u32x4*>(base) + vec_index;
  if constexpr (NT) return __builtin_nontemporal_load(p);
  return *p;
}
template <bool NT>
__device__ __forceinline__ void store16(void* base, size_t vec_index, u32x4 v) {
  u32x4* p = reinterpret_cast<u32x4*>(base) + vec_index;
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// 128-bit global access at an address that is aligned to the element only (the element paths):
// the hardware serves unaligned global accesses, so this is still one instruction.
__device__ __forceinline__ u32x4 load16_unaligned(const void* base, size_t byte_offset) {
  u32x4 v;
  __builtin_memcpy(&v, static_cast<const char*>(base) + byte_offset, 16);
  return v;
}
__device__ __forceinline__ void store16_unaligned(void* base, size_t byte_offset, u32x4 v) {
  __builtin_memcpy(static_cast<char*>(base) + byte_offset, &v, 16);
}

// A row of a row kernel as `pieces` 16-byte pieces followed by a tail shorter than 16 bytes.  AL:
// the row starts on a 16-byte boundary and has no tail (cache hints apply); otherwise the pieces
// sit at element-aligned addresses, which the hardware serves as one access all the same, so a
// row of 4104 bytes moves as fast as one of 4096.
typedef u32x4 u32x4_elem_aligned __attribute__((aligned(2)));       // 16 bytes at an address aligned to the element only
template <bool NT, bool AL>
__device__ __forceinline__ u32x4 load_piece(const void* row, uint32_t c) {
  if constexpr (AL) return load16<NT>(row, c);
  const u32x4_elem_aligned* p = reinterpret_cast<const u32x4_elem_aligned*>(static_cast<const char*>(row) + static_cast<size_t>(c) * 16);
  if constexpr (NT) return __builtin_nontemporal_load(p);
  return *p;
}
template <bool NT, bool AL>
__device__ __forceinline__ void store_piece(void* row, uint32_t c, u32x4 v) {
  if constexpr (AL) {
    store16<NT>(row, c, v);
  } else {
    u32x4_elem_aligned* p = reinterpret_cast<u32x4_elem_aligned*>(static_cast<char*>(row) + static_cast<size_t>(c) * 16);
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
  }
}
// Pieces [0, n) of one row copied by the BS threads of a workgroup, V pieces of a thread in flight.
template <int BS, int V, bool NTL, bool NTS, bool AL>
__device__ __forceinline__ void copy_row_pieces(void* drow, const void* srow, uint32_t n) {
  for (uint32_t c0 = threadIdx.x; c0 < n; c0 += V * BS) {
    u32x4 v[V];
#pragma unroll
    for (int u = 0; u < V; ++u)
      if (c0 + u * BS < n) v[u] = load_piece<NTL, AL>(srow, c0 + u * BS);
#pragma unroll
    for (int u = 0; u < V; ++u)
      if (c0 + u * BS < n) store_piece<NTS, AL>(drow, c0 + u * BS, v[u]);
  }
}

// The tail of a row as 2-byte units (every element type is a multiple of 2 bytes wide): unit `i` of
// the `tail2` units behind the `pieces` whole pieces.
__device__ __forceinline__ void copy_tail2(void* drow, const void* srow, uint32_t pieces, uint32_t i) {
  const size_t at = static_cast<size_t>(pieces) * 8 + i;
  static_cast<uint16_t*>(drow)[at] = static_cast<const uint16_t*>(srow)[at];
}
// Element `i` of a row of EB-byte elements, copied bit for bit.
template <int EB>
__device__ __forceinline__ void copy_elem(void* drow, const void* srow, size_t i) {
  if constexpr (EB == 4) static_cast<uint32_t*>(drow)[i] = static_cast<const uint32_t*>(srow)[i];
  else static_cast<uint16_t*>(drow)[i] = static_cast<const uint16_t*>(srow)[i];
}
__device__ __forceinline__ void zero_tail2(void* drow, uint32_t pieces, uint32_t i) {
  static_cast<uint16_t*>(drow)[static_cast<size_t>(pieces) * 8 + i] = 0;
}

// bf16 <-> binary32.  A bf16 is the upper half of a binary32 pattern.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Round to nearest even by adding the bias 0x7fff + (lsb of the kept part) and
// truncating; NaN is kept NaN by forcing the quiet bit.
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  const uint32_t nan = (u >> 16) | 0x0040u;
  return (f != f) ? nan : rounded;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (f32_to_bf16_rne(lo) & 0xffffu) | (f32_to_bf16_rne(hi) << 16);
}

// fp16 (IEEE binary16) <-> binary32 through the hardware conversions: widening is exact, narrowing
// rounds to nearest even, overflows to infinity and keeps NaN a NaN.
// The binary32 value passes through an empty asm statement on both sides.  Without it the
// compiler merges a conversion with a neighbouring multiply into one mixed-precision
// multiply-add whose addend is +0, and (-0) * g + (+0) is +0: the sign of a zero product
// would be lost.  The statement emits nothing; it only keeps the value in a register of its own.
__device__ __forceinline__ float f16_bits_to_f32(uint32_t h) {
  float f = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));
  asm volatile("" : "+v"(f));
  return f;
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {
  asm volatile("" : "+v"(f));
  return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f));
}

// Element traits: how many elements one 128-bit vector holds, the type the reduction is carried
// in (acc_t: binary32 for the floating types, int32 for int32), and how a vector is widened to /
// narrowed from lanes of that type.
template <int DT> struct Elem;
template <> struct Elem<MCR_F32> {
  static constexpr int kBytes = 4;
  static constexpr int kPerVec = 4;
  typedef float acc_t;
  __device__ static __forceinline__ void widen(u32x4 v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  __device__ static __forceinline__ u32x4 narrow(const float (&f)[4]) {
    u32x4 v;
    v.x = __float_as_uint(f[0]); v.y = __float_as_uint(f[1]);
    v.z = __float_as_uint(f[2]); v.w = __float_as_uint(f[3]);
    return v;
  }
  // one element as a bit pattern in the low bits of a word
  __device__ static __forceinline__ float widen1(uint32_t bits) { return __uint_as_float(bits); }
  __device__ static __forceinline__ uint32_t narrow1(float f) { return __float_as_uint(f); }
  __device__ static __forceinline__ float load1(const void* b, size_t i) {
    return reinterpret_cast<const float*>(b)[i];
  }
  __device__ static __forceinline__ void store1(void* b, size_t i, float f) {
    reinterpret_cast<float*>(b)[i] = f;
  }
};
template <> struct Elem<MCR_BF16> {
  static constexpr int kBytes = 2;
  static constexpr int kPerVec = 8;
  typedef float acc_t;
  __device__ static __forceinline__ void widen(u32x4 v, float (&f)[8]) {
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
  }
  __device__ static __forceinline__ u32x4 narrow(const float (&f)[8]) {
    u32x4 v;
    v.x = pack_bf16x2(f[0], f[1]); v.y = pack_bf16x2(f[2], f[3]);
    v.z = pack_bf16x2(f[4], f[5]); v.w = pack_bf16x2(f[6], f[7]);
    return v;
  }
  __device__ static __forceinline__ float widen1(uint32_t bits) { return __uint_as_float(bits << 16); }
  __device__ static __forceinline__ uint32_t narrow1(float f) { return f32_to_bf16_rne(f) & 0xffffu; }
  __device__ static __forceinline__ float load1(const void* b, size_t i) {
    return widen1(reinterpret_cast<const uint16_t*>(b)[i]);
  }
  __device__ static __forceinline__ void store1(void* b, size_t i, float f) {
    reinterpret_cast<uint16_t*>(b)[i] = static_cast<uint16_t>(narrow1(f));
  }
};
template <> struct Elem<MCR_F16> {
  static constexpr int kBytes = 2;
  static constexpr int kPerVec = 8;
  typedef float acc_t;
  __device__ static __forceinline__ void widen(u32x4 v, float (&f)[8]) {
    f[0] = f16_bits_to_f32(v.x & 0xffffu); f[1] = f16_bits_to_f32(v.x >> 16);
    f[2] = f16_bits_to_f32(v.y & 0xffffu); f[3] = f16_bits_to_f32(v.y >> 16);
    f[4] = f16_bits_to_f32(v.z & 0xffffu); f[5] = f16_bits_to_f32(v.z >> 16);
    f[6] = f16_bits_to_f32(v.w & 0xffffu); f[7] = f16_bits_to_f32(v.w >> 16);
  }
  __device__ static __forceinline__ u32x4 narrow(const float (&f)[8]) {
    u32x4 v;
    v.x = f32_to_f16_bits(f[0]) | (f32_to_f16_bits(f[1]) << 16);
    v.y = f32_to_f16_bits(f[2]) | (f32_to_f16_bits(f[3]) << 16);
    v.z = f32_to_f16_bits(f[4]) | (f32_to_f16_bits(f[5]) << 16);
    v.w = f32_to_f16_bits(f[6]) | (f32_to_f16_bits(f[7]) << 16);
    return v;
  }
  __device__ static __forceinline__ float widen1(uint32_t bits) { return f16_bits_to_f32(bits & 0xffffu); }
  __device__ static __forceinline__ uint32_t narrow1(float f) { return f32_to_f16_bits(f); }
  __device__ static __forceinline__ float load1(const void* b, size_t i) {
    return widen1(reinterpret_cast<const uint16_t*>(b)[i]);
  }
  __device__ static __forceinline__ void store1(void* b, size_t i, float f) {
    reinterpret_cast<uint16_t*>(b)[i] = static_cast<uint16_t>(narrow1(f));
  }
};
template <> struct Elem<MCR_I32> {
  static constexpr int kBytes = 4;
  static constexpr int kPerVec = 4;
  typedef int32_t acc_t;
  __device__ static __forceinline__ void widen(u32x4 v, int32_t (&f)[4]) {
    f[0] = static_cast<int32_t>(v.x); f[1] = static_cast<int32_t>(v.y);
    f[2] = static_cast<int32_t>(v.z); f[3] = static_cast<int32_t>(v.w);
  }
  __device__ static __forceinline__ u32x4 narrow(const int32_t (&f)[4]) {
    u32x4 v;
    v.x = static_cast<uint32_t>(f[0]); v.y = static_cast<uint32_t>(f[1]);
    v.z = static_cast<uint32_t>(f[2]); v.w = static_cast<uint32_t>(f[3]);
    return v;
  }
  __device__ static __forceinline__ int32_t widen1(uint32_t bits) { return static_cast<int32_t>(bits); }
  __device__ static __forceinline__ uint32_t narrow1(int32_t x) { return static_cast<uint32_t>(x); }
  __device__ static __forceinline__ int32_t load1(const void* b, size_t i) {
    return reinterpret_cast<const int32_t*>(b)[i];
  }
  __device__ static __forceinline__ void store1(void* b, size_t i, int32_t x) {
    reinterpret_cast<int32_t*>(b)[i] = x;
  }
};

// One step of the ReduceOp chain.  MAX and MIN let a NaN through from either side; between
// equal values the accumulated (earlier rank's) one stays.  `op` is uniform over the launch.
__device__ __forceinline__ float combine(float acc, float x, int op) {
  switch (op) {
    case MCR_MAX: return (x > acc || x != x) ? x : acc;
    case MCR_MIN: return (x < acc || x != x) ? x : acc;
    case MCR_PROD: return acc * x;
    default: return acc + x;
  }
}
// int32: sums and products wrap modulo 2^32.
__device__ __forceinline__ int32_t combine(int32_t acc, int32_t x, int op) {
  switch (op) {
    case MCR_MAX: return x > acc ? x : acc;
    case MCR_MIN: return x < acc ? x : acc;
    case MCR_PROD: return static_cast<int32_t>(static_cast<uint32_t>(acc) * static_cast<uint32_t>(x));
    default: return static_cast<int32_t>(static_cast<uint32_t>(acc) + static_cast<uint32_t>(x));
  }
}
__device__ __forceinline__ float plain_sum(float a, float b) { return a + b; }
__device__ __forceinline__ int32_t plain_sum(int32_t a, int32_t b) {
  return static_cast<int32_t>(static_cast<uint32_t>(a) + static_cast<uint32_t>(b));
}
// The AVG step; integers have no average (the entry points refuse it), so theirs is the identity.
__device__ __forceinline__ float avg_step(float acc, float scale) { return acc * scale; }
__device__ __forceinline__ int32_t avg_step(int32_t acc, float) { return acc; }

// Lanes of this wavefront with a lower lane id.
__device__ __forceinline__ uint64_t lanemask_lt() {
  const unsigned lane = __lane_id();
  return (lane == 0) ? 0ull : (~0ull >> (64 - lane));
}

}  // namespace mcr
