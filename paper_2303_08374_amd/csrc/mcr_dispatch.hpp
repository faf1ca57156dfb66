// Compile-time dispatch over rank count, element type and launch shape.
#pragma once
#include <type_traits>

#include "mcr_internal.hpp"

namespace mcr {

template <int N> using Int = std::integral_constant<int, N>;
template <bool B> using Bool = std::integral_constant<bool, B>;

// f(Int<P>) for P in 1..16
template <class F>
inline int dispatch_ranks(int P, F&& f) {
  switch (P) {
    case 1: return f(Int<1>{});   case 2: return f(Int<2>{});   case 3: return f(Int<3>{});
    case 4: return f(Int<4>{});   case 5: return f(Int<5>{});   case 6: return f(Int<6>{});
    case 7: return f(Int<7>{});   case 8: return f(Int<8>{});   case 9: return f(Int<9>{});
    case 10: return f(Int<10>{}); case 11: return f(Int<11>{}); case 12: return f(Int<12>{});
    case 13: return f(Int<13>{}); case 14: return f(Int<14>{}); case 15: return f(Int<15>{});
    case 16: return f(Int<16>{});
  }
  return MCR_EINVAL;
}

template <class F>
inline int dispatch_dtype(int dtype, F&& f) {
  if (dtype == MCR_F32) return f(Int<MCR_F32>{});
  if (dtype == MCR_BF16) return f(Int<MCR_BF16>{});
  if (dtype == MCR_F16) return f(Int<MCR_F16>{});
  if (dtype == MCR_I32) return f(Int<MCR_I32>{});
  return MCR_EDTYPE;
}

// the element types a gate weight can scale
template <class F>
inline int dispatch_float_dtype(int dtype, F&& f) {
  if (dtype == MCR_F32) return f(Int<MCR_F32>{});
  if (dtype == MCR_BF16) return f(Int<MCR_BF16>{});
  if (dtype == MCR_F16) return f(Int<MCR_F16>{});
  return MCR_EDTYPE;
}

// The reductions on the hot element types get every launch shape; on fp16 and int32 they are
// compiled like the generic ReduceOps: one shape, two vectors per thread, nontemporal loads and stores.
constexpr bool all_shapes(int dtype) { return dtype == MCR_F32 || dtype == MCR_BF16; }

// f(Int<U>, Bool<NT loads>, Bool<NT stores>) for the vector launch shapes
template <class F>
inline int dispatch_shape(int variant, F&& f) {
  switch (variant) {
    case SV_V1: return f(Int<1>{}, Bool<false>{}, Bool<false>{});
    case SV_V2: return f(Int<2>{}, Bool<false>{}, Bool<false>{});
    case SV_V4: return f(Int<4>{}, Bool<false>{}, Bool<false>{});
    case SV_V1NT: return f(Int<1>{}, Bool<true>{}, Bool<true>{});
    case SV_V2NT: return f(Int<2>{}, Bool<true>{}, Bool<true>{});
    case SV_V4NT: return f(Int<4>{}, Bool<true>{}, Bool<true>{});
    case SV_V1LN: return f(Int<1>{}, Bool<true>{}, Bool<false>{});
    case SV_V2LN: return f(Int<2>{}, Bool<true>{}, Bool<false>{});
    case SV_V4LN: return f(Int<4>{}, Bool<true>{}, Bool<false>{});
    case SV_V1SN: return f(Int<1>{}, Bool<false>{}, Bool<true>{});
    case SV_V2SN: return f(Int<2>{}, Bool<false>{}, Bool<true>{});
    case SV_V4SN: return f(Int<4>{}, Bool<false>{}, Bool<true>{});
  }
  return MCR_EVARIANT;
}

// The reductions are compiled for one plain shape (one vector per thread, what short messages take)
// and the fully nontemporal shape of each unroll; the ids of the other hint combinations ("v2", "v4",
// "ln", "sn"), which won no row of the tuning table at any scale, run the nontemporal kernel of
// their unroll.
template <class F>
inline int dispatch_reduce_shape(int variant, F&& f) {
  switch (variant) {
    case SV_V1: return f(Int<1>{}, Bool<false>{});
    case SV_V1NT: case SV_V1LN: case SV_V1SN: return f(Int<1>{}, Bool<true>{});
    case SV_V2: case SV_V2NT: case SV_V2LN: case SV_V2SN: return f(Int<2>{}, Bool<true>{});
    case SV_V4: case SV_V4NT: case SV_V4LN: case SV_V4SN: return f(Int<4>{}, Bool<true>{});
  }
  return MCR_EVARIANT;
}

// f(Bool<NT loads>, Bool<NT stores>): the cache hint of a shape, for kernels with a fixed unroll
template <class F>
inline int dispatch_hint(int variant, F&& f) {
  switch (variant) {
    case SV_V1NT: case SV_V2NT: case SV_V4NT: return f(Bool<true>{}, Bool<true>{});
    case SV_V1LN: case SV_V2LN: case SV_V4LN: return f(Bool<true>{}, Bool<false>{});
    case SV_V1SN: case SV_V2SN: case SV_V4SN: return f(Bool<false>{}, Bool<true>{});
  }
  return f(Bool<false>{}, Bool<false>{});
}

inline int shape_unroll(int variant) {
  switch (variant) {
    case SV_V2: case SV_V2NT: case SV_V2LN: case SV_V2SN: return 2;
    case SV_V4: case SV_V4NT: case SV_V4LN: case SV_V4SN: return 4;
  }
  return 1;
}

// Workgroups along x for `nvec` vectors per slice.
inline unsigned grid_x(size_t nvec, int variant) {
  const size_t per_block = static_cast<size_t>(shape_unroll(variant)) * kBlock;
  size_t blocks = (nvec + per_block - 1) / per_block;
  if (blocks == 0) blocks = 1;
  return static_cast<unsigned>(blocks);
}

}  // namespace mcr
