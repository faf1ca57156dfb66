// MoE token dispatch / combine around the Alltoall (paper Sec. II-C): routing
// (histogram + capacity clamp + exclusive scan -> pack slots and the split
// matrix), pack (row scatter by slot), unpack / gate-weighted combine (row
// gather by slot).
#include <mutex>

#include "mcr_dispatch.hpp"

namespace mcr {
namespace {

// ---- routing ---------------------------------------------------------------------
// One workgroup of 16 wavefronts per rank.  Wave w owns a contiguous run of
// tokens, so "earlier token" means: earlier wave, or earlier 64-token step of
// this wave, or lower lane in this step.  Within a step the lanes holding the
// same expert id are found with one ballot per id bit; a lane's position is
// the popcount of that mask below it.  Pass 1 counts per (wave, expert) in
// LDS; a scan over waves turns the counts into each wave's starting position;
// pass 2 replays the steps and emits slots.  Integer work on a few KB: bound
// by latency, not bandwidth.
constexpr int kRouteWaves = 16;
constexpr int kRouteBlock = kRouteWaves * kWave;
constexpr int kRouteBatch = 8;    // 64-token steps whose ids are loaded together

__device__ __forceinline__ uint64_t same_id_mask(int id, bool valid, int nbits) {
  uint64_t mask = __ballot(valid);
  for (int b = 0; b < nbits; ++b) {
    const bool bit = (id >> b) & 1;
    const uint64_t vote = __ballot(valid && bit);
    mask &= bit ? vote : ~vote;
  }
  return mask;
}

// Pass 1 of one wavefront over its 64-token steps [s_begin, s_end): counts per expert into `cnt`
// (this wave's row of the LDS table).  kRouteBatch steps at a time: all their ids are requested
// before the first is used, so the loop pays the memory latency once per batch, not once per step.
__device__ __forceinline__ void route_count(const int32_t* ids, int s_begin, int s_end, int T, int E, int nbits, int* cnt,
                                            int lane, uint64_t below) {
  for (int s0 = s_begin; s0 < s_end; s0 += kRouteBatch) {
    int idv[kRouteBatch];
#pragma unroll
    for (int j = 0; j < kRouteBatch; ++j) {
      const long long t = static_cast<long long>(s0 + j) * kWave + lane;
      idv[j] = (s0 + j < s_end && t < T) ? ids[t] : -1;
    }
#pragma unroll
    for (int j = 0; j < kRouteBatch; ++j) {
      if (s0 + j >= s_end) break;                                  // uniform over the wavefront
      const int id = idv[j];
      const bool valid = id >= 0 && id < E;
      const uint64_t mask = same_id_mask(id, valid, nbits);
      if (valid && (mask & below) == 0) cnt[id] += __popcll(mask);   // lowest lane of the group
    }
  }
}

// Pass 2: `pos` holds, per expert, the position of this wave's next token; slots go out.
__device__ __forceinline__ void route_emit(const int32_t* ids, int32_t* slot, int s_begin, int s_end, int T, int E, int C,
                                           int nbits, int* pos, const int* ebase, int lane, uint64_t below) {
  for (int s0 = s_begin; s0 < s_end; s0 += kRouteBatch) {
    int idv[kRouteBatch];
#pragma unroll
    for (int j = 0; j < kRouteBatch; ++j) {
      const long long t = static_cast<long long>(s0 + j) * kWave + lane;
      idv[j] = (s0 + j < s_end && t < T) ? ids[t] : -1;
    }
#pragma unroll
    for (int j = 0; j < kRouteBatch; ++j) {
      if (s0 + j >= s_end) break;                                  // uniform over the wavefront
      const long long t = static_cast<long long>(s0 + j) * kWave + lane;
      const int id = idv[j];
      const bool valid = id >= 0 && id < E;
      const uint64_t mask = same_id_mask(id, valid, nbits);
      int out = -1;
      if (valid) {
        const int at = pos[id] + __popcll(mask & below);
        if (at < C) out = ebase[id] + at;
      }
      // every lane has read the running position before the group's first lane moves it on
      __builtin_amdgcn_wave_barrier();
      if (valid && (mask & below) == 0) pos[id] += __popcll(mask);
      __builtin_amdgcn_wave_barrier();
      if (t < T) slot[t] = out;
    }
  }
}

// Exclusive scan of the kept counts over experts by one wavefront (E <= 512: 64 at a time), and
// the outputs that depend on them only.
__device__ __forceinline__ void route_expert_bases(const int* ecnt, int* ebase, int32_t* counts, bool write_counts, int E,
                                                   int lane) {
  int carry = 0;
  for (int e0 = 0; e0 < E; e0 += kWave) {
    const int e = e0 + lane;
    const int c = (e < E) ? ecnt[e] : 0;
    int incl = c;
    for (int d = 1; d < kWave; d <<= 1) {
      const int up = __shfl_up(incl, d);
      if (lane >= d) incl += up;
    }
    if (e < E) {
      ebase[e] = carry + incl - c;
      if (write_counts) counts[e] = c;
    }
    carry += __shfl(incl, kWave - 1);
  }
}

__global__ void __launch_bounds__(kRouteBlock)
moe_route_kernel(CPtrTab ids_tab, PtrTab slot_tab, PtrTab counts_tab, int64_t* splits, int T, int E,
                 int P, int C, int nbits) {
  __shared__ int wave_cnt[kRouteWaves][MCR_MAX_EXPERTS];   // count, then running start position
  __shared__ int ebase[MCR_MAX_EXPERTS];                   // first slot of each expert
  __shared__ int ecnt[MCR_MAX_EXPERTS];                    // kept tokens of each expert
  const int rank = blockIdx.x;
  const int32_t* ids = static_cast<const int32_t*>(ids_tab.p[rank]);
  int32_t* slot = static_cast<int32_t*>(slot_tab.p[rank]);
  int32_t* counts = static_cast<int32_t*>(counts_tab.p[rank]);
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const uint64_t below = lanemask_lt();

  for (int i = tid; i < kRouteWaves * E; i += kRouteBlock) wave_cnt[i / E][i % E] = 0;
  __syncthreads();

  // tokens of this wave: [t_begin, t_end), a multiple of 64 long except at the very end
  const int steps_total = (T + kWave - 1) / kWave;
  const int steps_per_wave = (steps_total + kRouteWaves - 1) / kRouteWaves;
  const int s_begin = wave * steps_per_wave;
  const int s_end = min(steps_total, s_begin + steps_per_wave);

  route_count(ids, s_begin, s_end, T, E, nbits, wave_cnt[wave], lane, below);
  __syncthreads();

  // per expert: exclusive scan over waves, then clamp the total to the capacity
  for (int e = tid; e < E; e += kRouteBlock) {
    int run = 0;
    for (int w = 0; w < kRouteWaves; ++w) {
      const int c = wave_cnt[w][e];
      wave_cnt[w][e] = run;
      run += c;
    }
    ecnt[e] = min(run, C);
  }
  __syncthreads();
  if (wave == 0) route_expert_bases(ecnt, ebase, counts, true, E, lane);
  __syncthreads();
  if (tid < P) {
    const int per = E / P;
    int64_t a = 0;
    for (int e = tid * per; e < (tid + 1) * per; ++e) a += ecnt[e];
    splits[static_cast<size_t>(rank) * P + tid] = a;
  }
  route_emit(ids, slot, s_begin, s_end, T, E, C, nbits, wave_cnt[wave], ebase, lane, below);
}

// ---- routing over several workgroups per rank --------------------------------------------------
// The one-workgroup kernel above is bound by the vector ALU of the one compute unit it runs on.
// With a workspace the tokens of a rank are cut into chunks of `chunk_steps` 64-token steps; a
// first launch counts per (rank, chunk, expert) into the workspace, a second launch gives every
// chunk its starting positions (the counts of the chunks before it) and emits the slots.  Same
// results as the kernel above, bit for bit.
constexpr int kChunkWaves = 4;
constexpr int kChunkBlock = kChunkWaves * kWave;

__device__ __forceinline__ void chunk_wave_range(int chunk, int chunk_steps, int steps_total, int wave, int* s_begin,
                                                 int* s_end) {
  const int c_begin = chunk * chunk_steps;
  const int c_end = min(steps_total, c_begin + chunk_steps);
  const int per_wave = (chunk_steps + kChunkWaves - 1) / kChunkWaves;
  *s_begin = min(c_end, c_begin + wave * per_wave);
  *s_end = min(c_end, *s_begin + per_wave);
}

// grid (chunks, P).  workspace[(rank * chunks + chunk) * E + e]
__global__ void __launch_bounds__(kChunkBlock)
moe_route_count_kernel(CPtrTab ids_tab, int32_t* workspace, int T, int E, int chunk_steps, int nbits) {
  __shared__ int wave_cnt[kChunkWaves][MCR_MAX_EXPERTS];
  const int rank = blockIdx.y, chunk = blockIdx.x, chunks = gridDim.x;
  const int32_t* ids = static_cast<const int32_t*>(ids_tab.p[rank]);
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  for (int i = tid; i < kChunkWaves * E; i += kChunkBlock) wave_cnt[i / E][i % E] = 0;
  __syncthreads();
  int s_begin, s_end;
  chunk_wave_range(chunk, chunk_steps, (T + kWave - 1) / kWave, wave, &s_begin, &s_end);
  route_count(ids, s_begin, s_end, T, E, nbits, wave_cnt[wave], lane, lanemask_lt());
  __syncthreads();
  int32_t* out = workspace + (static_cast<size_t>(rank) * chunks + chunk) * E;
  for (int e = tid; e < E; e += kChunkBlock) {
    int a = 0;
#pragma unroll
    for (int w = 0; w < kChunkWaves; ++w) a += wave_cnt[w][e];
    out[e] = a;
  }
}

__global__ void __launch_bounds__(kChunkBlock)
moe_route_slot_kernel(CPtrTab ids_tab, PtrTab slot_tab, PtrTab counts_tab, int64_t* splits, const int32_t* workspace, int T,
                      int E, int P, int C, int chunk_steps, int nbits) {
  __shared__ int wave_cnt[kChunkWaves][MCR_MAX_EXPERTS];
  __shared__ int ebase[MCR_MAX_EXPERTS];
  __shared__ int ecnt[MCR_MAX_EXPERTS];
  __shared__ int before[MCR_MAX_EXPERTS];                  // tokens of the expert in the chunks before this one
  const int rank = blockIdx.y, chunk = blockIdx.x, chunks = gridDim.x;
  const int32_t* ids = static_cast<const int32_t*>(ids_tab.p[rank]);
  int32_t* slot = static_cast<int32_t*>(slot_tab.p[rank]);
  int32_t* counts = static_cast<int32_t*>(counts_tab.p[rank]);
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const uint64_t below = lanemask_lt();
  const int32_t* hist = workspace + static_cast<size_t>(rank) * chunks * E;
  for (int e = tid; e < E; e += kChunkBlock) {
    int total = 0, bef = 0;
    for (int c = 0; c < chunks; ++c) {
      const int v = hist[static_cast<size_t>(c) * E + e];
      if (c < chunk) bef += v;
      total += v;
    }
    before[e] = bef;
    ecnt[e] = min(total, C);
  }
  for (int i = tid; i < kChunkWaves * E; i += kChunkBlock) wave_cnt[i / E][i % E] = 0;
  __syncthreads();
  int s_begin, s_end;
  chunk_wave_range(chunk, chunk_steps, (T + kWave - 1) / kWave, wave, &s_begin, &s_end);
  route_count(ids, s_begin, s_end, T, E, nbits, wave_cnt[wave], lane, below);
  if (wave == 0) route_expert_bases(ecnt, ebase, counts, chunk == 0, E, lane);
  __syncthreads();
  for (int e = tid; e < E; e += kChunkBlock) {
    int run = before[e];
#pragma unroll
    for (int w = 0; w < kChunkWaves; ++w) {
      const int c = wave_cnt[w][e];
      wave_cnt[w][e] = run;
      run += c;
    }
  }
  if (chunk == 0 && tid < P) {
    const int per = E / P;
    int64_t a = 0;
    for (int e = tid * per; e < (tid + 1) * per; ++e) a += ecnt[e];
    splits[static_cast<size_t>(rank) * P + tid] = a;
  }
  __syncthreads();
  route_emit(ids, slot, s_begin, s_end, T, E, C, nbits, wave_cnt[wave], ebase, lane, below);
}

// ---- pack / unpack -----------------------------------------------------------------
// A row is `upr` units; `tpr` threads (a power of two <= 256) share a row, so a
// workgroup covers 256/tpr rows.  blockIdx.y = rank.
template <int UB> struct RowUnit;
template <> struct RowUnit<16> { typedef u32x4 type; };
template <> struct RowUnit<4> { typedef uint32_t type; };
template <> struct RowUnit<2> { typedef uint16_t type; };

// Which row a thread works on and which units of it.  ONE (a row is wider than half a workgroup):
// the workgroup owns one row, so the row index is uniform and everything looked up by it (slot,
// gate) comes through scalar loads: a shorter dependent chain in front of the row's own loads,
// worth 7 % on 4 KiB rows.
template <bool ONE>
__device__ __forceinline__ void row_of_thread(uint32_t tpr, uint32_t tpr_shift, size_t* t, uint32_t* c0, uint32_t* step) {
  if constexpr (ONE) {
    *t = blockIdx.x;
    *c0 = threadIdx.x;
    *step = kBlock;
  } else {
    *t = static_cast<size_t>(blockIdx.x) * (kBlock >> tpr_shift) + (threadIdx.x >> tpr_shift);
    *c0 = threadIdx.x & (tpr - 1);
    *step = tpr;
  }
}

template <int UB, bool NTL, bool NTS, bool ONE>
__global__ void __launch_bounds__(kBlock)
pack_kernel(PtrTab out, CPtrTab in, CPtrTab slot_tab, size_t T, size_t out_rows, uint32_t upr,
            uint32_t tpr, uint32_t tpr_shift) {
  typedef typename RowUnit<UB>::type U;
  const unsigned rank = blockIdx.y;
  const int32_t* slot = static_cast<const int32_t*>(slot_tab.p[rank]);
  const U* src = static_cast<const U*>(in.p[rank]);
  U* dst = static_cast<U*>(out.p[rank]);
  size_t t;
  uint32_t c0, step;
  row_of_thread<ONE>(tpr, tpr_shift, &t, &c0, &step);
  if (t >= T) return;
  const int32_t s = slot[t];
  if (s < 0 || static_cast<size_t>(s) >= out_rows) return;
  const U* srow = src + t * upr;
  U* drow = dst + static_cast<size_t>(s) * upr;
  for (uint32_t c = c0; c < upr; c += step) {
    U v;
    if constexpr (NTL) v = __builtin_nontemporal_load(srow + c); else v = srow[c];
    if constexpr (NTS) __builtin_nontemporal_store(v, drow + c); else drow[c] = v;
  }
}

// pack_kernel for rows of any width and alignment from 64 bytes up: whole 16-byte pieces at the
// address the elements fall on, then `tail2` 2-byte units.
template <bool NTL, bool NTS>
__global__ void __launch_bounds__(kBlock)
pack_pieces_kernel(PtrTab out, CPtrTab in, CPtrTab slot_tab, size_t T, size_t out_rows, size_t row_bytes, uint32_t pieces,
                   uint32_t tail2, uint32_t tpr, uint32_t tpr_shift) {
  const unsigned rank = blockIdx.y;
  size_t t;
  uint32_t c0, step;
  row_of_thread<false>(tpr, tpr_shift, &t, &c0, &step);
  if (t >= T) return;
  const int32_t s = static_cast<const int32_t*>(slot_tab.p[rank])[t];
  if (s < 0 || static_cast<size_t>(s) >= out_rows) return;
  const char* srow = static_cast<const char*>(in.p[rank]) + t * row_bytes;
  char* drow = static_cast<char*>(out.p[rank]) + static_cast<size_t>(s) * row_bytes;
  for (uint32_t c = c0; c < pieces; c += step) store_piece<NTS, false>(drow, c, load_piece<NTL, false>(srow, c));
  if (c0 < tail2) copy_tail2(drow, srow, pieces, c0);
}

// pack for rows wider than half a workgroup: one row per workgroup, the slot through a scalar load.
// AL = false: rows of any width and alignment (16-byte pieces at element-aligned addresses, then
// `tail2` 2-byte units).
template <bool NTL, bool NTS, bool AL>
__global__ void __launch_bounds__(kBlock)
pack_row_kernel(PtrTab out, CPtrTab in, CPtrTab slot_tab, size_t out_rows, size_t row_bytes, uint32_t pieces, uint32_t tail2) {
  const unsigned rank = blockIdx.y;
  const size_t t = blockIdx.x;
  const int32_t s = static_cast<const int32_t*>(slot_tab.p[rank])[t];
  if (s < 0 || static_cast<size_t>(s) >= out_rows) return;
  const char* srow = static_cast<const char*>(in.p[rank]) + t * row_bytes;
  char* drow = static_cast<char*>(out.p[rank]) + static_cast<size_t>(s) * row_bytes;
  copy_row_pieces<kBlock, 1, NTL, NTS, AL>(drow, srow, pieces);
  if (!AL && threadIdx.x < tail2) copy_tail2(drow, srow, pieces, threadIdx.x);
}

template <int DT> __device__ __forceinline__ u32x4 scale_vec(u32x4 v, float g) {
  using E = Elem<DT>;
  float f[E::kPerVec];
  E::widen(v, f);
#pragma unroll
  for (int k = 0; k < E::kPerVec; ++k) f[k] = g * f[k];
  return E::narrow(f);
}

// GATE: 0 = plain gather, 1 = scale kept rows by gate[t].
template <int DT, int UB, bool NTL, bool NTS, bool GATE>
__global__ void __launch_bounds__(kBlock)
unpack_kernel(PtrTab out, CPtrTab in, CPtrTab slot_tab, CPtrTab gate_tab, size_t T, size_t in_rows,
              uint32_t upr, uint32_t tpr, uint32_t tpr_shift) {
  typedef typename RowUnit<UB>::type U;
  const unsigned rank = blockIdx.y;
  const int32_t* slot = static_cast<const int32_t*>(slot_tab.p[rank]);
  const U* src = static_cast<const U*>(in.p[rank]);
  U* dst = static_cast<U*>(out.p[rank]);
  size_t t;
  uint32_t c0, step;
  row_of_thread<false>(tpr, tpr_shift, &t, &c0, &step);
  if (t >= T) return;
  const int32_t s = slot[t];
  const bool kept = s >= 0 && static_cast<size_t>(s) < in_rows;
  U* drow = dst + t * upr;
  if (!kept) {
    U z = {};
    for (uint32_t c = c0; c < upr; c += step) {
      if constexpr (NTS) __builtin_nontemporal_store(z, drow + c); else drow[c] = z;
    }
    return;
  }
  const U* srow = src + static_cast<size_t>(s) * upr;
  float g = 1.0f;
  if constexpr (GATE) g = static_cast<const float*>(gate_tab.p[rank])[t];
  for (uint32_t c = c0; c < upr; c += step) {
    U v;
    if constexpr (NTL) v = __builtin_nontemporal_load(srow + c); else v = srow[c];
    if constexpr (GATE) {
      if constexpr (UB == 16) {
        v = scale_vec<DT>(v, g);
      } else {
        // one element per unit
        const float y = g * Elem<DT>::widen1(static_cast<uint32_t>(v));
        v = static_cast<U>(Elem<DT>::narrow1(y));
      }
    }
    if constexpr (NTS) __builtin_nontemporal_store(v, drow + c); else drow[c] = v;
  }
}

// unpack_kernel for rows of any width and alignment from 64 bytes up: 16-byte pieces, then the
// `tail` elements behind them one by one.
template <int DT, bool GATE>
__global__ void __launch_bounds__(kBlock)
unpack_pieces_kernel(PtrTab out, CPtrTab in, CPtrTab slot_tab, CPtrTab gate_tab, size_t T, size_t in_rows, size_t row_bytes,
                     uint32_t pieces, uint32_t tail, uint32_t tpr, uint32_t tpr_shift) {
  typedef Elem<DT> EL;
  const unsigned rank = blockIdx.y;
  size_t t;
  uint32_t c0, step;
  row_of_thread<false>(tpr, tpr_shift, &t, &c0, &step);
  if (t >= T) return;
  const int32_t s = static_cast<const int32_t*>(slot_tab.p[rank])[t];
  const bool kept = s >= 0 && static_cast<size_t>(s) < in_rows;
  char* drow = static_cast<char*>(out.p[rank]) + t * row_bytes;
  const size_t first_tail = static_cast<size_t>(pieces) * (16 / EL::kBytes);
  if (!kept) {
    const u32x4 z = {};
    for (uint32_t c = c0; c < pieces; c += step) store_piece<false, false>(drow, c, z);
    if (c0 < tail) {
      if constexpr (EL::kBytes == 4) reinterpret_cast<uint32_t*>(drow)[first_tail + c0] = 0u;
      else reinterpret_cast<uint16_t*>(drow)[first_tail + c0] = 0;
    }
    return;
  }
  const char* srow = static_cast<const char*>(in.p[rank]) + static_cast<size_t>(s) * row_bytes;
  float g = 1.0f;
  if constexpr (GATE) g = static_cast<const float*>(gate_tab.p[rank])[t];
  for (uint32_t c = c0; c < pieces; c += step) {
    u32x4 v = load_piece<false, false>(srow, c);
    if constexpr (GATE) v = scale_vec<DT>(v, g);
    store_piece<false, false>(drow, c, v);
  }
  if (c0 < tail) {
    const size_t i = first_tail + c0;
    if constexpr (GATE) EL::store1(drow, i, g * EL::load1(srow, i));
    else copy_elem<EL::kBytes>(drow, srow, i);
  }
}

// unpack for rows wider than half a workgroup: one row per workgroup of kRowGatherBlock threads (the
// slot and the gate come through scalar loads), kRowGatherVecs units per thread in flight.  A
// gather behind a lookup is bound by the rows a compute unit has in flight: the smaller workgroup
// doubles them (6.1 against 5.8 TB/s in a plain gather of 4 KiB rows).
template <int DT, bool NTL, bool NTS, bool GATE, bool AL>
__global__ void __launch_bounds__(kRowGatherBlock)
unpack_row_kernel(PtrTab out, CPtrTab in, CPtrTab slot_tab, CPtrTab gate_tab, size_t in_rows, size_t row_bytes, uint32_t upr,
                  uint32_t tail) {
  using E = Elem<DT>;
  constexpr int V = kRowGatherVecs;
  const unsigned rank = blockIdx.y;
  const size_t t = blockIdx.x;
  const int32_t s = static_cast<const int32_t*>(slot_tab.p[rank])[t];
  float g = 1.0f;
  if constexpr (GATE) g = static_cast<const float*>(gate_tab.p[rank])[t];
  char* drow = static_cast<char*>(out.p[rank]) + t * row_bytes;
  const bool kept = s >= 0 && static_cast<size_t>(s) < in_rows;
  const size_t first_tail = static_cast<size_t>(upr) * E::kPerVec;   // `tail` elements behind the whole pieces
  if (!kept) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (uint32_t c = threadIdx.x; c < upr; c += kRowGatherBlock) store_piece<NTS, AL>(drow, c, z);
    if (!AL && threadIdx.x < tail) E::store1(drow, first_tail + threadIdx.x, typename E::acc_t(0));
    return;
  }
  const char* srow = static_cast<const char*>(in.p[rank]) + static_cast<size_t>(s) * row_bytes;
  for (uint32_t c0 = threadIdx.x; c0 < upr; c0 += V * kRowGatherBlock) {
    u32x4 v[V];
#pragma unroll
    for (int u = 0; u < V; ++u) {
      const uint32_t c = c0 + u * kRowGatherBlock;
      if (c < upr) v[u] = load_piece<NTL, AL>(srow, c);
    }
#pragma unroll
    for (int u = 0; u < V; ++u) {
      const uint32_t c = c0 + u * kRowGatherBlock;
      if (c >= upr) continue;
      if constexpr (GATE) v[u] = scale_vec<DT>(v[u], g);
      store_piece<NTS, AL>(drow, c, v[u]);
    }
  }
  if (!AL && threadIdx.x < tail) {
    const size_t i = first_tail + threadIdx.x;
    if constexpr (GATE) E::store1(drow, i, g * E::load1(srow, i));
    else copy_elem<E::kBytes>(drow, srow, i);                        // a bit copy, whatever the pattern
  }
}

struct RowShape {
  uint32_t upr, tpr, shift;
  unsigned blocks;
};
inline RowShape row_shape(size_t T, size_t units_per_row) {
  RowShape s;
  s.upr = static_cast<uint32_t>(units_per_row);
  s.shift = 0;
  while ((1u << s.shift) < s.upr && s.shift < 8) ++s.shift;   // tpr = min(256, pow2 >= upr)
  s.tpr = 1u << s.shift;
  const size_t rows_per_block = kBlock >> s.shift;
  s.blocks = static_cast<unsigned>((T + rows_per_block - 1) / rows_per_block);
  if (s.blocks == 0) s.blocks = 1;
  return s;
}

}  // namespace

int launch_moe_route(mcr_ctx*, const CPtrTab& ids, int T, int E, int P, int capacity, const PtrTab& slot,
                     const PtrTab& counts, int64_t* splits, hipStream_t stream) {
  int nbits = 0;
  while ((1 << nbits) < E) ++nbits;
  hipLaunchKernelGGL(moe_route_kernel, dim3(P), dim3(kRouteBlock), 0, stream, ids, slot, counts, splits, T, E,
                     P, capacity, nbits);
  return launch_status();
}

// Chunks per rank of the several-workgroup routing: at least 2048 tokens each, at most 64 chunks;
// 1 means the one-workgroup kernel serves.
int route_chunks(int T, int* chunk_steps) {
  const int steps_total = (T + kWave - 1) / kWave;
  int cs = 32;
  if ((steps_total + cs - 1) / cs > 64) cs = (steps_total + 63) / 64;
  *chunk_steps = cs;
  const int chunks = (steps_total + cs - 1) / cs;
  return chunks < 1 ? 1 : chunks;
}

int launch_moe_route_chunked(mcr_ctx*, const CPtrTab& ids, int T, int E, int P, int capacity, const PtrTab& slot,
                             const PtrTab& counts, int64_t* splits, int32_t* workspace, hipStream_t stream) {
  int nbits = 0;
  while ((1 << nbits) < E) ++nbits;
  int chunk_steps;
  const int chunks = route_chunks(T, &chunk_steps);
  hipLaunchKernelGGL(moe_route_count_kernel, dim3(chunks, P), dim3(kChunkBlock), 0, stream, ids, workspace, T, E, chunk_steps,
                     nbits);
  int rc = launch_status();
  if (rc != MCR_OK) return rc;
  hipLaunchKernelGGL(moe_route_slot_kernel, dim3(chunks, P), dim3(kChunkBlock), 0, stream, ids, slot, counts, splits,
                     workspace, T, E, P, capacity, chunk_steps, nbits);
  return launch_status();
}

// ---- routing for callers that cannot allocate ---------------------------------------------------
// The chunk counters of the several-workgroup routing live in a static device array instead of
// a caller's workspace.  Every GPU the library runs on holds its own copy of the array at its
// own address until the process ends; the address is looked up once per device, with that device
// current, and host code uses that address only, never the array's name.
static __device__ __align__(256) int32_t scratch[MCR_ROUTE_SCRATCH_BYTES / sizeof(int32_t)];

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
int32_t* scratch_ptr[kMaxDevices] = {nullptr};
}  // namespace

// Device address of the calling thread's current device's copy of `scratch` (that device must be
// `device`), looked up on first use.  MCR_EHIP if the runtime cannot resolve the symbol.
int route_scratch_address(int device, int32_t** out) {
  if (device < 0 || device >= kMaxDevices) return MCR_EINVAL;
  std::lock_guard<std::mutex> lock(scratch_mu);
  if (!scratch_ptr[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MCR_EHIP;
    scratch_ptr[device] = static_cast<int32_t*>(p);
  }
  *out = scratch_ptr[device];
  return MCR_OK;
}

int launch_pack(mcr_ctx*, const PtrTab& out, const CPtrTab& in, const CPtrTab& slot, size_t T, size_t out_rows,
                size_t row_bytes, int elem_b, int P, int variant, hipStream_t stream) {
  if (T == 0 || row_bytes == 0) return MCR_OK;
  if (variant == SV_SCALAR && row_bytes / 16 > kBlock / 2) {
    // wide rows of any width and alignment: one row per workgroup, 16-byte pieces and a tail, nontemporal
    // both ways (what the tuning suite picks for the aligned rows of the workloads)
    hipLaunchKernelGGL((pack_row_kernel<true, true, false>), dim3(static_cast<unsigned>(T), P), dim3(kBlock), 0, stream, out, in, slot,
                       out_rows, row_bytes, static_cast<uint32_t>(row_bytes / 16), static_cast<uint32_t>((row_bytes % 16) / 2));
    return launch_status();
  }
  if (variant == SV_SCALAR && row_bytes >= 64) {
    const RowShape s = row_shape(T, row_bytes / 16);
    hipLaunchKernelGGL((pack_pieces_kernel<true, false>), dim3(s.blocks, P), dim3(kBlock), 0, stream, out, in, slot, T, out_rows,
                       row_bytes, s.upr, static_cast<uint32_t>((row_bytes % 16) / 2), s.tpr, s.shift);
    return launch_status();
  }
  if (variant == SV_SCALAR) {
    const RowShape s = row_shape(T, row_bytes / elem_b);
    if (elem_b == 4)
      hipLaunchKernelGGL((pack_kernel<4, false, false, false>), dim3(s.blocks, P), dim3(kBlock), 0, stream, out, in, slot, T, out_rows, s.upr, s.tpr, s.shift);
    else
      hipLaunchKernelGGL((pack_kernel<2, false, false, false>), dim3(s.blocks, P), dim3(kBlock), 0, stream, out, in, slot, T, out_rows, s.upr, s.tpr, s.shift);
    return launch_status();
  }
  const RowShape s = row_shape(T, row_bytes / 16);
  return dispatch_hint(variant, [&](auto ntl, auto nts) {
    if (s.tpr == kBlock)
      hipLaunchKernelGGL((pack_row_kernel<decltype(ntl)::value, decltype(nts)::value, true>), dim3(static_cast<unsigned>(T), P),
                         dim3(kBlock), 0, stream, out, in, slot, out_rows, row_bytes, s.upr, 0u);
    else
      hipLaunchKernelGGL((pack_kernel<16, decltype(ntl)::value, decltype(nts)::value, false>), dim3(s.blocks, P), dim3(kBlock), 0,
                         stream, out, in, slot, T, out_rows, s.upr, s.tpr, s.shift);
    return launch_status();
  });
}

int launch_unpack(mcr_ctx*, const PtrTab& out, const CPtrTab& in, const CPtrTab& slot, const CPtrTab* gate,
                  size_t T, size_t in_rows, size_t row_elems, int dtype, int P, int variant, hipStream_t stream) {
  if (T == 0 || row_elems == 0) return MCR_OK;
  CPtrTab g;
  for (int i = 0; i < MCR_MAX_RANKS; ++i) g.p[i] = gate ? gate->p[i] : nullptr;
  // without a gate the rows are copied, and only the element size matters
  const int kernel_dtype = gate ? dtype : (elem_bytes(dtype) == 4 ? MCR_F32 : MCR_BF16);
  return dispatch_float_dtype(kernel_dtype, [&](auto dt) {
    constexpr int DT = decltype(dt)::value;
    constexpr int EB = Elem<DT>::kBytes;
    const size_t row_bytes = row_elems * EB;
    auto go = [&](auto ub, auto ntl, auto nts, auto gc) {
      constexpr int UB = decltype(ub)::value;
      const RowShape s = row_shape(T, row_elems * EB / UB);
      if (UB == 16 && s.tpr == kBlock)
        hipLaunchKernelGGL((unpack_row_kernel<DT, decltype(ntl)::value, decltype(nts)::value, decltype(gc)::value, true>),
                           dim3(static_cast<unsigned>(T), P), dim3(kRowGatherBlock), 0, stream, out, in, slot, g, in_rows, row_bytes,
                           s.upr, 0u);
      else if (UB != 16 && row_bytes / 16 > kBlock / 2)
        // the element path on wide rows: 16-byte pieces at element-aligned addresses and a tail (plain
        // loads and stores: 291 us on the MoE workload with 4104-byte rows, 315-330 with nontemporal ones)
        hipLaunchKernelGGL((unpack_row_kernel<DT, false, false, decltype(gc)::value, false>), dim3(static_cast<unsigned>(T), P),
                           dim3(kRowGatherBlock), 0, stream, out, in, slot, g, in_rows, row_bytes,
                           static_cast<uint32_t>(row_bytes / 16), static_cast<uint32_t>((row_bytes % 16) / EB));
      else if (UB != 16 && row_bytes >= 64) {
        const RowShape sp = row_shape(T, row_bytes / 16);
        hipLaunchKernelGGL((unpack_pieces_kernel<DT, decltype(gc)::value>), dim3(sp.blocks, P), dim3(kBlock), 0, stream, out, in, slot,
                           g, T, in_rows, row_bytes, sp.upr, static_cast<uint32_t>((row_bytes % 16) / EB), sp.tpr, sp.shift);
      } else
        hipLaunchKernelGGL((unpack_kernel<DT, UB, decltype(ntl)::value, decltype(nts)::value, decltype(gc)::value>),
                           dim3(s.blocks, P), dim3(kBlock), 0, stream, out, in, slot, g, T, in_rows, s.upr, s.tpr, s.shift);
      return launch_status();
    };
    if (variant == SV_SCALAR)
      return gate ? go(Int<EB>{}, Bool<false>{}, Bool<false>{}, Bool<true>{}) : go(Int<EB>{}, Bool<false>{}, Bool<false>{}, Bool<false>{});
    return dispatch_hint(variant, [&](auto ntl, auto nts) {
      return gate ? go(Int<16>{}, ntl, nts, Bool<true>{}) : go(Int<16>{}, ntl, nts, Bool<false>{});
    });
  });
}

}  // namespace mcr
