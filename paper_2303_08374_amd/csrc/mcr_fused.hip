// Pipelines fused across op boundaries, which one address space allows and a
// library-per-operation runtime does not:
//   moe_dispatch  = pack + all_to_allv      (token rows go straight to their row in the
//                                            destination rank's receive buffer)
//   moe_combine   = all_to_allv(S^T) + gate-weighted unpack
//                                           (each token row is fetched from where the expert
//                                            left it on the destination rank and scaled)
//   dlrm_shuffle  = pack + all_to_allv + unpack of the embedding shuffle, forward or
//                   backward, as one row permutation across the rank buffers
// Each produces bit for bit what the unfused chain produces (paper Sec. II-C and II-D
// describe the chains), at 2 row transfers instead of 4 to 6.
#include "mcr_dispatch.hpp"

namespace mcr {
namespace {

template <int UB> struct RowUnit;
template <> struct RowUnit<16> { typedef u32x4 type; };
template <> struct RowUnit<4> { typedef uint32_t type; };
template <> struct RowUnit<2> { typedef uint16_t type; };

template <bool NT, class U> __device__ __forceinline__ U ldu(const U* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  return *p;
}
template <bool NT, class U> __device__ __forceinline__ void stu(U* p, U v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// Displacements of sender `p` for every receiver r, from the device split matrix:
//   sd[r] = sum_{q<r} S[p][q]  (sd[P] = rows rank p sends in all)
//   rd[r] = sum_{q<p} S[q][r]  (first row of rank p's block in receiver r's buffer)
// Entries are untrusted: negative counts as 0, nothing exceeds `cap` rows.
struct PairTables {
  int64_t sd[MCR_MAX_RANKS + 1];
  int64_t rd[MCR_MAX_RANKS];
};
__device__ __forceinline__ int64_t clamp_rows(int64_t s, int64_t cap) { return s < 0 ? 0 : (s > cap ? cap : s); }

__device__ __forceinline__ void build_pair_tables(PairTables& t, const int64_t* S, int p, int P, int64_t cap) {
  const int r = threadIdx.x;
  if (r <= P) {
    int64_t a = 0;
    for (int q = 0; q < r; ++q) a += clamp_rows(S[p * P + q], cap);
    t.sd[r] = a;
  }
  if (r < P) {
    int64_t a = 0;
    for (int q = 0; q < p; ++q) a += clamp_rows(S[q * P + r], cap);
    t.rd[r] = a;
  }
  __syncthreads();
}

// Receiver of packed row s of this sender, and its row in that receiver's buffer; false if the
// slot is not a row this sender owns or the row would leave the receive buffer.
// WAVE: every lane of the wavefront asks about the same row (a row is at least 64 threads wide),
// so lane q compares sd[q] once and a ballot counts the receivers that start at or below s,
// instead of every lane walking the table.
template <bool WAVE>
__device__ __forceinline__ bool locate(const PairTables& t, int P, int64_t s, int64_t send_rows, uint64_t recv_rows,
                                       int* r_out, uint64_t* row_out) {
  int r = 0;
  if constexpr (WAVE) {
    const int lane = __lane_id();
    const bool below = lane >= 1 && lane < P && t.sd[lane] <= s;
    r = __popcll(__ballot(below));
  }
  if (s < 0 || s >= t.sd[P] || s >= send_rows) return false;
  if constexpr (!WAVE) {
    for (int q = 1; q < P; ++q) r += (t.sd[q] <= s) ? 1 : 0;     // sd is non-decreasing
  }
  const uint64_t row = static_cast<uint64_t>(t.rd[r] + (s - t.sd[r]));
  if (row >= recv_rows) return false;
  *r_out = r;
  *row_out = row;
  return true;
}

constexpr int kRowsPerBlock = 32;   // token rows one workgroup walks (amortises the table build); <= 64
constexpr int kRowsInFlight = 4;   // rows whose loads are issued before the first store

// When a row is at least a wavefront wide, every wave fetches the slots of all the rows it will
// walk with one coalesced load (lane k holds the slot of the wave's k-th row) and hands them out
// by shuffle, so the row loop has no dependent slot load in it.
template <bool WAVE>
__device__ __forceinline__ int32_t prefetch_slots(const int32_t* slot, size_t t0, uint32_t rows_per_pass,
                                                  uint32_t tpr_shift, size_t T) {
  if constexpr (!WAVE) return -1;
  const unsigned lane = __lane_id();
  const size_t t = t0 + static_cast<size_t>(lane) * rows_per_pass + (threadIdx.x >> tpr_shift);
  return (lane < kRowsPerBlock && t < T) ? slot[t] : -1;
}
template <bool WAVE>
__device__ __forceinline__ int64_t row_slot(const int32_t* slot, int32_t my_slot, int k, size_t t, size_t T) {
  if constexpr (WAVE) return __shfl(my_slot, k);
  return t < T ? slot[t] : -1;
}

// blockIdx.y = sender p.  tpr threads (power of two) share a row of upr units.
template <int UB, bool NTL, bool NTS, bool WAVE>
__global__ void __launch_bounds__(kBlock)
moe_dispatch_kernel(PtrTab recv, CPtrTab tok, CPtrTab slot_tab, const int64_t* S, int P, size_t T,
                    uint64_t recv_rows, uint32_t upr, uint32_t tpr, uint32_t tpr_shift) {
  typedef typename RowUnit<UB>::type U;
  __shared__ PairTables tab;
  const int p = blockIdx.y;
  build_pair_tables(tab, S, p, P, static_cast<int64_t>(T));
  const int32_t* slot = static_cast<const int32_t*>(slot_tab.p[p]);
  const U* src = static_cast<const U*>(tok.p[p]);
  const uint32_t rows_per_pass = kBlock >> tpr_shift;
  const size_t t0 = static_cast<size_t>(blockIdx.x) * kRowsPerBlock * rows_per_pass;
  const int32_t my_slot = prefetch_slots<WAVE>(slot, t0, rows_per_pass, tpr_shift, T);
  for (int k0 = 0; k0 < kRowsPerBlock; k0 += kRowsInFlight) {
    const U* srow[kRowsInFlight];
    U* drow[kRowsInFlight];
    bool ok[kRowsInFlight];
#pragma unroll
    for (int j = 0; j < kRowsInFlight; ++j) {
      const size_t t = t0 + static_cast<size_t>(k0 + j) * rows_per_pass + (threadIdx.x >> tpr_shift);
      int r = 0;
      uint64_t row = 0;
      const int64_t sl = row_slot<WAVE>(slot, my_slot, k0 + j, t, T);       // -1: no such token
      ok[j] = locate<WAVE>(tab, P, sl, static_cast<int64_t>(T), recv_rows, &r, &row);
      srow[j] = src + t * upr;
      drow[j] = ok[j] ? static_cast<U*>(recv.p[r]) + row * upr : nullptr;
    }
    for (uint32_t c = threadIdx.x & (tpr - 1); c < upr; c += tpr) {
      U v[kRowsInFlight];
#pragma unroll
      for (int j = 0; j < kRowsInFlight; ++j)
        if (ok[j]) v[j] = ldu<NTL, U>(srow[j] + c);
#pragma unroll
      for (int j = 0; j < kRowsInFlight; ++j)
        if (ok[j]) stu<NTS, U>(drow[j] + c, v[j]);
    }
  }
}

template <int DT, int UB, class U> __device__ __forceinline__ U scale_unit(U v, float g) {
  if constexpr (UB == 16) {
    using E = Elem<DT>;
    float f[E::kPerVec];
    E::widen(v, f);
#pragma unroll
    for (int k = 0; k < E::kPerVec; ++k) f[k] = g * f[k];
    return E::narrow(f);
  } else {
    // one element per unit
    const float y = g * Elem<DT>::widen1(static_cast<uint32_t>(v));
    return static_cast<U>(Elem<DT>::narrow1(y));
  }
}

// out[p] row t = gate[p][t] * (row of expert_out[r] that token t was dispatched to), zeros if dropped.
template <int DT, int UB, bool NTL, bool NTS, bool GATE, bool WAVE>
__global__ void __launch_bounds__(kBlock)
moe_combine_kernel(PtrTab out, CPtrTab expert_out, CPtrTab slot_tab, CPtrTab gate_tab, const int64_t* S, int P,
                   size_t T, uint64_t recv_rows, uint32_t upr, uint32_t tpr, uint32_t tpr_shift) {
  typedef typename RowUnit<UB>::type U;
  __shared__ PairTables tab;
  const int p = blockIdx.y;
  build_pair_tables(tab, S, p, P, static_cast<int64_t>(T));
  const int32_t* slot = static_cast<const int32_t*>(slot_tab.p[p]);
  U* dst = static_cast<U*>(out.p[p]);
  const uint32_t rows_per_pass = kBlock >> tpr_shift;
  const size_t t0 = static_cast<size_t>(blockIdx.x) * kRowsPerBlock * rows_per_pass;
  const int32_t my_slot = prefetch_slots<WAVE>(slot, t0, rows_per_pass, tpr_shift, T);
  for (int k0 = 0; k0 < kRowsPerBlock; k0 += kRowsInFlight) {
    const U* srow[kRowsInFlight];
    U* drow[kRowsInFlight];
    bool live[kRowsInFlight], kept[kRowsInFlight];
    float g[kRowsInFlight];
#pragma unroll
    for (int j = 0; j < kRowsInFlight; ++j) {
      const size_t t = t0 + static_cast<size_t>(k0 + j) * rows_per_pass + (threadIdx.x >> tpr_shift);
      int r = 0;
      uint64_t row = 0;
      live[j] = t < T;
      const int64_t sl = row_slot<WAVE>(slot, my_slot, k0 + j, t, T);
      kept[j] = locate<WAVE>(tab, P, sl, static_cast<int64_t>(T), recv_rows, &r, &row);
      srow[j] = kept[j] ? static_cast<const U*>(expert_out.p[r]) + row * upr : nullptr;
      drow[j] = dst + t * upr;
      g[j] = 1.0f;
      if constexpr (GATE) {
        if (kept[j]) g[j] = static_cast<const float*>(gate_tab.p[p])[t];
      }
    }
    for (uint32_t c = threadIdx.x & (tpr - 1); c < upr; c += tpr) {
      U v[kRowsInFlight];
#pragma unroll
      for (int j = 0; j < kRowsInFlight; ++j) {
        v[j] = U{};
        if (kept[j]) v[j] = ldu<NTL, U>(srow[j] + c);
      }
#pragma unroll
      for (int j = 0; j < kRowsInFlight; ++j) {
        if (!live[j]) continue;
        U y = v[j];
        if constexpr (GATE) {
          if (kept[j]) y = scale_unit<DT, UB, U>(y, g[j]);
        }
        stu<NTS, U>(drow[j] + c, y);
      }
    }
  }
}

// ---- expert-major receive layout -------------------------------------------------------
// The expert FFN wants the tokens of one expert in one block.  The receive buffer of a rank is
// then ordered by (local expert, source rank, token order), and since the packed order of a
// sender is ordered by expert, row(p, t) = row_table[p][id] + slot[p][t] with
//   row_table[p][e] = first row of block (p, e) - (rows sender p packs before expert e).

// One workgroup of kLayoutBlock threads; thread e owns expert e.
constexpr int kLayoutBlock = 512;   // >= MCR_MAX_EXPERTS
constexpr int kLayoutWaves = kLayoutBlock / kWave;

// Inclusive prefix sum over the lanes of a wavefront.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  const unsigned lane = __lane_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int up = __shfl_up(v, d);
    if (lane >= static_cast<unsigned>(d)) v += up;
  }
  return v;
}

// Steps: (1) counts to LDS; (2) thread e walks its column: rows above each sender's block and the
// expert's total; (3) one workgroup-wide scan of the totals gives expert_first; (4) wave w turns
// the rows of senders w and w + 8 into exclusive prefix sums over the experts (what a sender packs
// before expert e), 64 experts at a time with a carry, no workgroup barrier inside; (5) thread e
// writes its column of the table.
__global__ void __launch_bounds__(kLayoutBlock)
moe_expert_layout_kernel(CPtrTab counts, int E, int P, int64_t* row_table, int64_t* expert_first, int64_t* expert_rows) {
  __shared__ int32_t cnt[MCR_MAX_RANKS][MCR_MAX_EXPERTS];
  __shared__ long long wave_total[kLayoutWaves];
  __shared__ long long before_expert[kLayoutBlock];
  const int e = threadIdx.x;
  const unsigned lane = __lane_id();
  const int wave = threadIdx.x / kWave;
  const bool live = e < E;
  const int per_rank = E / P;
  for (int p = 0; p < P; ++p) {
    int32_t x = 0;
    if (live) x = static_cast<const int32_t*>(counts.p[p])[e];
    cnt[p][e] = x > 0 ? x : 0;
  }
  __syncthreads();
  int32_t above[MCR_MAX_RANKS];
  long long rows = 0;
#pragma unroll
  for (int p = 0; p < MCR_MAX_RANKS; ++p) {
    above[p] = static_cast<int32_t>(rows);          // < 2^31: at most P * T rows reach one rank's expert
    if (p < P) rows += cnt[p][e];
  }
  // workgroup-wide exclusive scan of the experts' totals
  long long incl = rows;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const long long up = __shfl_up(incl, d);
    if (lane >= static_cast<unsigned>(d)) incl += up;
  }
  if (lane == kWave - 1) wave_total[wave] = incl;
  __syncthreads();
  long long before = 0;
  for (int w = 0; w < wave; ++w) before += wave_total[w];
  const long long excl = before + incl - rows;
  before_expert[e] = excl;
  // rows of cnt -> what each sender packs before the expert
  for (int p = wave; p < P; p += kLayoutWaves) {
    int carry = 0;
    for (int e0 = 0; e0 < E; e0 += kWave) {
      const int idx = e0 + static_cast<int>(lane);
      const int c = idx < E ? cnt[p][idx] : 0;
      const int inc = wave_inclusive_scan(c);
      if (idx < E) cnt[p][idx] = carry + inc - c;
      carry += __shfl(inc, kWave - 1);
    }
  }
  __syncthreads();
  if (!live) return;
  const long long first = excl - before_expert[(e / per_rank) * per_rank];
  expert_first[e] = first;
  expert_rows[e] = rows;
#pragma unroll
  for (int p = 0; p < MCR_MAX_RANKS; ++p)
    if (p < P) row_table[static_cast<size_t>(p) * E + e] = first + above[p] - cnt[p][e];
}

// The row table of the source-major layout, the one pack + all_to_allv leave behind: at receiver r
// the rows are ordered by (source rank, local expert, token order), so with S[p][r] = kept tokens
// of sender p for the experts of rank r,
//   row_table[p][e] = sum_{q<p} S[q][r(e)] - sum_{r'<r(e)} S[p][r'],
// and the by-expert dispatch / combine kernels, fed this table, reproduce that layout.
__global__ void __launch_bounds__(kLayoutBlock)
moe_source_layout_kernel(CPtrTab counts, int E, int P, int64_t* row_table) {
  __shared__ int32_t cnt[MCR_MAX_RANKS][MCR_MAX_EXPERTS];
  __shared__ long long S[MCR_MAX_RANKS][MCR_MAX_RANKS];
  const int e = threadIdx.x;
  const bool live = e < E;
  const int per_rank = E / P;
  for (int p = 0; p < P; ++p) {
    int32_t x = 0;
    if (live) x = static_cast<const int32_t*>(counts.p[p])[e];
    cnt[p][e] = x > 0 ? x : 0;
  }
  __syncthreads();
  if (threadIdx.x < P * P) {
    const int p = threadIdx.x / P, r = threadIdx.x % P;
    long long a = 0;
    for (int k = r * per_rank; k < (r + 1) * per_rank; ++k) a += cnt[p][k];
    S[p][r] = a;
  }
  __syncthreads();
  if (!live) return;
  const int r = e / per_rank;
  long long above = 0;                                   // rows of the senders before p at receiver r
  for (int p = 0; p < P; ++p) {
    long long left = 0;                                  // rows sender p packs for the receivers before r
    for (int q = 0; q < r; ++q) left += S[p][q];
    row_table[static_cast<size_t>(p) * E + e] = above - left;
    above += S[p][r];
  }
}

// Where token t of this sender goes: rank (negative: nowhere) and row in that rank's buffer.
struct RowDest {
  int32_t r;
  int64_t row;
};
__device__ __forceinline__ RowDest dest_of(const int64_t* table, const int32_t* ids, const int32_t* slot, size_t t, size_t T,
                                           int E, int per_rank, uint64_t recv_rows) {
  RowDest d{-1, 0};
  if (t >= T) return d;
  const int32_t sl = slot[t];
  const int32_t e = ids[t];
  if (sl < 0 || e < 0 || e >= E) return d;
  const int64_t row = table[e] + sl;
  if (row < 0 || static_cast<uint64_t>(row) >= recv_rows) return d;
  d.r = e / per_rank;
  d.row = row;
  return d;
}
// WAVE (a row is at least a wavefront wide): lane k resolves the wave's k-th row once, before the
// row loop, and the loop fetches the answer by shuffle.
template <bool WAVE>
__device__ __forceinline__ RowDest prefetch_dest(const int64_t* table, const int32_t* ids, const int32_t* slot, size_t t0,
                                                 uint32_t rows_per_pass, uint32_t tpr_shift, size_t T, int E, int per_rank,
                                                 uint64_t recv_rows) {
  if constexpr (!WAVE) return RowDest{-1, 0};
  const unsigned lane = __lane_id();
  const size_t t = t0 + static_cast<size_t>(lane) * rows_per_pass + (threadIdx.x >> tpr_shift);
  return dest_of(table, ids, slot, lane < kRowsPerBlock ? t : T, T, E, per_rank, recv_rows);
}
template <bool WAVE>
__device__ __forceinline__ RowDest row_dest(const RowDest& mine, int k, const int64_t* table, const int32_t* ids,
                                            const int32_t* slot, size_t t, size_t T, int E, int per_rank, uint64_t recv_rows) {
  if constexpr (WAVE) {
    RowDest d;
    d.r = __shfl(mine.r, k);
    const uint32_t lo = __shfl(static_cast<uint32_t>(mine.row), k);
    const uint32_t hi = __shfl(static_cast<uint32_t>(static_cast<uint64_t>(mine.row) >> 32), k);
    d.row = static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
    return d;
  } else {
    return dest_of(table, ids, slot, t, T, E, per_rank, recv_rows);
  }
}

__device__ __forceinline__ void stage_row_table(int64_t* lds, const int64_t* row_table, int p, int E) {
  for (int e = threadIdx.x; e < E; e += kBlock) lds[e] = row_table[static_cast<size_t>(p) * E + e];
  __syncthreads();
}

// A = K*T assignments per sender, choice-major (assignment a is choice a / T of token a mod T);
// the rows walked are assignments, the row read is the token's.
template <int UB, bool NTL, bool NTS, bool WAVE>
__global__ void __launch_bounds__(kBlock)
moe_dispatch_by_expert_kernel(PtrTab recv, CPtrTab tok, CPtrTab ids_tab, CPtrTab slot_tab, const int64_t* row_table, int E,
                              int P, size_t A, size_t T, uint64_t recv_rows, uint32_t upr, uint32_t tpr, uint32_t tpr_shift) {
  typedef typename RowUnit<UB>::type U;
  __shared__ int64_t table[MCR_MAX_EXPERTS];
  const int p = blockIdx.y;
  stage_row_table(table, row_table, p, E);
  const int per_rank = E / P;
  const int32_t* slot = static_cast<const int32_t*>(slot_tab.p[p]);
  const int32_t* ids = static_cast<const int32_t*>(ids_tab.p[p]);
  const U* src = static_cast<const U*>(tok.p[p]);
  const uint32_t rows_per_pass = kBlock >> tpr_shift;
  const size_t a0 = static_cast<size_t>(blockIdx.x) * kRowsPerBlock * rows_per_pass;
  const RowDest mine = prefetch_dest<WAVE>(table, ids, slot, a0, rows_per_pass, tpr_shift, A, E, per_rank, recv_rows);
  for (int k0 = 0; k0 < kRowsPerBlock; k0 += kRowsInFlight) {
    const U* srow[kRowsInFlight];
    U* drow[kRowsInFlight];
    bool ok[kRowsInFlight];
#pragma unroll
    for (int j = 0; j < kRowsInFlight; ++j) {
      const size_t a = a0 + static_cast<size_t>(k0 + j) * rows_per_pass + (threadIdx.x >> tpr_shift);
      const RowDest d = row_dest<WAVE>(mine, k0 + j, table, ids, slot, a, A, E, per_rank, recv_rows);
      ok[j] = d.r >= 0 && d.r < P;
      const size_t t = a < T ? a : a % T;
      srow[j] = src + t * upr;
      drow[j] = ok[j] ? static_cast<U*>(recv.p[d.r]) + static_cast<uint64_t>(d.row) * upr : nullptr;
    }
    for (uint32_t c = threadIdx.x & (tpr - 1); c < upr; c += tpr) {
      U v[kRowsInFlight];
#pragma unroll
      for (int j = 0; j < kRowsInFlight; ++j)
        if (ok[j]) v[j] = ldu<NTL, U>(srow[j] + c);
#pragma unroll
      for (int j = 0; j < kRowsInFlight; ++j)
        if (ok[j]) stu<NTS, U>(drow[j] + c, v[j]);
    }
  }
}

template <int DT, int UB, bool NTL, bool NTS, bool GATE, bool WAVE>
__global__ void __launch_bounds__(kBlock)
moe_combine_by_expert_kernel(PtrTab out, CPtrTab expert_out, CPtrTab ids_tab, CPtrTab slot_tab, CPtrTab gate_tab,
                             const int64_t* row_table, int E, int P, size_t T, uint64_t recv_rows, uint32_t upr,
                             uint32_t tpr, uint32_t tpr_shift) {
  typedef typename RowUnit<UB>::type U;
  __shared__ int64_t table[MCR_MAX_EXPERTS];
  const int p = blockIdx.y;
  stage_row_table(table, row_table, p, E);
  const int per_rank = E / P;
  const int32_t* slot = static_cast<const int32_t*>(slot_tab.p[p]);
  const int32_t* ids = static_cast<const int32_t*>(ids_tab.p[p]);
  U* dst = static_cast<U*>(out.p[p]);
  const uint32_t rows_per_pass = kBlock >> tpr_shift;
  const size_t t0 = static_cast<size_t>(blockIdx.x) * kRowsPerBlock * rows_per_pass;
  const RowDest mine = prefetch_dest<WAVE>(table, ids, slot, t0, rows_per_pass, tpr_shift, T, E, per_rank, recv_rows);
  for (int k0 = 0; k0 < kRowsPerBlock; k0 += kRowsInFlight) {
    const U* srow[kRowsInFlight];
    U* drow[kRowsInFlight];
    bool live[kRowsInFlight], kept[kRowsInFlight];
    float g[kRowsInFlight];
#pragma unroll
    for (int j = 0; j < kRowsInFlight; ++j) {
      const size_t t = t0 + static_cast<size_t>(k0 + j) * rows_per_pass + (threadIdx.x >> tpr_shift);
      const RowDest d = row_dest<WAVE>(mine, k0 + j, table, ids, slot, t, T, E, per_rank, recv_rows);
      live[j] = t < T;
      kept[j] = d.r >= 0 && d.r < P;
      srow[j] = kept[j] ? static_cast<const U*>(expert_out.p[d.r]) + static_cast<uint64_t>(d.row) * upr : nullptr;
      drow[j] = dst + t * upr;
      g[j] = 1.0f;
      if constexpr (GATE) {
        if (kept[j]) g[j] = static_cast<const float*>(gate_tab.p[p])[t];
      }
    }
    for (uint32_t c = threadIdx.x & (tpr - 1); c < upr; c += tpr) {
      U v[kRowsInFlight];
#pragma unroll
      for (int j = 0; j < kRowsInFlight; ++j) {
        v[j] = U{};
        if (kept[j]) v[j] = ldu<NTL, U>(srow[j] + c);
      }
#pragma unroll
      for (int j = 0; j < kRowsInFlight; ++j) {
        if (!live[j]) continue;
        U y = v[j];
        if constexpr (GATE) {
          if (kept[j]) y = scale_unit<DT, UB, U>(y, g[j]);
        }
        stu<NTS, U>(drow[j] + c, y);
      }
    }
  }
}

// Top-K combine: out[p] row t = round(sum over the kept choices k, in order, of gate[k*T + t] *
// f32(row of assignment k*T + t)): binary32 products and sums, the sum starting from the first kept
// product, one rounding at the end; all-zero bits when nothing was kept.  KU = compile-time bound
// on K.  One group of tpr threads per token row, kTopkRows rows per group and workgroup.
constexpr int kTopkRows = 16;   // rows one group of threads walks
constexpr int kTopkFly = 2;     // rows whose loads are in flight together (4 measured no faster)
template <int DT, int UB> struct UnitF32 {
  static constexpr int kN = UB / Elem<DT>::kBytes;
  typedef typename RowUnit<UB>::type U;
  __device__ static __forceinline__ void widen(U v, float (&f)[kN]) {
    if constexpr (UB == 16) Elem<DT>::widen(v, f);
    else f[0] = Elem<DT>::widen1(static_cast<uint32_t>(v));
  }
  __device__ static __forceinline__ U narrow(const float (&f)[kN]) {
    if constexpr (UB == 16) return Elem<DT>::narrow(f);
    else return static_cast<U>(Elem<DT>::narrow1(f[0]));
  }
};

// WAVE (a row is at least a wavefront wide): lane i*KU + k resolves choice k of the wave's i-th
// row (destination and gate) once, before the row loop, which fetches them by shuffle; kTopkFly
// rows have their K loads each in flight together.
template <int DT, int UB, int KU, bool NTL, bool NTS, bool WAVE>
__global__ void __launch_bounds__(kBlock)
moe_combine_topk_kernel(PtrTab out, CPtrTab expert_out, CPtrTab ids_tab, CPtrTab slot_tab, CPtrTab gate_tab,
                        const int64_t* row_table, int E, int P, size_t T, int K, uint64_t recv_rows, uint32_t upr,
                        uint32_t tpr, uint32_t tpr_shift) {
  typedef typename RowUnit<UB>::type U;
  typedef UnitF32<DT, UB> F;
  static_assert(kTopkRows * KU <= kWave, "one lane per (row, choice)");
  __shared__ int64_t table[MCR_MAX_EXPERTS];
  const int p = blockIdx.y;
  stage_row_table(table, row_table, p, E);
  const int per_rank = E / P;
  const int32_t* slot = static_cast<const int32_t*>(slot_tab.p[p]);
  const int32_t* ids = static_cast<const int32_t*>(ids_tab.p[p]);
  const float* gate = static_cast<const float*>(gate_tab.p[p]);
  U* dst = static_cast<U*>(out.p[p]);
  const uint32_t rows_per_pass = kBlock >> tpr_shift;
  const size_t A = T * static_cast<size_t>(K);
  const size_t t0 = static_cast<size_t>(blockIdx.x) * kTopkRows * rows_per_pass;
  const uint32_t group = threadIdx.x >> tpr_shift;
  RowDest mine{-1, 0};
  float my_gate = 1.0f;
  if constexpr (WAVE) {
    const int lane = static_cast<int>(__lane_id());
    const int li = lane / KU, lk = lane % KU;
    const size_t t = t0 + static_cast<size_t>(li) * rows_per_pass + group;
    if (li < kTopkRows && lk < K && t < T) {
      const size_t a = static_cast<size_t>(lk) * T + t;
      mine = dest_of(table, ids, slot, a, A, E, per_rank, recv_rows);
      if (mine.r >= 0 && mine.r < P && gate) my_gate = gate[a];
    }
  }
  for (int i0 = 0; i0 < kTopkRows; i0 += kTopkFly) {
    const U* srow[kTopkFly][KU];
    float g[kTopkFly][KU];
    bool kept[kTopkFly][KU];
    bool live[kTopkFly];
    U* drow[kTopkFly];
#pragma unroll
    for (int j = 0; j < kTopkFly; ++j) {
      const size_t t = t0 + static_cast<size_t>(i0 + j) * rows_per_pass + group;
      live[j] = t < T;
      drow[j] = dst + t * upr;
#pragma unroll
      for (int k = 0; k < KU; ++k) {
        RowDest d{-1, 0};
        g[j][k] = 1.0f;
        if constexpr (WAVE) {
          const int src_lane = (i0 + j) * KU + k;
          d.r = __shfl(mine.r, src_lane);
          const uint32_t lo = __shfl(static_cast<uint32_t>(mine.row), src_lane);
          const uint32_t hi = __shfl(static_cast<uint32_t>(static_cast<uint64_t>(mine.row) >> 32), src_lane);
          d.row = static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
          g[j][k] = __shfl(my_gate, src_lane);
        } else {
          if (k < K && live[j]) {
            const size_t a = static_cast<size_t>(k) * T + t;
            d = dest_of(table, ids, slot, a, A, E, per_rank, recv_rows);
            if (d.r >= 0 && d.r < P && gate) g[j][k] = gate[a];
          }
        }
        kept[j][k] = d.r >= 0 && d.r < P;
        srow[j][k] = kept[j][k] ? static_cast<const U*>(expert_out.p[d.r]) + static_cast<uint64_t>(d.row) * upr : nullptr;
      }
    }
    for (uint32_t c = threadIdx.x & (tpr - 1); c < upr; c += tpr) {
      U v[kTopkFly][KU];
#pragma unroll
      for (int j = 0; j < kTopkFly; ++j) {
#pragma unroll
        for (int k = 0; k < KU; ++k) {
          v[j][k] = U{};
          if (kept[j][k]) v[j][k] = ldu<NTL, U>(srow[j][k] + c);
        }
      }
#pragma unroll
      for (int j = 0; j < kTopkFly; ++j) {
        if (!live[j]) continue;
        float acc[F::kN];
        bool started = false;
#pragma unroll
        for (int k = 0; k < KU; ++k) {
          if (!kept[j][k]) continue;
          float f[F::kN];
          F::widen(v[j][k], f);
#pragma unroll
          for (int e = 0; e < F::kN; ++e) {
            const float term = g[j][k] * f[e];
            acc[e] = started ? acc[e] + term : term;
          }
          started = true;
        }
        U y = U{};
        if (started) y = F::narrow(acc);
        stu<NTS, U>(drow[j] + c, y);
      }
    }
  }
}

// ---- the same three operations for rows wider than half a workgroup: one row per workgroup.
// The row index is uniform over the workgroup, so id, slot, table entry and gate come through
// scalar loads and nothing is staged in LDS; a one-shot grid of one-row workgroups is also the
// shape in which 4 KiB rows move fastest on this GPU (6.0 TB/s against 5.0 for 32 rows per
// workgroup in a plain permutation of rows).
// Every lookup is written without a branch in front of it (indices are clamped, validity is
// decided afterwards), so that the loads of one level go out together: kernel arguments, then
// slot / id / gate of the row, then the table entry and the destination's base pointer, then the
// row itself.  With early exits between them the compiler strings the scalar loads into eight
// round trips, which made this shape slower than the one it replaces.
// `rank_magic` = ceil(2^32 / (E/P)): (e * rank_magic) >> 32 == e / (E/P) for every e < 2^23.
struct RowLookup {
  int64_t row;
  int r;
  bool ok;
};
__device__ __forceinline__ RowLookup lookup_row(const int64_t* table_p, int32_t sl, int32_t e, int E, uint64_t rank_magic,
                                                uint64_t recv_rows) {
  const int ec = e < 0 ? 0 : (e >= E ? E - 1 : e);
  RowLookup out;
  out.row = table_p[ec] + sl;
  out.r = static_cast<int>((static_cast<uint64_t>(ec) * rank_magic) >> 32);
  out.ok = sl >= 0 && e == ec && out.row >= 0 && static_cast<uint64_t>(out.row) < recv_rows;
  return out;
}

// blockIdx.x = token t, blockIdx.y = sender.  K choices (KU >= K at compile time): the token's row
// is read once and stored to the place of every kept choice.  AL = false: rows of any width and
// alignment, as 16-byte pieces at element-aligned addresses and `tail2` 2-byte units.
template <int KU, bool NTL, bool NTS, bool AL>
__global__ void __launch_bounds__(kBlock)
moe_dispatch_row_kernel(PtrTab recv, CPtrTab tok, CPtrTab ids_tab, CPtrTab slot_tab, const int64_t* row_table, int E,
                        uint64_t rank_magic, size_t T, int K, uint64_t recv_rows, size_t row_bytes, uint32_t pieces,
                        uint32_t tail2) {
  const int p = blockIdx.y;
  const size_t t = blockIdx.x;
  const int32_t* slot = static_cast<const int32_t*>(slot_tab.p[p]);
  const int32_t* ids = static_cast<const int32_t*>(ids_tab.p[p]);
  const int64_t* table = row_table + static_cast<size_t>(p) * E;
  int32_t sl[KU], e[KU];
#pragma unroll
  for (int k = 0; k < KU; ++k) {
    const size_t a = (k < K) ? static_cast<size_t>(k) * T + t : t;          // always a valid index
    sl[k] = slot[a];
    e[k] = ids[a];
  }
  char* drow[KU];
  bool kept[KU];
  bool any = false;
#pragma unroll
  for (int k = 0; k < KU; ++k) {
    const RowLookup d = lookup_row(table, sl[k], e[k], E, rank_magic, recv_rows);
    kept[k] = d.ok && k < K;
    drow[k] = static_cast<char*>(recv.p[d.r]) + static_cast<uint64_t>(kept[k] ? d.row : 0) * row_bytes;   // d.r < P whatever the id was
    any = any || kept[k];
  }
  if (!any) return;
  const char* srow = static_cast<const char*>(tok.p[p]) + t * row_bytes;
  constexpr int BS = kBlock, V = 1;
  for (uint32_t c0 = threadIdx.x; c0 < pieces; c0 += V * BS) {
    u32x4 v[V];
#pragma unroll
    for (int u = 0; u < V; ++u)
      if (c0 + u * BS < pieces) v[u] = load_piece<NTL, AL>(srow, c0 + u * BS);
#pragma unroll
    for (int k = 0; k < KU; ++k) {
      if (!kept[k]) continue;
#pragma unroll
      for (int u = 0; u < V; ++u)
        if (c0 + u * BS < pieces) store_piece<NTS, AL>(drow[k], c0 + u * BS, v[u]);
    }
  }
  if (!AL && threadIdx.x < tail2) {
#pragma unroll
    for (int k = 0; k < KU; ++k)
      if (kept[k]) copy_tail2(drow[k], srow, pieces, threadIdx.x);
  }
}

// The weighted sum of the kept choices' values, in choice order, starting from the first kept
// product; `started` tells whether anything was kept.
template <int KU, int N>
__device__ __forceinline__ bool weighted_sum(const float (&f)[KU][N], const float (&g)[KU], const bool (&kept)[KU], float (&acc)[N]) {
  bool started = false;
#pragma unroll
  for (int k = 0; k < KU; ++k) {
    if (!kept[k]) continue;
#pragma unroll
    for (int x = 0; x < N; ++x) {
      const float term = g[k] * f[k][x];
      acc[x] = started ? acc[x] + term : term;
    }
    started = true;
  }
  return started;
}

// blockIdx.x = token t.  K choices (KU >= K at compile time).  A gather with a chain of lookups in
// front of it is bound by how many rows a compute unit has in flight, so the workgroup is half the
// usual size (kRowGatherBlock threads, twice as many rows per compute unit) and every thread keeps
// the loads of kRowGatherVecs units of each kept row in flight (6.1 against 5.4 TB/s in a plain
// gather of 4 KiB rows behind a two-level lookup).  AL = false: rows of any width and alignment
// (16-byte pieces at element-aligned addresses, then `tail` single elements).
template <int DT, int KU, bool NTL, bool NTS, bool GATE, bool AL>
__global__ void __launch_bounds__(kRowGatherBlock)
moe_combine_row_kernel(PtrTab out, CPtrTab expert_out, CPtrTab ids_tab, CPtrTab slot_tab, CPtrTab gate_tab,
                       const int64_t* row_table, int E, uint64_t rank_magic, size_t T, int K, uint64_t recv_rows,
                       size_t row_bytes, uint32_t upr, uint32_t tail) {
  using EL = Elem<DT>;
  constexpr int N = EL::kPerVec;
  constexpr int V = kRowGatherVecs;
  const int p = blockIdx.y;
  const size_t t = blockIdx.x;
  const int32_t* slot = static_cast<const int32_t*>(slot_tab.p[p]);
  const int32_t* ids = static_cast<const int32_t*>(ids_tab.p[p]);
  const float* gate = static_cast<const float*>(gate_tab.p[p]);
  const int64_t* table = row_table + static_cast<size_t>(p) * E;
  char* drow = static_cast<char*>(out.p[p]) + t * row_bytes;
  int32_t sl[KU], e[KU];
  float g[KU];
#pragma unroll
  for (int k = 0; k < KU; ++k) {
    const size_t a = (k < K) ? static_cast<size_t>(k) * T + t : t;          // always a valid index
    sl[k] = slot[a];
    e[k] = ids[a];
    g[k] = 1.0f;
    if constexpr (GATE) g[k] = gate[a];
  }
  const char* srow[KU];
  bool kept[KU];
  bool any = false;
#pragma unroll
  for (int k = 0; k < KU; ++k) {
    const RowLookup d = lookup_row(table, sl[k], e[k], E, rank_magic, recv_rows);
    kept[k] = d.ok && k < K;
    srow[k] = static_cast<const char*>(expert_out.p[d.r]) + static_cast<uint64_t>(kept[k] ? d.row : 0) * row_bytes;
    any = any || kept[k];
  }
  const size_t first_tail = static_cast<size_t>(upr) * N;
  if (!any) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (uint32_t c = threadIdx.x; c < upr; c += kRowGatherBlock) store_piece<NTS, AL>(drow, c, z);
    if (!AL && threadIdx.x < tail) EL::store1(drow, first_tail + threadIdx.x, typename EL::acc_t(0));
    return;
  }
  for (uint32_t c0 = threadIdx.x; c0 < upr; c0 += V * kRowGatherBlock) {
    u32x4 v[V][KU];
#pragma unroll
    for (int u = 0; u < V; ++u) {
      const uint32_t c = c0 + u * kRowGatherBlock;
#pragma unroll
      for (int k = 0; k < KU; ++k) {
        v[u][k] = u32x4{0u, 0u, 0u, 0u};
        if (kept[k] && c < upr) v[u][k] = load_piece<NTL, AL>(srow[k], c);
      }
    }
#pragma unroll
    for (int u = 0; u < V; ++u) {
      const uint32_t c = c0 + u * kRowGatherBlock;
      if (c >= upr) continue;
      if constexpr (KU == 1 && !GATE) {                 // one choice and no weight: the row is copied bit for bit
        store_piece<NTS, AL>(drow, c, v[u][0]);
      } else {
        float f[KU][N], acc[N];
#pragma unroll
        for (int k = 0; k < KU; ++k) EL::widen(v[u][k], f[k]);
        weighted_sum<KU, N>(f, g, kept, acc);           // something was kept: `any`
        store_piece<NTS, AL>(drow, c, EL::narrow(acc));
      }
    }
  }
  if (!AL && threadIdx.x < tail) {
    const size_t i = first_tail + threadIdx.x;
    if constexpr (KU == 1 && !GATE) {
      copy_elem<EL::kBytes>(drow, srow[0], i);
    } else {
      float f[KU][1], acc[1];
#pragma unroll
      for (int k = 0; k < KU; ++k) f[k][0] = kept[k] ? EL::load1(srow[k], i) : 0.0f;
      weighted_sum<KU, 1>(f, g, kept, acc);
      EL::store1(drow, i, acc[0]);
    }
  }
}

// ---- the source-major fused pair on wide rows: one row per workgroup -------------------------
// mcr_moe_dispatch / mcr_moe_combine know a token's place only through its slot and the split
// matrix.  A first launch of one workgroup turns the matrix into the displacement tables of a
// PairSlot; the row kernels then find the receiver of a slot among the (at most 16) block starts of
// their sender and the row from one more entry, all through scalar loads of that table: the same
// three dependent steps (slot, table entry, row) as the table-driven kernels above.
__global__ void __launch_bounds__(kBlock)
moe_pair_tables_kernel(const int64_t* S, int P, int64_t cap, PairSlot* out) {
  __shared__ int64_t s[MCR_MAX_RANKS][MCR_MAX_RANKS];
  const int p = threadIdx.x / MCR_MAX_RANKS, r = threadIdx.x % MCR_MAX_RANKS;       // 256 threads: one per (p, r)
  s[p][r] = (p < P && r < P) ? clamp_rows(S[p * P + r], cap) : 0;                    // one load per thread, all in flight
  __syncthreads();
  constexpr int64_t kTop = 0x7fffffff;
  int64_t sd = 0, rd = 0;
  for (int q = 0; q < r; ++q) sd += s[p][q];
  for (int q = 0; q < p; ++q) rd += s[q][r];
  const bool live = p < P && r < P;
  out->start[p][r] = live ? static_cast<int32_t>(sd < kTop ? sd : kTop) : static_cast<int32_t>(kTop);
  out->delta[p][r] = live ? rd - sd : 0;
  if (r == MCR_MAX_RANKS - 1) {
    const int64_t all = sd + s[p][r];                                                // rows beyond P count 0
    out->start[p][MCR_MAX_RANKS] = p < P ? static_cast<int32_t>(all < kTop ? all : kTop) : 0;
  }
}

// Receiver and row of packed row `s` of sender p: the receiver is the number of block starts at or
// below s (the starts are non-decreasing; empty blocks share a start and the last of them, the one
// that holds the row, wins).  Lane q of the wavefront holds start q (lane 16 the total), one load
// for all of them, and a ballot counts; half of the workgroups of a dispatch carry a dropped token
// and do nothing but this, so it is kept to a handful of instructions and has no branch in it.
struct PairDest {
  int r;
  int64_t row;
  bool ok;
};
__device__ __forceinline__ PairDest pair_dest(const PairSlot* tab, int p, int32_t s, int64_t send_rows, uint64_t recv_rows) {
  const unsigned lane = __lane_id();
  const int32_t mine_start = tab->start[p][lane & 31u];                  // entries 17..31 of a row are never looked at
  const uint64_t at_or_below = __ballot(mine_start <= s);
  const int r = __popcll(at_or_below & 0xfffeull);                       // starts 1..15
  const bool in_range = ((at_or_below >> MCR_MAX_RANKS) & 1ull) == 0;    // s < all the rows p sends
  PairDest d;
  const bool mine = s >= 0 && in_range && s < send_rows;
  d.r = mine ? r : 0;
  d.row = s + tab->delta[p][d.r];
  d.ok = mine && d.row >= 0 && static_cast<uint64_t>(d.row) < recv_rows;
  return d;
}

template <bool NTL, bool NTS, bool AL>
__global__ void __launch_bounds__(kPairScatterBlock)
moe_dispatch_pairs_row_kernel(PtrTab recv, CPtrTab tok, CPtrTab slot_tab, const PairSlot* tab, size_t T,
                              uint64_t recv_rows, size_t row_bytes, uint32_t pieces, uint32_t tail2) {
  const int p = blockIdx.y;
  const size_t t = blockIdx.x;
  const int32_t s = static_cast<const int32_t*>(slot_tab.p[p])[t];
  const PairDest d = pair_dest(tab, p, s, static_cast<int64_t>(T), recv_rows);
  const char* srow = static_cast<const char*>(tok.p[p]) + t * row_bytes;
  char* drow = static_cast<char*>(recv.p[d.r]) + static_cast<uint64_t>(d.ok ? d.row : 0) * row_bytes;
  // a row that goes nowhere has no pieces: the loop bounds are the only branches
  const uint32_t n = d.ok ? pieces : 0, n_tail = d.ok ? tail2 : 0;
  copy_row_pieces<kPairScatterBlock, kPairScatterVecs, NTL, NTS, AL>(drow, srow, n);
  if (!AL && threadIdx.x < n_tail) copy_tail2(drow, srow, pieces, threadIdx.x);
}

template <int DT, bool NTL, bool NTS, bool GATE, bool AL>
__global__ void __launch_bounds__(kRowGatherBlock)
moe_combine_pairs_row_kernel(PtrTab out, CPtrTab expert_out, CPtrTab slot_tab, CPtrTab gate_tab, const PairSlot* tab,
                             size_t T, uint64_t recv_rows, size_t row_bytes, uint32_t upr, uint32_t tail) {
  using EL = Elem<DT>;
  constexpr int V = kRowGatherVecs;
  const int p = blockIdx.y;
  const size_t t = blockIdx.x;
  const int32_t s = static_cast<const int32_t*>(slot_tab.p[p])[t];
  float g = 1.0f;
  if constexpr (GATE) g = static_cast<const float*>(gate_tab.p[p])[t];
  const PairDest d = pair_dest(tab, p, s, static_cast<int64_t>(T), recv_rows);
  char* drow = static_cast<char*>(out.p[p]) + t * row_bytes;
  const char* srow = static_cast<const char*>(expert_out.p[d.r]) + static_cast<uint64_t>(d.ok ? d.row : 0) * row_bytes;
  const size_t first_tail = static_cast<size_t>(upr) * EL::kPerVec;
  if (!d.ok) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (uint32_t c = threadIdx.x; c < upr; c += kRowGatherBlock) store_piece<NTS, AL>(drow, c, z);
    if (!AL && threadIdx.x < tail) EL::store1(drow, first_tail + threadIdx.x, typename EL::acc_t(0));
    return;
  }
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
      if constexpr (GATE) v[u] = scale_unit<DT, 16, u32x4>(v[u], g);
      store_piece<NTS, AL>(drow, c, v[u]);
    }
  }
  if (!AL && threadIdx.x < tail) {
    const size_t i = first_tail + threadIdx.x;
    if constexpr (GATE) EL::store1(drow, i, g * EL::load1(srow, i));
    else copy_elem<EL::kBytes>(drow, srow, i);
  }
}

// DLRM shuffle.  Table t lives on rank t mod P as local table t div P; the table-major side is
// [T_p][batch][dim], the batch-major side [batch/P][n_tables][dim].  blockIdx.y = rank r of the
// batch-major side; rows j = b*n_tables + t of that side are walked in order.
//   forward : batch[r] row j  = table[t mod P] row (t div P)*batch + r*bl + b
//   backward: table[t mod P] row (...)        = batch[r] row j
template <int UB, bool NTL, bool NTS, bool BWD>
__global__ void __launch_bounds__(kBlock)
dlrm_shuffle_kernel(PtrTab dst_tab, CPtrTab src_tab, uint32_t n_tables, uint64_t batch, uint32_t P, uint32_t upr,
                    uint32_t tpr, uint32_t tpr_shift) {
  typedef typename RowUnit<UB>::type U;
  const uint32_t r = blockIdx.y;
  const uint64_t bl = batch / P;
  const uint64_t rows = bl * n_tables;
  const uint32_t rows_per_pass = kBlock >> tpr_shift;
  const uint64_t j = static_cast<uint64_t>(blockIdx.x) * rows_per_pass + (threadIdx.x >> tpr_shift);
  if (j >= rows) return;
  const uint64_t b = j / n_tables;
  const uint32_t t = static_cast<uint32_t>(j - b * n_tables);
  const uint32_t owner = t % P, local = t / P;
  const uint64_t trow = static_cast<uint64_t>(local) * batch + static_cast<uint64_t>(r) * bl + b;
  const U* s;
  U* d;
  if constexpr (BWD) {
    s = static_cast<const U*>(src_tab.p[r]) + j * upr;
    d = static_cast<U*>(dst_tab.p[owner]) + trow * upr;
  } else {
    s = static_cast<const U*>(src_tab.p[owner]) + trow * upr;
    d = static_cast<U*>(dst_tab.p[r]) + j * upr;
  }
  for (uint32_t c = threadIdx.x & (tpr - 1); c < upr; c += tpr) stu<NTS, U>(d + c, ldu<NTL, U>(s + c));
}

// The same walk for rows that are not a multiple of 16 bytes wide or not 16-byte aligned: whole
// 16-byte pieces at whatever address the elements fall on, then the `tail2` 2-byte units behind them
// (one element per access, the form for rows under 64 bytes, is what this replaces).
template <bool NTL, bool NTS, bool BWD>
__global__ void __launch_bounds__(kBlock)
dlrm_shuffle_pieces_kernel(PtrTab dst_tab, CPtrTab src_tab, uint32_t n_tables, uint64_t batch, uint32_t P, uint32_t row_bytes,
                           uint32_t pieces, uint32_t tail2, uint32_t tpr, uint32_t tpr_shift) {
  const uint32_t r = blockIdx.y;
  const uint64_t bl = batch / P;
  const uint64_t rows = bl * n_tables;
  const uint32_t rows_per_pass = kBlock >> tpr_shift;
  const uint64_t j = static_cast<uint64_t>(blockIdx.x) * rows_per_pass + (threadIdx.x >> tpr_shift);
  if (j >= rows) return;
  const uint64_t b = j / n_tables;
  const uint32_t t = static_cast<uint32_t>(j - b * n_tables);
  const uint32_t owner = t % P, local = t / P;
  const uint64_t trow = static_cast<uint64_t>(local) * batch + static_cast<uint64_t>(r) * bl + b;
  const char* s;
  char* d;
  if constexpr (BWD) {
    s = static_cast<const char*>(src_tab.p[r]) + j * row_bytes;
    d = static_cast<char*>(dst_tab.p[owner]) + trow * row_bytes;
  } else {
    s = static_cast<const char*>(src_tab.p[owner]) + trow * row_bytes;
    d = static_cast<char*>(dst_tab.p[r]) + j * row_bytes;
  }
  const uint32_t lane = threadIdx.x & (tpr - 1);
  for (uint32_t c = lane; c < pieces; c += tpr) store_piece<NTS, false>(d, c, load_piece<NTL, false>(s, c));
  if (lane < tail2) copy_tail2(d, s, pieces, lane);
}

struct RowShape {
  uint32_t upr, tpr, shift, rows_per_pass;
};
inline RowShape row_shape(size_t units_per_row) {
  RowShape s;
  s.upr = static_cast<uint32_t>(units_per_row);
  s.shift = 0;
  while ((1u << s.shift) < s.upr && s.shift < 8) ++s.shift;   // tpr = min(256, pow2 >= upr)
  s.tpr = 1u << s.shift;
  s.rows_per_pass = kBlock >> s.shift;
  return s;
}
// ceil(2^32 / (E/P)): the multiplier that turns an expert id into its rank without a division
inline uint64_t rank_magic(int E, int P) {
  const uint64_t per_rank = static_cast<uint64_t>(E / P);
  return ((uint64_t(1) << 32) + per_rank - 1) / per_rank;
}
inline unsigned blocks_for(size_t rows, size_t rows_per_block) {
  size_t b = (rows + rows_per_block - 1) / rows_per_block;
  return static_cast<unsigned>(b ? b : 1);
}

}  // namespace

// The next slot of the context's ring, filled with the displacement tables of `splits` by a launch
// on `stream` (the row kernels that follow on the same stream read it).
static int stage_pair_tables(mcr_ctx* ctx, const int64_t* splits, int P, size_t T, hipStream_t stream, const PairSlot** out) {
  PairSlot* slot = ctx->pair_ring + ctx->pair_next.fetch_add(1u) % kPairRingSlots;
  hipLaunchKernelGGL(moe_pair_tables_kernel, dim3(1), dim3(kBlock), 0, stream, splits, P, static_cast<int64_t>(T), slot);
  *out = slot;
  return launch_status();
}

int launch_moe_dispatch(mcr_ctx* ctx, const PtrTab& recv, const CPtrTab& tok, const CPtrTab& slot, const int64_t* splits,
                        size_t T, size_t recv_rows, size_t row_bytes, int elem_b, int P, int variant, hipStream_t stream) {
  if (T == 0 || row_bytes == 0) return MCR_OK;
  if (row_bytes / 16 > kBlock / 2) {
    // wide rows: one row per workgroup behind a launch that works the displacements out (187 against
    // 232 us on the MoE workload); the element path takes 16-byte pieces at element-aligned addresses
    const PairSlot* tab;
    const int rc = stage_pair_tables(ctx, splits, P, T, stream, &tab);
    if (rc != MCR_OK) return rc;
    auto one_row = [&](auto ntl, auto nts, auto al) {
      hipLaunchKernelGGL((moe_dispatch_pairs_row_kernel<decltype(ntl)::value, decltype(nts)::value, decltype(al)::value>),
                         dim3(static_cast<unsigned>(T), P), dim3(kPairScatterBlock), 0, stream, recv, tok, slot, tab, T,
                         static_cast<uint64_t>(recv_rows), row_bytes, static_cast<uint32_t>(row_bytes / 16),
                         static_cast<uint32_t>((row_bytes % 16) / 2));
      return launch_status();
    };
    if (variant == SV_SCALAR) return one_row(Bool<true>{}, Bool<true>{}, Bool<false>{});   // nontemporal, as tuned for aligned rows
    return dispatch_hint(variant, [&](auto ntl, auto nts) { return one_row(ntl, nts, Bool<true>{}); });
  }
  auto go = [&](auto ub, auto ntl, auto nts) {
    constexpr int UB = decltype(ub)::value;
    const RowShape s = row_shape(row_bytes / UB);
    const unsigned gx = blocks_for(T, static_cast<size_t>(kRowsPerBlock) * s.rows_per_pass);
    if (s.tpr >= kWave)
      hipLaunchKernelGGL((moe_dispatch_kernel<UB, decltype(ntl)::value, decltype(nts)::value, true>), dim3(gx, P), dim3(kBlock),
                         0, stream, recv, tok, slot, splits, P, T, static_cast<uint64_t>(recv_rows), s.upr, s.tpr, s.shift);
    else
      hipLaunchKernelGGL((moe_dispatch_kernel<UB, decltype(ntl)::value, decltype(nts)::value, false>), dim3(gx, P), dim3(kBlock),
                         0, stream, recv, tok, slot, splits, P, T, static_cast<uint64_t>(recv_rows), s.upr, s.tpr, s.shift);
    return launch_status();
  };
  if (variant == SV_SCALAR) return elem_b == 4 ? go(Int<4>{}, Bool<false>{}, Bool<false>{}) : go(Int<2>{}, Bool<false>{}, Bool<false>{});
  return dispatch_hint(variant, [&](auto ntl, auto nts) { return go(Int<16>{}, ntl, nts); });
}

int launch_moe_combine(mcr_ctx* ctx, const PtrTab& out, const CPtrTab& expert_out, const CPtrTab& slot, const CPtrTab* gate,
                       const int64_t* splits, size_t T, size_t recv_rows, size_t row_elems, int dtype, int P, int variant,
                       hipStream_t stream) {
  if (T == 0 || row_elems == 0) return MCR_OK;
  const int top_k = 1;
  CPtrTab g;
  for (int i = 0; i < MCR_MAX_RANKS; ++i) g.p[i] = gate ? gate->p[i] : nullptr;
  // without a gate (and with one choice per token) rows are copied: only the element size matters
  const int kernel_dtype = (gate || top_k > 1) ? dtype : (elem_bytes(dtype) == 4 ? MCR_F32 : MCR_BF16);
  return dispatch_float_dtype(kernel_dtype, [&](auto dt) {
    constexpr int DT = decltype(dt)::value;
    constexpr int EB = Elem<DT>::kBytes;
    const size_t row_bytes = row_elems * EB;
    if (row_bytes / 16 > kBlock / 2) {                  // wide rows: one row per workgroup (see launch_moe_dispatch)
      const PairSlot* tab;
      const int rc = stage_pair_tables(ctx, splits, P, T, stream, &tab);
      if (rc != MCR_OK) return rc;
      auto one_row = [&](auto ntl, auto nts, auto al) {
        auto launch = [&](auto gc) {
          hipLaunchKernelGGL((moe_combine_pairs_row_kernel<DT, decltype(ntl)::value, decltype(nts)::value, decltype(gc)::value,
                                                           decltype(al)::value>),
                             dim3(static_cast<unsigned>(T), P), dim3(kRowGatherBlock), 0, stream, out, expert_out, slot, g, tab, T,
                             static_cast<uint64_t>(recv_rows), row_bytes, static_cast<uint32_t>(row_bytes / 16),
                             static_cast<uint32_t>((row_bytes % 16) / EB));
        };
        if (gate) launch(Bool<true>{});
        else launch(Bool<false>{});
        return launch_status();
      };
      if (variant == SV_SCALAR) return one_row(Bool<true>{}, Bool<true>{}, Bool<false>{});   // nontemporal, as tuned for aligned rows
      return dispatch_hint(variant, [&](auto ntl, auto nts) { return one_row(ntl, nts, Bool<true>{}); });
    }
    auto go = [&](auto ub, auto ntl, auto nts, auto gc) {
      constexpr int UB = decltype(ub)::value;
      const RowShape s = row_shape(row_elems * EB / UB);
      const unsigned gx = blocks_for(T, static_cast<size_t>(kRowsPerBlock) * s.rows_per_pass);
      if (s.tpr >= kWave)
        hipLaunchKernelGGL((moe_combine_kernel<DT, UB, decltype(ntl)::value, decltype(nts)::value, decltype(gc)::value, true>),
                           dim3(gx, P), dim3(kBlock), 0, stream, out, expert_out, slot, g, splits, P, T,
                           static_cast<uint64_t>(recv_rows), s.upr, s.tpr, s.shift);
      else
        hipLaunchKernelGGL((moe_combine_kernel<DT, UB, decltype(ntl)::value, decltype(nts)::value, decltype(gc)::value, false>),
                           dim3(gx, P), dim3(kBlock), 0, stream, out, expert_out, slot, g, splits, P, T,
                           static_cast<uint64_t>(recv_rows), s.upr, s.tpr, s.shift);
      return launch_status();
    };
    if (variant == SV_SCALAR)
      return gate ? go(Int<EB>{}, Bool<false>{}, Bool<false>{}, Bool<true>{}) : go(Int<EB>{}, Bool<false>{}, Bool<false>{}, Bool<false>{});
    return dispatch_hint(variant, [&](auto ntl, auto nts) {
      return gate ? go(Int<16>{}, ntl, nts, Bool<true>{}) : go(Int<16>{}, ntl, nts, Bool<false>{});
    });
  });
}

int launch_moe_expert_layout(mcr_ctx*, const CPtrTab& counts, int E, int P, int64_t* row_table, int64_t* expert_first,
                             int64_t* expert_rows, hipStream_t stream) {
  hipLaunchKernelGGL(moe_expert_layout_kernel, dim3(1), dim3(kLayoutBlock), 0, stream, counts, E, P, row_table, expert_first,
                     expert_rows);
  return launch_status();
}

int launch_moe_source_layout(mcr_ctx*, const CPtrTab& counts, int E, int P, int64_t* row_table, hipStream_t stream) {
  hipLaunchKernelGGL(moe_source_layout_kernel, dim3(1), dim3(kLayoutBlock), 0, stream, counts, E, P, row_table);
  return launch_status();
}

int launch_moe_dispatch_by_expert(mcr_ctx*, const PtrTab& recv, const CPtrTab& tok, const CPtrTab& ids, const CPtrTab& slot,
                                  const int64_t* row_table, int E, size_t T, int K, size_t recv_rows, size_t row_bytes,
                                  int elem_b, int P, int variant, hipStream_t stream) {
  if (T == 0 || row_bytes == 0) return MCR_OK;
  const size_t A = T * static_cast<size_t>(K);
  // one row per workgroup (193 against 212 us on the MoE workload); with several choices per
  // token the workgroup reads the token's row once and stores it to every kept choice's place.
  // al = false: the element path on wide rows, 16-byte pieces at element-aligned addresses and a tail
  auto one_row = [&](auto ntl, auto nts, auto al) {
    auto launch = [&](auto ku) {
      hipLaunchKernelGGL((moe_dispatch_row_kernel<decltype(ku)::value, decltype(ntl)::value, decltype(nts)::value, decltype(al)::value>),
                         dim3(static_cast<unsigned>(T), P), dim3(kBlock), 0, stream, recv, tok, ids, slot, row_table, E,
                         rank_magic(E, P), T, K, static_cast<uint64_t>(recv_rows), row_bytes, static_cast<uint32_t>(row_bytes / 16),
                         static_cast<uint32_t>((row_bytes % 16) / 2));
    };
    if (K == 1) launch(Int<1>{});
    else if (K == 2) launch(Int<2>{});
    else launch(Int<MCR_MAX_TOPK>{});
    return launch_status();
  };
  const bool wide = row_bytes / 16 > kBlock / 2;
  if (variant == SV_SCALAR && wide) return one_row(Bool<true>{}, Bool<true>{}, Bool<false>{});   // nontemporal, as tuned for aligned rows
  auto go = [&](auto ub, auto ntl, auto nts) {
    constexpr int UB = decltype(ub)::value;
    const RowShape s = row_shape(row_bytes / UB);
    if (UB == 16 && s.tpr == kBlock) return one_row(ntl, nts, Bool<true>{});
    const unsigned gx = blocks_for(A, static_cast<size_t>(kRowsPerBlock) * s.rows_per_pass);
    if (s.tpr >= kWave)
      hipLaunchKernelGGL((moe_dispatch_by_expert_kernel<UB, decltype(ntl)::value, decltype(nts)::value, true>), dim3(gx, P),
                         dim3(kBlock), 0, stream, recv, tok, ids, slot, row_table, E, P, A, T,
                         static_cast<uint64_t>(recv_rows), s.upr, s.tpr, s.shift);
    else
      hipLaunchKernelGGL((moe_dispatch_by_expert_kernel<UB, decltype(ntl)::value, decltype(nts)::value, false>), dim3(gx, P),
                         dim3(kBlock), 0, stream, recv, tok, ids, slot, row_table, E, P, A, T,
                         static_cast<uint64_t>(recv_rows), s.upr, s.tpr, s.shift);
    return launch_status();
  };
  if (variant == SV_SCALAR) return elem_b == 4 ? go(Int<4>{}, Bool<false>{}, Bool<false>{}) : go(Int<2>{}, Bool<false>{}, Bool<false>{});
  return dispatch_hint(variant, [&](auto ntl, auto nts) {
    // rows narrower than a workgroup with several choices per token: every token row is read once
    // per choice, so the nontemporal load hint is dropped
    if (K > 1 && row_shape(row_bytes / 16).tpr != kBlock) return go(Int<16>{}, Bool<false>{}, nts);
    return go(Int<16>{}, ntl, nts);
  });
}

int launch_moe_combine_by_expert(mcr_ctx*, const PtrTab& out, const CPtrTab& expert_out, const CPtrTab& ids,
                                 const CPtrTab& slot, const CPtrTab* gate, const int64_t* row_table, int E, size_t T, int K,
                                 size_t recv_rows, size_t row_elems, int dtype, int P, int variant, hipStream_t stream) {
  if (T == 0 || row_elems == 0) return MCR_OK;
  const int top_k = K;
  CPtrTab g;
  for (int i = 0; i < MCR_MAX_RANKS; ++i) g.p[i] = gate ? gate->p[i] : nullptr;
  // without a gate (and with one choice per token) rows are copied: only the element size matters
  const int kernel_dtype = (gate || top_k > 1) ? dtype : (elem_bytes(dtype) == 4 ? MCR_F32 : MCR_BF16);
  return dispatch_float_dtype(kernel_dtype, [&](auto dt) {
    constexpr int DT = decltype(dt)::value;
    constexpr int EB = Elem<DT>::kBytes;
    const size_t row_bytes = row_elems * EB;
    if (row_bytes / 16 > kBlock / 2) {     // one row per workgroup; on the element path with pieces at element-aligned addresses
      const uint32_t upr = static_cast<uint32_t>(row_bytes / 16);
      auto one_row = [&](auto ntl, auto nts, auto al) {
        auto launch = [&](auto ku, auto gc) {
          hipLaunchKernelGGL((moe_combine_row_kernel<DT, decltype(ku)::value, decltype(ntl)::value, decltype(nts)::value,
                                                     decltype(gc)::value, decltype(al)::value>),
                             dim3(static_cast<unsigned>(T), P), dim3(kRowGatherBlock), 0, stream, out, expert_out, ids, slot, g,
                             row_table, E, rank_magic(E, P), T, K, static_cast<uint64_t>(recv_rows), row_bytes, upr,
                             static_cast<uint32_t>((row_bytes % 16) / EB));
        };
        auto by_k = [&](auto gc) {
          if (K == 1) launch(Int<1>{}, gc);
          else if (K == 2) launch(Int<2>{}, gc);
          else launch(Int<MCR_MAX_TOPK>{}, gc);
        };
        if (gate) by_k(Bool<true>{});
        else by_k(Bool<false>{});
        return launch_status();
      };
      if (variant == SV_SCALAR) return one_row(Bool<true>{}, Bool<true>{}, Bool<false>{});   // nontemporal, as tuned for aligned rows
      return dispatch_hint(variant, [&](auto ntl, auto nts) { return one_row(ntl, nts, Bool<true>{}); });
    }
    if (K > 1) {
      auto topk = [&](auto ub, auto ntl, auto nts) {
        constexpr int UB = decltype(ub)::value;
        const RowShape s = row_shape(row_elems * EB / UB);
        const unsigned gx = blocks_for(T, static_cast<size_t>(kTopkRows) * s.rows_per_pass);
        auto launch = [&](auto ku, auto wv) {
          hipLaunchKernelGGL((moe_combine_topk_kernel<DT, UB, decltype(ku)::value, decltype(ntl)::value, decltype(nts)::value,
                                                      decltype(wv)::value>),
                             dim3(gx, P), dim3(kBlock), 0, stream, out, expert_out, ids, slot, g, row_table, E, P, T, K,
                             static_cast<uint64_t>(recv_rows), s.upr, s.tpr, s.shift);
        };
        if (K <= 2) {
          if (s.tpr >= kWave) launch(Int<2>{}, Bool<true>{});
          else launch(Int<2>{}, Bool<false>{});
        } else {
          if (s.tpr >= kWave) launch(Int<MCR_MAX_TOPK>{}, Bool<true>{});
          else launch(Int<MCR_MAX_TOPK>{}, Bool<false>{});
        }
        return launch_status();
      };
      if (variant == SV_SCALAR) return topk(Int<EB>{}, Bool<false>{}, Bool<false>{});
      return dispatch_hint(variant, [&](auto ntl, auto nts) { return topk(Int<16>{}, ntl, nts); });
    }
    auto go = [&](auto ub, auto ntl, auto nts, auto gc) {
      constexpr int UB = decltype(ub)::value;
      const RowShape s = row_shape(row_elems * EB / UB);
      const unsigned gx = blocks_for(T, static_cast<size_t>(kRowsPerBlock) * s.rows_per_pass);
      if (s.tpr >= kWave)
        hipLaunchKernelGGL(
            (moe_combine_by_expert_kernel<DT, UB, decltype(ntl)::value, decltype(nts)::value, decltype(gc)::value, true>),
            dim3(gx, P), dim3(kBlock), 0, stream, out, expert_out, ids, slot, g, row_table, E, P, T,
            static_cast<uint64_t>(recv_rows), s.upr, s.tpr, s.shift);
      else
        hipLaunchKernelGGL(
            (moe_combine_by_expert_kernel<DT, UB, decltype(ntl)::value, decltype(nts)::value, decltype(gc)::value, false>),
            dim3(gx, P), dim3(kBlock), 0, stream, out, expert_out, ids, slot, g, row_table, E, P, T,
            static_cast<uint64_t>(recv_rows), s.upr, s.tpr, s.shift);
      return launch_status();
    };
    if (variant == SV_SCALAR)
      return gate ? go(Int<EB>{}, Bool<false>{}, Bool<false>{}, Bool<true>{}) : go(Int<EB>{}, Bool<false>{}, Bool<false>{}, Bool<false>{});
    return dispatch_hint(variant, [&](auto ntl, auto nts) {
      return gate ? go(Int<16>{}, ntl, nts, Bool<true>{}) : go(Int<16>{}, ntl, nts, Bool<false>{});
    });
  });
}

int launch_dlrm_shuffle(mcr_ctx*, const PtrTab& dst, const CPtrTab& src, int n_tables, size_t batch, size_t row_bytes,
                        int elem_b, int P, bool backward, int variant, hipStream_t stream) {
  const size_t rows = (batch / P) * static_cast<size_t>(n_tables);
  if (rows == 0 || row_bytes == 0) return MCR_OK;
  auto go = [&](auto ub, auto ntl, auto nts) {
    constexpr int UB = decltype(ub)::value;
    const RowShape s = row_shape(row_bytes / UB);
    const unsigned gx = blocks_for(rows, s.rows_per_pass);
    if (backward)
      hipLaunchKernelGGL((dlrm_shuffle_kernel<UB, decltype(ntl)::value, decltype(nts)::value, true>), dim3(gx, P), dim3(kBlock),
                         0, stream, dst, src, static_cast<uint32_t>(n_tables), static_cast<uint64_t>(batch),
                         static_cast<uint32_t>(P), s.upr, s.tpr, s.shift);
    else
      hipLaunchKernelGGL((dlrm_shuffle_kernel<UB, decltype(ntl)::value, decltype(nts)::value, false>), dim3(gx, P), dim3(kBlock),
                         0, stream, dst, src, static_cast<uint32_t>(n_tables), static_cast<uint64_t>(batch),
                         static_cast<uint32_t>(P), s.upr, s.tpr, s.shift);
    return launch_status();
  };
  if (variant == SV_SCALAR && row_bytes >= 64) {
    const uint32_t pieces = static_cast<uint32_t>(row_bytes / 16), tail2 = static_cast<uint32_t>(row_bytes % 16) / 2;
    const RowShape s = row_shape(pieces);
    const unsigned gx = blocks_for(rows, s.rows_per_pass);
    auto odd = [&](auto bwd) {
      hipLaunchKernelGGL((dlrm_shuffle_pieces_kernel<true, false, decltype(bwd)::value>), dim3(gx, P), dim3(kBlock), 0, stream, dst,
                         src, static_cast<uint32_t>(n_tables), static_cast<uint64_t>(batch), static_cast<uint32_t>(P),
                         static_cast<uint32_t>(row_bytes), pieces, tail2, s.tpr, s.shift);
      return launch_status();
    };
    return backward ? odd(Bool<true>{}) : odd(Bool<false>{});
  }
  if (variant == SV_SCALAR) return elem_b == 4 ? go(Int<4>{}, Bool<false>{}, Bool<false>{}) : go(Int<2>{}, Bool<false>{}, Bool<false>{});
  return dispatch_hint(variant, [&](auto ntl, auto nts) { return go(Int<16>{}, ntl, nts); });
}

}  // namespace mcr
