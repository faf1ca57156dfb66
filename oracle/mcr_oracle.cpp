// CPU oracle for the local data movement and reduction inside the collectives
// that MCR-DL dispatches (its API listing, Sec. IV-A "MCR-DL API"), computed
// over P simulated rank buffers held in host memory.
//
// THIS IS TEST INFRASTRUCTURE.  It is a checker, not a product path: only the
// test-suite, the smoke check and the benchmark's CPU-baseline leg may call
// it.  It shares no source, header, table or helper with the GPU library.
//
// Style: every function is the plain definition of the operation written as
// the obvious loop nest, single-threaded, one element at a time.  Sums are
// taken in IEEE binary32 in rank order 0,1,...,P-1 starting from rank 0's
// value (not from 0.0f), and compiled with -ffp-contract=off so that no
// multiply-add is fused.  bf16 and fp16 are carried as uint16_t.  fp16 (IEEE binary16) is
// reduced like bf16: widened exactly, combined in binary32, rounded once.  int32 is reduced in
// two's-complement arithmetic that wraps (sums and products modulo 2^32), which does not depend
// on the order; AVG of integers and gate-scaling of integers are not defined and are refused.
//
// The paper delegates the semantics of each collective to MPI/NCCL
// (Sec. II-B "Communication Backends"); the definitions below are the MPI
// ones, with the vector displacements fixed to packed prefix sums.
//
// Pin status: every function here is pinned by tests that do not call it to
// produce their own expectation (closed forms, involutions, brute force,
// library routines); none is "parity unpinned".

#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

enum { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2, DT_I32 = 3 };
enum { OP_SUM = 0, OP_AVG = 1, OP_MAX = 2, OP_MIN = 3, OP_PROD = 4 };

// bf16 is the upper half of a binary32 pattern.
inline float bf16_bits_to_float(uint16_t h) {
  uint32_t u = static_cast<uint32_t>(h) << 16;
  float f;
  std::memcpy(&f, &u, sizeof f);
  return f;
}

// Round-to-nearest, ties-to-even, from binary32 to bf16, by definition:
// the two candidates are the truncated pattern and its successor in
// magnitude; the discarded 16 bits decide.  A carry out of the 7-bit
// significand runs into the exponent, which is the correct successor
// (and reaches infinity from the largest finite value).  NaN stays NaN
// (quiet bit forced so that a payload living only in the low half does
// not turn into infinity).
inline uint16_t float_to_bf16_bits(float f) {
  uint32_t u;
  std::memcpy(&u, &f, sizeof u);
  const uint32_t mag = u & 0x7fffffffu;
  if (mag > 0x7f800000u) {
    return static_cast<uint16_t>((u >> 16) | 0x0040u);
  }
  uint32_t kept = u >> 16;
  const uint32_t discarded = u & 0xffffu;
  const uint32_t half = 0x8000u;
  bool round_up;
  if (discarded > half) {
    round_up = true;
  } else if (discarded < half) {
    round_up = false;
  } else {
    round_up = (kept & 1u) != 0u;  // tie: go to the even neighbour
  }
  if (round_up) kept += 1u;
  return static_cast<uint16_t>(kept);
}

// IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.
inline float half_bits_to_float(uint16_t h) {
  const uint32_t sign = static_cast<uint32_t>(h & 0x8000u) << 16;
  const int exp = (h >> 10) & 0x1f;
  const uint32_t frac = h & 0x3ffu;
  if (exp == 31) {                                   // infinity or NaN (payload kept)
    const uint32_t u = sign | 0x7f800000u | (frac << 13);
    float f;
    std::memcpy(&f, &u, sizeof f);
    return f;
  }
  // value = frac * 2^-24 (subnormal) or (1024 + frac) * 2^(exp-25): exact in binary32
  const float mag = exp == 0 ? std::ldexp(static_cast<float>(frac), -24)
                             : std::ldexp(static_cast<float>(1024u + frac), exp - 25);
  return sign ? -mag : mag;
}

// Round to nearest, ties to even, from binary32 to binary16, by definition: in the binade
// 2^E <= |f| < 2^(E+1) the representable values are multiples of the quantum 2^(E-10); below
// 2^-14 (subnormal results) the quantum stays 2^-24.  |f| / quantum is exact in binary64, its
// fractional part decides, a tie goes to the even multiple; 2048 quanta are 1024 of the next
// binade; past the largest exponent the result is infinity.
inline uint16_t float_to_half_bits(float f) {
  uint32_t u;
  std::memcpy(&u, &f, sizeof u);
  const uint16_t sign = static_cast<uint16_t>((u >> 16) & 0x8000u);
  const uint32_t mag = u & 0x7fffffffu;
  if (mag > 0x7f800000u) return static_cast<uint16_t>(sign | 0x7e00u | ((mag >> 13) & 0x3ffu));   // NaN, quiet bit forced
  if (mag == 0x7f800000u) return static_cast<uint16_t>(sign | 0x7c00u);
  const double a = std::fabs(static_cast<double>(f));
  if (a == 0.0) return sign;
  int e2;
  std::frexp(a, &e2);                                // a = m * 2^e2, 0.5 <= m < 1
  int E = e2 - 1;
  if (E < -14) E = -14;
  const double scaled = a / std::ldexp(1.0, E - 10);
  double n = std::floor(scaled);
  const double rem = scaled - n;
  if (rem > 0.5 || (rem == 0.5 && std::fmod(n, 2.0) == 1.0)) n += 1.0;
  if (n == 2048.0) {
    E += 1;
    n = 1024.0;
  }
  if (E > 15) return static_cast<uint16_t>(sign | 0x7c00u);
  const uint32_t q = static_cast<uint32_t>(n);
  if (q < 1024u) return static_cast<uint16_t>(sign | q);                     // subnormal (E == -14)
  return static_cast<uint16_t>(sign | (static_cast<uint32_t>(E + 15) << 10) | (q - 1024u));
}

inline float load_elem(const void* base, size_t i, int dtype) {
  if (dtype == DT_F32) return static_cast<const float*>(base)[i];
  if (dtype == DT_F16) return half_bits_to_float(static_cast<const uint16_t*>(base)[i]);
  return bf16_bits_to_float(static_cast<const uint16_t*>(base)[i]);
}

inline void store_elem(void* base, size_t i, int dtype, float v) {
  if (dtype == DT_F32) {
    static_cast<float*>(base)[i] = v;
  } else if (dtype == DT_F16) {
    static_cast<uint16_t*>(base)[i] = float_to_half_bits(v);
  } else {
    static_cast<uint16_t*>(base)[i] = float_to_bf16_bits(v);
  }
}

inline size_t elem_bytes(int dtype) { return (dtype == DT_F32 || dtype == DT_I32) ? 4u : 2u; }

inline bool bad_dtype(int dtype) { return dtype < DT_F32 || dtype > DT_I32; }
inline bool bad_op(int op) { return op < OP_SUM || op > OP_PROD; }

// One step of the ReduceOp chain (API listing: all_reduce / reduce / reduce_scatter take a
// ReduceOp).  MAX and MIN let a NaN through from either side, so a NaN anywhere in the chain
// reaches the result; between equal values (+0 and -0 included) the earlier rank's value stays.
inline float combine(float acc, float x, int op) {
  switch (op) {
    case OP_MAX: return (x > acc || x != x) ? x : acc;
    case OP_MIN: return (x < acc || x != x) ? x : acc;
    case OP_PROD: return acc * x;
    default: return acc + x;
  }
}

// Reduction of element i over ranks 0..P-1, canonical order.
inline float reduce_at(const void* const* bufs, size_t i, int dtype, int op, int P) {
  float acc = load_elem(bufs[0], i, dtype);
  for (int p = 1; p < P; ++p) {
    acc = combine(acc, load_elem(bufs[p], i, dtype), op);
  }
  if (op == OP_AVG) {
    const float scale = 1.0f / static_cast<float>(P);
    acc = acc * scale;
  }
  return acc;
}

// The same for int32: sums and products wrap modulo 2^32 (computed on the unsigned patterns),
// MAX and MIN compare as signed integers.
inline int32_t combine_i32(int32_t acc, int32_t x, int op) {
  switch (op) {
    case OP_MAX: return x > acc ? x : acc;
    case OP_MIN: return x < acc ? x : acc;
    case OP_PROD: return static_cast<int32_t>(static_cast<uint32_t>(acc) * static_cast<uint32_t>(x));
    default: return static_cast<int32_t>(static_cast<uint32_t>(acc) + static_cast<uint32_t>(x));
  }
}

inline int32_t reduce_at_i32(const void* const* bufs, size_t i, int op, int P) {
  int32_t acc = static_cast<const int32_t*>(bufs[0])[i];
  for (int p = 1; p < P; ++p) {
    acc = combine_i32(acc, static_cast<const int32_t*>(bufs[p])[i], op);
  }
  return acc;
}

// int32 has no average and no gate-scaling.
inline bool int_refused(int dtype, int op) { return dtype == DT_I32 && op == OP_AVG; }

}  // namespace

extern "C" {

// ---- bf16 conversions (exposed so the rounding itself can be pinned) -------
uint16_t orc_f32_to_bf16(float f) { return float_to_bf16_bits(f); }
float orc_bf16_to_f32(uint16_t h) { return bf16_bits_to_float(h); }

void orc_f32_to_bf16_array(const float* in, uint16_t* out, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = float_to_bf16_bits(in[i]);
}
void orc_bf16_to_f32_array(const uint16_t* in, float* out, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = bf16_bits_to_float(in[i]);
}

uint16_t orc_f32_to_f16(float f) { return float_to_half_bits(f); }
float orc_f16_to_f32(uint16_t h) { return half_bits_to_float(h); }
void orc_f32_to_f16_array(const float* in, uint16_t* out, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = float_to_half_bits(in[i]);
}
void orc_f16_to_f32_array(const uint16_t* in, float* out, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = half_bits_to_float(in[i]);
}

// ---- all_reduce (API listing, all_reduce) ------------------------------------
// In place: every rank's buffer ends up holding the reduction.
int orc_allreduce(void* const* bufs, size_t n, int dtype, int op, int P) {
  if (!bufs || P < 1 || bad_dtype(dtype) || bad_op(op)) return -1;
  if (int_refused(dtype, op)) return -3;
  for (size_t i = 0; i < n; ++i) {
    if (dtype == DT_I32) {
      const int32_t y = reduce_at_i32(bufs, i, op, P);
      for (int r = 0; r < P; ++r) static_cast<int32_t*>(bufs[r])[i] = y;
      continue;
    }
    const float y = reduce_at(bufs, i, dtype, op, P);
    for (int r = 0; r < P; ++r) store_elem(bufs[r], i, dtype, y);
  }
  return 0;
}

// Double-precision reference of the same reduction, for tolerance checks of
// any re-associated sum: out[i] = sum_p x_p[i] (times 1/P for AVG) in
// binary64, mag[i] = sum_p |x_p[i]| (the error-bound denominator).
int orc_allreduce_ref64(const void* const* bufs, size_t n, int dtype, int op, int P,
                        double* out, double* mag) {
  if (!bufs || P < 1 || bad_dtype(dtype) || dtype == DT_I32 || bad_op(op)) return -1;
  for (size_t i = 0; i < n; ++i) {
    double acc = 0.0, m = 0.0;
    for (int p = 0; p < P; ++p) {
      const double x = static_cast<double>(load_elem(bufs[p], i, dtype));
      acc += x;
      m += x < 0 ? -x : x;
    }
    if (op == OP_AVG) {
      acc /= static_cast<double>(P);
      m /= static_cast<double>(P);
    }
    out[i] = acc;
    if (mag) mag[i] = m;
  }
  return 0;
}

// ---- reduce (API listing, reduce) : only the root's buffer receives the result --
int orc_reduce(void* const* bufs, size_t n, int dtype, int op, int P, int root) {
  if (!bufs || P < 1 || root < 0 || root >= P || bad_dtype(dtype) || bad_op(op)) return -1;
  if (int_refused(dtype, op)) return -3;
  for (size_t i = 0; i < n; ++i) {
    if (dtype == DT_I32) {
      static_cast<int32_t*>(bufs[root])[i] = reduce_at_i32(bufs, i, op, P);
      continue;
    }
    const float y = reduce_at(bufs, i, dtype, op, P);
    store_elem(bufs[root], i, dtype, y);
  }
  return 0;
}

// ---- bcast (API listing, bcast) : every buffer becomes a bit copy of the root's --
int orc_bcast(void* const* bufs, size_t n, int dtype, int P, int root) {
  if (!bufs || P < 1 || root < 0 || root >= P || bad_dtype(dtype)) return -1;
  const size_t s = elem_bytes(dtype);
  for (int r = 0; r < P; ++r) {
    if (r == root) continue;
    for (size_t i = 0; i < n; ++i)
      std::memcpy(static_cast<char*>(bufs[r]) + i * s, static_cast<const char*>(bufs[root]) + i * s, s);
  }
  return 0;
}

// ---- gatherv / scatterv / all_gatherv (API listing) with packed displacements ----
// counts[p] elements belong to rank p; displ[p] = sum_{q<p} counts[q].
//   gatherv   : root_out[displ[p] + j] = in[p][j]
//   scatterv  : out[r][j] = root_in[displ[r] + j]
//   allgatherv: out[r][displ[p] + j] = in[p][j] for every r
// gather / scatter are the equal-count cases.
int orc_gatherv(void* root_out, const void* const* in, const uint64_t* counts, int dtype, int P) {
  if (!in || !counts || P < 1 || bad_dtype(dtype)) return -1;
  const size_t s = elem_bytes(dtype);
  uint64_t displ = 0;
  for (int p = 0; p < P; ++p) {
    for (uint64_t j = 0; j < counts[p]; ++j)
      std::memcpy(static_cast<char*>(root_out) + (displ + j) * s, static_cast<const char*>(in[p]) + j * s, s);
    displ += counts[p];
  }
  return 0;
}

int orc_scatterv(void* const* out, const void* root_in, const uint64_t* counts, int dtype, int P) {
  if (!out || !counts || P < 1 || bad_dtype(dtype)) return -1;
  const size_t s = elem_bytes(dtype);
  uint64_t displ = 0;
  for (int r = 0; r < P; ++r) {
    for (uint64_t j = 0; j < counts[r]; ++j)
      std::memcpy(static_cast<char*>(out[r]) + j * s, static_cast<const char*>(root_in) + (displ + j) * s, s);
    displ += counts[r];
  }
  return 0;
}

int orc_allgatherv(void* const* out, const void* const* in, const uint64_t* counts, int dtype, int P) {
  if (!out || !in || !counts || P < 1 || bad_dtype(dtype)) return -1;
  for (int r = 0; r < P; ++r) {
    const int rc = orc_gatherv(out[r], in, counts, dtype, P);
    if (rc != 0) return rc;
  }
  return 0;
}

// ---- the same with displacements chosen by the caller (the displs / sdispls / rdispls
// arguments of the API listing), in elements (rows for all_to_allv) from the buffer start.
// Gaps between blocks are left untouched; blocks of one destination must not overlap.
//   gatherv   : root_out[displs[p] + j] = in[p][j]                       j < counts[p]
//   scatterv  : out[r][j] = root_in[displs[r] + j]                       j < counts[r]
//   allgatherv: out[r][displs[p] + j] = in[p][j] for every r
//   alltoallv : out[r][rdispls[r*P + p] + k] = in[p][sdispls[p*P + r] + k]   k < counts[p*P + r] rows
int orc_gatherv_displs(void* root_out, const void* const* in, const uint64_t* counts, const uint64_t* displs, int dtype,
                       int P) {
  if (!in || !counts || !displs || P < 1 || bad_dtype(dtype)) return -1;
  const size_t s = elem_bytes(dtype);
  for (int p = 0; p < P; ++p)
    for (uint64_t j = 0; j < counts[p]; ++j)
      std::memcpy(static_cast<char*>(root_out) + (displs[p] + j) * s, static_cast<const char*>(in[p]) + j * s, s);
  return 0;
}

int orc_scatterv_displs(void* const* out, const void* root_in, const uint64_t* counts, const uint64_t* displs, int dtype,
                        int P) {
  if (!out || !counts || !displs || P < 1 || bad_dtype(dtype)) return -1;
  const size_t s = elem_bytes(dtype);
  for (int r = 0; r < P; ++r)
    for (uint64_t j = 0; j < counts[r]; ++j)
      std::memcpy(static_cast<char*>(out[r]) + j * s, static_cast<const char*>(root_in) + (displs[r] + j) * s, s);
  return 0;
}

int orc_allgatherv_displs(void* const* out, const void* const* in, const uint64_t* counts, const uint64_t* displs,
                          int dtype, int P) {
  if (!out || !in || !counts || !displs || P < 1 || bad_dtype(dtype)) return -1;
  for (int r = 0; r < P; ++r) {
    const int rc = orc_gatherv_displs(out[r], in, counts, displs, dtype, P);
    if (rc != 0) return rc;
  }
  return 0;
}

int orc_alltoallv_displs(void* const* out, const void* const* in, const int64_t* counts, const int64_t* sdispls,
                         const int64_t* rdispls, size_t row_elems, int dtype, int P) {
  if (!out || !in || !counts || !sdispls || !rdispls || P < 1 || bad_dtype(dtype)) return -1;
  for (int i = 0; i < P * P; ++i)
    if (counts[i] < 0 || sdispls[i] < 0 || rdispls[i] < 0) return -2;
  const size_t rb = row_elems * elem_bytes(dtype);
  for (int r = 0; r < P; ++r) {
    for (int p = 0; p < P; ++p) {
      const int64_t cnt = counts[p * P + r];
      const int64_t from = sdispls[p * P + r];
      const int64_t to = rdispls[r * P + p];
      for (int64_t k = 0; k < cnt; ++k) {
        std::memcpy(static_cast<char*>(out[r]) + static_cast<size_t>(to + k) * rb,
                    static_cast<const char*>(in[p]) + static_cast<size_t>(from + k) * rb, rb);
      }
    }
  }
  return 0;
}

// ---- reduce_scatter (API listing, reduce_scatter; the root it prints is ------
// a slip, there is none) : rank r receives slice r of the reduction.
int orc_reduce_scatter(void* const* out, const void* const* in, size_t n, int dtype,
                       int op, int P) {
  if (!out || !in || P < 1 || bad_dtype(dtype) || bad_op(op)) return -1;
  if (n % static_cast<size_t>(P) != 0) return -2;
  if (int_refused(dtype, op)) return -3;
  const size_t b = n / static_cast<size_t>(P);
  for (int r = 0; r < P; ++r) {
    for (size_t j = 0; j < b; ++j) {
      if (dtype == DT_I32) {
        static_cast<int32_t*>(out[r])[j] = reduce_at_i32(in, static_cast<size_t>(r) * b + j, op, P);
        continue;
      }
      const float y = reduce_at(in, static_cast<size_t>(r) * b + j, dtype, op, P);
      store_elem(out[r], j, dtype, y);
    }
  }
  return 0;
}

// ---- all_gather (API listing, all_gather) : bit copy -------------------------
int orc_allgather(void* const* out, const void* const* in, size_t m, int dtype, int P) {
  if (!out || !in || P < 1 || bad_dtype(dtype)) return -1;
  const size_t s = elem_bytes(dtype);
  for (int r = 0; r < P; ++r) {
    for (int p = 0; p < P; ++p) {
      for (size_t j = 0; j < m; ++j) {
        std::memcpy(static_cast<char*>(out[r]) + (static_cast<size_t>(p) * m + j) * s,
                    static_cast<const char*>(in[p]) + j * s, s);
      }
    }
  }
  return 0;
}

// ---- all_to_all_single, equal split : P x P block transpose ------------------
int orc_alltoall(void* const* out, const void* const* in, size_t n, int dtype, int P) {
  if (!out || !in || P < 1 || bad_dtype(dtype)) return -1;
  if (n % static_cast<size_t>(P) != 0) return -2;
  const size_t s = elem_bytes(dtype);
  const size_t b = n / static_cast<size_t>(P);
  for (int r = 0; r < P; ++r) {
    for (int p = 0; p < P; ++p) {
      for (size_t k = 0; k < b; ++k) {
        std::memcpy(static_cast<char*>(out[r]) + (static_cast<size_t>(p) * b + k) * s,
                    static_cast<const char*>(in[p]) + (static_cast<size_t>(r) * b + k) * s, s);
      }
    }
  }
  return 0;
}

// ---- all_to_allv with packed displacements -----------------------------------
// S is P x P, row-major, S[p*P + r] = rows rank p sends to rank r.  A row is
// row_elems elements.  sdispl[p][r] = sum_{q<r} S[p][q];
// rdispl[r][p] = sum_{q<p} S[q][r].  Rows of out[r] past sum_p S[p][r] are
// not written.
int orc_alltoallv(void* const* out, const void* const* in, const int64_t* S,
                  size_t row_elems, int dtype, int P) {
  if (!out || !in || !S || P < 1 || bad_dtype(dtype)) return -1;
  for (int i = 0; i < P * P; ++i)
    if (S[i] < 0) return -2;
  const size_t rb = row_elems * elem_bytes(dtype);
  for (int r = 0; r < P; ++r) {
    int64_t rdispl = 0;
    for (int p = 0; p < P; ++p) {
      int64_t sdispl = 0;
      for (int q = 0; q < r; ++q) sdispl += S[p * P + q];
      const int64_t cnt = S[p * P + r];
      for (int64_t k = 0; k < cnt; ++k) {
        std::memcpy(static_cast<char*>(out[r]) + static_cast<size_t>(rdispl + k) * rb,
                    static_cast<const char*>(in[p]) + static_cast<size_t>(sdispl + k) * rb, rb);
      }
      rdispl += cnt;
    }
  }
  return 0;
}

// The way back (the second Alltoall of Sec. II-C "Mixture-of-Experts", which returns the expert
// outputs): the same exchange with the roles of the matrix swapped, rank r now sending
// S[p][r] rows to rank p.  With T[a][b] = S[b][a]: sender a's rows for receiver b start at
// sum_{q<b} T[a][q] and land at sum_{q<a} T[q][b].
int orc_alltoallv_transposed(void* const* out, const void* const* in, const int64_t* S,
                             size_t row_elems, int dtype, int P) {
  if (!out || !in || !S || P < 1 || bad_dtype(dtype)) return -1;
  for (int i = 0; i < P * P; ++i)
    if (S[i] < 0) return -2;
  const size_t rb = row_elems * elem_bytes(dtype);
  for (int b = 0; b < P; ++b) {          // receiver
    int64_t rdispl = 0;
    for (int a = 0; a < P; ++a) {        // sender
      int64_t sdispl = 0;
      for (int q = 0; q < b; ++q) sdispl += S[q * P + a];
      const int64_t back = S[b * P + a];
      for (int64_t k = 0; k < back; ++k) {
        std::memcpy(static_cast<char*>(out[b]) + static_cast<size_t>(rdispl + k) * rb,
                    static_cast<const char*>(in[a]) + static_cast<size_t>(sdispl + k) * rb, rb);
      }
      rdispl += back;
    }
  }
  return 0;
}

// ---- MoE routing of one rank's tokens (Sec. II-C "Mixture-of-Experts": --------
// tokens are routed to experts by a gate and exchanged with Alltoall) ----------
// ids[t] in [0,E) is token t's expert (top-1).  Capacity C per expert per
// source rank; within an expert, tokens are kept first-come in token order.
// Experts are laid out on ranks in contiguous groups of E/P.
//   pos[t]  = number of earlier tokens with the same expert
//   kept[t] = pos[t] < C
//   cnt[e]  = min(#tokens of e, C),  base[e] = sum_{e'<e} cnt[e']
//   slot[t] = kept ? base[ids[t]] + pos[t] : -1
//   srow[r] = sum of cnt[e] over the experts living on rank r
// A token whose id is outside [0,E) is dropped and counted nowhere.
int orc_moe_route(const int32_t* ids, int T, int E, int P, int C, int32_t* slot,
                  int32_t* counts, int64_t* srow) {
  if (!ids || !slot || !counts || !srow || T < 0 || E < 1 || P < 1 || C < 0) return -1;
  if (E % P != 0) return -2;
  std::vector<int64_t> seen(static_cast<size_t>(E), 0);
  std::vector<int64_t> pos(static_cast<size_t>(T), 0);
  for (int t = 0; t < T; ++t) {
    const int32_t e = ids[t];
    if (e < 0 || e >= E) continue;
    pos[static_cast<size_t>(t)] = seen[static_cast<size_t>(e)];
    seen[static_cast<size_t>(e)] += 1;
  }
  std::vector<int64_t> base(static_cast<size_t>(E), 0);
  int64_t run = 0;
  for (int e = 0; e < E; ++e) {
    const int64_t c = seen[static_cast<size_t>(e)] < C ? seen[static_cast<size_t>(e)] : C;
    counts[e] = static_cast<int32_t>(c);
    base[static_cast<size_t>(e)] = run;
    run += c;
  }
  for (int t = 0; t < T; ++t) {
    const int32_t e = ids[t];
    if (e < 0 || e >= E || pos[static_cast<size_t>(t)] >= C) {
      slot[t] = -1;
    } else {
      slot[t] = static_cast<int32_t>(base[static_cast<size_t>(e)] + pos[static_cast<size_t>(t)]);
    }
  }
  const int per_rank = E / P;
  for (int r = 0; r < P; ++r) {
    int64_t s = 0;
    for (int e = r * per_rank; e < (r + 1) * per_rank; ++e) s += counts[e];
    srow[r] = s;
  }
  return 0;
}

// ---- expert-major receive layout (the other half of MoE dispatch: the expert FFN wants all
// the tokens of one expert in one block) ------------------------------------------------------
// counts[p*E + e] = kept tokens of source rank p for expert e (as orc_moe_route gives them).
// At the rank that owns expert e (rank e / (E/P)) the receive buffer is ordered by
// (local expert, source rank, token order within the source):
//   expert_rows[e]  = sum_p counts[p][e]
//   expert_first[e] = sum of expert_rows over the experts of the same rank before e
//   block_first[p*E + e] = expert_first[e] + sum_{q<p} counts[q][e]     (first row of (p, e))
int orc_moe_expert_layout(const int32_t* counts, int E, int P, int64_t* block_first, int64_t* expert_first,
                          int64_t* expert_rows) {
  if (!counts || !block_first || !expert_first || !expert_rows || E < 1 || P < 1 || E % P != 0) return -1;
  const int per_rank = E / P;
  for (int e = 0; e < E; ++e) {
    int64_t rows = 0;
    for (int p = 0; p < P; ++p) rows += counts[p * E + e];
    expert_rows[e] = rows;
  }
  for (int e = 0; e < E; ++e) {
    int64_t first = 0;
    for (int e2 = (e / per_rank) * per_rank; e2 < e; ++e2) first += expert_rows[e2];
    expert_first[e] = first;
    int64_t above = 0;
    for (int p = 0; p < P; ++p) {
      block_first[p * E + e] = first + above;
      above += counts[p * E + e];
    }
  }
  return 0;
}

// Dispatch into that layout with top-K gating.  Every token has K assignments; ids[p], slot[p]
// (and gate[p] below) are K blocks of T entries, choice-major: entry a = k*T + t is choice k of
// token t, which is also the order the routing walked them in (all first choices before any second
// choice, so first choices fill an expert's capacity first).  An assignment is kept when its slot is
// >= 0.  The j-th kept assignment (in that order) of source p for expert e puts a copy of its token
// row in row block_first[p][e] + j of the receive buffer of rank e / (E/P).  Rows of recv that
// receive nothing are left untouched.  K = 1 is plain top-1 dispatch.
int orc_moe_dispatch_by_expert(void* const* recv, const void* const* tok, const int32_t* const* ids,
                               const int32_t* const* slot, const int32_t* counts, int64_t T, int K, int E, int P,
                               size_t row_elems, int dtype) {
  if (!recv || !tok || !ids || !slot || !counts || T < 0 || K < 1 || E < 1 || P < 1 || E % P != 0 || bad_dtype(dtype))
    return -1;
  std::vector<int64_t> block_first(static_cast<size_t>(P) * E), ef(E), er(E);
  if (orc_moe_expert_layout(counts, E, P, block_first.data(), ef.data(), er.data()) != 0) return -1;
  const size_t rb = row_elems * elem_bytes(dtype);
  const int per_rank = E / P;
  for (int p = 0; p < P; ++p) {
    std::vector<int64_t> seen(static_cast<size_t>(E), 0);
    for (int k = 0; k < K; ++k) {
      for (int64_t t = 0; t < T; ++t) {
        const int64_t a = static_cast<int64_t>(k) * T + t;
        if (slot[p][a] < 0) continue;
        const int e = ids[p][a];
        const int64_t row = block_first[static_cast<size_t>(p) * E + e] + seen[e];
        seen[e] += 1;
        std::memcpy(static_cast<char*>(recv[e / per_rank]) + static_cast<size_t>(row) * rb,
                    static_cast<const char*>(tok[p]) + static_cast<size_t>(t) * rb, rb);
      }
    }
  }
  return 0;
}

// Combine out of that layout.  For token t of rank p, over its kept assignments in choice order
// k = 0..K-1:  acc = gate_k * f32(row_k) for the first kept one, acc = acc + gate_k * f32(row_k)
// for each later one (binary32 multiply and add, each rounded once), then one rounding to the
// element type.  No kept assignment: all-zero bits.  gate == nullptr stands for gates of 1
// (with K = 1 the row is then copied bit for bit).
int orc_moe_combine_by_expert(void* const* out, const void* const* expert_out, const int32_t* const* ids,
                              const int32_t* const* slot, const float* const* gate, const int32_t* counts, int64_t T,
                              int K, int E, int P, size_t row_elems, int dtype) {
  if (!out || !expert_out || !ids || !slot || !counts || T < 0 || K < 1 || E < 1 || P < 1 || E % P != 0 || bad_dtype(dtype))
    return -1;
  if (dtype == DT_I32 && (gate || K > 1)) return -4;
  std::vector<int64_t> block_first(static_cast<size_t>(P) * E), ef(E), er(E);
  if (orc_moe_expert_layout(counts, E, P, block_first.data(), ef.data(), er.data()) != 0) return -1;
  const size_t rb = row_elems * elem_bytes(dtype);
  const int per_rank = E / P;
  for (int p = 0; p < P; ++p) {
    // first pass, in routing order: where every kept assignment's row is
    std::vector<int64_t> seen(static_cast<size_t>(E), 0);
    std::vector<const char*> src(static_cast<size_t>(K) * static_cast<size_t>(T), nullptr);
    for (int64_t a = 0; a < static_cast<int64_t>(K) * T; ++a) {
      if (slot[p][a] < 0) continue;
      const int e = ids[p][a];
      const int64_t row = block_first[static_cast<size_t>(p) * E + e] + seen[e];
      seen[e] += 1;
      src[static_cast<size_t>(a)] = static_cast<const char*>(expert_out[e / per_rank]) + static_cast<size_t>(row) * rb;
    }
    for (int64_t t = 0; t < T; ++t) {
      char* dst = static_cast<char*>(out[p]) + static_cast<size_t>(t) * rb;
      int kept = 0;
      for (int k = 0; k < K; ++k) kept += src[static_cast<size_t>(k) * T + t] ? 1 : 0;
      if (kept == 0) {
        std::memset(dst, 0, rb);
        continue;
      }
      if (K == 1 && !gate) {
        std::memcpy(dst, src[static_cast<size_t>(t)], rb);
        continue;
      }
      for (size_t c = 0; c < row_elems; ++c) {
        float acc = 0.0f;
        bool first = true;
        for (int k = 0; k < K; ++k) {
          const size_t a = static_cast<size_t>(k) * T + t;
          if (!src[a]) continue;
          const float g = gate ? gate[p][a] : 1.0f;
          const float term = g * load_elem(src[a], c, dtype);
          acc = first ? term : acc + term;
          first = false;
        }
        store_elem(dst, c, dtype, acc);
      }
    }
  }
  return 0;
}

// ---- pack / unpack / gate-weighted combine ------------------------------------
// pack:   Packed[slot[t]][:] = Tok[t][:] for kept t (slot >= 0).
int orc_pack(void* out, const void* in, const int32_t* slot, int64_t T, size_t row_elems,
             int dtype) {
  if (!out || !in || !slot || T < 0 || bad_dtype(dtype)) return -1;
  const size_t rb = row_elems * elem_bytes(dtype);
  for (int64_t t = 0; t < T; ++t) {
    if (slot[t] < 0) continue;
    std::memcpy(static_cast<char*>(out) + static_cast<size_t>(slot[t]) * rb,
                static_cast<const char*>(in) + static_cast<size_t>(t) * rb, rb);
  }
  return 0;
}

// unpack: Out[t][:] = kept ? Packed[slot[t]][:] : +0.  With a gate vector,
// Out[t][c] = round_to_dtype( gate[t] * f32(Packed[slot[t]][c]) ), one
// binary32 multiply and one rounding.
int orc_unpack(void* out, const void* in, const int32_t* slot, const float* gate, int64_t T,
               size_t row_elems, int dtype) {
  if (!out || !in || !slot || T < 0 || bad_dtype(dtype)) return -1;
  if (gate && dtype == DT_I32) return -4;
  const size_t s = elem_bytes(dtype);
  const size_t rb = row_elems * s;
  for (int64_t t = 0; t < T; ++t) {
    char* dst = static_cast<char*>(out) + static_cast<size_t>(t) * rb;
    if (slot[t] < 0) {
      std::memset(dst, 0, rb);
      continue;
    }
    const char* src = static_cast<const char*>(in) + static_cast<size_t>(slot[t]) * rb;
    if (!gate) {
      std::memcpy(dst, src, rb);
    } else {
      const float g = gate[t];
      for (size_t c = 0; c < row_elems; ++c) {
        const float x = load_elem(src, c, dtype);
        const float y = g * x;
        store_elem(dst, c, dtype, y);
      }
    }
  }
  return 0;
}

// ---- DLRM embedding shuffle (Sec. II-D: tables are split across processes ----
// and shuffled with an Alltoall before the top MLP) ----------------------------
// n_tables tables, table t lives on rank t mod P as that rank's local table
// t div P.  Rank p's source is [T_p][batch][dim] (table-major).  Rank r's
// output is its batch shard [batch/P][n_tables][dim], table index natural.
//   Out[r][b][t][:] = Src[t mod P][t div P][r*(batch/P) + b][:]
int orc_dlrm_forward(void* const* out, const void* const* src, int n_tables, int64_t batch,
                     size_t dim, int dtype, int P) {
  if (!out || !src || P < 1 || n_tables < 0 || batch < 0 || bad_dtype(dtype)) return -1;
  if (batch % P != 0) return -2;
  const int64_t bl = batch / P;
  const size_t rb = dim * elem_bytes(dtype);
  for (int r = 0; r < P; ++r) {
    for (int64_t b = 0; b < bl; ++b) {
      for (int t = 0; t < n_tables; ++t) {
        const int owner = t % P;
        const int local = t / P;
        const size_t src_row = static_cast<size_t>(local) * static_cast<size_t>(batch) +
                               static_cast<size_t>(r) * static_cast<size_t>(bl) + static_cast<size_t>(b);
        const size_t dst_row = static_cast<size_t>(b) * static_cast<size_t>(n_tables) + static_cast<size_t>(t);
        std::memcpy(static_cast<char*>(out[r]) + dst_row * rb,
                    static_cast<const char*>(src[owner]) + src_row * rb, rb);
      }
    }
  }
  return 0;
}

// Backward: the gradient of a permutation is the inverse permutation.
//   GradSrc[t mod P][t div P][r*(batch/P) + b][:] = GradOut[r][b][t][:]
int orc_dlrm_backward(void* const* grad_src, const void* const* grad_out, int n_tables,
                      int64_t batch, size_t dim, int dtype, int P) {
  if (!grad_src || !grad_out || P < 1 || n_tables < 0 || batch < 0 || bad_dtype(dtype)) return -1;
  if (batch % P != 0) return -2;
  const int64_t bl = batch / P;
  const size_t rb = dim * elem_bytes(dtype);
  for (int r = 0; r < P; ++r) {
    for (int64_t b = 0; b < bl; ++b) {
      for (int t = 0; t < n_tables; ++t) {
        const int owner = t % P;
        const int local = t / P;
        const size_t src_row = static_cast<size_t>(local) * static_cast<size_t>(batch) +
                               static_cast<size_t>(r) * static_cast<size_t>(bl) + static_cast<size_t>(b);
        const size_t dst_row = static_cast<size_t>(b) * static_cast<size_t>(n_tables) + static_cast<size_t>(t);
        std::memcpy(static_cast<char*>(grad_src[owner]) + src_row * rb,
                    static_cast<const char*>(grad_out[r]) + dst_row * rb, rb);
      }
    }
  }
  return 0;
}

// ---- Tensor fusion (Sec. IV-D: small tensors are combined into a buffer of ---
// at most B elements) -----------------------------------------------------------
// Greedy, order preserving, no tensor is split and no padding is inserted:
// walk the list; a tensor larger than B closes the open bucket and forms a
// bucket by itself; otherwise, if it does not fit in the open bucket, close
// that first; then append.  tensor_offset is the offset inside its bucket.
int orc_fuse_plan(const uint64_t* numel, int n_tensors, uint64_t B, int32_t* tensor_bucket,
                  uint64_t* tensor_offset, int32_t* n_buckets, uint64_t* bucket_numel) {
  if (n_tensors < 0 || B == 0 || (n_tensors > 0 && (!numel || !tensor_bucket || !tensor_offset)))
    return -1;
  int32_t cur_bucket = 0;
  uint64_t cur_fill = 0;
  bool open = false;  // does bucket cur_bucket hold anything yet
  for (int i = 0; i < n_tensors; ++i) {
    const uint64_t n = numel[i];
    if (open && (n > B || cur_fill + n > B)) {
      if (bucket_numel) bucket_numel[cur_bucket] = cur_fill;
      cur_bucket += 1;
      cur_fill = 0;
      open = false;
    }
    tensor_bucket[i] = cur_bucket;
    tensor_offset[i] = cur_fill;
    cur_fill += n;
    open = true;
    if (n > B) {  // oversize tensor: alone in its bucket
      if (bucket_numel) bucket_numel[cur_bucket] = cur_fill;
      cur_bucket += 1;
      cur_fill = 0;
      open = false;
    }
  }
  if (open) {
    if (bucket_numel) bucket_numel[cur_bucket] = cur_fill;
    cur_bucket += 1;
  }
  if (n_buckets) *n_buckets = cur_bucket;
  return 0;
}

// fuse: Flat[off_i + j] = Tensor_i[j] for the tensors of one bucket.
int orc_fuse(void* flat, const void* const* tensors, const uint64_t* numel,
             const uint64_t* offset, int n_in_bucket, int dtype) {
  if (bad_dtype(dtype) || n_in_bucket < 0) return -1;
  const size_t s = elem_bytes(dtype);
  for (int i = 0; i < n_in_bucket; ++i) {
    for (uint64_t j = 0; j < numel[i]; ++j) {
      std::memcpy(static_cast<char*>(flat) + (offset[i] + j) * s,
                  static_cast<const char*>(tensors[i]) + j * s, s);
    }
  }
  return 0;
}

// unfuse: Tensor_i[j] = Flat[off_i + j].
int orc_unfuse(void* const* tensors, const void* flat, const uint64_t* numel,
               const uint64_t* offset, int n_in_bucket, int dtype) {
  if (bad_dtype(dtype) || n_in_bucket < 0) return -1;
  const size_t s = elem_bytes(dtype);
  for (int i = 0; i < n_in_bucket; ++i) {
    for (uint64_t j = 0; j < numel[i]; ++j) {
      std::memcpy(static_cast<char*>(tensors[i]) + j * s,
                  static_cast<const char*>(flat) + (offset[i] + j) * s, s);
    }
  }
  return 0;
}

// ---- Static tuning table lookup (Sec. IV-E "Communication Tuning", Table II) --
// Rows (message size in bytes -> choice) sorted by size.  The row with the
// largest size not above the message is taken; a message below the first
// row takes the first, above the last takes the last; an empty table gives
// choice 0.
int orc_tune_lookup(const uint64_t* sizes, const int32_t* choice, int n_rows, uint64_t bytes) {
  if (n_rows <= 0) return 0;
  int pick = 0;
  for (int i = 0; i < n_rows; ++i) {
    if (sizes[i] <= bytes) pick = i;
  }
  return choice[pick];
}

}  // extern "C"
