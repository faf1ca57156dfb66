/*
 * mcr.h -- C ABI of the MI355X-native local data movement and reduction that
 * sits inside the collectives of MCR-DL's API (paper Sec. IV-A, "High-level
 * MCR-DL API" listing).
 *
 * Model.  The paper's calls are per rank (get_rank, one tensor per call) and
 * hand the bytes to NCCL/MPI.  Here all P ranks are simulated in one GPU's
 * memory: every collective takes a HOST array of P DEVICE pointers, one per
 * rank, and performs the whole P-rank operation in one stream-ordered launch.
 *
 * Conventions that hold for every entry point unless stated otherwise:
 *   - Return value: 0 (MCR_OK) or a negative mcr_status.  On any error nothing
 *     has been launched and no output has been touched.  Nothing throws or
 *     aborts.  mcr_strerror() names a code.
 *   - Pointer arguments named *bufs / *in / *out / *slot / *gate / *flat are
 *     HOST arrays holding DEVICE addresses; the arrays are read before the
 *     call returns and may be reused at once.  The device memory they point to
 *     is owned by the caller and must stay valid until the stream has passed
 *     the launch.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  The
 *     call enqueues and returns; ordering and completion are the stream's.
 *     This is the paper's non-blocking model (Sec. IV-C: the operation is
 *     posted to a stream and waited for through an event): the caller records
 *     an event on `stream` as its work handle.
 *   - No entry point allocates or frees device memory except mcr_init,
 *     mcr_finalize, mcr_fuse_plan_create/bind/destroy.
 *   - P is 1..MCR_MAX_RANKS.  Rank pointer tables travel as kernel arguments.
 *   - `variant` selects the kernel: a non-negative id from mcr_get_variants,
 *     or MCR_AUTO, which consults the tuning table (the paper's "auto"
 *     backend, Sec. IV-A and IV-E) and falls back to a safe choice when the
 *     shape or the pointer alignment rules the tabled variant out.  An
 *     explicit variant that cannot handle the shape/alignment gives
 *     MCR_EVARIANT.
 *   - Except for mcr_allreduce (in place by definition) inputs and outputs
 *     must not overlap; overlap is not detected.
 *   - Element counts are in elements of `dtype`, never bytes.
 */
#ifndef MCR_H_
#define MCR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mcr_ctx mcr_ctx;             /* library-owned: variant registry + tuning table */
typedef struct mcr_fuse_plan mcr_fuse_plan; /* library-owned: bucket plan + device descriptors */

/* Element types.  bf16 and fp16 (IEEE binary16) are widened exactly to binary32, combined in
 * binary32 and rounded once (to nearest even) when stored.  int32 is combined in two's-complement
 * arithmetic that wraps (sums and products modulo 2^32; MAX and MIN compare as signed), which
 * does not depend on the order; MCR_AVG of int32 gives MCR_EOP, and the calls that scale rows by
 * a gate weight (mcr_unpack, mcr_moe_combine, mcr_moe_combine_by_expert with a gate or K > 1)
 * give MCR_EDTYPE for it.  The reductions (SUM / AVG) on MCR_F32 and MCR_BF16 are compiled for
 * "v1" with plain accesses, for the nontemporal shape of every unroll ("v2", "v4" and the "ln" /
 * "sn" variants run the nontemporal kernel of their unroll: the other hint combinations won no row
 * of the tuning table) and for "pk8" and "w64"; on MCR_F16 and MCR_I32, and for the other
 * ReduceOps, every vector variant runs one shape ("v2nt").  mcr_allreduce_multi is compiled for
 * plain and for nontemporal accesses; its "ln" / "sn" variants run the nontemporal kernel. */
typedef enum { MCR_F32 = 0, MCR_BF16 = 1, MCR_F16 = 2, MCR_I32 = 3 } mcr_dtype;

/* ReduceOp of the API listing; every op runs as a left-to-right chain in rank order in
 * binary32 with one final rounding.  MCR_AVG is the sum multiplied (before that rounding) by
 * the binary32 value 1.0f/P.  MCR_MAX / MCR_MIN let a NaN through from either side, and
 * between equal values (+0 and -0 included) the earlier rank's value stays. */
typedef enum { MCR_SUM = 0, MCR_AVG = 1, MCR_MAX = 2, MCR_MIN = 3, MCR_PROD = 4 } mcr_redop;

typedef enum {
  MCR_OP_ALLREDUCE = 0,
  MCR_OP_REDUCE_SCATTER = 1,
  MCR_OP_ALLGATHER = 2,
  MCR_OP_ALLTOALL = 3,
  MCR_OP_ALLTOALLV = 4,
  MCR_OP_PACK = 5,
  MCR_OP_UNPACK = 6,
  MCR_OP_FUSE = 7,
  MCR_OP_UNFUSE = 8,
  MCR_OP_ALLREDUCE_MULTI = 9,
  MCR_OP_MOE_ROUTE = 10,
  MCR_OP_MOE_DISPATCH = 11,
  MCR_OP_MOE_COMBINE = 12,
  MCR_OP_DLRM_SHUFFLE = 13,
  MCR_OP_MOE_DISPATCH_BY_EXPERT = 14,
  MCR_OP_MOE_COMBINE_BY_EXPERT = 15,
  MCR_OP_COUNT = 16
} mcr_op;

typedef enum {
  MCR_OK = 0,
  MCR_EINVAL = -1,   /* null pointer, P out of range, count not divisible by P, negative split, ... */
  MCR_EDTYPE = -2,   /* unknown dtype */
  MCR_EOP = -3,      /* unknown reduce op / op id */
  MCR_EVARIANT = -4, /* unknown variant, or variant not applicable to this shape/alignment */
  MCR_ESPLIT = -5,   /* host-resident split matrix inconsistent with the declared buffer rows */
  MCR_EHIP = -6,     /* the HIP runtime reported an error (launch, copy, allocation) */
  MCR_ENOMEM = -7,   /* host allocation failed */
  MCR_EIO = -8,      /* tuning-table file could not be read / written / parsed */
  MCR_ESTATE = -9,   /* call order: plan not bound, wrong P for a bound plan, ... */
  MCR_ELIMIT = -10   /* the problem needs more than a fixed-size static scratch array holds */
} mcr_status;

#define MCR_AUTO (-1)
#define MCR_NO_DEVICE (-1)
#define MCR_MAX_RANKS 16
#define MCR_MAX_EXPERTS 512
#define MCR_MAX_TOPK 4

/* ---- lifecycle (API listing: init, finalize, synchronize, get_backends) ---- */

/* Creates a context on HIP device `device` (made current for the call).  If the
 * environment variable MCR_TUNING_TABLE names a readable table file it is
 * loaded; otherwise the table starts empty (MCR_AUTO then uses built-in
 * defaults).  *out is written only on success.
 * device == MCR_NO_DEVICE gives a host-only context that touches no GPU: the
 * tuning table, mcr_get_variants, mcr_fuse_plan_create/info and all argument
 * validation work as usual, and any call that would launch or bind returns
 * MCR_ESTATE instead (after its validation has passed). */
int mcr_init(mcr_ctx** out, int device);

/* Destroys the context.  Plans created from it must be destroyed first. */
int mcr_finalize(mcr_ctx* ctx);

/* Blocks the host until `stream` has drained (hipStreamSynchronize). */
int mcr_synchronize(mcr_ctx* ctx, void* stream);

/* The kernel variants of one op, the analogue of get_backends().  On entry *n is
 * the capacity of names[]; on return *n is the number of variants, and the
 * first min(capacity, *n) entries of names[] point to static strings.  The
 * index in names[] is the variant id. */
int mcr_get_variants(mcr_ctx* ctx, int op_id, const char** names, int* n);

const char* mcr_strerror(int status);

/* ---- collectives ------------------------------------------------------------ */

/* all_reduce (API listing).  bufs[r], r<P: `count` elements each, reduced in
 * place: every bufs[r][i] becomes x_0[i] (+) x_1[i] (+) ... (+) x_{P-1}[i], taken left
 * to right in rank order in binary32 (bf16 widened first, rounded once to
 * nearest-even at the end).  Every element index is read (all P) and then
 * written (all P) by one thread, so in-place is race free.
 * Alignment: buffers need only be aligned to the element.  The 128-bit variants apply when all
 * P buffers are 16-byte aligned, and also when all of them miss that alignment by the same
 * number of bytes (the same view of a tensor on every rank) and the message reaches the next
 * 16-byte boundary; otherwise only the element path ("scalar") applies.  `count` may be any
 * number.
 * Two variants beyond the common launch shapes (all_reduce, reduce, reduce_scatter): "pk8", a
 * persistent form with one workgroup of 1024 threads per compute unit, each walking a contiguous
 * run of the message in rounds (read and reduce 8 steps of one vector per thread, then store
 * them), and "w64", workgroups of one wavefront with two vectors per thread.  The ids behind them,
 * named "<shape>.x<KiB>" ("v1nt.x1024", "w64.x512", ...), run that shape with its tiles dealt to
 * the 8 XCDs in contiguous units of that many KiB of every rank buffer instead of every eighth
 * tile; which of them wins depends on the message size, and the tuning table chooses. */
int mcr_allreduce(mcr_ctx* ctx, void* const* bufs, size_t count, mcr_dtype dtype,
                  mcr_redop op, int P, int variant, void* stream);

/* reduce_scatter (API listing; it has no root).  in[p]: `count` elements;
 * out[r]: count/P elements = slice r of the reduction.  P must divide count. */
int mcr_reduce_scatter(mcr_ctx* ctx, void* const* out, const void* const* in, size_t count,
                       mcr_dtype dtype, mcr_redop op, int P, int variant, void* stream);

/* all_gather (API listing; Table II is its tuning table).  in[p]: `count`
 * elements; out[r]: P*count elements, out[r][p*count + j] = in[p][j].  Bit copy.
 * Variants beyond the common launch shapes: "sc4", "sc8", "sc16" copy one super-chunk of 4, 8 or
 * 16 MiB of a source to one destination after the other (one read and one write stream at a time,
 * the re-reads served by the cache); "sc16x" is "sc16" with the tiles of a super-chunk dealt to the
 * 8 XCDs in contiguous units of 512 KiB. */
int mcr_allgather(mcr_ctx* ctx, void* const* out, const void* const* in, size_t count,
                  mcr_dtype dtype, int P, int variant, void* stream);

/* all_to_all_single (API listing; "shuffles the tensor elements themselves"),
 * equal split.  in[p], out[r]: `count` elements, P divides count, b = count/P:
 * out[r][p*b + k] = in[p][r*b + k].  Bit copy.
 * Variants beyond the common launch shapes: "flat" (threads numbered along the output of a
 * destination, so that blocks shorter than a workgroup leave no lane idle), "w64" (the same with
 * workgroups of one wavefront) and "lds" ("flat" with four vectors per thread staged through LDS
 * between the workgroup's loads and its stores). */
int mcr_alltoall(mcr_ctx* ctx, void* const* out, const void* const* in, size_t count,
                 mcr_dtype dtype, int P, int variant, void* stream);

/* all_to_allv (API listing) with packed displacements.  The unit is a row of
 * `row_elems` elements.  splits is P x P row-major int64, splits[p*P + r] = rows
 * rank p sends to rank r (row p is rank p's scounts, column r is rank r's
 * rcounts).  sdispl[p][r] = sum_{q<r} splits[p][q], rdispl[r][p] =
 * sum_{q<p} splits[q][r]:
 *     out[r] row (rdispl[r][p] + k) = in[p] row (sdispl[p][r] + k),  k < splits[p][r].
 * Rows of out[r] beyond its received total are left untouched.
 * splits_flags is a sum of:
 *   MCR_SPLITS_ON_DEVICE: splits is DEVICE memory (e.g. written by mcr_moe_route earlier on the
 *     same stream) and is read by the kernel; no host synchronisation happens.  The kernel
 *     itself skips any row that would fall outside in_rows / out_rows and treats negative
 *     entries as 0.  Without the flag splits is HOST memory, read before return and validated:
 *     a negative entry gives MCR_EINVAL; a sender's total above in_rows or a receiver's total
 *     above out_rows gives MCR_ESPLIT.
 *   MCR_SPLITS_TRANSPOSED: the matrix is read transposed, splits[r*P + p] = rows rank p sends to
 *     rank r.  This is the way back of an exchange that went out with the same matrix (the
 *     second Alltoall of paper Sec. II-C, which returns the expert outputs): every rank sends
 *     back what it received, and nobody has to transpose the matrix in between.
 * Any other bit gives MCR_EINVAL.
 *   splits == NULL: equal split, every pair exchanges in_rows/P rows (P must
 *     divide in_rows, and out_rows >= in_rows).
 * in_rows / out_rows: capacity, in rows, of every in[p] / out[r]. */
#define MCR_SPLITS_ON_DEVICE 1
#define MCR_SPLITS_TRANSPOSED 2
int mcr_alltoallv(mcr_ctx* ctx, void* const* out, const void* const* in, const int64_t* splits,
                  int splits_flags, size_t in_rows, size_t out_rows, size_t row_elems,
                  mcr_dtype dtype, int P, int variant, void* stream);

/* ---- rooted and vector collectives (API listing: reduce, bcast, gather, scatter, gatherv,
 * scatterv, all_gatherv; the paper names the vectored ones as what other frameworks lack,
 * Sec. I).  Displacements are packed: displ[p] = sum_{q<p} counts[q].  Counts are in
 * elements.  MCR_AUTO looks these up under MCR_OP_ALLREDUCE (reduce) and MCR_OP_ALLTOALLV
 * (the others), whose kernels they run on. ------------------------------------------------- */

/* reduce: bufs[root][i] = x_0[i] (+) ... (+) x_{P-1}[i] with the arithmetic of mcr_allreduce; the
 * other buffers are read only. */
int mcr_reduce(mcr_ctx* ctx, void* const* bufs, size_t count, mcr_dtype dtype, mcr_redop op,
               int root, int P, int variant, void* stream);

/* bcast: bufs[r][i] = bufs[root][i] for every r != root.  Bit copy.
 * In bcast and the all_gatherv calls a message longer than 16 MiB that goes to two receivers or
 * more is copied 16 MiB at a time to each receiver in turn, so that it is fetched from memory
 * once; a vector variant then selects the 128-bit path only (its cache hints and unroll apply to
 * shorter messages). */
int mcr_bcast(mcr_ctx* ctx, void* const* bufs, size_t count, mcr_dtype dtype, int root, int P,
              int variant, void* stream);

/* gather / gatherv: out (the root's receive buffer, DEVICE memory, sum of counts elements)
 * [displ[p] + j] = in[p][j], j < counts[p] (gather: every count is `count`).  counts: HOST
 * array of P.  in[p] may be NULL where counts[p] == 0. */
int mcr_gather(mcr_ctx* ctx, void* out, const void* const* in, size_t count, mcr_dtype dtype,
               int P, int variant, void* stream);
int mcr_gatherv(mcr_ctx* ctx, void* out, const void* const* in, const size_t* counts,
                mcr_dtype dtype, int P, int variant, void* stream);

/* scatter / scatterv: out[r][j] = in (the root's send buffer)[displ[r] + j], j < counts[r]. */
int mcr_scatter(mcr_ctx* ctx, void* const* out, const void* in, size_t count, mcr_dtype dtype,
                int P, int variant, void* stream);
int mcr_scatterv(mcr_ctx* ctx, void* const* out, const void* in, const size_t* counts,
                 mcr_dtype dtype, int P, int variant, void* stream);

/* all_gatherv (it has no root): out[r][displ[p] + j] = in[p][j] for every r. */
int mcr_allgatherv(mcr_ctx* ctx, void* const* out, const void* const* in, const size_t* counts,
                   mcr_dtype dtype, int P, int variant, void* stream);

/* ---- the vector collectives with displacements chosen by the caller (API listing: the
 * displs of gatherv / scatterv / all_gatherv, the sdispls and rdispls of all_to_allv) ------
 * Offsets count from the start of the buffer, in elements (rows of row_elems elements for
 * all_to_allv); gaps between blocks are left untouched.  The caller states the extent of the
 * buffers that displacements point into (out_elems, in_elems, in_rows, out_rows); a block that
 * leaves it gives MCR_ESPLIT and two blocks that overlap in one destination MCR_EINVAL, before
 * anything is launched.  counts, displs, sdispls, rdispls: HOST arrays.  Counts and offsets that
 * are not all multiples of 16 bytes take the element path (variant "scalar").
 *
 * mcr_alltoallv_displs: out[r] rows rdispls[r*P + p] + k = in[p] rows sdispls[p*P + r] + k for
 * k < counts[p*P + r]. */
int mcr_alltoallv_displs(mcr_ctx* ctx, void* const* out, const void* const* in,
                         const int64_t* counts, const int64_t* sdispls, const int64_t* rdispls,
                         size_t in_rows, size_t out_rows, size_t row_elems, mcr_dtype dtype, int P,
                         int variant, void* stream);

/* out[displs[p] + j] = in[p][j], j < counts[p]; out holds out_elems elements. */
int mcr_gatherv_displs(mcr_ctx* ctx, void* out, size_t out_elems, const void* const* in,
                       const size_t* counts, const size_t* displs, mcr_dtype dtype, int P,
                       int variant, void* stream);

/* out[r][j] = in[displs[r] + j], j < counts[r]; in holds in_elems elements. */
int mcr_scatterv_displs(mcr_ctx* ctx, void* const* out, const void* in, size_t in_elems,
                        const size_t* counts, const size_t* displs, mcr_dtype dtype, int P,
                        int variant, void* stream);

/* out[r][displs[p] + j] = in[p][j] for every r; every out[r] holds out_elems elements. */
int mcr_allgatherv_displs(mcr_ctx* ctx, void* const* out, size_t out_elems, const void* const* in,
                          const size_t* counts, const size_t* displs, mcr_dtype dtype, int P,
                          int variant, void* stream);

/* ---- MoE dispatch / combine (paper Sec. II-C: routing of tokens to experts and
 * the combination of the expert outputs each need an Alltoall) -------------------
 *
 * mcr_moe_route: for every rank p independently, from top-1 expert ids
 * expert_ids[p][t], t<T (ids outside [0,E) drop the token):
 *   pos[t]  = number of earlier tokens of rank p with the same expert
 *   kept[t] = pos[t] < capacity
 *   counts[p][e] = min(#tokens of e, capacity); base[e] = sum_{e'<e} counts[p][e']
 *   slot[p][t] = kept ? base[id] + pos[t] : -1      (row in rank p's packed send buffer)
 *   splits[p*P + r] = sum of counts[p][e] over the E/P experts living on rank r
 * so the packed buffer is ordered by (expert, token index), hence by
 * destination rank.  P must divide E; E <= MCR_MAX_EXPERTS; T < 2^31.
 * expert_ids, slot, counts: host arrays of P device pointers (T, T, E int32
 * each); splits: DEVICE memory, P*P int64, fully overwritten. */
int mcr_moe_route(mcr_ctx* ctx, const int32_t* const* expert_ids, int T, int E, int P,
                  int capacity, int32_t* const* slot, int32_t* const* counts, int64_t* splits,
                  void* stream);

/* mcr_moe_route_ws: the same results as mcr_moe_route, bit for bit, computed by several
 * workgroups per rank (chunks of at least 2048 tokens, two launches) with a caller-owned
 * workspace between them: DEVICE memory, 4-byte aligned, at least
 * mcr_moe_route_workspace_bytes(T, E, P) bytes, contents irrelevant before and after; calls that
 * may overlap in time need a workspace each.  workspace == NULL, or a T for which the byte count
 * is 0 (fewer than two chunks), runs mcr_moe_route itself; a workspace that is too small gives
 * MCR_EINVAL.  For callers who route tens of thousands of tokens per rank: the one-workgroup
 * kernel is bound by the vector ALU of one compute unit. */
size_t mcr_moe_route_workspace_bytes(int T, int E, int P);
int mcr_moe_route_ws(mcr_ctx* ctx, const int32_t* const* expert_ids, int T, int E, int P,
                     int capacity, int32_t* const* slot, int32_t* const* counts, int64_t* splits,
                     void* workspace, size_t workspace_bytes, void* stream);

/* mcr_moe_route_static: for callers that cannot allocate device memory or own a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The same
 * results as mcr_moe_route_ws, bit for bit, by the same kernels; the chunk counters sit in a
 * static device array of MCR_ROUTE_SCRATCH_BYTES that each GPU the library runs on holds until
 * the process ends.  Neither this call nor anything it calls allocates or frees memory.
 * A routing whose counters need more (mcr_moe_route_workspace_bytes(T, E, P) >
 * MCR_ROUTE_SCRATCH_BYTES) gives MCR_ELIMIT and launches nothing; a T with fewer than two chunks
 * runs mcr_moe_route's one-workgroup kernel, which uses no scratch.  All calls on one GPU share
 * that GPU's array: two calls that may overlap in time there (different streams, or threads)
 * race; calls on one stream are ordered and safe.  Nothing has to be cleared between calls: the
 * first launch overwrites every counter the second one reads. */
#define MCR_ROUTE_SCRATCH_BYTES (1u << 20)
int mcr_moe_route_static(mcr_ctx* ctx, const int32_t* const* expert_ids, int T, int E, int P,
                         int capacity, int32_t* const* slot, int32_t* const* counts,
                         int64_t* splits, void* stream);

/* mcr_pack, batched over P ranks: out[p] row slot[p][t] = in[p] row t for every t<T
 * with 0 <= slot[p][t] < out_rows; other rows of out[p] are left untouched. */
int mcr_pack(mcr_ctx* ctx, void* const* out, const void* const* in, const int32_t* const* slot,
             size_t T, size_t out_rows, size_t row_elems, mcr_dtype dtype, int P, int variant,
             void* stream);

/* mcr_unpack, batched over P ranks: out[p] row t = in[p] row slot[p][t] if
 * 0 <= slot[p][t] < in_rows, else all-zero bits.  With gate != NULL (host array of
 * P device pointers to T binary32 weights) the kept rows are scaled:
 * out = round_to_dtype(gate[p][t] * f32(in)), one binary32 multiply and one
 * rounding (the gate-weighted combine). */
int mcr_unpack(mcr_ctx* ctx, void* const* out, const void* const* in, const int32_t* const* slot,
               const float* const* gate, size_t T, size_t in_rows, size_t row_elems,
               mcr_dtype dtype, int P, int variant, void* stream);

/* ---- pipelines fused across op boundaries ----------------------------------------
 * One address space lets a row go straight from where it is to where it is needed;
 * each call below writes bit for bit what the chain of calls it replaces writes, for
 * split matrices as mcr_moe_route produces them (entries within [0, T]).
 *
 * mcr_moe_dispatch = mcr_pack followed by mcr_alltoallv(splits on device): for every rank
 * p and token t with 0 <= slot[p][t] < T, the token row is written to row
 * rdispl[r][p] + (slot - sdispl[p][r]) of recv[r], r being the rank whose block of rank
 * p's packed order holds that slot.  Rows that would fall outside recv_rows are skipped;
 * other rows of recv are left untouched.  splits: DEVICE memory, P*P int64.
 * On rows wider than 2 KiB this call and mcr_moe_combine launch two kernels: a one-workgroup
 * kernel turns `splits` into displacement tables in the next of the context's 64 table slots
 * (device memory the context owns), and the row kernel reads them.  Both are ordered on
 * `stream`; only more than 64 such calls in flight at once on different streams would meet in
 * one slot.  A captured graph keeps the slot it was captured with. */
int mcr_moe_dispatch(mcr_ctx* ctx, void* const* recv, const void* const* tokens,
                     const int32_t* const* slot, const int64_t* splits, size_t T, size_t recv_rows,
                     size_t row_elems, mcr_dtype dtype, int P, int variant, void* stream);

/* mcr_moe_combine = mcr_alltoallv(transposed splits) followed by mcr_unpack with a gate:
 * out[p] row t = round_to_dtype(gate[p][t] * f32(row of expert_out[r] that token t was
 * dispatched to)), all-zero bits for a dropped token.  expert_out[r] has the layout of
 * recv[r] above (the experts' outputs, row for row).  gate may be NULL (no scaling). */
int mcr_moe_combine(mcr_ctx* ctx, void* const* out, const void* const* expert_out,
                    const int32_t* const* slot, const float* const* gate, const int64_t* splits,
                    size_t T, size_t recv_rows, size_t row_elems, mcr_dtype dtype, int P, int variant,
                    void* stream);

/* ---- expert-major receive layout ---------------------------------------------------
 * The expert FFN that follows the dispatch Alltoall of paper Sec. II-C works on the tokens of
 * one expert at a time.  The calls below deliver every expert's tokens as one block:
 * the receive buffer of rank r is ordered by (local expert, source rank, token order).
 *
 * mcr_moe_expert_layout: from counts[p][e] (kept tokens per source rank and expert, as
 * mcr_moe_route leaves them; negative entries count as 0), with per = E/P:
 *   expert_rows[e]  = sum_p counts[p][e]
 *   expert_first[e] = sum of expert_rows[e'] for per*(e/per) <= e' < e
 *   row_table[p*E + e] = expert_first[e] + sum_{q<p} counts[q][e] - sum_{e'<e} counts[p][e']
 * so that token t of rank p (kept, expert id) lands in row row_table[p*E + id] + slot[p][t]
 * of rank id/per.  counts: host array of P device pointers (E int32 each); row_table,
 * expert_first, expert_rows: DEVICE memory, 8-byte aligned, P*E, E and E int64, overwritten.
 * One small launch; nothing is synchronised. */
int mcr_moe_expert_layout(mcr_ctx* ctx, const int32_t* const* counts, int E, int P,
                          int64_t* row_table, int64_t* expert_first, int64_t* expert_rows,
                          void* stream);

/* mcr_moe_source_layout: the row table of the OTHER receive layout, the one mcr_pack followed by
 * mcr_alltoallv (and mcr_moe_dispatch) produces: at rank r the rows are ordered by (source rank,
 * local expert, token order).  With S[p][r] = sum of counts[p][e] over the experts of rank r:
 *   row_table[p*E + e] = sum_{q<p} S[q][e/(E/P)] - sum_{r'<e/(E/P)} S[p][r'].
 * mcr_moe_dispatch_by_expert / mcr_moe_combine_by_expert fed this table move the same rows to the
 * same places as mcr_moe_dispatch / mcr_moe_combine, bit for bit (for a caller that keeps the
 * table over several calls).  Arguments as for mcr_moe_expert_layout. */
int mcr_moe_source_layout(mcr_ctx* ctx, const int32_t* const* counts, int E, int P,
                          int64_t* row_table, void* stream);

/* Top-K gating: every token has K choices (1 <= K <= MCR_MAX_TOPK).  expert_ids[p], slot[p] and
 * gate[p] then hold K*T entries, choice-major: entry a = k*T + t is choice k of token t.  Routing
 * is mcr_moe_route over those K*T entries (its T argument = K*T), which walks them in that order,
 * so first choices fill an expert's capacity before any second choice; mcr_moe_expert_layout is
 * unchanged.  K*T < 2^31.
 *
 * mcr_moe_dispatch_by_expert: for every rank p and assignment a < K*T with slot[p][a] >= 0 and
 * 0 <= id = expert_ids[p][a] < E, row (a mod T) of tokens[p] is written to row
 * row_table[p*E + id] + slot[p][a] of recv[id / (E/P)]; a row outside [0, recv_rows) is
 * skipped, other rows of recv are left untouched.  expert_ids, slot: as for
 * mcr_moe_route; row_table: DEVICE memory as mcr_moe_expert_layout writes it. */
int mcr_moe_dispatch_by_expert(mcr_ctx* ctx, void* const* recv, const void* const* tokens,
                               const int32_t* const* expert_ids, const int32_t* const* slot,
                               const int64_t* row_table, size_t T, int K, int E, size_t recv_rows,
                               size_t row_elems, mcr_dtype dtype, int P, int variant, void* stream);

/* mcr_moe_combine_by_expert: the way back.  With x_k = f32(row row_table[p*E + id_k] + slot_k of
 * expert_out[id_k/(E/P)]) for the dispatched choices k of token t, in choice order:
 * out[p] row t = round_to_dtype(g_0*x_0 + g_1*x_1 + ...), binary32 products and sums, the sum
 * starting from the first dispatched product, one rounding; all-zero bits when no choice of the
 * token was dispatched.  gate: host array of P device pointers to K*T binary32 weights, or NULL
 * (weights of 1; with K = 1 the row is then copied bit for bit). */
int mcr_moe_combine_by_expert(mcr_ctx* ctx, void* const* out, const void* const* expert_out,
                              const int32_t* const* expert_ids, const int32_t* const* slot,
                              const float* const* gate, const int64_t* row_table, size_t T, int K,
                              int E, size_t recv_rows, size_t row_elems, mcr_dtype dtype, int P,
                              int variant, void* stream);

/* mcr_dlrm_shuffle: the embedding shuffle of paper Sec. II-D as one row permutation.
 * n_tables tables, table t on rank t mod P as its local table t div P.
 *   backward == 0: in[p] is [T_p][batch][dim] (table-major pooled rows), out[r] is
 *     [batch/P][n_tables][dim]; out[r][b][t][:] = in[t mod P][t div P][r*(batch/P) + b][:].
 *   backward != 0: the inverse (gradients): in[r] is [batch/P][n_tables][dim], out[p] is
 *     [T_p][batch][dim].
 * P must divide batch.  Equals pack + all_to_allv + unpack of the same rows. */
int mcr_dlrm_shuffle(mcr_ctx* ctx, void* const* out, const void* const* in, int n_tables,
                     size_t batch, size_t dim, mcr_dtype dtype, int P, int backward, int variant,
                     void* stream);

/* ---- tensor fusion (paper Sec. IV-D: small tensors are combined into a fusion
 * buffer of at most B elements; the wait-time parameter T is not modelled) -------
 *
 * Plan: walk numel[0..n_tensors) in order; a tensor larger than bucket_elems
 * closes the open bucket and is a bucket by itself (never split); otherwise, if
 * it does not fit in the open bucket, that bucket is closed first; then it is
 * appended.  Offsets inside a bucket are running sums, no padding. */
int mcr_fuse_plan_create(mcr_ctx* ctx, const size_t* numel, int n_tensors, size_t bucket_elems,
                         mcr_dtype dtype, mcr_fuse_plan** out);

/* Any output pointer may be NULL.  bucket_numel needs n_buckets entries,
 * tensor_bucket and tensor_offset n_tensors entries. */
int mcr_fuse_plan_info(const mcr_fuse_plan* plan, int* n_buckets, size_t* bucket_numel,
                       int* tensor_bucket, size_t* tensor_offset);

/* Binds the tensors of P ranks to the plan: tensors is a HOST array of
 * P*n_tensors DEVICE pointers, rank-major (tensors[p*n_tensors + i]).  The table
 * is copied to plan-owned device memory synchronously (the call blocks until
 * the copy is done; it may allocate on its first use or when P grows).  Rebind
 * whenever an address changes; do not rebind while launches that use the plan
 * are still in flight. */
int mcr_fuse_plan_bind(mcr_ctx* ctx, mcr_fuse_plan* plan, void* const* tensors, int P);

/* fuse: flat[p][off_i + j] = tensor_i^p[j] for the tensors of `bucket`, all bound
 * ranks in one launch.  flat: host array of P device pointers, each with room
 * for bucket_numel[bucket] elements.  P must equal the bound P. */
int mcr_fuse(mcr_ctx* ctx, const mcr_fuse_plan* plan, int bucket, void* const* flat, int P,
             int variant, void* stream);

/* unfuse: the inverse, writes the bound tensors. */
int mcr_unfuse(mcr_ctx* ctx, const mcr_fuse_plan* plan, int bucket, const void* const* flat, int P,
               int variant, void* stream);

/* The small-message path (paper Sec. IV-C: concurrency only helps small
 * messages; Sec. IV-D: fusion exists to avoid many tiny operations): one launch
 * all-reduces, in place and with the arithmetic of mcr_allreduce, every bound
 * tensor of `bucket` (or of the whole plan when bucket == -1) across the bound
 * P ranks, reading and writing the tensors where they lie -- no flat buffer. */
int mcr_allreduce_multi(mcr_ctx* ctx, const mcr_fuse_plan* plan, int bucket, mcr_redop op,
                        int variant, void* stream);

int mcr_fuse_plan_destroy(mcr_fuse_plan* plan);

/* ---- diagnostic: what the dispatch layer costs (paper Sec. V-B compares the runtime with a
 * C-level micro-benchmark of the same operation and reports 5 % overhead for small, 1 % for
 * large messages).  Runs `iters` back-to-back all_to_all_single operations on `stream` twice:
 * through mcr_alltoall with MCR_AUTO (validation, table lookup, pointer-table marshalling,
 * launch) and as bare launches of the kernel that call resolves to, each followed by one
 * stream synchronisation, the two loops swapping places from round to round; reports the best
 * of four rounds as microseconds per operation:
 * us_auto / us_direct from the first call to the end of the synchronisation (what an
 * application sees), host_us_auto / host_us_direct (either may be NULL) up to the return of
 * the last enqueueing call (the CPU cost per call while the hardware queue has room; it moves
 * by a microsecond with the state of the runtime's queue), and dispatch_only_us (may be NULL):
 * the CPU time per call of everything mcr_alltoall does before its launch (checks, pointer
 * tables, table lookup), timed in a loop of 20 * iters calls that launches nothing, which is
 * the dispatch layer's cost with no noise from the GPU in it.
 * Arguments as for mcr_alltoall; the buffers are overwritten. */
int mcr_dispatch_overhead(mcr_ctx* ctx, void* const* out, const void* const* in, size_t count,
                          mcr_dtype dtype, int P, int iters, void* stream, double* us_auto,
                          double* us_direct, double* host_us_auto, double* host_us_direct,
                          double* dispatch_only_us);

/* ---- static tuning table (paper Sec. IV-E, Table II) ---------------------------
 * One table per (op, dtype, P): rows (message bytes -> variant), kept sorted by
 * size.  Lookup takes the row with the largest size not above the message; a
 * message below the first row takes the first, above the last the last; no rows
 * gives MCR_EVARIANT from mcr_tune_get.  MCR_AUTO, finding no table for its rank count,
 * takes the table of the closest rank count of the same op and dtype, and its built-in
 * default (one vector per thread below 1 MiB, four above) when there is none at all.
 * "Message bytes" is one rank's send-buffer size: count*elem for allreduce,
 * reduce_scatter, allgather, alltoall; in_rows*row bytes for alltoallv;
 * T*row bytes for pack/unpack; bucket bytes for fuse/unfuse/allreduce_multi. */
int mcr_tune_set(mcr_ctx* ctx, int op_id, mcr_dtype dtype, int P, size_t bytes, int variant);
int mcr_tune_get(mcr_ctx* ctx, int op_id, mcr_dtype dtype, int P, size_t bytes, int* variant);
/* What MCR_AUTO would choose for this key and size: the table's row if there is one, else
 * the built-in default; the scalar variant when vec_ok == 0 (shape or alignment rules the
 * 128-bit variants out). */
int mcr_auto_variant(mcr_ctx* ctx, int op_id, mcr_dtype dtype, int P, size_t bytes, int vec_ok, int* variant);
int mcr_tune_clear(mcr_ctx* ctx);
/* Number of rows over all tables (Num_Collectives x Num_Scales x Num_Message_Sizes). */
int mcr_tune_count(mcr_ctx* ctx, size_t* n_rows);
/* Text file, one row per line: "<op name> <dtype name> <P> <bytes> <variant name>". */
int mcr_tune_save(mcr_ctx* ctx, const char* path);
int mcr_tune_load(mcr_ctx* ctx, const char* path);

#ifdef __cplusplus
}
#endif
#endif /* MCR_H_ */
