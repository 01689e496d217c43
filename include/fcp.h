/*
 * libfcp -- rank-local attention of Flexible Context Parallelism on MI355X (gfx950).
 *
 * The paper assigns every packed sequence to a context-parallel (CP) group whose degree
 * may be ANY positive integer (Sec. 4.2) and computes attention (Eq. 1, Sec. 3.1; causal
 * for language models, Sec. 4.3) ring-style: each rank keeps its share of the queries
 * while key/value blocks travel round the group (Sec. 3.2, Sec. 4.3 communication cost).
 * This library is the work ONE rank does: a shard plan, one partial attention result per
 * ring step, the log-sum-exp merge of those partials, and the matching backward.
 * Two forms of the device calls: the plain ones (fcp_attn_fwd_step, fcp_lse_merge, fcp_attn_bwd_step,
 * fcp_grad_finalize) work one or several ring steps per call and combine across calls; the *_direct ones take a
 * rank's whole work list at once and write every row that a single work item feeds - in a packed batch, most -
 * in its final form straight from the attention kernel.
 *
 * Conventions
 *   - plain C ABI, no exceptions; every call returns 0 (FCP_OK) or a negative FCP_ERR_*;
 *     fcp_last_error() returns a thread-local message for the last failing call.
 *   - the CALLER owns all memory, host and device.  The library allocates no device memory;
 *     kernels that need a work area take `scratch` sized by fcp_scratch_bytes().
 *   - "device" pointers are HIP device memory of the current device; "host" pointers are
 *     ordinary host memory.  Device calls enqueue work on `stream` (a hipStream_t passed as
 *     void*, NULL = default stream) and return without synchronising.  Outputs are
 *     undefined after an error return.
 *   - bf16 tensors are raw 16-bit patterns; fp32 is IEEE binary32.
 *   - layouts (row-major, last index fastest):
 *       Q, dO, O, dQ      [tq , hq , head_dim]   rows = the rank's local (packed) query rows
 *       K, V, dK, dV      [tkv, hkv, head_dim]   the resident pool: every sequence unsharded,
 *                                                in input order; sequence n starts at row
 *                                                cu_seqlens_kv[n]
 *       LSE, Delta        [hq, tq]  fp32 (head-major)
 *       partial O         [n_parts][tq, hq, head_dim]  fp32
 *       partial LSE       [n_parts][hq, tq]            fp32
 *   - query head h reads KV head h / (hq / hkv); hq % hkv == 0; head_dim is 64 or 128.
 *   - LSE is the natural log of the sum of exp of the SCALED scores; -inf marks "no key".
 */
#ifndef FCP_H_
#define FCP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FCP_OK 0
#define FCP_ERR_INVALID_ARG (-1)
#define FCP_ERR_CAPACITY (-2)
#define FCP_ERR_UNSUPPORTED (-3)
#define FCP_ERR_HIP (-4)

/* One per (sequence, zigzag chunk), sorted by (rank, seq, chunk).  24 bytes. */
typedef struct fcp_chunk_desc {
  int32_t seq;        /* index into seq_lens                                             */
  int32_t rank;       /* base_rank[seq] + group-local rank                               */
  int32_t chunk;      /* 0 .. 2d-1 (0 only when the degree d is 1)                       */
  int32_t seq_start;  /* first token position of the chunk inside its sequence          */
  int32_t len;        /* tokens in the chunk (0 is possible when L < 2d)                 */
  int32_t local_off;  /* row offset of the chunk in that rank's packed Q/O/dO/dQ buffers */
} fcp_chunk_desc;

/* One per (rank, ring step, sequence, query chunk) that sees at least one key.  44 bytes.
 * The mask is implied by positions: a key is visible iff k_pos <= q_pos, where
 * q_pos = q_seq_start + row and k_pos = k_seq_start[s] + key inside segment s (with full-attention spans:
 * iff k_pos <= limit(q_pos), see fcp_shard_plan_mixed).
 * Sorted by (rank, step, seq, q_seq_start).  Unused segment fields are 0. */
typedef struct fcp_work_desc {
  int32_t seq, rank, step;      /* step s reads the KV chunks of group-local rank (i - s) mod d;
                                   it is also the partial slot this item writes            */
  int32_t q_local_off, q_seq_start, q_len;
  int32_t n_seg;                /* 1 or 2 key/value segments, increasing positions         */
  int32_t k_seq_start[2], k_len[2];
} fcp_work_desc;

/* Message of the last error on the calling thread ("" if none).  Never NULL. */
const char* fcp_last_error(void);

/*
 * fcp_shard_plan -- HOST ONLY, integer exact.
 * Splits every sequence for its CP degree (the paper: an even split over the d ranks of
 * the group, Sec. 4.3; any integer d, Sec. 4.2) in the load-balanced zigzag form:
 * degree 1 -> one chunk; degree d > 1 -> 2d chunks, the first (L mod 2d) one token longer,
 * group-local rank i owning chunks i and 2d-1-i.  Emits the chunk table and, per
 * (rank, ring step), the work items (query chunk x visible KV segments).
 *   seq_lens, cp_degree [n_seqs] host, lengths >= 1, degrees >= 1
 *   base_rank [n_seqs] host or NULL (all 0): first global rank of each sequence's group
 *   chunks / work: host output arrays of chunk_cap / work_cap entries, or NULL to only count
 *   n_chunks / n_work: host, always written with the required counts
 * Returns FCP_ERR_CAPACITY if a non-NULL array is too small (counts are still written).
 */
int fcp_shard_plan(const int32_t* seq_lens, const int32_t* cp_degree, const int32_t* base_rank,
                   int32_t n_seqs, fcp_chunk_desc* chunks, int64_t chunk_cap, int64_t* n_chunks,
                   fcp_work_desc* work, int64_t work_cap, int64_t* n_work);

/* Scratch size in bytes for `which` = FCP_SCRATCH_FWD or FCP_SCRATCH_BWD. */
#define FCP_SCRATCH_FWD 0
#define FCP_SCRATCH_BWD 1
size_t fcp_scratch_bytes(int which, int32_t tq, int32_t tkv, int32_t hq, int32_t hkv,
                         int32_t head_dim, int64_t n_work, int32_t n_parts);

/*
 * fcp_attn_fwd_step -- partial attention of one rank for one or several ring steps.
 * For every work item, every row of its query chunk and every head: softmax(scale q.K^T)
 * V over the item's VISIBLE keys only (Eq. 1 restricted to the keys present in that ring
 * step), normalised by that step's own sum, written to partial slot `step` together with
 * LSE_step.  Rows that no item of a slot covers get LSE = -inf in that slot and their
 * partial O rows are left unwritten (fcp_lse_merge never reads them).
 *   q [tq,hq,D], k, v [tkv,hkv,D]           bf16 device
 *   cu_seqlens_kv [n_seqs+1]                 int32 device
 *   work [n_work]                            device; this rank's items, any subset of steps
 *   n_parts                                  number of partial slots; every item needs step < n_parts
 *   o_part [n_parts][tq,hq,D] fp32, lse_part [n_parts][hq,tq] fp32       device outputs
 *   scratch                                  device, >= fcp_scratch_bytes(FCP_SCRATCH_FWD, ...), 256-byte aligned
 * Items are checked on the device against tq, tkv, n_seqs and n_parts; an item that fails is
 * skipped and counted (see fcp_scratch_status); no access leaves the given extents.
 * Two items that cover the same (row, step) are a caller error (last writer wins).
 * Limits: n_work <= 2^24 items (FCP_ERR_UNSUPPORTED beyond); a key segment of an item at most 2^30 bytes of pool
 * rows (2^30 / (hkv * head_dim * 2) keys; longer segments are rejected on the device and counted); the CP degree
 * itself is not limited (any integer, Sec. 4.2) beyond n_parts partial slots of memory.
 */
int fcp_attn_fwd_step(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                      int32_t n_seqs, const fcp_work_desc* work, int64_t n_work, int32_t n_parts,
                      int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                      float softmax_scale, float* o_part, float* lse_part,
                      void* scratch, size_t scratch_bytes, void* stream);

/*
 * fcp_attn_fwd_step_static -- fcp_attn_fwd_step for callers that cannot allocate device memory or carry a work
 * area around: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * function, arguments, results and errors as fcp_attn_fwd_step, except that the scheduler's work area is a static
 * device array inside the library (FCP_STATIC_SCRATCH_BYTES, held on every GPU the library runs on until the
 * process ends) instead of `scratch`.  The call allocates nothing and frees nothing.
 *   - a call that needs more than FCP_STATIC_SCRATCH_BYTES (see fcp_scratch_bytes(FCP_SCRATCH_FWD, ...)) returns
 *     FCP_ERR_CAPACITY and launches nothing;
 *   - every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two streams, two threads)
 *     race and give undefined results; calls on one stream are ordered and safe.  Nothing has to be cleared between
 *     calls;
 *   - fcp_scratch_status has no access to the static area.
 */
#define FCP_STATIC_SCRATCH_BYTES (2 * 1024 * 1024)
int fcp_attn_fwd_step_static(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                             int32_t n_seqs, const fcp_work_desc* work, int64_t n_work, int32_t n_parts,
                             int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                             float softmax_scale, float* o_part, float* lse_part, void* stream);

/*
 * fcp_lse_merge -- combine the partials of the ring steps (online-softmax rescaling):
 *   LSE = ln sum_s exp(LSE_s),   O = sum_s exp(LSE_s - LSE) O_s.
 * A slot with LSE_s = -inf contributes nothing and its O rows are not read; a row whose
 * slots are all -inf gets O = 0, LSE = -inf.  o [tq,hq,D] bf16 (round to nearest even),
 * lse [hq,tq] fp32.  All pointers device.
 * Limit: n_parts <= 16 per call (FCP_ERR_UNSUPPORTED beyond) - a ring of more than 16 steps merges in rounds, the
 * result of a round being one more partial (the merge is associative), or uses fcp_attn_fwd_step_running.
 */
int fcp_lse_merge(const float* o_part, const float* lse_part, int32_t n_parts, int32_t tq,
                  int32_t hq, int32_t head_dim, void* o, float* lse, void* stream);

/*
 * fcp_attn_fwd_step_direct / fcp_lse_merge_direct -- the whole forward of a rank with final results written once.
 * Same function as fcp_attn_fwd_step (+ _mixed when q_limit is given) followed by fcp_lse_merge, for a work list that
 * carries ALL ring steps.  Rows that get all their keys from one work item (every sequence that is not sharded,
 * paper Sec. 4.1; no other item of the call covers the item's query rows) need no partial result and no merge
 * (Sec. 3.2: the rescaling combines the steps of a ring): the kernel writes their normalised O as bf16 into o and
 * their LSE into lse.  The other rows get partial results in o_part / lse_part as in fcp_attn_fwd_step;
 * fcp_lse_merge_direct merges those, gives rows that no item covers O = 0 and LSE = -inf, and leaves the directly
 * written rows alone.  The row states stay in `scratch` between the two calls.
 *   o [tq,hq,D] bf16, lse [hq,tq] fp32: device, complete after fcp_lse_merge_direct;  o_part / lse_part: defined only
 *   for the rows that are merged.  n_work <= 1024 (FCP_ERR_UNSUPPORTED beyond).  Other arguments, alignment and errors
 *   as in fcp_attn_fwd_step; fcp_lse_merge_direct takes the same n_parts, tq, tkv, n_work and scratch.
 */
int fcp_attn_fwd_step_direct(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                             int32_t n_seqs, const fcp_work_desc* work, int64_t n_work, int32_t n_parts,
                             int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                             float softmax_scale, const int32_t* q_limit, float* o_part, float* lse_part,
                             void* o, float* lse, void* scratch, size_t scratch_bytes, void* stream);
int fcp_lse_merge_direct(const float* o_part, const float* lse_part, int32_t n_parts, int32_t tq,
                         int32_t tkv, int32_t hq, int32_t head_dim, void* o, float* lse, void* scratch,
                         int64_t n_work, void* stream);

/* Backward prologue: delta[h, i] = sum_c dO[i,h,c] * O[i,h,c]  (fp32).  Device pointers. */
int fcp_attn_bwd_delta(const void* o, const void* d_o, int32_t tq, int32_t hq, int32_t head_dim,
                       float* delta, void* stream);

/*
 * fcp_attn_bwd_step -- gradient contributions of one rank for one or several ring steps.
 * With P = exp(scale q.K^T - LSE) on the visible pairs of each work item (LSE = merged),
 *   dV += P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dQ += scale dS K,  dK += scale dS^T Q,
 * dK/dV summed over the hq/hkv query heads of a KV head.  The three fp32 accumulators are
 * ADDED to (caller zeroes them before the first step): dq_acc [tq,hq,D], dk_acc, dv_acc
 * [tkv,hkv,D].  Rows (keys) that only one work item of the call touches are read, added to and
 * written back with plain loads and stores; the others use fp32 atomics, so their summation
 * order varies run to run.  While the call runs nobody else may write the accumulators.
 * Limits: tq*hq*head_dim below 2^30 - 2^21 elements (the bf16 rows of a work item are addressed with 32-bit byte
 * offsets), n_work <= 2^24 items (FCP_ERR_UNSUPPORTED).
 * Other arguments as in fcp_attn_fwd_step; scratch sized with FCP_SCRATCH_BWD.
 */
int fcp_attn_bwd_step(const void* q, const void* k, const void* v, const void* d_o,
                      const float* lse, const float* delta, const int32_t* cu_seqlens_kv,
                      int32_t n_seqs, const fcp_work_desc* work, int64_t n_work,
                      int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                      float softmax_scale, float* dq_acc, float* dk_acc, float* dv_acc,
                      void* scratch, size_t scratch_bytes, void* stream);

/*
 * Mixed masks (paper Sec. 4.3, time estimation before Eq. 8: multimodal models give some tokens full
 * attention; the mask efficiency factor eta_k of Eq. 8 follows from the shape of the mask).  Reading: the
 * tokens [start, start + len) of a span see each other in BOTH directions, every other pair of a sequence is
 * causal.  Such a mask keeps two monotone properties the kernels use: the query at position i sees exactly
 * the keys 0 .. limit(i), and the key at position j is seen by exactly the queries from(j) .. L-1, where
 * limit / from are the position itself outside a span and the span's last / first position inside one.
 */
typedef struct fcp_span {
  int32_t seq;    /* index into seq_lens          */
  int32_t start;  /* first token of the span      */
  int32_t len;    /* tokens in the span, >= 1     */
} fcp_span;

/*
 * fcp_shard_plan_mixed -- fcp_shard_plan for sequences with full-attention spans.  HOST ONLY, integer exact.
 * The chunks are those of fcp_shard_plan; a work item lists every key chunk of its ring step of which the
 * query chunk's last row sees at least the first key, which may include a LATER chunk when a span crosses the
 * chunk border.  The work descriptors keep their meaning, except that inside a (query row, segment) pair a key
 * is visible iff k_pos <= limit(q_pos) instead of k_pos <= q_pos.
 *   spans [n_spans] host, sorted by (seq, start), not overlapping, inside their sequences (else
 *   FCP_ERR_INVALID_ARG); n_spans = 0 gives fcp_shard_plan's result.  Other arguments as in fcp_shard_plan.
 */
int fcp_shard_plan_mixed(const int32_t* seq_lens, const int32_t* cp_degree, const int32_t* base_rank,
                         int32_t n_seqs, const fcp_span* spans, int32_t n_spans, fcp_chunk_desc* chunks,
                         int64_t chunk_cap, int64_t* n_chunks, fcp_work_desc* work, int64_t work_cap,
                         int64_t* n_work);

/*
 * fcp_mask_tables -- HOST ONLY, integer exact.  The per-row form of a mixed mask for one rank:
 *   q_limit [n_q] out (or NULL): for every local query row of `rank` (rows as laid out by the chunk table,
 *            n_q = the rank's row count, written to *n_q if non-NULL) the sequence position of the last key
 *            the row sees; q_limit_cap = entries available (FCP_ERR_CAPACITY if fewer than n_q)
 *   k_from  [sum of seq_lens] out (or NULL): for every row of the KV pool the sequence position of the first
 *            query that sees the key
 *   eta     [n_seqs] out (or NULL): visible pairs of the sequence over its causal count L (L + 1) / 2, minus 1
 *            (the factor of Eq. 8; feeds fcp_plan_groups)
 *   chunks [n_chunks]: the chunk table of fcp_shard_plan(_mixed) for the same lengths; spans as above.
 */
int fcp_mask_tables(const int32_t* seq_lens, int32_t n_seqs, const fcp_span* spans, int32_t n_spans,
                    const fcp_chunk_desc* chunks, int64_t n_chunks, int32_t rank, int32_t* q_limit,
                    int64_t q_limit_cap, int64_t* n_q, int32_t* k_from, float* eta);

/*
 * fcp_attn_fwd_step_mixed / fcp_attn_bwd_step_mixed -- the two attention steps under a mixed mask.  As
 * fcp_attn_fwd_step / fcp_attn_bwd_step with the work items of fcp_shard_plan_mixed and
 *   q_limit [tq]  int32 device: fcp_mask_tables' q_limit of this rank
 *   k_from  [tkv] int32 device: fcp_mask_tables' k_from (backward only)
 * Both tables must be non-decreasing along a chunk / a sequence and describe the same mask; values are only
 * compared with positions, never used as addresses, so wrong tables give wrong numbers but no access outside
 * the given extents.
 */
int fcp_attn_fwd_step_mixed(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                            int32_t n_seqs, const fcp_work_desc* work, int64_t n_work, int32_t n_parts,
                            int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                            float softmax_scale, const int32_t* q_limit, float* o_part, float* lse_part,
                            void* scratch, size_t scratch_bytes, void* stream);
int fcp_attn_bwd_step_mixed(const void* q, const void* k, const void* v, const void* d_o,
                            const float* lse, const float* delta, const int32_t* cu_seqlens_kv,
                            int32_t n_seqs, const fcp_work_desc* work, int64_t n_work,
                            int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                            float softmax_scale, const int32_t* q_limit, const int32_t* k_from,
                            float* dq_acc, float* dk_acc, float* dv_acc,
                            void* scratch, size_t scratch_bytes, void* stream);

/*
 * fcp_attn_fwd_step_running -- one ring step fused with the running merge (no partial results, no
 * fcp_lse_merge): the alternative to the partial + merge pair, for a caller that runs the ring steps of
 * Sec. 3.2 one after the other.  (o_run, lse_run) hold the merged attention over the keys of the ring steps so
 * far; for every row of every work item of the call they are replaced by the merge with this step's keys:
 *   LSE' = ln(exp(LSE) + sum_j exp(s_j)),  O' = (exp(LSE - LSE') O + sum_j exp(s_j - LSE') V_j).
 * Inside the kernel the previous result simply is the initial state of the online softmax.
 *   o_run [tq,hq,D] fp32, lse_run [hq,tq] fp32 device, in/out.  Before the first step the caller sets lse_run
 *         to -inf (o_run of a row with lse_run = -inf is not read).  Rows that no item of the call covers are
 *         left as they are.
 *   o_out [tq,hq,D] bf16 device or NULL: the covered rows' O' rounded to bf16 as well (pass it in every call, or
 *         at least in the last call that covers a row: a row's last visit may come before the last ring step)
 *   q_limit: NULL (causal) or as in fcp_attn_fwd_step_mixed.  The items' `step` fields are ignored.
 * Two items of one call must not share a row (the steps of a ring never do); one call per ring step, in any
 * order, on one stream.  scratch as for fcp_attn_fwd_step with n_parts = 1.
 */
int fcp_attn_fwd_step_running(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                              int32_t n_seqs, const fcp_work_desc* work, int64_t n_work,
                              int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                              float softmax_scale, const int32_t* q_limit, float* o_run, float* lse_run,
                              void* o_out, void* scratch, size_t scratch_bytes, void* stream);

/* Cast n fp32 accumulator values to bf16, round to nearest even.  Device pointers. */
int fcp_grad_finalize(const float* acc, void* out_bf16, int64_t n, void* stream);

/*
 * fcp_attn_bwd_step_direct -- the whole backward of a rank in one call, final bf16 results without a pass over all
 * accumulators.  Same function as fcp_attn_bwd_step (mask as in fcp_attn_bwd_step_mixed when q_limit / k_from are
 * given, causal when both are NULL), for a work list that carries ALL ring steps (paper Sec. 3.2: a rank's dQ rows
 * and, after the ring has returned them, its dK/dV rows are the sums over the steps).  Most rows of a packed batch get
 * their whole result from one unit of work (every sequence that is not sharded, Sec. 4.1): the kernel that computes
 * such a row writes it as bf16 at once.  Per query row and per pool key:
 *   - no work item of the call touches it: the result is zero;
 *   - one work item owns it (no other item of the call covers the same query rows / key segment): written to
 *     dq_out / dk_out / dv_out directly, the fp32 accumulator row is neither read nor written;
 *   - otherwise: accumulated in fp32 in dq_acc / dk_acc / dv_acc (this call clears those rows first; the caller need
 *     not) with atomics.
 * fcp_grad_finalize_direct then completes the outputs: accumulated rows are converted (round to nearest even),
 * untouched rows zeroed, directly written rows left alone.  The row states stay in `scratch` between the two calls.
 *   dq_acc [tq,hq,D], dk_acc, dv_acc [tkv,hkv,D] fp32 device, contents on entry irrelevant, on exit defined only
 *   for the accumulated rows;  dq_out [tq,hq,D], dk_out, dv_out [tkv,hkv,D] bf16 device, complete after the finalize.
 * Limits: those of fcp_attn_bwd_step, and n_work <= 1024 (FCP_ERR_UNSUPPORTED beyond: use the accumulating call).
 * Other arguments, alignment and errors as in fcp_attn_bwd_step; scratch sized with FCP_SCRATCH_BWD.
 */
int fcp_attn_bwd_step_direct(const void* q, const void* k, const void* v, const void* d_o,
                             const float* lse, const float* delta, const int32_t* cu_seqlens_kv,
                             int32_t n_seqs, const fcp_work_desc* work, int64_t n_work,
                             int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                             float softmax_scale, const int32_t* q_limit, const int32_t* k_from,
                             float* dq_acc, float* dk_acc, float* dv_acc, void* dq_out, void* dk_out,
                             void* dv_out, void* scratch, size_t scratch_bytes, void* stream);

/* Second half of the direct backward: see fcp_attn_bwd_step_direct.  Same scratch, n_work, sizes and stream. */
int fcp_grad_finalize_direct(const float* dq_acc, const float* dk_acc, const float* dv_acc, void* dq_out,
                             void* dk_out, void* dv_out, void* scratch, int64_t n_work, int32_t tq,
                             int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim, void* stream);

/* Coefficients of the scheduler's time model (paper Eq. 8-9), all >= 0, in the caller's time unit. */
typedef struct fcp_cost_model {
  double alpha1;         /* attention compute per (1 + eta_k) |s_k|^2                         */
  double alpha2;         /* linear-layer compute per token                                     */
  double beta1;          /* constant compute overhead of a group                               */
  double alpha3_over_v;  /* KV exchange per token: alpha3 / v_p, one link speed for all groups */
  double beta2;          /* constant exchange overhead of a group with a ring (degree > 1)     */
} fcp_cost_model;

/*
 * fcp_plan_groups -- HOST ONLY.  The scheduler's two stages (paper Sec. 4.4) for one micro-batch:
 *  1. atomic sequence groups by best-fit decreasing: sequences in decreasing length (equal lengths in
 *     input order); each goes into the open group with the least remaining room that still holds it
 *     (the group opened first among equals), otherwise it opens a group of
 *     d_min = ceil(len / tokens_per_rank) ranks and d_min * tokens_per_rank tokens;
 *  2. the 2D dynamic programme of Eq. 11 / Alg. 1 over (groups, ranks): every group gets a degree
 *     d >= d_min, at most n_ranks in total (Cond. 6), so that the largest group time is least; among
 *     equal makespans the fewest ranks, and inside the recurrence the smallest degree, win.
 * Group time at degree d (Eq. 8-10; the compute terms divided by d, no exchange at d = 1, the exchange
 * hidden behind the attention compute as far as it goes):
 *   T_cpa = sum_k alpha1 (1 + eta_k) len_k^2 / d,   T_cp = T_cpa + sum_k alpha2 len_k / d + beta1,
 *   T_cm = d == 1 ? 0 : alpha3_over_v * sum_k len_k + beta2,   T = T_cp + T_cm - min(T_cpa, T_cm).
 * tokens_per_rank = (E - M_ms) / M_token of Cond. 3 / Eq. 7: a rank's activation budget in tokens.
 *   seq_lens [n_seqs] host, >= 1;  eta [n_seqs] host or NULL (all 0: causal masks), >= 0
 *   group_of_seq [n_seqs] out: group index (in order of opening) of every sequence
 *   n_groups out;  group_d_min, group_degree, group_base_rank: out arrays of at least n_seqs entries,
 *   the first n_groups are written; base ranks are the running sums of the degrees
 *   makespan out: the largest group time of the plan
 * A sequence of a group runs at the group's degree on ranks base .. base + degree - 1 (the paper's atomic
 * groups); cp_degree / base_rank for fcp_shard_plan follow from group_of_seq.
 * Returns FCP_ERR_CAPACITY if the minimum degrees do not fit n_ranks (n_groups and group_d_min are valid
 * then unless a single sequence alone needs more than n_ranks).
 */
int fcp_plan_groups(const int32_t* seq_lens, const float* eta, int32_t n_seqs, int32_t n_ranks,
                    int64_t tokens_per_rank, const fcp_cost_model* cm, int32_t* group_of_seq,
                    int32_t* n_groups, int32_t* group_d_min, int32_t* group_degree,
                    int32_t* group_base_rank, double* makespan);

/*
 * fcp_group_shard_args -- HOST ONLY.  The paper executes an atomic group as ONE CP group (Sec. 4.4): every
 * sequence packed into a group, short ones included, is split over the group's degree.  Turns the result of
 * fcp_plan_groups into the per-sequence arguments of fcp_shard_plan:
 *   cp_degree[k] = group_degree[group_of_seq[k]],  base_rank[k] = group_base_rank[group_of_seq[k]].
 * (fcp_shard_plan itself takes any per-sequence degrees, e.g. short sequences of a group left at degree 1.)
 *   group_of_seq [n_seqs], group_degree, group_base_rank [n_groups] host in; cp_degree, base_rank [n_seqs] host out.
 */
int fcp_group_shard_args(const int32_t* group_of_seq, int32_t n_seqs, const int32_t* group_degree,
                         const int32_t* group_base_rank, int32_t n_groups, int32_t* cp_degree,
                         int32_t* base_rank);

/*
 * Reads back what the last fwd/bwd step that used `scratch` recorded: the number of
 * scheduled tiles and the number of rejected work items.  Synchronises `stream`.
 * Either output pointer (host) may be NULL.
 */
int fcp_scratch_status(const void* scratch, void* stream, int32_t* n_tiles, int32_t* n_rejected);

#ifdef __cplusplus
}
#endif
#endif /* FCP_H_ */
