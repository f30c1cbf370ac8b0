/* dssd.h - C ABI of the batched speculative-decoding verification step of DSSD
 * (Distributed Split Speculative Decoding, arXiv 2507.12000) for AMD MI355X (gfx950).
 *
 * The paper cuts one verification round in two (Sec. 3, Algorithm 2):
 *   edge   : accept/reject every draft token against the target model's distributions and,
 *            if all are accepted, draw the bonus token           -> dssd_verify_batch,
 *                                                                   dssd_bonus_sample
 *   device : if a draft was rejected at position j, redraw it from
 *            norm(max(0, P_j - Q_j))                             -> dssd_residual_sample
 * Running the three calls back to back on one GPU is the unsplit scheme (Sec. 2.1, Algorithm 1).
 *
 * Conventions
 *   - Every pointer inside dssd_batch / dssd_out is a DEVICE pointer owned by the caller; the
 *     library never frees or reallocates it.  The structs themselves live in HOST memory and
 *     are read during the call only.
 *   - All three hot calls are asynchronous on `hip_stream` (a hipStream_t, NULL = default
 *     stream); they never synchronise, never allocate and never touch host copies of the data.
 *   - dssd_residual_sample and dssd_bonus_sample must follow dssd_verify_batch for the same
 *     batch on the same context and stream: they act on the per-session record (row to draw
 *     from, its softmax statistics) that verify left in the context's workspace, not on the
 *     caller's copies of accepted_len / rejected.
 *   - One context serves one stream at a time (its workspace is shared by consecutive calls).
 *     A context belongs to the device it was created on: that device must be the current one
 *     when its calls are made (dssd_create itself leaves the caller's current device as it was).
 *   - Positions are 0-based: accepted_len = j - 1 in the paper's numbering.
 *   - Host-checkable errors return a negative status before anything is launched.  Errors that
 *     only the device can see (token id outside [0,V), inconsistent offsets, a logits row whose
 *     softmax is not finite) set status[b] and give that session accepted_len = 0,
 *     rejected = 1, out_token = -1; the samplers skip it.  A bad token or row counts where the
 *     loop of Algorithm 2 looks ("while j <= gamma and Flag = 1"): at positions and rows up to
 *     the first rejected draft (whose row feeds the redraw), and at the bonus row when every
 *     draft is accepted.  What lies after the first rejection is never looked at, so a fault
 *     there changes nothing, on any entry point and in any mode.
 */
#ifndef DSSD_H
#define DSSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dssd_ctx dssd_ctx; /* opaque: device workspace, settings, timing events */

typedef enum { DSSD_F32 = 0, DSSD_BF16 = 1, DSSD_F16 = 2 /* IEEE binary16: downlink P rows only */ } dssd_dtype;

typedef enum {
  DSSD_OK = 0,
  DSSD_EINVAL = -1,       /* NULL required pointer, negative size, unknown dtype        */
  DSSD_EALIGN = -2,       /* a pointer is not aligned to its element size                */
  DSSD_ENOMEM = -3,       /* batch larger than the context's workspace / allocation failed */
  DSSD_EHIP = -4,         /* a HIP runtime call failed                                   */
  DSSD_EUNSUPPORTED = -5
} dssd_status;

/* Per-session bits written to dssd_out.status (device side). */
enum {
  DSSD_SESSION_BAD_TOKEN = 1,    /* a draft token outside [0, V)                          */
  DSSD_SESSION_ZERO_RESIDUAL = 2,/* residual mass rounded to 0: token drawn from P_j       */
  DSSD_SESSION_BAD_OFFSETS = 4,  /* draft_offsets not monotone or beyond total_drafts      */
  DSSD_SESSION_BAD_ROW = 8,      /* a softmax sum or maximum that is not finite/positive,
                                    or an inverse temperature that is not finite/positive  */
  DSSD_SESSION_SUPPORT_OVERFLOW = 16 /* DSSD_FLAG_SPARSE_SUPPORT was set but the row to draw
                                    from has more than DSSD_MAX_SUPPORT finite logits        */
};

/* dssd_batch.flags */
enum {
  /* The caller promises that every logits row has at most DSSD_MAX_SUPPORT entries above -inf,
   * e.g. after top-k filtering upstream (the paper's experiments sample with k = 10; Sec. 4).
   * verify then also records each row's support while it streams the row, and the two samplers
   * draw from those few entries instead of passing over the vocabulary again.  Same results as
   * without the flag up to summation order. */
  DSSD_FLAG_SPARSE_SUPPORT = 1,
  /* Early exit: the caller allows the library to take the loop of Algorithm 2 ("while j <=
   * gamma and Flag = 1") at its word and read a session's logits rows only about as far as its
   * first rejected draft.  The rows are visited in rounds of growing blocks (by default [0,2),
   * [2,6), the rest; two blocks [0,3), the rest for smaller batches; none where the extra
   * launches are expected to cost more than the unread rows save: the choice prices unread rows at
   * a per-position acceptance of 0.8 against 140 MB of streaming per extra round, figures tuned
   * on MI355X; dssd_set_early_exit_schedule of dssd_aux.h overrides it), and a session leaves as
   * soon as a block holds its first rejection or its bonus row.  accepted_len, rejected and out_token are bit-identical to the default path,
   * and so are row_stats, p_tok and q_tok for the rows and positions of the blocks that were
   * visited; entries of later blocks are NaN.  Honoured by dssd_verify_batch and
   * dssd_step_fused; combines with DSSD_FLAG_SPARSE_SUPPORT. */
  DSSD_FLAG_EARLY_EXIT = 2
};
#define DSSD_MAX_SUPPORT 64

/* Input of one verification step for B sessions (Sec. 2.1 "Verification Process";
 * Algorithm 2, inputs of the edge: tokens x_1..x_gamma, values q_j(x_j), and P_1..P_{gamma+1}).
 *
 * Session b owns draft rows [off_b, off_b + gamma_b) and logits rows
 * [off_b + b, off_b + b + gamma_b]  (gamma_b + 1 of them), where off_b = draft_offsets[b]
 * and gamma_b = draft_offsets[b+1] - draft_offsets[b], or off_b = b*gamma, gamma_b = gamma
 * when draft_offsets is NULL.  R_Q = total_drafts rows of drafts, R_L = R_Q + B rows of logits.
 */
typedef struct {
  int32_t B;                    /* sessions; 0 is a no-op                                          */
  int32_t V;                    /* vocabulary size |V|, >= 1                                       */
  int32_t gamma;                /* drafts per session when draft_offsets == NULL, >= 0             */
  int32_t logits_dtype;         /* dssd_dtype of `logits`                                          */
  int64_t total_drafts;         /* R_Q = sum of gamma_b (must equal B*gamma when offsets == NULL)  */
  const int32_t *draft_offsets; /* [B+1] prefix sums of gamma_b, or NULL for uniform gamma         */
  const void *logits;           /* [R_L, V] row-major contiguous target logits, fp32 or bf16       */
  const float *draft_probs;     /* [R_Q, V] row-major fp32 draft distributions Q_i, each row
                                   already a probability vector; used as given.  May be NULL for
                                   dssd_verify_batch / dssd_bonus_sample / dssd_export_p_rows when
                                   draft_q_tok is given (the edge of DSSD never sees Q rows)       */
  const int32_t *draft_tokens;  /* [R_Q] draft token ids x_i in [0, V)                             */
  const float *inv_temperature; /* [B] 1/T_b > 0 multiplying the target logits before the softmax,
                                   or NULL for T = 1 (the paper's setting)                         */
  uint64_t seed;                /* Philox4x32-10 key (lo, hi)                                      */
  uint64_t step;                /* verify-step number; Philox counter = (session_base + b,
                                   position, step lo, step hi).  Word 0 of the block drives the
                                   accept test at that position, word 1 the residual draw at that
                                   position, word 2 the bonus draw (position gamma_b)              */
  uint32_t session_base;        /* global id of session 0 (keeps results independent of sharding)  */
  uint32_t flags;               /* DSSD_FLAG_* bits, 0 for none                                    */
  const float *draft_q_tok;     /* [R_Q] or NULL: the scalars q_i(x_i) that DSSD uploads with the
                                   tokens (Sec. 3 "Uplink Transmission"); read only when
                                   draft_probs is NULL                                             */
  const uint64_t *step_counter; /* device, 8-byte aligned, or NULL: a counter read by the kernels
                                   when they run and ADDED to `step` (64-bit wrap).  For callers
                                   that record the calls into a HIP graph: `step` is frozen into
                                   the graph, this is not, so bumping it between replays gives
                                   every replay fresh random numbers.  It must not change while
                                   the calls of one step are in flight                             */
} dssd_batch;

/* Output of one step: the paper's (x_j, j) record per session plus what the samplers and the
 * parity checks need.  Required: accepted_len, rejected, out_token.  Optional (may be NULL):
 * row_stats, p_tok, q_tok, status.
 */
typedef struct {
  int32_t *accepted_len; /* [B] n_b in [0, gamma_b]: number of accepted drafts (j - 1)             */
  int32_t *rejected;     /* [B] 1 iff n_b < gamma_b (Flag = 0; the indicator `a` of Sec. 3.1)      */
  int32_t *out_token;    /* [B] redrawn token (rejected) or bonus token (all accepted)             */
  float *row_stats;      /* [R_L, 2]: (m, Z) with m = max_v z_v/T, Z = sum_v exp(z_v/T - m), so
                            P(v) = exp(z_v/T - m)/Z                                                */
  float *p_tok;          /* [R_Q] p_i(x_i) for every draft position                                */
  float *q_tok;          /* [R_Q] q_i(x_i): the scalars DSSD uploads instead of the Q rows         */
  int32_t *status;       /* [B] DSSD_SESSION_* bits, 0 when fine                                   */
} dssd_out;

/* Bytes of device workspace a context needs for up to max_rows logits rows of max_V entries. */
size_t dssd_workspace_bytes(int64_t max_rows, int32_t max_V, int32_t logits_dtype);

/* Create a context on HIP device `device`, with workspace for batches of up to max_rows logits
 * rows (R_L) and vocabularies up to max_V, for either logits dtype.  The only call that
 * allocates device memory.  Fails with DSSD_EHIP when no usable GPU is present. */
dssd_status dssd_create(dssd_ctx **ctx, int device, int64_t max_rows, int32_t max_V);
void dssd_destroy(dssd_ctx *ctx);

/* Edge side, Algorithm 2 "Verification Process": softmax statistics of all R_L logits rows
 * (each row is read from memory once), then per draft position
 *   accept_i  <=>  r_i * q_i(x_i) < p_i(x_i)     (r_i < min(1, p/q), r_i in [0,1))
 * and n_b = index of the first rejected draft, or gamma_b.  Writes accepted_len, rejected and
 * the optional outputs.  out_token is written only for sessions with a device-side error. */
dssd_status dssd_verify_batch(dssd_ctx *ctx, const dssd_batch *batch, dssd_out *out, void *hip_stream);

/* Device side, Algorithm 2 "Resample" (Algorithm 1 "Reject and Resample"): for every session
 * with rejected = 1, out_token = x ~ norm(max(0, P_n - Q_n)) at n = accepted_len, by inverse
 * CDF in vocabulary order with r = word 1 of the position-n block: the smallest k whose
 * inclusive prefix sum exceeds r * R, R the residual mass.  Other sessions are untouched. */
dssd_status dssd_residual_sample(dssd_ctx *ctx, const dssd_batch *batch, dssd_out *out, void *hip_stream);

/* Edge side, Algorithm 2: for every session with rejected = 0, out_token = x ~ P_{gamma_b+1}
 * (the last logits row of the session) by the same inverse-CDF rule with r = word 2 of the
 * position-gamma_b block.  Other sessions are untouched. */
dssd_status dssd_bonus_sample(dssd_ctx *ctx, const dssd_batch *batch, dssd_out *out, void *hip_stream);

/* The whole step in one call, as in Algorithm 1 where the edge does all of it: equivalent to
 * dssd_verify_batch, dssd_residual_sample, dssd_bonus_sample in a row on the same stream, with
 * bit-identical outputs.  Batches with uniform gamma (draft_offsets == NULL) that are small
 * (B * ceil((gamma+1) * chunks_per_row / 4) <= 512 unless dssd_set_fused_limit of dssd_aux.h says
 * otherwise; a chunk is 8 KiB of logits) and whose rows are short (V * (logit bytes + 4) <= 384
 * KiB: what one workgroup streams quickly when it finishes a session alone) run as ONE kernel
 * launch, which is what matters when a step is bound by launch latency rather than bandwidth;
 * small batches with longer rows run as TWO launches (statistics + accept + bonus, then the
 * redraw of rejected sessions); all others run the kernels of the three calls, with the bonus
 * draw folded into the accept launch when the rows are dense (one launch fewer).  Needs the full
 * Q rows (draft_probs). */
dssd_status dssd_step_fused(dssd_ctx *ctx, const dssd_batch *batch, dssd_out *out, void *hip_stream);
/* The whole step for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs and bit-identical
 * results as dssd_step_fused, but it takes no context: the workspace (chunk statistics, chunk
 * masses, per-session job records, arrival counters) is a static device array of
 * DSSD_STATIC_SCRATCH_BYTES that is part of the library's code object, so every GPU the library
 * runs on holds it until the process ends.  The call allocates and frees nothing, on the host or
 * on the device, and does not synchronise.
 *   - The current HIP device must be the one `hip_stream` and every buffer belong to.
 *   - A batch needs 8 bytes per chunk of every logits row (a chunk is 8 KiB of logits: 4096 bf16
 *     or 2048 fp32 entries) plus about 48 bytes per session and 4 bytes per session and chunk;
 *     one that needs more than DSSD_STATIC_SCRATCH_BYTES is refused with DSSD_ENOMEM before
 *     anything is launched (the five benchmark workloads fit: the largest, 9 705 bf16 rows of
 *     256 000 entries, takes 5.2 MB).
 *   - batch->flags must be 0 (DSSD_EUNSUPPORTED otherwise: both modes keep lists elsewhere).
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU
 *     (different streams or threads) race.  Calls in stream order on one stream are fine; the
 *     array keeps the last call's contents and the call clears what it needs cleared.
 *   - The first call on a device looks the array's address up (no allocation); dssd_create on
 *     that device does it too, so either may come first. */
#define DSSD_STATIC_SCRATCH_BYTES (8u << 20)
dssd_status dssd_step_static(const dssd_batch *batch, dssd_out *out, void *hip_stream);

/* Edge side, Algorithm 2 "Downlink Transmission": after dssd_verify_batch, for every session
 * with rejected = 1 write the distribution at the rejected position, P_n(v) for v in [0, V), into
 * p_rows[b*V + v] as b_prob-bit values: p_dtype = DSSD_F32 (b_prob = 32) or DSSD_F16 (b_prob = 16,
 * round to nearest even from the fp32 value).  p_rows is a device buffer of B*V values owned by
 * the caller; rows of sessions that were not rejected are left untouched. */
dssd_status dssd_export_p_rows(dssd_ctx *ctx, const dssd_batch *batch, void *p_rows, int32_t p_dtype,
                               void *hip_stream);

/* What the device of DSSD holds when it redraws (Sec. 3 "Verification Process (on Device)"): its
 * own Q rows, the received j (accepted_len = j - 1, rejected) and the received P_j rows.  All
 * pointers are device pointers owned by the caller; layout of sessions as in dssd_batch. */
typedef struct {
  int32_t B, V, gamma;          /* as in dssd_batch                                                 */
  int32_t p_dtype;              /* DSSD_F32 or DSSD_F16: type of p_rows                             */
  int64_t total_drafts;         /* R_Q                                                              */
  const int32_t *draft_offsets; /* [B+1] or NULL                                                    */
  const float *draft_probs;     /* [R_Q, V] fp32 Q rows                                             */
  const void *p_rows;           /* [B, V] received P_n of session b (read for rejected sessions)    */
  const int32_t *accepted_len;  /* [B] received n_b                                                 */
  const int32_t *rejected;      /* [B] received flag                                                */
  uint64_t seed, step;          /* same Philox key / step as the edge used                          */
  uint32_t session_base, reserved;
  int32_t *out_token;           /* [B] written for rejected sessions only                           */
  int32_t *status;              /* [B] or NULL: DSSD_SESSION_* bits (written for rejected sessions) */
  const uint64_t *step_counter; /* device or NULL: as in dssd_batch                                 */
} dssd_device_batch;

/* Device side, Algorithm 2 "Resample" from what crossed the link: for every rejected session,
 * out_token = x ~ norm(max(0, P~_n - Q_n)) with P~_n the received row, same inverse-CDF rule and
 * the same random word (word 1 of the position-n block) as dssd_residual_sample.  Needs a context
 * (for its workspace) but no preceding verify call on it.  A record with n_b outside [0, gamma_b)
 * sets DSSD_SESSION_BAD_OFFSETS and out_token = -1. */
dssd_status dssd_residual_sample_from_p(dssd_ctx *ctx, const dssd_device_batch *batch, void *hip_stream);

const char *dssd_status_str(dssd_status s);

/* The step on top-k lists (the paper's experiments sample with top-k = 10, Sec. 4): both models'
 * rows arrive as k (token id, value) pairs instead of V values.  It computes what the dense step
 * computes on rows that are -inf (target logits) / 0 (draft probabilities) outside the lists:
 * P_i = softmax of the k listed logits times 1/T, accept iff r*q < p with p, q = 0 for a token
 * outside the respective list, redraw from norm(max(0, P_n - Q_n)) (its support lies inside the
 * target's list) or bonus token from P_gamma, both by inverse CDF in vocabulary order, the same
 * Philox blocks.  One launch; rows after a session's first rejection are not used (at most four
 * are fetched ahead), and their row_stats / p_tok / q_tok entries are NaN.  Ids within one list must be distinct; -1 marks an
 * unused entry; the lists need not be sorted.  Layout of sessions, rows and outputs as in
 * dssd_batch / dssd_out.  All pointers are device pointers, 4-byte aligned. */
typedef struct {
  int32_t B, k, gamma, V;       /* k in [1, 64] entries per list; V > 0 range-checks the draft
                                   tokens, V = 0 does not                                          */
  int64_t total_drafts;         /* R_Q                                                             */
  const int32_t *draft_offsets; /* [B+1] or NULL                                                   */
  const int32_t *p_idx;         /* [R_L, k] token ids of the target's list                         */
  const float *p_logit;         /* [R_L, k] their logits                                           */
  const int32_t *q_idx;         /* [R_Q, k] token ids of the draft's list                          */
  const float *q_prob;          /* [R_Q, k] their probabilities, as the draft sampled from them    */
  const int32_t *draft_tokens;  /* [R_Q]                                                           */
  const float *inv_temperature; /* [B] or NULL                                                     */
  uint64_t seed, step;
  uint32_t session_base, reserved;
  const uint64_t *step_counter; /* device or NULL: as in dssd_batch                                */
} dssd_topk_batch;
dssd_status dssd_step_topk(dssd_ctx *ctx, const dssd_topk_batch *batch, dssd_out *out, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DSSD_H */
