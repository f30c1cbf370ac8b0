/* dssd_aux.h - what sits beside the verification step of dssd.h without being part of the
 * method: tuning knobs of the launch strategy, a kernel-timing aid, and two checking aids.
 * Same conventions as dssd.h (C ABI, device pointers owned by the caller, status codes).
 */
#ifndef DSSD_AUX_H
#define DSSD_AUX_H

#include "dssd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- tuning knobs (per context; defaults suit MI355X) ---- */

/* Largest batch, counted as B * ceil((gamma+1) * chunks_per_row / 4), that dssd_step_fused runs
 * as a single launch (default 512: beyond it the streaming kernels were measured faster on
 * MI355X); 0 disables the single-launch path; a negative value sets the limit to its magnitude
 * and lifts the row-length rule (for tests and measurements). */
dssd_status dssd_set_fused_limit(dssd_ctx *ctx, int64_t max_blocks);
/* Blocks of DSSD_FLAG_EARLY_EXIT: begin[0..n) are the first rows of the blocks, strictly
 * increasing from begin[0] = 0, the last block open-ended; n in [2, 8] (one block would be the
 * default path).  n = 0 returns to the automatic choice by batch size. */
dssd_status dssd_set_early_exit_schedule(dssd_ctx *ctx, const int32_t *begin, int32_t n);
/* Largest batch (counted the same way, default 512) that dssd_step_fused runs as two launches
 * when the single-launch rule does not apply; 0 disables the two-launch path.  Negative values
 * are DSSD_EINVAL. */
dssd_status dssd_set_fused_pair_limit(dssd_ctx *ctx, int64_t max_blocks);

/* Waves per compute unit that the two streaming kernels (row statistics; residual masses) keep
 * resident: read throughput on this chip peaks at a moderate number of bytes in flight per unit
 * and loses several percent towards full occupancy, so the library caps them (by requesting LDS
 * the kernels never touch).  0 = no cap (whatever the registers allow).  Values are rounded
 * down to whole workgroups (two waves for the statistics, four for the residual masses), never
 * below two workgroups per unit.  Until this is called the statistics run at 12 waves per unit
 * for bf16 logits and 10 for fp32, the residual masses at 12 and 16 (the best settings measured
 * on MI355X over batches from 160 MB to 5 GB of logits). */
dssd_status dssd_set_stream_occupancy(dssd_ctx *ctx, int32_t stats_waves_per_cu, int32_t resid_waves_per_cu);

/* ---- kernel timing ---- */

/* Bit k of kernel_mask brackets every launch of kernel k with a pair of HIP events on the launch
 * stream (0 = off).  Each bracket costs a few microseconds of queue time, so time only the
 * kernels a measurement needs.  The events come from a pool of 2048 pairs per kernel that
 * dssd_profile_enable creates the first time a kernel is asked for (the only call here that
 * creates anything; the hot calls never do): launches beyond the pool go untimed until
 * dssd_profile_reset, and dssd_profile_read then returns DSSD_ENOMEM with the figures of the
 * launches that were timed.  A stream that is being captured into a graph is not bracketed.  If
 * an event cannot be recorded the hot call returns DSSD_EHIP.  Kernel ids: 0 row softmax statistics,
 * 1 accept / first-reject, 2 residual chunk masses (for small batches also the pick, in one
 * launch), 3 residual pick, 4 bonus pick, 5 export of P rows, 6 and 7 chunk masses and pick of
 * the device-side redraw, 8 the single-launch step of dssd_step_fused, 9 the read probe, 10 row statistics of an early-exit
 * block, 11 the step on top-k lists. */
enum { DSSD_K_ROW_STATS = 0, DSSD_K_ACCEPT = 1, DSSD_K_RESID_MASS = 2, DSSD_K_RESID_PICK = 3,
       DSSD_K_BONUS_PICK = 4, DSSD_K_EXPORT_P = 5, DSSD_K_DEVICE_MASS = 6, DSSD_K_DEVICE_PICK = 7,
       DSSD_K_FUSED_STEP = 8, DSSD_K_READ_PROBE = 9, DSSD_K_ROW_STATS_BLOCK = 10, DSSD_K_TOPK_STEP = 11,
       DSSD_K_COUNT = 12 };
dssd_status dssd_profile_enable(dssd_ctx *ctx, uint32_t kernel_mask);
/* Synchronises the recorded events, returns the summed duration (ms) and number of timed
 * launches of one kernel since the last reset. */
dssd_status dssd_profile_read(dssd_ctx *ctx, int kernel_id, double *total_ms, int64_t *launches);
dssd_status dssd_profile_reset(dssd_ctx *ctx);
const char *dssd_kernel_name(int kernel_id);

/* Measurement aid: read `bytes` (rounded down to whole waves' shares) of device memory at `buf`
 * (16-byte aligned) the way the row-statistics kernel reads, with no arithmetic: one wave per
 * loads_per_lane KiB (1, 2, 4 or 8 non-temporal 128-bit loads per lane, all in flight), at most
 * waves_per_cu waves resident per compute unit (0 = no cap; rounded as in
 * dssd_set_stream_occupancy).  The best rate over these settings is the read ceiling that kernel
 * can be held against on the chip at hand. */
dssd_status dssd_probe_read(dssd_ctx *ctx, const void *buf, size_t bytes, int32_t loads_per_lane,
                            int32_t waves_per_cu, void *hip_stream);

/* ---- checking aids ---- */

/* The Philox4x32-10 blocks the step draws from, for the rectangle of sessions
 * [session_first, +n_sessions) x positions [position_first, +n_positions) (32-bit wrap-around),
 * counter = (session_base + b, position, step low, step high), key = (seed low, seed high).
 * words (device, 4-byte aligned) receives n_sessions * n_positions * 4 uint32: word 0 feeds the
 * accept test r_j of Algorithm 2, word 1 the redraw, word 2 the bonus draw, word 3 is unused. */
dssd_status dssd_random_words(dssd_ctx *ctx, uint64_t seed, uint64_t step, uint32_t session_first,
                              uint32_t position_first, int32_t n_sessions, int32_t n_positions,
                              uint32_t *words, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DSSD_AUX_H */
