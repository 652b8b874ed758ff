/*
 * asd_testing.h -- hooks of libasd.so for its tests and for profiling.  Not part of the
 * sampling boundary (that is asd.h): raw generator output for bit-exact comparison with an
 * independent implementation of the counter-based generator of Alg. 1's u_{1:K}, xi_{1:K},
 * per-kernel event timing, and queries of which code path a context takes.
 */
#ifndef ASD_TESTING_H
#define ASD_TESTING_H

#include "asd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* 1 if the next asd_sample on this context runs whole chains inside one workgroup (shape fits, switch on,
 * profiling off). */
ASD_API int32_t asd_resident_active(const asd_ctx* ctx);
/* Non-zero if the verify call of this context runs the split-operand kernels of the Gaussian-mixture denoiser: the
 * number of 16-bit matrix-core products they spend on one fp32 product -- 3 (two fp16 terms per operand: d and C
 * multiples of 32, both model calls) or 6 (three bf16 terms: multiples of 16, the verify call only). */
ASD_API int32_t asd_split_gemm_active(const asd_ctx* ctx);

/* The second GEMM of the split-operand mixture denoiser (softmax weights times means) skips the stretches of
 * components whose weights are exactly 0.0f for every row of a tile (the denoiser takes a weight below 2^-40 of its
 * row's largest as zero -- that moves a result by less than 2 C 2^-40 of the largest |mean| -- and once a posterior
 * has narrowed most are).  The skipped products are zeros, so results are identical bit for bit; on = 0 makes
 * the kernel visit every component anyway (for tests and timing comparisons).  Default: on.  The same switch covers
 * the closed form for rows with a single non-zero weight (asd_profile_model_work). */
ASD_API asd_status asd_use_sparse_combine(asd_ctx* ctx, int32_t on);

/* Screening of the verify call's first GEMM in the split-operand mixture denoiser: an int8 GEMM with a
 * rigorous error bound finds the tiles of logits (128 components x 128 rows, or 64 rows: the halves of a row tile
 * are judged separately) that lie so far below their rows' maxima that every softmax weight in them is exactly 0.0f,
 * and the exact GEMM leaves those tiles out.  Results are identical bit for bit.  While it is on and L is a multiple
 * of 64, the verify call's row plan starts every chain's rows at a multiple of 64 rows (filling up with repeats of
 * the chain's last row), so that a row tile holds rows of two chains.  mode 0: off; 1 (default): a verify call is screened when the draft call before it found its rows'
 * posteriors collapsed; 2: every verify call is screened.  Needs the second GEMM's skipping
 * (asd_use_sparse_combine) switched on, d a multiple of 128 (at most 2048) and C a multiple of 256; otherwise it
 * stays off.
 * asd_logit_screen_active: the mode in force (0 when the shape or the other switches rule it out). */
ASD_API asd_status asd_use_logit_screen(asd_ctx* ctx, int32_t mode);
ASD_API int32_t asd_logit_screen_active(const asd_ctx* ctx);

/* One-hot certificate of the screened verify call (split-operand mixture denoiser).  Before any matrix work, a row
 * tile (128 rows) whose rows all lie so close to the mean their chain's last draft-call row was found one-hot on
 * that the distance from that mean to its nearest neighbour alone proves every other softmax weight exactly 0.0f
 * (Cauchy-Schwarz on x - s mu_b; one float per component, made at asd_init) is written in closed form,
 * c_x' x + c_m' mu_b, and skips the screening pass and both GEMMs.  Results are identical bit for bit: it certifies
 * what the exact path would have found.  Works inside asd_sample and the stage calls (the row plan names every row's
 * chain), not in asd_denoise.  Default: on; needs the screening pass (asd_logit_screen_active != 0) and at most 64
 * groups of 64 components (C <= 4096); otherwise it stays off.
 * asd_onehot_certificate_active: 1 if the verify calls of this context run it. */
ASD_API asd_status asd_use_onehot_certificate(asd_ctx* ctx, int32_t on);
ASD_API int32_t asd_onehot_certificate_active(const asd_ctx* ctx);

/* Verify calls of the split-operand mixture denoiser on fp16 terms whose every tile is wanted -- calls that are not
 * screened, by the draft call's verdict or at all -- run their two GEMMs on 256 x 256 tiles (eight wavefronts of
 * 128 x 64, fragments streamed one plane pair at a time) when the context has at least 16384 model rows per call
 * (chains * L); otherwise, and for every other launch, on 128 x 128 tiles.  The same terms are added in the same order
 * per output element: results are identical bit for bit.  on = 0 keeps every launch on the small tiles (for tests and
 * timing comparisons).  Default: on.  asd_tall_tiles_active: 1 if this context's dense verify calls take them. */
ASD_API asd_status asd_use_tall_tiles(asd_ctx* ctx, int32_t on);
ASD_API int32_t asd_tall_tiles_active(const asd_ctx* ctx);

/* Early accept (inside asd_sample and asd_sample_noalloc; mixture denoiser with the one-hot certificate on fp16
 * terms, d a multiple of 4 and at most 1024, more than 16384 model rows per call, no model-call reuse).  A certified
 * row's model value is c_x' x + c_m' mu_b, which the accept stage can form itself, and a drafted row is a recurrence
 * on the row before it.  So after the draft call one kernel takes every chain it can through its whole round: it
 * drafts a slot from the slot before it in registers, certifies it, forms its model value and takes the accept test,
 * stopping at the first rejection like the accept stage proper; only the rows the chain keeps go to the trajectory.
 * Chains with a slot it cannot certify are left as they were and go through the draft kernel, the verify call and the
 * accept kernel, which then take those chains only.  A chain's round is the same either way, bit for bit: the same
 * sums in the same order on the same values.  Late in a sample, when every row is certifiable, a round then writes
 * the dozen rows per chain it keeps, instead of writing the whole window, reading it, writing its model values and
 * reading a third of those back.  Once a round has left no chain to the kernels behind it, the rounds that follow are
 * this kernel alone -- it then certifies y_a as well and forms the draft call's model value itself -- until one reports
 * a chain it could not take; that chain has not moved and is taken up by the next full round.  Default: on.  asd_early_accept_active: 1 if asd_sample of
 * this context does it.
 * asd_profile_early_accept (while asd_profile_enable is on): model rows the kernel formed itself, chain-rounds it
 * committed, the rows of their windows (slots 1 .. w - 1) and the rows it resampled since then.  asd_profile_rows
 * counts those window rows among the verify rows all the same, so that figure stays the number of rows Alg. 1
 * verifies; asd_profile_accept_rows likewise covers both accept kernels. */
ASD_API asd_status asd_use_early_accept(asd_ctx* ctx, int32_t on);
ASD_API int32_t asd_early_accept_active(const asd_ctx* ctx);
ASD_API asd_status asd_profile_early_accept(asd_ctx* ctx, int64_t* model_rows, int64_t* chain_rounds, int64_t* window_rows,
                                            int64_t* resampled_rows);

/* Raw generator output: out DEV uint32 [nblk, 4] = Philox4x32-10 words for
 * counters (blk, step, chain, stream_id), blk = 0..nblk-1, key = seed. */
ASD_API asd_status asd_debug_philox(uint64_t seed, uint32_t chain, uint32_t step, uint32_t stream_id,
                            int32_t nblk, uint32_t* out, void* stream);
/* xi DEV fp32 [d] = the normals of (chain, step); u DEV fp32 [1] = the uniform. */
ASD_API asd_status asd_debug_randoms(uint64_t seed, uint32_t chain, uint32_t step, int32_t d,
                             float* xi, float* u, void* stream);

/* ---- per-kernel timing -------------------------------------------------------
 * When enabled, every kernel launch of the sampling path is bracketed by HIP
 * events on its own stream.  asd_profile_read synchronises the device and
 * returns, for one kernel kind within one of the two model calls (call = 0:
 * the draft call on one row per chain, call = 1: the batched verify call;
 * kinds that belong to no model call use call = 0), the number of launches
 * and their summed duration since the last asd_profile_enable(ctx, on).
 * on = 1 times the kernels of the denoisers and the draft and accept kernels; on = 2 also the scopes around
 * them (ASD_PROF_MODEL: a whole model call) and the row planning (ASD_PROF_PLAN) -- every scope costs two
 * events on the stream, a few microseconds each, which shows in a round of a millisecond.
 * asd_profile_rows returns the number of live rows (rows inside a window of an
 * unfinished chain) the two model calls were asked to evaluate since then. */
typedef enum {
  ASD_PROF_MODEL = 0,        /* a whole model call (all its kernels)          */
  ASD_PROF_PLAN = 1,         /* row planning                                  */
  ASD_PROF_GMM_ROWWISE = 2,  /* GMM denoiser, one wavefront per row           */
  ASD_PROF_GMM_LOGITS = 3,   /* GMM logits GEMM  X M^T (+ the rows' fp16 scales) */
  ASD_PROF_GMM_SOFTMAX = 4,  /* GMM, between the two GEMMs: row maxima, one-hot rows */
  ASD_PROF_GMM_COMBINE = 5,  /* GMM  P M  GEMM + affine combination           */
  ASD_PROF_MLP_PACK = 6,     /* MLP input packing (bf16 x ; time embedding)   */
  ASD_PROF_MLP_GEMM_IN = 7,  /* MLP first layer                               */
  ASD_PROF_MLP_GEMM_BLK = 8, /* MLP residual blocks (one launch per block)    */
  ASD_PROF_MLP_GEMM_OUT = 9, /* MLP output layer                              */
  ASD_PROF_DRAFT = 10,       /* fused draft kernel                            */
  ASD_PROF_ACCEPT = 11,      /* fused accept / scan / resample kernel         */
  ASD_PROF_GMM_SCREEN = 12,  /* GMM screening pass of the verify call's logits */
  ASD_PROF_GMM_CERT = 13,    /* GMM one-hot certificate (rows it passes are written by it) */
  ASD_PROF_ACCEPT_EARLY = 14, /* accept stage of certified chains, ahead of the verify call (asd_use_early_accept) */
  ASD_PROF_KINDS = 16
} asd_prof_kernel;
ASD_API asd_status asd_profile_enable(asd_ctx* ctx, int32_t on);
/* Which scopes are timed while timing is enabled: bit (kernel + 16 * call) of `slots` (all by default).  An event
 * on the stream ends the overlap of the kernels on either side of it and costs a few microseconds itself -- at two
 * thousand scopes per sample of the largest workload, a tenth of the sample -- so a caller that wants the durations
 * of one kernel selects it alone.  The counters of rows and of executed work run either way.  Takes effect with the
 * next launch and lasts until changed. */
ASD_API asd_status asd_profile_select(asd_ctx* ctx, uint32_t slots);
ASD_API asd_status asd_profile_read(asd_ctx* ctx, int32_t kernel, int32_t call, int64_t* launches, double* total_ms);
ASD_API asd_status asd_profile_rows(asd_ctx* ctx, int64_t* draft_rows, int64_t* verify_rows);
/* What the accept kernel touched since then: x0hat rows it read for the accept test (it examines a window eight
 * slots at a time and stops at the group that holds the first rejection) and rows it resampled (one per
 * chain-round that ended in a rejection). */
ASD_API asd_status asd_profile_accept_rows(asd_ctx* ctx, int64_t* examined_rows, int64_t* resampled_rows);
/* Matrix work the mixture denoiser's verify calls left out since then (split-operand kernels only; all zero
 * otherwise).  logit_tiles_done / logit_tiles: half tiles (64 rows x 128 components) of logits the first GEMM computed
 * and how many there were, over the calls that went through the screening pass (asd_use_logit_screen; a call it was switched off for by
 * the draft call's verdict counts all its tiles as done).  combine_slabs_done / combine_slabs: K slabs (32 components
 * with fp16 terms, 16 with bf16 terms: asd_split_gemm_active) the second GEMM's workgroups visited and how many there
 * were (asd_use_sparse_combine).
 * (Workgroups of row tiles written in closed form count in neither.)
 * screened_tiles: the part of logit_tiles the screening GEMM looked at (calls it ran for, row tiles not certified).
 * onehot_row_tiles: tiles of 128 rows whose rows all have one softmax weight of 1.0 and zeros, which the second GEMM
 * leaves to a kernel that writes  c_x' x + c_m' mu_b  directly (same switch as the sparse second GEMM).
 * certified_row_tiles: the part of onehot_row_tiles that was proven one-hot before any matrix work
 * (asd_use_onehot_certificate); their half tiles of logits count in logit_tiles, none in logit_tiles_done. */
ASD_API asd_status asd_profile_model_work(asd_ctx* ctx, int64_t* logit_tiles_done, int64_t* logit_tiles,
                                          int64_t* combine_slabs_done, int64_t* combine_slabs, int64_t* screened_tiles,
                                          int64_t* onehot_row_tiles, int64_t* certified_row_tiles);

#ifdef __cplusplus
}
#endif
#endif /* ASD_TESTING_H */
