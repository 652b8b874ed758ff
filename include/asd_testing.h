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
/* 1 if the verify call of this context runs the split-operand bf16 kernels. */
ASD_API int32_t asd_split_gemm_active(const asd_ctx* ctx);

/* The second GEMM of the split-operand mixture denoiser (softmax weights times means) skips the stretches of
 * components whose weights are exactly 0.0f for every row of a tile (2^(logit - row maximum) underflows once a
 * posterior has collapsed).  The skipped products are zeros, so results are identical bit for bit; on = 0 makes
 * the kernel visit every component anyway (for tests and timing comparisons).  Default: on. */
ASD_API asd_status asd_use_sparse_combine(asd_ctx* ctx, int32_t on);

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
 * and their summed duration since the last asd_profile_enable(ctx, 1).
 * asd_profile_rows returns the number of live rows (rows inside a window of an
 * unfinished chain) the two model calls were asked to evaluate since then. */
typedef enum {
  ASD_PROF_MODEL = 0,        /* a whole model call (all its kernels)          */
  ASD_PROF_PLAN = 1,         /* row planning                                  */
  ASD_PROF_GMM_ROWWISE = 2,  /* GMM denoiser, one wavefront per row           */
  ASD_PROF_GMM_LOGITS = 3,   /* GMM logits GEMM  X M^T  (fp32 MFMA)           */
  ASD_PROF_GMM_SOFTMAX = 4,  /* GMM row softmax                               */
  ASD_PROF_GMM_COMBINE = 5,  /* GMM  P M  GEMM + affine combination           */
  ASD_PROF_MLP_PACK = 6,     /* MLP input packing (bf16 x ; time embedding)   */
  ASD_PROF_MLP_GEMM_IN = 7,  /* MLP first layer                               */
  ASD_PROF_MLP_GEMM_BLK = 8, /* MLP residual blocks (one launch per block)    */
  ASD_PROF_MLP_GEMM_OUT = 9, /* MLP output layer                              */
  ASD_PROF_DRAFT = 10,       /* fused draft kernel                            */
  ASD_PROF_ACCEPT = 11,      /* fused accept / scan / resample kernel         */
  ASD_PROF_KINDS = 16
} asd_prof_kernel;
ASD_API asd_status asd_profile_enable(asd_ctx* ctx, int32_t on);
ASD_API asd_status asd_profile_read(asd_ctx* ctx, int32_t kernel, int32_t call, int64_t* launches, double* total_ms);
ASD_API asd_status asd_profile_rows(asd_ctx* ctx, int64_t* draft_rows, int64_t* verify_rows);
/* What the accept kernel touched since then: x0hat rows it read for the accept test (it examines a window eight
 * slots at a time and stops at the group that holds the first rejection) and rows it resampled (one per
 * chain-round that ended in a rejection). */
ASD_API asd_status asd_profile_accept_rows(asd_ctx* ctx, int64_t* examined_rows, int64_t* resampled_rows);

#ifdef __cplusplus
}
#endif
#endif /* ASD_TESTING_H */
