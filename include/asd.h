/*
 * asd.h -- C boundary of the MI355X (gfx950) implementation of one round of
 * Autospeculative Decoding (ASD) for DDPM sampling over a batch of chains.
 *
 * The library samples the Euler chain
 *     y_{i+1} = c_x[i] y_i + c_0[i] D(y_i, tau[i]) + sigma[i] xi_{i+1}
 * (Eq. euler-sde written in the x0-prediction form of the Remark after
 * Alg. 3; D is the denoiser E[x_0 | y_i], the paper's "model call") with
 * Alg. 1: draft a window of L steps from one model call, evaluate the model at
 * all drafted points in one batched pass, run the Gaussian Rejection Sampler
 * (Alg. 3) on every slot, advance to the first rejection (Alg. 2) and
 * resample that step by reflection.
 *
 * Conventions
 *  - "HOST" pointers are read during the call and may be freed afterwards.
 *    "DEV" pointers are device (HBM) memory owned by the caller; the library
 *    never frees them.  The denoiser's DEV parameters given to asd_init (GMM:
 *    means, log_w; MLP: biases and the time-embedding table; the MLP weight
 *    matrices are copied) must stay valid until asd_destroy; every other
 *    pointer is only used by the call it is passed to (asynchronously, on
 *    `stream`).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Stage calls are asynchronous; only asd_sample synchronises (it polls a
 *    per-round live-chain count).
 *  - All state is fp32; trajectories are row-major traj[chain][step][dim] with
 *    step = 0..K (K+1 rows per chain).  Random numbers come from a
 *    counter-based Philox4x32-10 keyed by `seed` with counter
 *    (block = dim/4, step, chain, stream-id): Alg. 1 draws u_{1:K}, xi_{1:K}
 *    once and indexes them by step, never by round.
 *  - No call throws or aborts: every entry returns an asd_status.  Argument
 *    errors are detected on the host before any launch.  A ctx is bound to the
 *    device that was current at asd_init and is not thread-safe.
 */
#ifndef ASD_H
#define ASD_H

#include <stdint.h>

#if defined(__GNUC__)
#define ASD_API __attribute__((visibility("default")))
#else
#define ASD_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct asd_ctx asd_ctx; /* opaque, owned by the library */

typedef enum {
  ASD_OK = 0,
  ASD_EINVAL = -1,       /* NULL pointer, size or value out of range          */
  ASD_ENOMEM = -2,       /* host or device allocation failed                  */
  ASD_EDEVICE = -3,      /* a HIP call failed (no device, launch error, ...)  */
  ASD_ESTATE = -4,       /* stage calls out of order (draft->verify->accept)  */
  ASD_EUNSUPPORTED = -5  /* valid request this build does not implement       */
} asd_status;

/* Alg. 1 inputs "steps K, step sizes, variances", in x0-prediction form.
 * All arrays HOST, length K; copied by asd_init.
 *   c_x, c_0 : coefficients of y_i and of D(y_i, tau[i]) in the mean of step i
 *   sigma    : standard deviation of the noise of step i (>= 0; 0 allowed:
 *              such a slot is treated as the sigma -> 0 limit of Alg. 3)
 *   tau      : time index fed to the denoiser at step i, in [0, n_tau) */
typedef struct {
  int32_t K;
  const float* c_x;
  const float* c_0;
  const float* sigma;
  const int32_t* tau;
} asd_schedule;

typedef enum { ASD_DEN_GMM = 1, ASD_DEN_MLP = 2 } asd_den_kind;

/* The model g of Alg. 1, as a denoiser D(x, tau) = E[x_0 | x_tau = x].
 *
 * GMM: data law sum_k w_k N(mu_k, var I) observed as
 *   x_tau = sqrt(abar[tau]) x_0 + sqrt(1 - abar[tau]) eps; D is the exact
 *   posterior mean (the mean function m(t, y) of Eq. sl-defn for this law).
 *   means DEV fp32 [C, d] row-major; log_w DEV fp32 [C] (unnormalised logs
 *   allowed); abar HOST fp32 [n_tau], values in (0, 1].
 *   Alternatively (abar NULL) the chain may run in the paper's own stochastic-
 *   localization coordinates: sl_time HOST fp32 [n_tau], values t >= 0, and D
 *   is the mean function itself, m(t, y) = E[x* | t x* + sqrt(t) xi = y] of
 *   Eq. sl-defn; the schedule is then the Euler chain of Eq. euler-sde
 *   (c_x = 1, c_0 = eta_i, sigma = sqrt(eta_i)).  Exactly one of abar and
 *   sl_time is given.
 * MLP: in = [bf16(x) ; temb[tau]] (d + temb_dim), h = W_in in + b_in,
 *   n_blocks times h += SiLU(W_l bf16(h) + b_l), out = W_out bf16(h) + b_out,
 *   D = clamp(out, -out_clip, out_clip) if out_clip > 0 (the usual clipping of
 *   the predicted x_0 to the data range), D = out if out_clip == 0.
 *   predict_eps = 1: the network predicts the noise of x_tau = sqrt(abar) x_0 +
 *   sqrt(1 - abar) eps instead (the parametrisation of the paper's image
 *   models); then out is replaced by (x - sqrt(1 - abar[tau]) out) / sqrt(abar[tau])
 *   before the clip, and abar (HOST fp32 [n_tau], values in (0, 1]) is required.
 *   Weights DEV bf16 row-major [out, in]: w_in [width, d+temb_dim],
 *   w_blk [n_blocks, width, width], w_out [d, width]; biases DEV fp32 or NULL
 *   (= 0): b_in [width], b_blk [n_blocks, width], b_out [d];
 *   temb DEV bf16 [n_tau, temb_dim].  Products accumulate in fp32.
 *   act_terms (1 or 2): how an fp32 activation v (x, h) enters a product.  1: as bf16(v), the formulas
 *   above.  2: as the sum of two bf16 numbers, bf16(v) + bf16(v - bf16(v)) (16 significant bits; round to
 *   nearest even both times), twice the matrix-core work.  With one term, the rounding of the activations
 *   is amplified by a random-weight residual network to ~2e-3 of its output scale whatever the
 *   accumulation order; with two it is ~4e-6.
 *   linears_per_block must be 1.  d, temb_dim and width must be multiples of 8. */
typedef struct {
  int32_t kind; /* asd_den_kind */
  int32_t d;
  int32_t n_tau;
  /* GMM */
  int32_t C;
  const float* means;
  const float* log_w;
  float var;
  const float* abar;
  const float* sl_time;
  /* MLP */
  int32_t width, n_blocks, linears_per_block, temb_dim;
  float out_clip;
  int32_t predict_eps;
  int32_t act_terms;
  const void* w_in;
  const void* w_blk;
  const void* w_out;
  const float* b_in;
  const float* b_blk;
  const float* b_out;
  const void* temb;
} asd_denoiser;

/* Problem statement of Alg. 1 for a batch: schedule, model, speculation
 * length L (the paper's theta; L >= 1; windows are cut at K, so L >= K is the
 * paper's ASD-infinity: every round speculates to the end of the chain),
 * number of chains, seed.  Scratch memory grows with chains * L. */
typedef struct {
  asd_schedule sched;
  asd_denoiser den;
  int32_t L;
  int32_t chains;
  uint64_t seed;
} asd_config;

/* Validates the configuration (ASD_EINVAL / ASD_EUNSUPPORTED before touching
 * the device), copies the tables to the device and allocates all scratch
 * (sized for chains*L rows; the stage and sampling calls allocate no device
 * memory).  chains <= 65535 (ASD_EUNSUPPORTED above).  *out is NULL on failure. */
ASD_API asd_status asd_init(const asd_config* cfg, asd_ctx** out);
ASD_API asd_status asd_destroy(asd_ctx* ctx); /* NULL is allowed */

/* Re-key the random streams; the next asd_sample / stage calls use it.  Waits for
 * the work this context has queued (it may still read the old key). */
ASD_API asd_status asd_set_seed(asd_ctx* ctx, uint64_t seed);

/* ---- one round (body of the while-loop of Alg. 1), three stages ----------
 * a DEV int32 [chains]: current index a_c of each chain (0 <= a_c <= K; a
 * chain with a_c == K is finished and is left untouched).
 * Call order draft -> verify -> accept is enforced (ASD_ESTATE otherwise).
 *
 * asd_draft: model call 1 and the proposal samples.  Reads traj[c][a_c],
 *   evaluates x0a_c = D(y_a, tau[a_c]) (kept in ctx scratch) and writes the
 *   proposal samples yhat_{a+1..b}, b = min(K, a+L), into traj[c][a_c+1..b]:
 *   yhat_{i+1} = c_x[i] yhat_i + c_0[i] x0a + sigma[i] xi_{i+1}. */
ASD_API asd_status asd_draft(asd_ctx* ctx, float* traj, const int32_t* a, void* stream);

/* asd_verify: model call 2, the batched target-mean evaluation.
 *   x0hat DEV fp32 [chains, L, d]; slot 0 receives a copy of x0a (proposal
 *   mean == target mean for step a+1, so it is not recomputed); slot s in
 *   1..b-a-1 receives D(yhat_{a+s}, tau[a+s]).  Slots >= b-a are unspecified. */
ASD_API asd_status asd_verify(asd_ctx* ctx, const float* traj, const int32_t* a, float* x0hat, void* stream);

/* asd_accept: Alg. 3 on every slot, first-rejection scan (Alg. 2), resample,
 *   advance.  Slot a+1 is accepted; for s >= 1, v = c_0 (x0a - x0hat[s]),
 *   accept iff log u <= -(<v,xi>/sigma + |v|^2 / (2 sigma^2)); sigma == 0
 *   rejects.  With j the end of the accepted prefix: if j < b the row
 *   traj[c][j+1] is overwritten by the reflected sample and a_c = j+1, else
 *   a_c = j.  accepted (DEV int32 [chains], may be NULL) receives j - a_c(old)
 *   (-1 for finished chains).
 *   stats (DEV fp32 [chains, L, 4], may be NULL) receives per examined slot
 *   (<d,xi>, |d|^2, log u, rho) with d = x0a - x0hat[s]  (slot 0: zeros).
 *   The window is examined in order, eight slots at a time, up to the group
 *   that holds the first rejection; entries of later slots are left as they
 *   were. */
ASD_API asd_status asd_accept(asd_ctx* ctx, float* traj, int32_t* a, const float* x0hat,
                      int32_t* accepted, float* stats, void* stream);

/* ---- whole sample (Alg. 1) ------------------------------------------------
 * y0 DEV fp32 [chains, d] or NULL (then y_0 ~ N(0, I) from the Philox stream
 * at step 0).  Fills traj DEV fp32 [chains, K+1, d] and rounds DEV int32
 * [chains] (iterations of the while-loop each chain took; may be NULL).
 * Rounds are lock-step launches over all unfinished chains. */
ASD_API asd_status asd_sample(asd_ctx* ctx, const float* y0, float* traj, int32_t* rounds, void* stream);

/* asd_sample for callers that cannot allocate (code under HIP graph capture of their own, tight serving loops,
 * harnesses that forbid hipMalloc): the same sample on the same kernels, with the batched verify call's outputs
 * (x0hat [chains, L, d], the only buffer asd_sample needs beyond what asd_init set up) in a static device array
 * of 32 MiB that every GPU the library runs on holds until the process ends.  The call makes no hipMalloc /
 * hipFree, creates no stream, event or graph (rounds are plain launches on `stream`, lock-step round kernels
 * only) and returns ASD_EUNSUPPORTED when chains*L*d*4 bytes exceed the 32 MiB, ASD_ESTATE while per-kernel
 * timing is on.  Results equal asd_sample's with asd_use_graphs(0) and asd_use_resident(0).  All contexts on a
 * GPU share that GPU's array, and it keeps the last call's contents (no slot is read before the same round has
 * written it, so nothing is cleared): calls that overlap in time on one GPU race. */
ASD_API asd_status asd_sample_noalloc(asd_ctx* ctx, const float* y0, float* traj, int32_t* rounds, void* stream);

/* asd_sample launches the rounds of launch-bound workloads as one captured HIP graph per round
 * (kernels only; the graph is rebuilt when traj, rounds or the stream change).  on = 0 switches to
 * plain kernel launches; the results are identical.  Default: on. */
ASD_API asd_status asd_use_graphs(asd_ctx* ctx, int32_t on);

/* Window control for asd_sample (an extension; Alg. 1 takes the speculation length as a fixed input).
 * on = 1: each chain chooses the window of its next round from its own past, never longer than L: three
 * quarters of a running mean of its accepted run length (integers: state <- state - state/4 + obs, obs =
 * accepted slots, or twice the window when all of it was accepted; window = clamp(3 state / 16, min(4, L),
 * L); state starts at 4 L).  A window that depends on the chain's past only leaves the law of every
 * step intact (the correctness proof conditions on the past), so samples stay exact; the model calls a
 * round spends on slots behind the first rejection shrink.  Default: off (every window is L).  The stage
 * calls always use L. */
ASD_API asd_status asd_use_adaptive_window(asd_ctx* ctx, int32_t on);

/* Model-call reuse across rounds in asd_sample (the paper counts "sequential network calls" as if evaluations
 * were carried from one iteration of Alg. 1 to the next; Alg. 1 as printed makes two calls per iteration).
 * on = 1: the batched verify call also evaluates the model at the last proposal sample yhat_b of every window
 * that ends before K (one more row per chain); a chain whose whole window is accepted starts its next round at
 * y_b = yhat_b with that value as x0a and is left out of the next draft call.  The samples are the same function
 * of the random inputs (to the rounding difference between the two calls' GEMM tilings); what changes is the
 * number of rows each call evaluates.  With a noalloc sample the scratch bound counts L + 1 slots per chain.
 * Default: off.  The stage calls and the chain-resident path do not reuse. */
ASD_API asd_status asd_use_call_reuse(asd_ctx* ctx, int32_t on);

/* For a Gaussian-mixture denoiser small enough to sit in one CU's LDS (with the window of a chain),
 * asd_sample runs Alg. 1 for each chain inside one workgroup: one launch per sample instead of
 * several per round (chains do not interact, so no step of the method changes; rounds[c] keeps its
 * meaning and asd_last_round_count returns the largest of them).  on = 0 forces the lock-step
 * round kernels; the two paths agree to rounding.  Default: on.  Other shapes ignore the switch. */
ASD_API asd_status asd_use_resident(asd_ctx* ctx, int32_t on);

/* Model-call GEMMs of the large Gaussian-mixture denoiser on the 16-bit matrix pipes with every fp32
 * operand split into 16-bit terms, fp32 accumulation.  d and C multiples of 32: two fp16 terms per operand
 * (the nearest fp16 and the nearest fp16 of the remainder, operands scaled by powers of two into fp16's range) and
 * three products per fp32 product, in both model calls; what is left out is 2^-23 of |a||b| per product on
 * average and never above 3 * 2^-22, a few units of fp32 rounding.  Multiples of 16 only: three bf16 terms and
 * six products (2^-23 on average, never above 2^-21), in the verify call.  Nothing in the method changes: it is
 * another way to evaluate the same fp32 contraction, about 2.3x (1.5x) faster on this chip than its fp32 matrix
 * pipe.  on = 0 selects the fp32 MFMA kernels.  Default: on.  Other shapes ignore the switch. */
ASD_API asd_status asd_use_split_gemm(asd_ctx* ctx, int32_t on);

/* Sequential chain with the same random inputs (one model call per step, K
 * launches): the baseline ASD is compared against in the paper's speedups. */
ASD_API asd_status asd_sample_sequential(asd_ctx* ctx, const float* y0, float* traj, void* stream);

/* Number of lock-step rounds launched by the last asd_sample (host value): the largest rounds[c], or a few more
 * where early accept is at work (asd_testing.h) -- a round launched without the verify call may leave a chain
 * waiting for the next full one, which rounds[c] does not count. */
ASD_API int32_t asd_last_round_count(const asd_ctx* ctx);

/* ---- the model call on its own ---------------------------------------------
 * asd_denoise: out[n] = D(x[n], tau[n]) for n rows (n <= chains*L), through the
 *   kernels of the batched verify call.
 *   x, out DEV fp32 [n, d]; tau DEV int32 [n]. */
ASD_API asd_status asd_denoise(asd_ctx* ctx, const float* x, const int32_t* tau, int32_t n, float* out, void* stream);

/* ---- host-only helpers -----------------------------------------------------
 * DDPM linear-beta schedule (beta_tau from beta_min to beta_max over tau=1..K)
 * in the x0-prediction form, computed in double and rounded to fp32:
 * the coefficients obtained by mapping a DDPM iterate to Stochastic
 * Localization, taking one Euler step there and mapping back (Sec. 3), which
 * is ancestral sampling with the posterior variance.  Step i handles
 * tau[i] = K - i.  Arrays HOST: c_x, c_0, sigma, tau [K]; abar [K+1]
 * (abar[0] = 1).  Any output pointer may be NULL. */
ASD_API asd_status asd_schedule_ddpm_linear(int32_t K, double beta_min, double beta_max,
                                    float* c_x, float* c_0, float* sigma, int32_t* tau, float* abar);

/* The same coefficients for any variance-preserving schedule given by its abar[0..K] (HOST, double; abar[0] = 1,
 * strictly decreasing, abar[K] > 0): beta_tau = 1 - abar[tau]/abar[tau-1].  Cosine, sigmoid, learned ... schedules
 * enter through this.  Outputs as above (any may be NULL; abar_f32 [K+1] is the fp32 copy a GMM or
 * noise-predicting denoiser takes). */
ASD_API asd_status asd_schedule_from_abar(int32_t K, const double* abar, float* c_x, float* c_0, float* sigma,
                                  int32_t* tau, float* abar_f32);
/* The Euler chain of Eq. euler-sde on the stochastic-localization process itself, for a mixture denoiser given
 * sl_time: times t[0..K] (HOST, double; positive, strictly increasing), step i goes from t[i] to t[i+1] with
 * c_x = 1, c_0 = eta_i = t[i+1] - t[i], sigma = sqrt(eta_i), tau[i] = i (the index into sl_time).  A
 * variance-exploding diffusion x = x_0 + s eps is this process at t = 1/s^2, y = x/s^2.  Outputs HOST [K]
 * (t_f32 [K+1]); any may be NULL. */
ASD_API asd_status asd_schedule_sl_euler(int32_t K, const double* t, float* c_x, float* c_0, float* sigma,
                                 int32_t* tau, float* t_f32);
/* abar[0..K] (HOST, double) of the cosine schedule, abar ~ cos^2(((tau/K + s)/(1 + s)) pi/2), with every beta
 * clipped at beta_clip (Nichol & Dhariwal 2021 use s = 0.008, beta_clip = 0.999). */
ASD_API asd_status asd_abar_cosine(int32_t K, double s, double beta_clip, double* abar);

ASD_API const char* asd_status_string(asd_status s);
/* Message of the last failure on this thread ("" if none). */
ASD_API const char* asd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ASD_H */
