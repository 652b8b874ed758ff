// Shared declarations of the ASD library internals (host side + launchers).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string>
#include <vector>

#include "../../include/asd_testing.h"
#include "gmm_cert.h"
#include "rng.h"

namespace asd {

// ---- error plumbing ---------------------------------------------------------
void set_error(const char* fmt, ...);

#define ASD_HIP(...)                                                               \
  do {                                                                             \
    hipError_t e__ = (__VA_ARGS__);                                                       \
    if (e__ != hipSuccess) {                                                       \
      ::asd::set_error("%s failed: %s (%s:%d)", #__VA_ARGS__, hipGetErrorString(e__), __FILE__, __LINE__); \
      return ASD_EDEVICE;                                                          \
    }                                                                              \
  } while (0)

#define ASD_TRY(call)                 \
  do {                                \
    asd_status s__ = (call);          \
    if (s__ != ASD_OK) return s__;    \
  } while (0)

// ---- row plans written by the round kernels themselves (asd_sample) ------------------------------
// The stage entries plan their model calls with a scan over the chains (plan_rows_kernel, ordered rows).
// Inside asd_sample the kernels that already visit every chain append the rows of the *next* model
// call with one atomic add per chain: the accept kernel lists y_{a_next} of every unfinished chain for
// the next round's draft call, the draft kernel lists the drafted slots for this round's verify call.
// The order of the rows then varies from run to run; a row's result does not depend on its position.
struct PlanOut {
  int64_t* in_off = nullptr;    // NULL: the kernel writes no plan
  int64_t* out_off = nullptr;
  int32_t* row_tau = nullptr;
  int32_t* row_chain = nullptr; // chain of every row (a hint for the denoiser: rows of one chain are alike)
  int32_t* n_rows = nullptr;    // [2]: rows of the draft call, rows of the verify call
  const int32_t* tau = nullptr; // step -> time index
  int64_t* row_counts = nullptr;  // [2] running totals for the profiler, or NULL
  int32_t* ring = nullptr;      // round index + live-chain ring, advanced once per round
};

// ---- a row of a batched model call -----------------------------------------
// The denoiser is always evaluated on a *list of rows*: row n is read at
// in_base + in_off[n] (d floats), its time index is tau[n], and its result is
// written at out_base + out_off[n].  Draft call: one row per chain (y_a);
// verify call: the drafted samples of slots 1..L-1 of every chain, read in
// place from the trajectory and written into x0hat.
struct RowPlan {
  int n;                  // upper bound on the number of rows (grid sizing)
  const int32_t* n_dev;   // DEV: actual number of rows (the plan is compacted on the device)
  const float* in_base;   // DEV
  float* out_base;        // DEV
  const int64_t* in_off;  // DEV [n], in floats
  const int64_t* out_off; // DEV [n]
  const int32_t* tau;     // DEV [n]
  int call;               // 0: draft model call (one row per chain), 1: verify (batched)
  // DEV [n] or NULL: the chain (0 .. chains-1) every row belongs to.  Only a hint: a denoiser may use what it learnt
  // about a chain's earlier rows to guess -- never to decide -- something about this one.
  const int32_t* chain = nullptr;
};

struct GmmState;
struct MlpState;

// Optional per-kernel timing with HIP events recorded on the launch stream.
// Slot = kernel kind + 16 * call kind (see asd_prof_kernel in asd.h).
struct Profiler {
  struct Rec {
    int slot;
    hipEvent_t e0, e1;
  };
  bool on = false;
  bool outer = false;   // also time the scopes that enclose other scopes (a whole model call) and the row planning
  uint32_t slots = ~0u; // bit (kind + 16 call): that slot's scopes are timed (asd_profile_select)
  std::vector<Rec> recs;
  std::vector<hipEvent_t> pool;
  size_t used = 0;
  hipEvent_t take() {
    if (used == pool.size()) {
      hipEvent_t e = nullptr;
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
      pool.push_back(e);
    }
    return pool[used++];
  }
  void reset() {
    recs.clear();
    used = 0;
  }
  void destroy() {
    for (hipEvent_t e : pool) (void)hipEventDestroy(e);
    pool.clear();
    reset();
  }
};

}  // namespace asd

// The context behind the opaque handle.
struct asd_ctx {
  int device = 0;
  int32_t K = 0, L = 0, B = 0, d = 0, n_tau = 0;
  int64_t n_rows_max = 0;  // B * L
  asd::Key key{0, 0};
  asd::Key* key_dev = nullptr;    // DEV copy of the key: kernels read it, so launches do not depend on the seed
  bool key_dirty = false;         // key differs from *key_dev: the next launching call stores it first
  int kind = 0;
  // schedule on the device
  float* c_x = nullptr;
  float* c_0 = nullptr;
  float* sigma = nullptr;
  int32_t* tau = nullptr;
  // row plan scratch
  int64_t* in_off = nullptr;
  int64_t* out_off = nullptr;
  int32_t* row_tau = nullptr;
  int32_t* row_chain = nullptr;   // chain of every row of the current plan
  int32_t* n_rows_dev = nullptr;  // DEV [2]: rows of the current draft-call / verify-call plan
  // x0a: model value at y_a of every chain [B, d]
  float* x0a = nullptr;
  // owned by asd_sample
  float* x0hat = nullptr;  // [B, L, d]
  int32_t* a = nullptr;    // [B]
  int32_t* live = nullptr;       // DEV [1 + 2 kLiveRing]: round index, the ring of live-chain counters, the ring of
                                 // chains a round's early accept kernel left pending
  int32_t* live_host = nullptr;  // pinned mirror
  hipEvent_t* live_ev = nullptr;
  int32_t last_rounds = 0;
  // one round of the cheap-round path as an instantiated HIP graph, valid for (g_traj, g_rounds, g_stream)
  hipGraphExec_t gexec = nullptr;
  hipGraphExec_t gexec_light = nullptr;   // the light round (draft call + early accept kernel only), same validity
  const void* g_traj = nullptr;
  const void* g_rounds = nullptr;
  hipStream_t g_stream = nullptr;
  hipStream_t own_stream = nullptr;  // used instead of the legacy default stream, which cannot be captured
  bool graphs_enabled = true;
  unsigned long long* chain_max = nullptr;  // DEV: (launch id << 32 | largest round count) of the chain-resident sampler
  uint32_t chain_launches = 0;
  int32_t* win = nullptr;      // DEV [2 B]: window of each chain, then the controller's state (asd_sample, adaptive)
  int32_t* cur_win = nullptr;  // what the round kernels are given: win while an adaptive sample runs, else NULL (= L)
  bool adaptive = false;
  const void* g_win = nullptr; // cur_win the round graph was captured with
  bool g_reuse = false;        // reuse_now the round graph was captured with
  bool fold_plans = false;     // set while asd_sample's rounds run: see PlanOut
  // Model-call reuse across rounds (asd_use_call_reuse): the verify call also evaluates the last proposal sample
  // yhat_b of every window (slot w of x0hat, hence L + 1 slots per chain there); a chain whose whole window was
  // accepted takes that value as its next x0a and is left out of the next draft call (carry[c] = 1).
  bool reuse = false;          // the switch
  bool reuse_now = false;      // set while asd_sample's rounds run with the switch on (the stage calls never reuse)
  int32_t* carry = nullptr;    // DEV [B]
  // Early accept (asd_use_early_accept): chains whose rows the denoiser can certify one-hot have their accept stage
  // before the verify call, on model values formed in the accept kernel; the verify call sees the other chains only.
  bool early = true;           // the switch
  bool early_now = false;      // set while asd_sample's rounds run with it
  bool g_early = false;        // early_now the round graph was captured with
  int32_t* pending = nullptr;  // DEV [B]: 1 = the chain still needs this round's verify call and accept kernel
  bool resident_enabled = true;  // asd_sample may run whole chains in one launch (gmm_chain.hip) when the shape allows
  int stage = 0;  // 0: expect draft, 1: expect verify, 2: expect accept
  asd::Profiler prof;
  int64_t* row_counts = nullptr;  // DEV [8], summed over launches while profiling: live rows of the draft call, of the verify
                                  // call, x0hat rows the accept kernel read for its tests, rows it resampled; model rows
                                  // the early accept kernel formed itself, chain-rounds it committed, window rows of those, rows it resampled
  double model_macs_per_row = 0.0;  // multiply-adds of one denoiser row (set by the denoiser)
  asd::GmmState* gmm = nullptr;
  asd::MlpState* mlp = nullptr;
};

namespace asd {

constexpr int kLiveRing = 8;

// Whether kernels get the device-side counters of rows and executed work (asd_profile_rows, asd_profile_model_work).
inline bool prof_counting(const asd_ctx* ctx) { return ctx->prof.on; }

// Times everything launched on `st` during its lifetime under `slot`.
struct ProfScope {
  asd_ctx* ctx;
  hipStream_t st;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int slot;
  ProfScope(asd_ctx* c, int kernel, int call, hipStream_t s) : ctx(c), st(s), slot(kernel + 16 * call) {
    if (!ctx->prof.on) return;
    if ((kernel == ASD_PROF_MODEL || kernel == ASD_PROF_PLAN) && !ctx->prof.outer) return;
    if (!((ctx->prof.slots >> slot) & 1u)) return;
    e0 = ctx->prof.take();
    e1 = ctx->prof.take();
    if (e0 && e1) (void)hipEventRecord(e0, st);
  }
  ~ProfScope() {
    if (e0 && e1) {
      (void)hipEventRecord(e1, st);
      ctx->prof.recs.push_back({slot, e0, e1});
    }
  }
};


// denoisers (gmm.hip / mlp.hip)
asd_status gmm_create(asd_ctx* ctx, const asd_denoiser& den);
void gmm_destroy(asd_ctx* ctx);
asd_status gmm_eval(asd_ctx* ctx, const RowPlan& rows, hipStream_t st);
// chain-resident sampler (gmm_chain.hip): all of Alg. 1 for a chain in one workgroup, one launch per sample
bool gmm_chain_supported(const asd_ctx* ctx);
asd_status gmm_chain_sample(asd_ctx* ctx, const float* y0, float* traj, int32_t* rounds, hipStream_t st);  // honours ctx->adaptive

asd_status mlp_create(asd_ctx* ctx, const asd_denoiser& den);
void mlp_destroy(asd_ctx* ctx);
asd_status mlp_eval(asd_ctx* ctx, const RowPlan& rows, hipStream_t st);

// What a kernel outside the mixture denoiser needs to certify rows one-hot and form their model values (gmm_cert.h);
// false when the denoiser's own verify call would not do the same, bit for bit.
bool gmm_onehot_cert(const asd_ctx* ctx, asd::OneHotCert* out);
inline bool model_onehot_cert(const asd_ctx* ctx, asd::OneHotCert* out) {
  return ctx->kind == ASD_DEN_GMM && gmm_onehot_cert(ctx, out);
}
// Rows per chain block the denoiser would like the verify call's plan laid out in (0: as they come): see gmm.hip.
int gmm_row_block(const asd_ctx* ctx);
inline int model_row_block(const asd_ctx* ctx) { return ctx->kind == ASD_DEN_GMM ? gmm_row_block(ctx) : 0; }

inline asd_status model_eval(asd_ctx* ctx, const RowPlan& rows, hipStream_t st) {
  if (rows.n <= 0) return ASD_OK;
  ProfScope ps(ctx, ASD_PROF_MODEL, rows.call, st);
  return ctx->kind == ASD_DEN_GMM ? gmm_eval(ctx, rows, st) : mlp_eval(ctx, rows, st);
}

// round kernels (round.hip)
asd_status launch_init_state(asd_ctx* ctx, const float* y0, float* traj, int32_t* a, int32_t* rounds, hipStream_t st);
asd_status launch_plan_draft(asd_ctx* ctx, const int32_t* a, hipStream_t st, int32_t* zero_me = nullptr);
asd_status launch_plan_verify(asd_ctx* ctx, const int32_t* a, hipStream_t st, const int32_t* pending = nullptr);
asd_status launch_draft(asd_ctx* ctx, float* traj, const int32_t* a, hipStream_t st, int32_t* ring = nullptr,
                        const int32_t* pending = nullptr);
asd_status launch_copy_slot0(asd_ctx* ctx, float* x0hat, hipStream_t st);
// x0_slots: slots per chain of x0hat (L for the caller's array of the stage calls, L + 1 with model-call reuse)
asd_status launch_accept(asd_ctx* ctx, float* traj, int32_t* a, const float* x0hat, int x0_slots, int32_t* accepted,
                         float* stats, int32_t* rounds, int32_t* live, hipStream_t st, const int32_t* pending = nullptr);
// Draft and accept stage of the chains the denoiser's one-hot certificate covers, ahead of the draft kernel and the
// verify call; leaves ctx->pending[c] = 1 for every chain that still needs those and launch_accept (accept_early_kernel).
asd_status launch_accept_early(asd_ctx* ctx, float* traj, int32_t* a, int32_t* rounds, int32_t* live, hipStream_t st,
                               bool light = false);
asd_status launch_seq_step(asd_ctx* ctx, float* traj, int32_t step, hipStream_t st);
asd_status launch_plan_seq(asd_ctx* ctx, int32_t step, hipStream_t st);
asd_status launch_debug_philox(Key key, uint32_t chain, uint32_t step, uint32_t stream_id, int32_t nblk,
                               uint32_t* out, hipStream_t st);
asd_status launch_debug_randoms(Key key, uint32_t chain, uint32_t step, int32_t d, float* xi, float* u,
                                hipStream_t st);

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace asd
