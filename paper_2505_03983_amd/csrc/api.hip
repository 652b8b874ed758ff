// C entry points of the ASD library: validation, context life cycle, the three
// stages of a round and the whole-sample driver (the while-loop of Alg. 1 run
// in lock step over a batch of independent chains).
#include <math.h>
#include <stdarg.h>
#include <string.h>

#include <new>

#include "common.h"
#include "gmm_state.h"

// Scratch of asd_sample_noalloc: the verify call's outputs x0hat [chains, L, d] of a sample whose caller may
// not allocate.  One copy per GPU, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address of each GPU's copy is kept in g_scratch_ptr and is what kernels and
// copies are given.
constexpr size_t kNoallocScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];

namespace asd {

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU (set by asd_init)

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

static asd_status fail(asd_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return s;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// ---- validation (host only; no HIP call) -------------------------------------
static asd_status validate(const asd_config* cfg) {
  if (!cfg) return fail(ASD_EINVAL, "cfg is NULL");
  const asd_schedule& s = cfg->sched;
  const asd_denoiser& m = cfg->den;
  if (s.K < 1) return fail(ASD_EINVAL, "K must be >= 1 (got %d)", s.K);
  if (cfg->L < 1) return fail(ASD_EINVAL, "L must be >= 1 (got %d)", cfg->L);
  if (cfg->chains < 1) return fail(ASD_EINVAL, "chains must be >= 1 (got %d)", cfg->chains);
  if (!s.c_x || !s.c_0 || !s.sigma || !s.tau) return fail(ASD_EINVAL, "schedule table is NULL");
  if (m.d < 1) return fail(ASD_EINVAL, "d must be >= 1 (got %d)", m.d);
  if (m.n_tau < 1) return fail(ASD_EINVAL, "n_tau must be >= 1 (got %d)", m.n_tau);
  for (int i = 0; i < s.K; ++i) {
    if (!isfinite(s.c_x[i]) || !isfinite(s.c_0[i]) || !isfinite(s.sigma[i]))
      return fail(ASD_EINVAL, "schedule entry %d is not finite", i);
    if (s.sigma[i] < 0.f) return fail(ASD_EINVAL, "sigma[%d] is negative", i);
    if (s.tau[i] < 0 || s.tau[i] >= m.n_tau) return fail(ASD_EINVAL, "tau[%d]=%d outside [0,%d)", i, s.tau[i], m.n_tau);
  }
  if ((double)cfg->chains * cfg->L > 1.0e9 || (double)cfg->chains * ((double)s.K + 1.0) * m.d > 4.0e12)
    return fail(ASD_EINVAL, "problem too large");
  if (m.kind == ASD_DEN_GMM) {
    if (m.C < 1) return fail(ASD_EINVAL, "C must be >= 1 (got %d)", m.C);
    if (!m.means || !m.log_w) return fail(ASD_EINVAL, "GMM parameter pointer is NULL");
    if ((m.abar != nullptr) == (m.sl_time != nullptr))
      return fail(ASD_EINVAL, "a GMM denoiser takes exactly one of abar and sl_time");
    if (!(m.var >= 0.f) || !isfinite(m.var)) return fail(ASD_EINVAL, "var must be finite and >= 0");
    for (int t = 0; t < m.n_tau; ++t) {
      if (m.abar) {
        const float ab = m.abar[t];
        if (!(ab > 0.f) || !(ab <= 1.f)) return fail(ASD_EINVAL, "abar[%d] outside (0,1]", t);
        if ((double)ab * m.var + 1.0 - ab <= 0.0) return fail(ASD_EINVAL, "abar[%d]=1 with var=0 is degenerate", t);
      } else {
        const float tt = m.sl_time[t];
        if (!(tt >= 0.f) || !isfinite(tt)) return fail(ASD_EINVAL, "sl_time[%d] must be finite and >= 0", t);
      }
    }
  } else if (m.kind == ASD_DEN_MLP) {
    if (m.width < 1 || m.n_blocks < 0 || m.temb_dim < 0) return fail(ASD_EINVAL, "bad MLP shape");
    if (!m.w_in || !m.w_out || (m.n_blocks > 0 && !m.w_blk) || (m.temb_dim > 0 && !m.temb))
      return fail(ASD_EINVAL, "MLP parameter pointer is NULL");
    if (!(m.out_clip >= 0.f)) return fail(ASD_EINVAL, "out_clip must be >= 0");
    if (m.predict_eps) {
      if (!m.abar) return fail(ASD_EINVAL, "predict_eps needs abar");
      for (int t = 0; t < m.n_tau; ++t)
        if (!(m.abar[t] > 0.f) || !(m.abar[t] <= 1.f)) return fail(ASD_EINVAL, "abar[%d] outside (0,1]", t);
    }
    if (m.act_terms != 1 && m.act_terms != 2) return fail(ASD_EINVAL, "act_terms must be 1 or 2 (got %d)", m.act_terms);
    if (m.linears_per_block != 1) return fail(ASD_EUNSUPPORTED, "linears_per_block must be 1");
    if (m.d % 8 || m.temb_dim % 8 || m.width % 8)
      return fail(ASD_EUNSUPPORTED, "MLP needs d, temb_dim and width to be multiples of 8");
  } else {
    return fail(ASD_EINVAL, "unknown denoiser kind %d", m.kind);
  }
  if (cfg->chains > 65535) return fail(ASD_EUNSUPPORTED, "chains > 65535 (got %d)", cfg->chains);
  return ASD_OK;
}

static asd_status check_ctx(asd_ctx* ctx) {
  if (!ctx) return fail(ASD_EINVAL, "ctx is NULL");
  ASD_HIP(hipSetDevice(ctx->device));
  return ASD_OK;
}

static asd_status check_rows_ptr(const asd_ctx* ctx, const void* p, const char* name) {
  if (!p) return fail(ASD_EINVAL, "%s is NULL", name);
  if ((ctx->d & 3) == 0 && !aligned16(p)) return fail(ASD_EINVAL, "%s must be 16-byte aligned", name);
  return ASD_OK;
}

template <class T>
static asd_status upload(T** dst, const T* src, size_t n) {
  ASD_HIP(hipMalloc(dst, sizeof(T) * n));
  ASD_HIP(hipMemcpy(*dst, src, sizeof(T) * n, hipMemcpyHostToDevice));
  return ASD_OK;
}

static asd_status build(asd_ctx* ctx, const asd_config* cfg) {
  ASD_HIP(hipGetDevice(&ctx->device));
  if (ctx->device >= 0 && ctx->device < kMaxDevices && !g_scratch_ptr[ctx->device]) {
    void* p = nullptr;
    ASD_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));   // this device's copy (the device is current)
    g_scratch_ptr[ctx->device] = p;
  }
  ctx->K = cfg->sched.K;
  ctx->L = cfg->L;
  ctx->B = cfg->chains;
  ctx->d = cfg->den.d;
  ctx->n_tau = cfg->den.n_tau;
  ctx->n_rows_max = (int64_t)cfg->chains * cfg->L;
  ctx->key = make_key(cfg->seed);
  ctx->kind = cfg->den.kind;
  const size_t K = (size_t)ctx->K, rows = (size_t)ctx->n_rows_max;
  ASD_TRY(upload(&ctx->c_x, cfg->sched.c_x, K));
  ASD_TRY(upload(&ctx->c_0, cfg->sched.c_0, K));
  ASD_TRY(upload(&ctx->sigma, cfg->sched.sigma, K));
  ASD_TRY(upload(&ctx->tau, cfg->sched.tau, K));
  ASD_HIP(hipMalloc(&ctx->in_off, sizeof(int64_t) * rows));
  ASD_HIP(hipMalloc(&ctx->out_off, sizeof(int64_t) * rows));
  ASD_HIP(hipMalloc(&ctx->row_tau, sizeof(int32_t) * rows));
  ASD_HIP(hipMalloc(&ctx->row_chain, sizeof(int32_t) * rows));
  ASD_HIP(hipMalloc(&ctx->n_rows_dev, sizeof(int32_t) * 2));
  ASD_HIP(hipMemset(ctx->n_rows_dev, 0, sizeof(int32_t) * 2));
  ASD_HIP(hipMalloc(&ctx->x0a, sizeof(float) * (size_t)ctx->B * ctx->d));
  // one more slot per chain than the window: with model-call reuse slot w holds the model value at yhat_b
  ASD_HIP(hipMalloc(&ctx->x0hat, sizeof(float) * (size_t)ctx->B * ((size_t)ctx->L + 1) * (size_t)ctx->d));
  ASD_HIP(hipMalloc(&ctx->carry, sizeof(int32_t) * (size_t)ctx->B));
  ASD_HIP(hipMemset(ctx->carry, 0, sizeof(int32_t) * (size_t)ctx->B));
  ASD_HIP(hipMalloc(&ctx->a, sizeof(int32_t) * (size_t)ctx->B));
  ASD_HIP(hipMalloc(&ctx->row_counts, sizeof(int64_t) * 8));
  ASD_HIP(hipMemset(ctx->row_counts, 0, sizeof(int64_t) * 8));
  ASD_HIP(hipMalloc(&ctx->pending, sizeof(int32_t) * (size_t)ctx->B));
  ASD_HIP(hipMemset(ctx->pending, 0, sizeof(int32_t) * (size_t)ctx->B));
  ASD_HIP(hipMalloc(&ctx->live, sizeof(int32_t) * (1 + 2 * kLiveRing)));
  ASD_HIP(hipMemset(ctx->live, 0, sizeof(int32_t) * (1 + 2 * kLiveRing)));
  ASD_HIP(hipMalloc(&ctx->win, sizeof(int32_t) * 2 * (size_t)ctx->B));
  ASD_HIP(hipMalloc(&ctx->chain_max, sizeof(unsigned long long)));
  ASD_HIP(hipMemset(ctx->chain_max, 0, sizeof(unsigned long long)));
  ASD_HIP(hipMalloc(&ctx->key_dev, sizeof(Key)));
  ASD_HIP(hipMemcpy(ctx->key_dev, &ctx->key, sizeof(Key), hipMemcpyHostToDevice));
  ASD_HIP(hipHostMalloc((void**)&ctx->live_host, sizeof(int32_t) * 2 * kLiveRing, hipHostMallocDefault));
  ctx->live_ev = new (std::nothrow) hipEvent_t[kLiveRing]();
  if (!ctx->live_ev) return ASD_ENOMEM;
  for (int i = 0; i < kLiveRing; ++i) ASD_HIP(hipEventCreateWithFlags(&ctx->live_ev[i], hipEventDisableTiming));
  if (ctx->kind == ASD_DEN_GMM) return gmm_create(ctx, cfg->den);
  return mlp_create(ctx, cfg->den);
}

// The captured rounds hold the launch arguments and kernels of the settings they were captured under.
static void drop_round_graphs(asd_ctx* ctx) {
  if (ctx->gexec) (void)hipGraphExecDestroy(ctx->gexec);
  if (ctx->gexec_light) (void)hipGraphExecDestroy(ctx->gexec_light);
  ctx->gexec = nullptr;
  ctx->gexec_light = nullptr;
}

static void teardown(asd_ctx* ctx) {
  if (!ctx) return;
  gmm_destroy(ctx);
  mlp_destroy(ctx);
  (void)hipFree(ctx->c_x);
  (void)hipFree(ctx->c_0);
  (void)hipFree(ctx->sigma);
  (void)hipFree(ctx->tau);
  (void)hipFree(ctx->in_off);
  (void)hipFree(ctx->out_off);
  (void)hipFree(ctx->row_tau);
  (void)hipFree(ctx->row_chain);
  (void)hipFree(ctx->n_rows_dev);
  (void)hipFree(ctx->x0a);
  (void)hipFree(ctx->x0hat);
  (void)hipFree(ctx->carry);
  (void)hipFree(ctx->a);
  (void)hipFree(ctx->live);
  (void)hipFree(ctx->chain_max);
  (void)hipFree(ctx->win);
  (void)hipFree(ctx->key_dev);
  drop_round_graphs(ctx);
  if (ctx->own_stream) (void)hipStreamDestroy(ctx->own_stream);
  (void)hipFree(ctx->row_counts);
  (void)hipFree(ctx->pending);
  ctx->prof.destroy();
  if (ctx->live_host) (void)hipHostFree(ctx->live_host);
  if (ctx->live_ev) {
    for (int i = 0; i < kLiveRing; ++i)
      if (ctx->live_ev[i]) (void)hipEventDestroy(ctx->live_ev[i]);
    delete[] ctx->live_ev;
  }
  delete ctx;
}

static RowPlan draft_rows(asd_ctx* ctx, const float* traj) {
  return RowPlan{ctx->B, ctx->n_rows_dev + 0, traj, ctx->x0a, ctx->in_off, ctx->out_off, ctx->row_tau, 0, ctx->row_chain};
}

static RowPlan verify_rows(asd_ctx* ctx, const float* traj, float* x0hat) {
  int per_chain = ctx->L - 1 + (ctx->reuse_now ? 1 : 0);   // tested slots, plus yhat_b with model-call reuse
  const int block = ctx->cur_win ? 0 : model_row_block(ctx);    // the planner's filling of each chain's block (launch_plan_verify)
  if (block > 0) per_chain = (per_chain + block - 1) / block * block;
  return RowPlan{ctx->B * per_chain, ctx->n_rows_dev + 1, traj, x0hat, ctx->in_off, ctx->out_off, ctx->row_tau, 1,
                 ctx->row_chain};
}

__global__ void set_key_kernel(Key* dst, Key key) { *dst = key; }

// The kernels read the key from device memory (so that a captured round does not depend on the seed); a new
// key travels as a kernel argument and is stored in stream order ahead of the launches that read it.
static asd_status flush_key(asd_ctx* ctx, hipStream_t st) {
  if (!ctx->key_dirty) return ASD_OK;
  hipLaunchKernelGGL(set_key_kernel, dim3(1), dim3(1), 0, st, ctx->key_dev, ctx->key);
  ASD_HIP(hipGetLastError());
  ctx->key_dirty = false;
  return ASD_OK;
}

__global__ void plan_dense_kernel(int n, int d, int n_tau, const int32_t* __restrict__ tau,
                                  int64_t* __restrict__ in_off, int64_t* __restrict__ out_off,
                                  int32_t* __restrict__ row_tau, int32_t* __restrict__ n_rows) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i == 0) *n_rows = n;
  if (i >= n) return;
  in_off[i] = (int64_t)i * d;
  out_off[i] = (int64_t)i * d;
  row_tau[i] = min(max(tau[i], 0), n_tau - 1);
}

}  // namespace asd

using namespace asd;

extern "C" {

asd_status asd_init(const asd_config* cfg, asd_ctx** out) {
  if (!out) return fail(ASD_EINVAL, "out is NULL");
  *out = nullptr;
  ASD_TRY(validate(cfg));
  asd_ctx* ctx = new (std::nothrow) asd_ctx();
  if (!ctx) return fail(ASD_ENOMEM, "host allocation failed");
  asd_status s = build(ctx, cfg);
  if (s != ASD_OK) {
    teardown(ctx);
    return s;
  }
  *out = ctx;
  return ASD_OK;
}

asd_status asd_destroy(asd_ctx* ctx) {
  if (!ctx) return ASD_OK;
  (void)hipSetDevice(ctx->device);
  (void)hipDeviceSynchronize();
  teardown(ctx);
  return ASD_OK;
}

asd_status asd_set_seed(asd_ctx* ctx, uint64_t seed) {
  if (!ctx) return fail(ASD_EINVAL, "ctx is NULL");
  ctx->key = make_key(seed);
  ctx->key_dirty = true;   // written to the device by the next call that launches kernels, in stream order
  return ASD_OK;
}

asd_status asd_draft(asd_ctx* ctx, float* traj, const int32_t* a, void* stream) {
  ASD_TRY(check_ctx(ctx));
  ASD_TRY(check_rows_ptr(ctx, traj, "traj"));
  if (!a) return fail(ASD_EINVAL, "a is NULL");
  if (ctx->stage != 0) return fail(ASD_ESTATE, "asd_draft called out of order (expected stage %d)", ctx->stage);
  hipStream_t st = (hipStream_t)stream;
  ASD_TRY(flush_key(ctx, st));
  ASD_TRY(launch_plan_draft(ctx, a, st));
  ASD_TRY(model_eval(ctx, draft_rows(ctx, traj), st));
  ASD_TRY(launch_draft(ctx, traj, a, st));
  ctx->stage = 1;
  return ASD_OK;
}

asd_status asd_verify(asd_ctx* ctx, const float* traj, const int32_t* a, float* x0hat, void* stream) {
  ASD_TRY(check_ctx(ctx));
  ASD_TRY(check_rows_ptr(ctx, traj, "traj"));
  ASD_TRY(check_rows_ptr(ctx, x0hat, "x0hat"));
  if (!a) return fail(ASD_EINVAL, "a is NULL");
  if (ctx->stage != 1) return fail(ASD_ESTATE, "asd_verify called out of order (expected stage %d)", ctx->stage);
  hipStream_t st = (hipStream_t)stream;
  ASD_TRY(launch_copy_slot0(ctx, x0hat, st));
  if (ctx->L > 1) {
    ASD_TRY(launch_plan_verify(ctx, a, st));
    ASD_TRY(model_eval(ctx, verify_rows(ctx, traj, x0hat), st));
  }
  ctx->stage = 2;
  return ASD_OK;
}

asd_status asd_accept(asd_ctx* ctx, float* traj, int32_t* a, const float* x0hat, int32_t* accepted, float* stats,
                      void* stream) {
  ASD_TRY(check_ctx(ctx));
  ASD_TRY(check_rows_ptr(ctx, traj, "traj"));
  ASD_TRY(check_rows_ptr(ctx, x0hat, "x0hat"));
  if (!a) return fail(ASD_EINVAL, "a is NULL");
  if (ctx->stage != 2) return fail(ASD_ESTATE, "asd_accept called out of order (expected stage %d)", ctx->stage);
  ASD_TRY(flush_key(ctx, (hipStream_t)stream));
  ASD_TRY(launch_accept(ctx, traj, a, x0hat, ctx->L, accepted, stats, nullptr, nullptr, (hipStream_t)stream));
  ctx->stage = 0;
  return ASD_OK;
}

// All launches of one round of Alg. 1 on `st`, plus the copy of the live-chain ring to the host.
// light (early accept only): the early accept kernel alone (behind the planning kernel, which starts the round) --
// for rounds in which, as far as the host knows, that kernel takes every chain.  A chain it does not take stays where
// it is until the next full round.
static asd_status enqueue_round(asd_ctx* ctx, float* traj, int32_t* rounds, float* x0hat, hipStream_t st, bool light) {
  // No planning kernels here: the rows of the draft call were listed by the previous round's accept
  // kernel (by init_state before round 0), those of the verify call are listed by the draft kernel.
  // (or, for large batches, by the planning kernels: see fold_plans)
  const int32_t* pending = ctx->early_now ? ctx->pending : nullptr;
  if (!ctx->fold_plans) ASD_TRY(launch_plan_draft(ctx, ctx->a, st, ctx->live));
  // (a light round has no draft call either: the early accept kernel forms the model value at y_a itself)
  if (!(pending && light)) ASD_TRY(model_eval(ctx, draft_rows(ctx, traj), st));
  // chains the denoiser can certify have their draft and accept stage in one kernel now; the draft kernel, the verify
  // call and the accept kernel take the others only
  if (pending) ASD_TRY(launch_accept_early(ctx, traj, ctx->a, rounds, ctx->live, st, light));
  if (!(pending && light)) {
    ASD_TRY(launch_draft(ctx, traj, ctx->a, st, ctx->live, pending));
    if (ctx->L > 1 || ctx->reuse_now) {
      if (!ctx->fold_plans) ASD_TRY(launch_plan_verify(ctx, ctx->a, st, pending));
      ASD_TRY(model_eval(ctx, verify_rows(ctx, traj, x0hat), st));
    }
    ASD_TRY(launch_accept(ctx, traj, ctx->a, x0hat, ctx->L + (ctx->reuse_now ? 1 : 0), nullptr, nullptr, rounds,
                          ctx->live, st, pending));
  }
  // The whole ring is copied: slot r % kLiveRing keeps its value until round r + kLiveRing overwrites it,
  // long after the host has read it.
  ASD_HIP(hipMemcpyAsync(ctx->live_host, ctx->live + 1, sizeof(int32_t) * 2 * kLiveRing, hipMemcpyDeviceToHost, st));
  return ASD_OK;
}

// Capture one round into a graph (launch-bound workloads: one graph launch instead of ~8 kernel launches).
// Every launch argument of a round is the same in every round: the round index and the live ring are
// advanced on the device, the seed is read from device memory.
static asd_status ensure_round_graph(asd_ctx* ctx, float* traj, int32_t* rounds, hipStream_t st, bool light) {
  const bool valid = ctx->g_traj == traj && ctx->g_rounds == rounds && ctx->g_stream == st &&
                     ctx->g_win == ctx->cur_win && ctx->g_reuse == ctx->reuse_now && ctx->g_early == ctx->early_now;
  if (!valid) drop_round_graphs(ctx);   // both forms were captured for other arguments
  hipGraphExec_t& exec = light ? ctx->gexec_light : ctx->gexec;
  if (exec) return ASD_OK;
  hipGraph_t graph = nullptr;
  ASD_HIP(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
  asd_status s = enqueue_round(ctx, traj, rounds, ctx->x0hat, st, light);
  hipError_t e = hipStreamEndCapture(st, &graph);
  if (s != ASD_OK) {
    if (graph) (void)hipGraphDestroy(graph);
    return s;
  }
  ASD_HIP(e);
  e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  ASD_HIP(e);
  ctx->g_traj = traj;
  ctx->g_rounds = rounds;
  ctx->g_stream = st;
  ctx->g_win = ctx->cur_win;
  ctx->g_reuse = ctx->reuse_now;
  ctx->g_early = ctx->early_now;
  return ASD_OK;
}

// Whether asd_sample's rounds may take certified chains through their accept stage ahead of the verify call.
static bool early_accept_possible(const asd_ctx* ctx) {
  asd::OneHotCert oc;
  return ctx->early && ctx->pending && ctx->L > 1 && ctx->d % 4 == 0 && ctx->d / 4 <= 256 && model_onehot_cert(ctx, &oc);
}

// The while-loop of Alg. 1 in lock step over the chains, on the round kernels.  x0hat: where the verify call
// leaves its outputs; allow_setup: the call may create streams and graphs and take the one-launch path.
static asd_status sample_rounds(asd_ctx* ctx, const float* y0, float* traj, int32_t* rounds, float* x0hat,
                                bool allow_setup, hipStream_t st) {
  struct WinScope {  // the round kernels see the per-chain windows only while this sample runs
    asd_ctx* c;
    explicit WinScope(asd_ctx* x) : c(x) {
      c->cur_win = c->adaptive ? c->win : nullptr;
      // Appending the row plans from the draft / accept kernels saves two launches per round but costs
      // those kernels an atomic per chain and the index writes: a gain for launch-bound rounds (cfg 3:
      // -5% per sample), a wash for large batches, whose draft / accept kernels run near their own
      // limits (cfg 5: +13 and +18 us on them against 27 us of planning kernels).
      c->fold_plans = c->n_rows_max <= 16384;
      c->reuse_now = c->reuse;
      c->early_now = early_accept_possible(c) && !c->fold_plans && !c->reuse_now;
    }
    ~WinScope() {
      c->cur_win = nullptr;
      c->fold_plans = false;
      c->reuse_now = false;
      c->early_now = false;
    }
  } win_scope(ctx);
  // The live-chain count of a round is read back `lag` rounds later, so the host never waits for the
  // round it has just queued; a finished batch then runs `lag` empty rounds, which cost next to nothing
  // (every kernel exits at once on finished chains and the model calls see zero rows).
  const int lag = 2;
  const bool use_graph = allow_setup && ctx->graphs_enabled && !ctx->prof.on;
  hipStream_t caller = st;
  if (use_graph && st == nullptr) {
    // the legacy default stream cannot be captured: run on a stream of our own, ordered after the caller's work
    if (!ctx->own_stream) ASD_HIP(hipStreamCreateWithFlags(&ctx->own_stream, hipStreamNonBlocking));
    ASD_HIP(hipEventRecord(ctx->live_ev[0], caller));
    ASD_HIP(hipStreamWaitEvent(ctx->own_stream, ctx->live_ev[0], 0));
    st = ctx->own_stream;
  }
  ASD_TRY(flush_key(ctx, st));
  ASD_TRY(launch_init_state(ctx, y0, traj, ctx->a, rounds, st));
  int r = 0;
  int done_at = -1;
  bool light = false;
  // Alg. 1 ends within K iterations (correctness theorem); a light round may leave a chain waiting, at most `lag`
  // rounds in a row before a full one comes
  const int r_cap = (ctx->early_now ? (lag + 2) : 1) * ctx->K + lag + 1;
  for (; r < r_cap; ++r) {
    const int slot = r % kLiveRing;
    if (use_graph && r > 0) {
      ASD_TRY(ensure_round_graph(ctx, traj, rounds, st, light));  // round 0 ran eagerly (first-use set-up)
      ASD_HIP(hipGraphLaunch(light ? ctx->gexec_light : ctx->gexec, st));
    } else {
      ASD_TRY(enqueue_round(ctx, traj, rounds, x0hat, st, light));
    }
    ASD_HIP(hipEventRecord(ctx->live_ev[slot], st));
    if (r >= lag) {
      const int q = (r - lag) % kLiveRing;
      ASD_HIP(hipEventSynchronize(ctx->live_ev[q]));
      if (ctx->live_host[q] == 0) {
        done_at = r - lag;
        break;
      }
      // the early accept kernel took every chain of round r - lag: the rounds to come are launched without the
      // kernels behind it, until one of them reports a chain it could not take (which has waited since)
      light = ctx->early_now && ctx->live_host[kLiveRing + q] == 0;
    }
  }
  ASD_HIP(hipStreamSynchronize(st));
  if (done_at < 0) return fail(ASD_EDEVICE, "asd_sample: chains did not finish within %d rounds", r_cap);
  ctx->last_rounds = done_at + 1;
  return ASD_OK;
}

asd_status asd_sample(asd_ctx* ctx, const float* y0, float* traj, int32_t* rounds, void* stream) {
  ASD_TRY(check_ctx(ctx));
  ASD_TRY(check_rows_ptr(ctx, traj, "traj"));
  if (y0) ASD_TRY(check_rows_ptr(ctx, y0, "y0"));
  if (ctx->stage != 0) return fail(ASD_ESTATE, "asd_sample called between stage calls");
  hipStream_t st = (hipStream_t)stream;
  // Small mixtures: the whole sample is one launch, a workgroup per chain (profiling wants the
  // stand-alone kernels, whose times it reports).
  if (ctx->resident_enabled && !ctx->prof.on && gmm_chain_supported(ctx)) {
    ASD_TRY(flush_key(ctx, st));
    return gmm_chain_sample(ctx, y0, traj, rounds, st);
  }
  return sample_rounds(ctx, y0, traj, rounds, ctx->x0hat, true, st);
}

asd_status asd_sample_noalloc(asd_ctx* ctx, const float* y0, float* traj, int32_t* rounds, void* stream) {
  ASD_TRY(check_ctx(ctx));
  ASD_TRY(check_rows_ptr(ctx, traj, "traj"));
  if (y0) ASD_TRY(check_rows_ptr(ctx, y0, "y0"));
  if (ctx->stage != 0) return fail(ASD_ESTATE, "asd_sample_noalloc called between stage calls");
  if (ctx->prof.on) return fail(ASD_ESTATE, "asd_sample_noalloc: per-kernel timing creates events; switch it off");
  const size_t need = sizeof(float) * (size_t)ctx->B * ((size_t)ctx->L + (ctx->reuse ? 1 : 0)) * (size_t)ctx->d;
  if (need > kNoallocScratchBytes)
    return fail(ASD_EUNSUPPORTED, "asd_sample_noalloc: chains*L*d*4 = %zu bytes exceeds the %zu-byte static scratch",
                need, kNoallocScratchBytes);
  float* x0hat = (ctx->device >= 0 && ctx->device < kMaxDevices) ? (float*)g_scratch_ptr[ctx->device] : nullptr;
  if (!x0hat) return fail(ASD_EDEVICE, "asd_sample_noalloc: no static scratch on device %d", ctx->device);
  // Nothing in the scratch has to start at zero: every slot the accept kernel reads was written by the
  // verify call of the same round.
  return sample_rounds(ctx, y0, traj, rounds, x0hat, false, (hipStream_t)stream);
}

asd_status asd_sample_sequential(asd_ctx* ctx, const float* y0, float* traj, void* stream) {
  ASD_TRY(check_ctx(ctx));
  ASD_TRY(check_rows_ptr(ctx, traj, "traj"));
  if (y0) ASD_TRY(check_rows_ptr(ctx, y0, "y0"));
  if (ctx->stage != 0) return fail(ASD_ESTATE, "asd_sample_sequential called between stage calls");
  hipStream_t st = (hipStream_t)stream;
  ASD_TRY(flush_key(ctx, st));
  ASD_TRY(launch_init_state(ctx, y0, traj, ctx->a, nullptr, st));
  for (int i = 0; i < ctx->K; ++i) {
    ASD_TRY(launch_plan_seq(ctx, i, st));
    ASD_TRY(model_eval(ctx, draft_rows(ctx, traj), st));
    ASD_TRY(launch_seq_step(ctx, traj, i, st));
  }
  ASD_HIP(hipStreamSynchronize(st));
  return ASD_OK;
}

asd_status asd_use_graphs(asd_ctx* ctx, int32_t on) {
  if (!ctx) return fail(ASD_EINVAL, "ctx is NULL");
  ctx->graphs_enabled = on != 0;
  return ASD_OK;
}

asd_status asd_use_adaptive_window(asd_ctx* ctx, int32_t on) {
  if (!ctx) return fail(ASD_EINVAL, "ctx is NULL");
  ctx->adaptive = on != 0;
  return ASD_OK;
}

asd_status asd_use_call_reuse(asd_ctx* ctx, int32_t on) {
  if (!ctx) return fail(ASD_EINVAL, "ctx is NULL");
  ctx->reuse = on != 0;
  return ASD_OK;
}

asd_status asd_use_resident(asd_ctx* ctx, int32_t on) {
  if (!ctx) return fail(ASD_EINVAL, "ctx is NULL");
  ctx->resident_enabled = on != 0;
  return ASD_OK;
}

asd_status asd_use_split_gemm(asd_ctx* ctx, int32_t on) {
  if (!ctx) return fail(ASD_EINVAL, "ctx is NULL");
  if (ctx->gmm && ctx->gmm->split_ok && ctx->gmm->use_split != (on != 0)) {
    ctx->gmm->use_split = on != 0;
    drop_round_graphs(ctx);   // the captured round holds the other kernels
  }
  return ASD_OK;
}

asd_status asd_use_sparse_combine(asd_ctx* ctx, int32_t on) {
  if (!ctx) return fail(ASD_EINVAL, "ctx is NULL");
  if (ctx->gmm && ctx->gmm->sparse_combine != (on != 0)) {
    ctx->gmm->sparse_combine = on != 0;
    drop_round_graphs(ctx);   // the captured round holds the other launch arguments
  }
  return ASD_OK;
}

asd_status asd_use_logit_screen(asd_ctx* ctx, int32_t mode) {
  if (!ctx) return fail(ASD_EINVAL, "ctx is NULL");
  if (mode < 0 || mode > 2) return fail(ASD_EINVAL, "asd_use_logit_screen: mode is 0 (off), 1 (when it pays) or 2 (always)");
  if (ctx->gmm && ctx->gmm->screen_mode != mode) {
    ctx->gmm->screen_mode = mode;
    drop_round_graphs(ctx);   // the captured round holds the other launches
  }
  return ASD_OK;
}

asd_status asd_use_onehot_certificate(asd_ctx* ctx, int32_t on) {
  if (!ctx) return fail(ASD_EINVAL, "ctx is NULL");
  if (ctx->gmm && ctx->gmm->cert_on != (on != 0)) {
    ctx->gmm->cert_on = on != 0;
    drop_round_graphs(ctx);   // the captured round holds the other launches
  }
  return ASD_OK;
}

asd_status asd_use_tall_tiles(asd_ctx* ctx, int32_t on) {
  if (!ctx) return fail(ASD_EINVAL, "ctx is NULL");
  if (ctx->gmm && ctx->gmm->big_on != (on != 0)) {
    ctx->gmm->big_on = on != 0;
    drop_round_graphs(ctx);   // the captured round holds the other launches
  }
  return ASD_OK;
}

int32_t asd_tall_tiles_active(const asd_ctx* ctx) {
  const asd::GmmState* g = ctx ? ctx->gmm : nullptr;
  return (g && g->use_split && g->two_ok && g->big_ok && g->big_on) ? 1 : 0;
}

int32_t asd_onehot_certificate_active(const asd_ctx* ctx) {
  const asd::GmmState* g = ctx ? ctx->gmm : nullptr;
  return (asd_logit_screen_active(ctx) != 0 && g->cert_ok && g->cert_on) ? 1 : 0;
}

int32_t asd_logit_screen_active(const asd_ctx* ctx) {
  const asd::GmmState* g = ctx ? ctx->gmm : nullptr;
  return (g && g->use_split && g->screen_ok && g->screen_mode != 0 && g->sparse_combine) ? g->screen_mode : 0;
}

int32_t asd_split_gemm_active(const asd_ctx* ctx) {
  if (!ctx || !ctx->gmm || !ctx->gmm->use_split) return 0;
  return ctx->gmm->two_ok ? 3 : 6;
}

int32_t asd_resident_active(const asd_ctx* ctx) {
  return (ctx && ctx->resident_enabled && !ctx->prof.on && gmm_chain_supported(ctx)) ? 1 : 0;
}

int32_t asd_last_round_count(const asd_ctx* ctx) { return ctx ? ctx->last_rounds : -1; }

asd_status asd_denoise(asd_ctx* ctx, const float* x, const int32_t* tau, int32_t n, float* out, void* stream) {
  ASD_TRY(check_ctx(ctx));
  ASD_TRY(check_rows_ptr(ctx, x, "x"));
  ASD_TRY(check_rows_ptr(ctx, out, "out"));
  if (!tau) return fail(ASD_EINVAL, "tau is NULL");
  if (n < 0 || n > ctx->n_rows_max) return fail(ASD_EINVAL, "n=%d outside [0, chains*L=%lld]", n, (long long)ctx->n_rows_max);
  if (ctx->stage != 0) return fail(ASD_ESTATE, "asd_denoise called between stage calls");
  if (n == 0) return ASD_OK;
  hipStream_t st = (hipStream_t)stream;
  hipLaunchKernelGGL(plan_dense_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, st, n, ctx->d, ctx->n_tau,
                     tau, ctx->in_off, ctx->out_off, ctx->row_tau, ctx->n_rows_dev + 1);
  ASD_HIP(hipGetLastError());
  return model_eval(ctx, RowPlan{n, ctx->n_rows_dev + 1, x, out, ctx->in_off, ctx->out_off, ctx->row_tau, 1}, st);
}

asd_status asd_profile_enable(asd_ctx* ctx, int32_t on) {
  ASD_TRY(check_ctx(ctx));
  ASD_HIP(hipDeviceSynchronize());
  ctx->prof.reset();
  ctx->prof.on = on != 0;
  ctx->prof.outer = on >= 2;
  ASD_HIP(hipMemset(ctx->row_counts, 0, sizeof(int64_t) * 8));
  if (ctx->gmm && ctx->gmm->work_counts) ASD_HIP(hipMemset(ctx->gmm->work_counts, 0, 8 * sizeof(unsigned long long)));
  return ASD_OK;
}

asd_status asd_use_early_accept(asd_ctx* ctx, int32_t on) {
  ASD_TRY(check_ctx(ctx));
  ctx->early = on != 0;
  return ASD_OK;
}

int32_t asd_early_accept_active(const asd_ctx* ctx) {
  if (!ctx) return 0;
  // (as asd_sample decides it: plans folded into the round kernels and model-call reuse exclude it)
  return (early_accept_possible(ctx) && ctx->n_rows_max > 16384 && !ctx->reuse) ? 1 : 0;
}

asd_status asd_profile_early_accept(asd_ctx* ctx, int64_t* model_rows, int64_t* chain_rounds, int64_t* window_rows,
                                    int64_t* resampled_rows) {
  ASD_TRY(check_ctx(ctx));
  int64_t h[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  ASD_HIP(hipMemcpy(h, ctx->row_counts, sizeof(h), hipMemcpyDeviceToHost));
  if (model_rows) *model_rows = h[4];
  if (chain_rounds) *chain_rounds = h[5];
  if (window_rows) *window_rows = h[6];
  if (resampled_rows) *resampled_rows = h[7];
  return ASD_OK;
}

asd_status asd_profile_select(asd_ctx* ctx, uint32_t slots) {
  ASD_TRY(check_ctx(ctx));
  ctx->prof.slots = slots;
  return ASD_OK;
}

asd_status asd_profile_read(asd_ctx* ctx, int32_t kernel, int32_t call, int64_t* launches, double* total_ms) {
  ASD_TRY(check_ctx(ctx));
  if (kernel < 0 || kernel >= ASD_PROF_KINDS || call < 0 || call > 1) return fail(ASD_EINVAL, "bad profile slot");
  ASD_HIP(hipDeviceSynchronize());
  int64_t n = 0;
  double ms = 0.0;
  for (const Profiler::Rec& r : ctx->prof.recs) {
    if (r.slot != kernel + 16 * call) continue;
    float t = 0.f;
    ASD_HIP(hipEventElapsedTime(&t, r.e0, r.e1));
    ms += t;
    ++n;
  }
  if (launches) *launches = n;
  if (total_ms) *total_ms = ms;
  return ASD_OK;
}

asd_status asd_profile_rows(asd_ctx* ctx, int64_t* draft_rows, int64_t* verify_rows) {
  ASD_TRY(check_ctx(ctx));
  int64_t h[2] = {0, 0};
  ASD_HIP(hipMemcpy(h, ctx->row_counts, sizeof(h), hipMemcpyDeviceToHost));
  if (draft_rows) *draft_rows = h[0];
  if (verify_rows) *verify_rows = h[1];
  return ASD_OK;
}

asd_status asd_profile_accept_rows(asd_ctx* ctx, int64_t* examined_rows, int64_t* resampled_rows) {
  ASD_TRY(check_ctx(ctx));
  int64_t h[4] = {0, 0, 0, 0};
  ASD_HIP(hipMemcpy(h, ctx->row_counts, sizeof(h), hipMemcpyDeviceToHost));
  if (examined_rows) *examined_rows = h[2];
  if (resampled_rows) *resampled_rows = h[3];
  return ASD_OK;
}

asd_status asd_profile_model_work(asd_ctx* ctx, int64_t* logit_tiles_done, int64_t* logit_tiles,
                                  int64_t* combine_slabs_done, int64_t* combine_slabs, int64_t* screened_tiles,
                                  int64_t* onehot_row_tiles, int64_t* certified_row_tiles) {
  ASD_TRY(check_ctx(ctx));
  unsigned long long h[7] = {0, 0, 0, 0, 0, 0, 0};
  if (ctx->gmm && ctx->gmm->work_counts) ASD_HIP(hipMemcpy(h, ctx->gmm->work_counts, sizeof(h), hipMemcpyDeviceToHost));
  int64_t* out[7] = {logit_tiles_done, logit_tiles, combine_slabs_done, combine_slabs, screened_tiles, onehot_row_tiles,
                     certified_row_tiles};
  for (int i = 0; i < 7; ++i)
    if (out[i]) *out[i] = (int64_t)h[i];
  return ASD_OK;
}

asd_status asd_debug_philox(uint64_t seed, uint32_t chain, uint32_t step, uint32_t stream_id, int32_t nblk,
                            uint32_t* out, void* stream) {
  if (!out || nblk < 1) return fail(ASD_EINVAL, "asd_debug_philox: bad arguments");
  return launch_debug_philox(make_key(seed), chain, step, stream_id, nblk, out, (hipStream_t)stream);
}

asd_status asd_debug_randoms(uint64_t seed, uint32_t chain, uint32_t step, int32_t d, float* xi, float* u,
                             void* stream) {
  if (d < 0 || (!xi && !u) || (xi && d < 1)) return fail(ASD_EINVAL, "asd_debug_randoms: bad arguments");
  return launch_debug_randoms(make_key(seed), chain, step, d, xi, u, (hipStream_t)stream);
}

asd_status asd_schedule_ddpm_linear(int32_t K, double beta_min, double beta_max, float* c_x, float* c_0,
                                    float* sigma, int32_t* tau, float* abar) {
  if (K < 1) return fail(ASD_EINVAL, "K must be >= 1");
  if (!(beta_min > 0.0) || !(beta_max < 1.0) || !(beta_min <= beta_max))
    return fail(ASD_EINVAL, "need 0 < beta_min <= beta_max < 1");
  // abar_t = prod_{s<=t} (1 - beta_s), walked from t = 1 up; step i = K - t.
  double ab_prev = 1.0;
  if (abar) abar[0] = 1.0f;
  for (int t = 1; t <= K; ++t) {
    const double beta = (K > 1) ? beta_min + (double)(t - 1) * (beta_max - beta_min) / (double)(K - 1) : beta_min;
    const double ab = ab_prev * (1.0 - beta);
    const int i = K - t;
    const double shrink = (1.0 - ab_prev) / (1.0 - ab);
    if (c_x) c_x[i] = (float)(sqrt(1.0 - beta) * shrink);
    if (c_0) c_0[i] = (float)(sqrt(ab_prev) * beta / (1.0 - ab));
    if (sigma) sigma[i] = (float)sqrt(beta * shrink);
    if (tau) tau[i] = t;
    if (abar) abar[t] = (float)ab;
    ab_prev = ab;
  }
  return ASD_OK;
}

asd_status asd_schedule_from_abar(int32_t K, const double* abar, float* c_x, float* c_0, float* sigma, int32_t* tau,
                                  float* abar_f32) {
  if (K < 1 || !abar) return fail(ASD_EINVAL, "K must be >= 1 and abar non-NULL");
  if (abar[0] != 1.0) return fail(ASD_EINVAL, "abar[0] must be 1");
  for (int t = 1; t <= K; ++t)
    if (!(abar[t] > 0.0) || !(abar[t] < abar[t - 1])) return fail(ASD_EINVAL, "abar must decrease strictly and stay positive (tau = %d)", t);
  if (abar_f32) abar_f32[0] = 1.0f;
  for (int t = 1; t <= K; ++t) {
    const double alpha = abar[t] / abar[t - 1];
    const double shrink = (1.0 - abar[t - 1]) / (1.0 - abar[t]);
    const int i = K - t;
    if (c_x) c_x[i] = (float)(sqrt(alpha) * shrink);
    if (c_0) c_0[i] = (float)(sqrt(abar[t - 1]) * (1.0 - alpha) / (1.0 - abar[t]));
    if (sigma) sigma[i] = (float)sqrt((1.0 - alpha) * shrink);
    if (tau) tau[i] = t;
    if (abar_f32) abar_f32[t] = (float)abar[t];
  }
  return ASD_OK;
}

asd_status asd_schedule_sl_euler(int32_t K, const double* t, float* c_x, float* c_0, float* sigma, int32_t* tau,
                                 float* t_f32) {
  if (K < 1 || !t) return fail(ASD_EINVAL, "K must be >= 1 and t non-NULL");
  if (!(t[0] > 0.0)) return fail(ASD_EINVAL, "t[0] must be positive");
  for (int i = 0; i < K; ++i)
    if (!(t[i + 1] > t[i])) return fail(ASD_EINVAL, "t must increase strictly (index %d)", i + 1);
  for (int i = 0; i < K; ++i) {
    const double eta = t[i + 1] - t[i];
    if (c_x) c_x[i] = 1.0f;
    if (c_0) c_0[i] = (float)eta;
    if (sigma) sigma[i] = (float)sqrt(eta);
    if (tau) tau[i] = i;
  }
  if (t_f32)
    for (int i = 0; i <= K; ++i) t_f32[i] = (float)t[i];
  return ASD_OK;
}

asd_status asd_abar_cosine(int32_t K, double s, double beta_clip, double* abar) {
  if (K < 1 || !abar) return fail(ASD_EINVAL, "K must be >= 1 and abar non-NULL");
  if (!(s >= 0.0) || !(beta_clip > 0.0) || !(beta_clip < 1.0)) return fail(ASD_EINVAL, "need s >= 0 and 0 < beta_clip < 1");
  const double half_pi = 1.5707963267948966;
  auto f = [&](int t) {
    const double c = cos(((double)t / (double)K + s) / (1.0 + s) * half_pi);
    return c * c;
  };
  abar[0] = 1.0;
  double prev = f(0);
  for (int t = 1; t <= K; ++t) {
    const double cur = f(t);
    double beta = 1.0 - cur / prev;
    if (beta > beta_clip) beta = beta_clip;
    abar[t] = abar[t - 1] * (1.0 - beta);
    prev = cur;
  }
  return ASD_OK;
}

const char* asd_status_string(asd_status s) {
  switch (s) {
    case ASD_OK: return "ASD_OK";
    case ASD_EINVAL: return "ASD_EINVAL";
    case ASD_ENOMEM: return "ASD_ENOMEM";
    case ASD_EDEVICE: return "ASD_EDEVICE";
    case ASD_ESTATE: return "ASD_ESTATE";
    case ASD_EUNSUPPORTED: return "ASD_EUNSUPPORTED";
  }
  return "ASD_UNKNOWN";
}

const char* asd_last_error(void) { return g_err; }

}  // extern "C"
