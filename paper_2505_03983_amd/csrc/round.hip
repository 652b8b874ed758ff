// Round kernels of ASD: state initialisation, row planning for the two model
// calls, the fused draft kernel (Alg. 1, proposal means and samples) and the
// fused accept / first-rejection scan / reflection-resample kernel
// (Alg. 3 on every slot, Alg. 2, and the advance rule of Alg. 1).
#include "common.h"
#include "device_util.h"

namespace asd {

// ----------------------------------------------------------------------------
// y_0, a = 0, rounds = 0
// ----------------------------------------------------------------------------
__global__ void init_state_kernel(int B, int K, int d, const Key* __restrict__ key_p, const float* __restrict__ y0,
                                  float* __restrict__ traj, int32_t* __restrict__ a,
                                  int32_t* __restrict__ rounds, int32_t* __restrict__ round_idx, int L,
                                  int32_t* __restrict__ win, int32_t* __restrict__ carry, PlanOut plan) {
  const int c = blockIdx.x;
  const Key key = *key_p;
  if (c == 0 && threadIdx.x == 0 && round_idx) *round_idx = 0;
  if (plan.in_off && threadIdx.x == 0) {  // the draft call of round 0: y_0 of every chain
    plan.in_off[c] = (int64_t)c * (K + 1) * d;
    plan.out_off[c] = (int64_t)c * d;
    plan.row_tau[c] = plan.tau[0];
    plan.row_chain[c] = c;
    if (c == 0) {
      plan.n_rows[0] = B;
      plan.n_rows[1] = 0;
      if (plan.row_counts) atomicAdd((unsigned long long*)&plan.row_counts[0], (unsigned long long)B);
    }
  }
  const int nblk = (d + 3) >> 2;
  const bool vec = (d & 3) == 0;
  float* row = traj + (int64_t)c * (K + 1) * d;
  for (int blk = threadIdx.x; blk < nblk; blk += blockDim.x) {
    float4 v = y0 ? load4(y0 + (int64_t)c * d, blk, d, vec) : normal4(key, (uint32_t)c, 0u, (uint32_t)blk);
    store4(row, blk, d, vec, v);
  }
  if (threadIdx.x == 0) {
    a[c] = 0;
    if (carry) carry[c] = 0;
    if (rounds) rounds[c] = 0;
    if (win) {
      win[B + c] = 4 * L;
      win[c] = window_of(4 * L, L);
    }
  }
}

static PlanOut plan_out(asd_ctx* ctx, int32_t* ring) {
  PlanOut p;
  if (!ctx->fold_plans) return p;
  p.in_off = ctx->in_off;
  p.out_off = ctx->out_off;
  p.row_tau = ctx->row_tau;
  p.row_chain = ctx->row_chain;
  p.n_rows = ctx->n_rows_dev;
  p.tau = ctx->tau;
  p.row_counts = prof_counting(ctx) ? ctx->row_counts : nullptr;
  p.ring = ring;
  return p;
}

asd_status launch_init_state(asd_ctx* ctx, const float* y0, float* traj, int32_t* a, int32_t* rounds,
                             hipStream_t st) {
  hipLaunchKernelGGL(init_state_kernel, dim3(ctx->B), dim3(256), 0, st, ctx->B, ctx->K, ctx->d, ctx->key_dev, y0,
                     traj, a, rounds, ctx->live, ctx->L, ctx->cur_win, ctx->carry, plan_out(ctx, nullptr));
  ASD_HIP(hipGetLastError());
  return ASD_OK;
}

// ----------------------------------------------------------------------------
// Row plans.  A model call evaluates a list of rows; the list is built on the
// device and is *compacted*: only rows inside the window of an unfinished
// chain are listed (finished chains and the tail of a window cut by K cost
// nothing), and their number is left in device memory for the model kernels.
// Draft call: row = y_a of live chain c.  Verify call: rows = proposal samples
// of slots s = 1..w-1 of live chain c (slot 0 reuses the draft call's value).
// One workgroup scans the chains in chunks of 1024.
// ----------------------------------------------------------------------------
__device__ __forceinline__ int block_exclusive_scan(int v, int* s_wave, int* s_total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  if (lane == 63) s_wave[wave] = inc;
  __syncthreads();
  if (wave == 0) {
    const int wv = (lane < 16) ? s_wave[lane] : 0;
    int winc = wv;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      const int t = __shfl_up(winc, o, 64);
      if (lane >= o) winc += t;
    }
    if (lane < 16) s_wave[lane] = winc - wv;
    if (lane == 15) *s_total = winc;
  }
  __syncthreads();
  return inc - v + s_wave[wave];
}

// MODE 0: draft call, MODE 1: verify call
template <int MODE>
__global__ __launch_bounds__(1024) void plan_rows_kernel(int B, int K, int L, int d, const int32_t* __restrict__ a,
                                                         const int32_t* __restrict__ tau,
                                                         int64_t* __restrict__ in_off, int64_t* __restrict__ out_off,
                                                         int32_t* __restrict__ row_tau,
                                                         int32_t* __restrict__ row_chain, int32_t* __restrict__ n_rows,
                                                         int32_t* __restrict__ ring,
                                                         int64_t* __restrict__ row_counts,
                                                         const int32_t* __restrict__ win,
                                                         const int32_t* __restrict__ carry, int extra, int slots,
                                                         int pad, const int32_t* __restrict__ pending) {
  // pending (verify call, or NULL): only chains with pending[c] != 0 are listed -- the others have had their round
  // already (accept_early_kernel) and their a[c] is the next round's.
  // carry (draft call): chains whose x0a was handed over by the last round are not listed.  extra (verify call):
  // 1 = also list the last proposal sample yhat_b of a window that ends before K.  slots: slots per chain of x0hat.
  // pad (verify call; 0 = none): every chain's rows start at a multiple of `pad` rows -- its block is filled up with
  // repeats of its last row (same input, same output address, same value) -- so that a row tile of the model call
  // holds rows of few chains: what a tile of the mixture denoiser can leave out depends on how alike its rows are.
  __shared__ int s_wave[16];
  __shared__ int s_total;
  __shared__ int s_off[1024], s_cnt[1024], s_ac[1024];
  // A round starts here: advance the round index and clear this round's slot of the live-chain ring
  // (ring[0] = index of the next round, ring[1 + r % kLiveRing] = chains still unfinished after round r).
  if (threadIdx.x == 0 && blockIdx.x == 0 && ring) {
    const int r = ring[0];
    ring[0] = r + 1;
    ring[1 + (r % kLiveRing)] = 0;
    ring[1 + kLiveRing + (r % kLiveRing)] = 0;
  }
  __shared__ int s_pc[1024];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int base = 0, real = 0;
  for (int c0 = 0; c0 < B; c0 += 1024) {
    const int c = c0 + threadIdx.x;
    int ac = K, cnt = 0;
    if (c < B) {
      ac = min(max(a[c], 0), K);
      if (ac < K) {
        const int w = min(win ? win[c] : L, K - ac);
        cnt = (MODE == 0) ? ((carry && carry[c]) ? 0 : 1) : w - 1 + ((extra && ac + w < K) ? 1 : 0);
        if (MODE == 1 && pending && !pending[c]) cnt = 0;
      }
    }
    // rows of the chain's block (a window cut short by the end of the chain is not worth filling up: the blocks
    // behind it merely lose their alignment)
    const int pc = (MODE == 1 && pad > 0 && 2 * cnt > pad) ? (cnt + pad - 1) / pad * pad : cnt;
    if (MODE == 1 && pad > 0) {   // the rows asked for, without the filling
      (void)block_exclusive_scan(cnt, s_wave, &s_total);
      real += s_total;
      __syncthreads();
    }
    const int off = base + block_exclusive_scan(pc, s_wave, &s_total);
    if (MODE == 0) {
      if (cnt) {
        in_off[off] = ((int64_t)c * (K + 1) + ac) * d;
        out_off[off] = (int64_t)c * d;
        row_tau[off] = tau[ac];
        row_chain[off] = c;
      }
    } else {
      // the rows of a chain are written by a whole wavefront (consecutive entries, coalesced)
      s_off[threadIdx.x] = off;
      s_cnt[threadIdx.x] = cnt;
      s_pc[threadIdx.x] = pc;
      s_ac[threadIdx.x] = ac;
      __syncthreads();
      // (every workgroup of the launch computes the whole scan -- it is a thousand integers -- and fills the rows of
      // its share of the chains, so nothing has to pass between workgroups)
      for (int t = wave + 16 * (int)blockIdx.x; t < 1024 && c0 + t < B; t += 16 * (int)gridDim.x) {
        const int n_t = s_cnt[t], p_t = s_pc[t], o_t = s_off[t], a_t = s_ac[t], c_t = c0 + t;
        for (int s = 1 + lane; s <= p_t; s += 64) {
          const int sr = min(s, n_t);   // past the chain's rows: its last row again
          const int i = a_t + sr;
          in_off[o_t + s - 1] = ((int64_t)c_t * (K + 1) + i) * d;
          out_off[o_t + s - 1] = ((int64_t)c_t * slots + sr) * d;
          row_tau[o_t + s - 1] = tau[i];
          row_chain[o_t + s - 1] = c_t;
        }
      }
    }
    base += s_total;
    __syncthreads();
  }
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    *n_rows = base;
    if (row_counts) atomicAdd((unsigned long long*)&row_counts[MODE], (unsigned long long)((MODE == 1 && pad > 0) ? real : base));
  }
}

asd_status launch_plan_draft(asd_ctx* ctx, const int32_t* a, hipStream_t st, int32_t* ring) {
  ProfScope ps(ctx, ASD_PROF_PLAN, 0, st);
  hipLaunchKernelGGL(plan_rows_kernel<0>, dim3(1), dim3(1024), 0, st, ctx->B, ctx->K, ctx->L, ctx->d, a, ctx->tau,
                     ctx->in_off, ctx->out_off, ctx->row_tau, ctx->row_chain, ctx->n_rows_dev + 0, ring,
                     prof_counting(ctx) ? ctx->row_counts : nullptr, ctx->cur_win,
                     ctx->reuse_now ? ctx->carry : (const int32_t*)nullptr, 0, ctx->L, 0, (const int32_t*)nullptr);
  ASD_HIP(hipGetLastError());
  return ASD_OK;
}

asd_status launch_plan_verify(asd_ctx* ctx, const int32_t* a, hipStream_t st, const int32_t* pending) {
  if (ctx->L <= 1 && !ctx->reuse_now) return ASD_OK;
  ProfScope ps(ctx, ASD_PROF_PLAN, 1, st);
  // up to 64 workgroups share the filling of a large plan (a chain per wavefront at a time, see the kernel)
  const unsigned wgs = (unsigned)std::min<int64_t>(64, std::max<int64_t>(1, ctx->n_rows_max / 1024));
  hipLaunchKernelGGL(plan_rows_kernel<1>, dim3(wgs), dim3(1024), 0, st, ctx->B, ctx->K, ctx->L, ctx->d, a, ctx->tau,
                     ctx->in_off, ctx->out_off, ctx->row_tau, ctx->row_chain, ctx->n_rows_dev + 1, (int32_t*)nullptr,
                     prof_counting(ctx) ? ctx->row_counts : nullptr, ctx->cur_win, (const int32_t*)nullptr,
                     ctx->reuse_now ? 1 : 0, ctx->L + (ctx->reuse_now ? 1 : 0), ctx->cur_win ? 0 : model_row_block(ctx),
                     pending);
  ASD_HIP(hipGetLastError());
  return ASD_OK;
}

// ----------------------------------------------------------------------------
// Draft (Alg. 1, proposal loop): for k = 0..w-1, i = a+k,
//   yhat_{i+1} = c_x[i] yhat_i + c_0[i] x0a + sigma[i] xi_{i+1},
// written straight into traj[c][i+1].  A first-order linear recurrence along
// the window, independent per coordinate: one thread owns four coordinates and
// walks the window; rows are written coalesced.  HBM-bound: reads 2 rows,
// writes w rows per chain.
// ----------------------------------------------------------------------------
template <bool FOLD>  // FOLD: also list this chain's rows of the verify call and keep the round's books (see PlanOut)
__global__ __launch_bounds__(256) void draft_kernel(int K, int Lwin, int d, const Key* __restrict__ key_p,
                                                    const int32_t* __restrict__ a,
                                                    const float* __restrict__ c_x,
                                                    const float* __restrict__ c_0,
                                                    const float* __restrict__ sigma,
                                                    const float* __restrict__ x0a, float* __restrict__ traj,
                                                    const int32_t* __restrict__ win, PlanOut plan, int extra,
                                                    const int32_t* __restrict__ pending) {
  // extra (FOLD only): 1 = the verify call also evaluates yhat_b of a window that ends before K (slot w of
  // x0hat, which then has Lwin + 1 slots per chain).  pending (or NULL; not with FOLD): chains with pending[c] == 0
  // have had their round already (accept_early_kernel).
  const int c = blockIdx.y;
  const int blk = blockIdx.x * blockDim.x + threadIdx.x;
  const int nblk = (d + 3) >> 2;
  const int ac = a[c];
  const bool live = ac < K && ac >= 0 && !(pending && !pending[c]);
  const int w = live ? min(win ? win[c] : Lwin, K - ac) : 0;
  if (FOLD && blockIdx.x == 0) {
    // Bookkeeping of the round, once: the draft call has consumed its row count; the round index
    // advances and this round's slot of the live-chain ring starts at zero (the accept kernel adds to it).
    if (c == 0 && threadIdx.x == 0) {
      plan.n_rows[0] = 0;
      if (plan.ring) {
        const int r = plan.ring[0];
        plan.ring[0] = r + 1;
        plan.ring[1 + (r % kLiveRing)] = 0;
        plan.ring[1 + kLiveRing + (r % kLiveRing)] = 0;
      }
    }
    // This chain's rows of the verify call: the drafted samples of slots 1..w-1, read in place from the
    // trajectory, results to x0hat[c][slot].  One atomic add reserves the range; the first wavefront fills it.
    const int cnt = w - 1 + ((extra && live && ac + w < K) ? 1 : 0);
    if (threadIdx.x < 64 && cnt > 0) {
      int base = 0;
      if (threadIdx.x == 0) {
        base = atomicAdd(&plan.n_rows[1], cnt);
        if (plan.row_counts) atomicAdd((unsigned long long*)&plan.row_counts[1], (unsigned long long)cnt);
      }
      base = __shfl(base, 0, 64);
      for (int s = 1 + (int)threadIdx.x; s <= cnt; s += 64) {
        const int i = ac + s;
        plan.in_off[base + s - 1] = ((int64_t)c * (K + 1) + i) * d;
        plan.out_off[base + s - 1] = ((int64_t)c * (Lwin + extra) + s) * d;
        plan.row_tau[base + s - 1] = plan.tau[i];
        plan.row_chain[base + s - 1] = c;
      }
    }
  }
  if (blk >= nblk || !live) return;
  const Key key = *key_p;
  const bool vec = (d & 3) == 0;
  float* row = traj + ((int64_t)c * (K + 1) + ac) * d;
  float4 y = load4(row, blk, d, vec);
  const float4 g = load4(x0a + (int64_t)c * d, blk, d, vec);
  for (int k = 0; k < w; ++k) {
    const int i = ac + k;
    const float cx = c_x[i], c0 = c_0[i], sg = sigma[i];
    const float4 xi = normal4(key, (uint32_t)c, (uint32_t)(i + 1), (uint32_t)blk);
    y.x = fmaf(sg, xi.x, fmaf(cx, y.x, c0 * g.x));
    y.y = fmaf(sg, xi.y, fmaf(cx, y.y, c0 * g.y));
    y.z = fmaf(sg, xi.z, fmaf(cx, y.z, c0 * g.z));
    y.w = fmaf(sg, xi.w, fmaf(cx, y.w, c0 * g.w));
    row += d;
    store4(row, blk, d, vec, y);
  }
}

asd_status launch_draft(asd_ctx* ctx, float* traj, const int32_t* a, hipStream_t st, int32_t* ring, const int32_t* pending) {
  const int nblk = (ctx->d + 3) / 4;
  const int threads = nblk >= 256 ? 256 : (int)(ceil_div(nblk, 64) * 64);
  dim3 grid((unsigned)ceil_div(nblk, threads), (unsigned)ctx->B);
  ProfScope ps(ctx, ASD_PROF_DRAFT, 0, st);
  const PlanOut plan = plan_out(ctx, ring);
  if (plan.in_off)
    hipLaunchKernelGGL(draft_kernel<true>, grid, dim3(threads), 0, st, ctx->K, ctx->L, ctx->d, ctx->key_dev, a, ctx->c_x,
                       ctx->c_0, ctx->sigma, ctx->x0a, traj, ctx->cur_win, plan, ctx->reuse_now ? 1 : 0, (const int32_t*)nullptr);
  else
    hipLaunchKernelGGL(draft_kernel<false>, grid, dim3(threads), 0, st, ctx->K, ctx->L, ctx->d, ctx->key_dev, a, ctx->c_x,
                       ctx->c_0, ctx->sigma, ctx->x0a, traj, ctx->cur_win, plan, 0, pending);
  ASD_HIP(hipGetLastError());
  return ASD_OK;
}

// Sequential baseline: every chain takes step `step` (window of one).
__global__ void fill_i32_kernel(int n, int32_t v, int32_t* p) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

asd_status launch_plan_seq(asd_ctx* ctx, int32_t step, hipStream_t st) {
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)ceil_div(ctx->B, 256)), dim3(256), 0, st, ctx->B, step,
                     ctx->a);
  ASD_HIP(hipGetLastError());
  return launch_plan_draft(ctx, ctx->a, st);
}

asd_status launch_seq_step(asd_ctx* ctx, float* traj, int32_t step, hipStream_t st) {
  (void)step;
  const int nblk = (ctx->d + 3) / 4;
  const int threads = nblk >= 256 ? 256 : (int)(ceil_div(nblk, 64) * 64);
  dim3 grid((unsigned)ceil_div(nblk, threads), (unsigned)ctx->B);
  hipLaunchKernelGGL(draft_kernel<false>, grid, dim3(threads), 0, st, ctx->K, 1, ctx->d, ctx->key_dev, ctx->a, ctx->c_x,
                     ctx->c_0, ctx->sigma, ctx->x0a, traj, (const int32_t*)nullptr, PlanOut(), 0, (const int32_t*)nullptr);
  ASD_HIP(hipGetLastError());
  return ASD_OK;
}

// x0hat[c][0][:] = x0a[c][:]
__global__ void copy_slot0_kernel(int B, int L, int d, const float* __restrict__ x0a, float* __restrict__ x0hat) {
  const int c = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < d) x0hat[(int64_t)c * L * d + j] = x0a[(int64_t)c * d + j];
}

asd_status launch_copy_slot0(asd_ctx* ctx, float* x0hat, hipStream_t st) {
  dim3 grid((unsigned)ceil_div(ctx->d, 256), (unsigned)ctx->B);
  hipLaunchKernelGGL(copy_slot0_kernel, grid, dim3(256), 0, st, ctx->B, ctx->L, ctx->d, ctx->x0a, x0hat);
  ASD_HIP(hipGetLastError());
  return ASD_OK;
}

// ----------------------------------------------------------------------------
// Accept + scan + resample + advance.  One workgroup per chain; its size follows d
// (one thread per four coordinates, 1 to 16 wavefronts).
//
// The window is examined kAcceptChunk slots at a time, in order, and the walk stops at the
// chunk that holds the first rejection: Alg. 2 only needs the accepted prefix, and the slots
// behind the first rejection (most of the window, typically) are never read.
// Per chunk:
//   Alg. 3, accept test: with D = x0a - x0hat[k] (so v = c_0 D) every thread adds its
//   coordinates' share of <D, xi> and |D|^2 for each slot k of the chunk, regenerating
//   xi_{a+k+1} from the counter; the wavefront totals go to LDS and one thread per slot evaluates
//       rho = -( c_0 <D,xi> / sigma + c_0^2 |D|^2 / (2 sigma^2) ),
//       bit = [ log u_{a+k+1} <= rho ].
//   Slot 0 (step a+1) has v == 0 by construction and is accepted; a slot with
//   sigma == 0 is rejected (sigma -> 0 limit of the test).
//   Alg. 2: the wavefront ballots the chunk's bits and counts the trailing ones.
// Then (Alg. 3 reject branch + advance rule of Alg. 1): if n_acc < w the
//   row of step r = a + n_acc + 1 becomes
//       m + sigma (xi - 2 v <v,xi>/|v|^2) = yhat_r - D (c_0 + 2 sigma <D,xi>/|D|^2)
//   (using yhat = m + v + sigma xi), and a <- r; else a <- a + w.
// HBM-bound: reads x0a, the examined rows of x0hat and one trajectory row, writes one row.
// ----------------------------------------------------------------------------
constexpr int kAcceptChunk = 8;

template <bool FOLD>  // FOLD: also list this chain's row of the next round's draft call (see PlanOut)
__global__ __launch_bounds__(1024) void accept_kernel(int K, int L, int d, const Key* __restrict__ key_p,
                                                      int32_t* __restrict__ a,
                                                      const float* __restrict__ c_0,
                                                      const float* __restrict__ sigma,
                                                      float* x0a, int32_t* __restrict__ carry,
                                                      const float* __restrict__ x0hat, int x0_slots,
                                                      float* __restrict__ traj,
                                                      int32_t* __restrict__ accepted, float* __restrict__ stats,
                                                      int32_t* __restrict__ rounds, int32_t* __restrict__ live,
                                                      int32_t* __restrict__ win, PlanOut plan,
                                                      int64_t* __restrict__ prof_counts,
                                                      const int32_t* __restrict__ pending) {
  // pending (or NULL): chains with pending[c] == 0 have had their round already (accept_early_kernel)
  __shared__ float s_part[kAcceptChunk][16][2];  // per slot of the chunk, per wavefront: partial <D,xi>, |D|^2
  __shared__ float s_rej[2];                     // <D,xi>, |D|^2 of the first rejected slot
  __shared__ int s_first;                        // index inside the chunk of the first rejection, 64 if none

  const int c = blockIdx.x;
  const int tid = threadIdx.x;
  const int nthreads = blockDim.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int nwaves = nthreads >> 6;
  const int ac = a[c];
  // the verify call has consumed its row count: the draft kernel of the next round starts from zero
  if constexpr (FOLD) {
    if (c == 0 && tid == 0) plan.n_rows[1] = 0;
  }
  if (ac >= K || ac < 0) {
    if (tid == 0 && accepted) accepted[c] = -1;
    return;
  }
  if (pending && !pending[c]) return;
  const Key key = *key_p;
  const int w = min(win ? win[c] : L, K - ac);
  const int nblk = (d + 3) >> 2;
  const bool vec = (d & 3) == 0;
  const float* g_a = x0a + (int64_t)c * d;
  const float* g_w = x0hat + (int64_t)c * x0_slots * d;

  auto slot_terms = [&](float4 ga, float4 gk, float4 xi, float& dot, float& vv) {
    // coordinates past d load as zero in both rows, so they add nothing
    const float dx = ga.x - gk.x, dy = ga.y - gk.y, dz = ga.z - gk.z, dw = ga.w - gk.w;
    dot = fmaf(dx, xi.x, dot);
    dot = fmaf(dy, xi.y, dot);
    dot = fmaf(dz, xi.z, dot);
    dot = fmaf(dw, xi.w, dot);
    vv = fmaf(dx, dx, vv);
    vv = fmaf(dy, dy, vv);
    vv = fmaf(dz, dz, vv);
    vv = fmaf(dw, dw, vv);
  };
  const bool single = nblk <= nthreads;  // one coordinate block per thread: x0a stays in registers
  const float4 ga1 = (single && tid < nblk) ? load4(g_a, tid, d, vec) : make_float4(0.f, 0.f, 0.f, 0.f);

  int n_acc = w;
  int examined = 0;   // slots whose x0hat row was read for the test
  for (int base = 0; base < w; base += kAcceptChunk) {
    examined = min(w, base + kAcceptChunk) - 1;
    // every thread walks the chunk's slots over its own coordinate blocks; the loads of the slots are
    // independent, so a whole chunk of rows is in flight per wavefront
    float dot[kAcceptChunk], vv[kAcceptChunk];
#pragma unroll
    for (int kk = 0; kk < kAcceptChunk; ++kk) dot[kk] = vv[kk] = 0.f;
    if (single) {
      if (tid < nblk) {
#pragma unroll
        for (int kk = 0; kk < kAcceptChunk; ++kk) {
          const int k = base + kk;
          if (k >= 1 && k < w) {
            const float4 gk = load4(g_w + (int64_t)k * d, tid, d, vec);
            const float4 xi = normal4(key, (uint32_t)c, (uint32_t)(ac + k + 1), (uint32_t)tid);
            slot_terms(ga1, gk, xi, dot[kk], vv[kk]);
          }
        }
      }
    } else {
      for (int blk = tid; blk < nblk; blk += nthreads) {
        const float4 ga = load4(g_a, blk, d, vec);
#pragma unroll
        for (int kk = 0; kk < kAcceptChunk; ++kk) {
          const int k = base + kk;
          if (k >= 1 && k < w) {
            const float4 gk = load4(g_w + (int64_t)k * d, blk, d, vec);
            const float4 xi = normal4(key, (uint32_t)c, (uint32_t)(ac + k + 1), (uint32_t)blk);
            slot_terms(ga, gk, xi, dot[kk], vv[kk]);
          }
        }
      }
    }
#pragma unroll
    for (int kk = 0; kk < kAcceptChunk; ++kk) {
      const float ds = wave_sum(dot[kk]), vs = wave_sum(vv[kk]);
      if (lane == 0) {
        s_part[kk][wave][0] = ds;
        s_part[kk][wave][1] = vs;
      }
    }
    __syncthreads();

    // Alg. 3 accept test, one thread per slot of the chunk
    if (tid < 64) {
      const int k = base + lane;
      const bool valid = lane < kAcceptChunk && k < w;
      float sd = 0.f, sv = 0.f, rho = -INFINITY, logu = 0.f;
      int bit = 1;  // slot 0, and the lanes that stand for no slot
      if (valid && k >= 1) {
        for (int q = 0; q < nwaves; ++q) {
          sd += s_part[lane][q][0];
          sv += s_part[lane][q][1];
        }
        const int i = ac + k;
        const float sg = sigma[i], c0 = c_0[i];
        bit = 0;
        if (sg > 0.f) {
          const float vxi = c0 * sd;
          const float v2 = c0 * c0 * sv;
          rho = -(vxi / sg + v2 / (2.0f * sg * sg));
          logu = logf(uniform1(key, (uint32_t)c, (uint32_t)(i + 1)));
          bit = (logu <= rho) ? 1 : 0;
        }
      }
      if (stats && valid) {
        float* sp = stats + ((int64_t)c * L + k) * 4;
        sp[0] = sd;
        sp[1] = sv;
        sp[2] = (k == 0) ? 0.f : logu;
        sp[3] = (k == 0) ? 0.f : rho;
      }
      // Alg. 2: accepted prefix = trailing ones of the ballot
      const unsigned long long inv = ~__ballot(bit);
      const int first = inv ? (__ffsll((long long)inv) - 1) : 64;
      if (lane == first) {
        s_rej[0] = sd;
        s_rej[1] = sv;
      }
      if (lane == 0) s_first = first;
    }
    __syncthreads();
    if (s_first < 64) {
      n_acc = base + s_first;
      break;
    }
  }

  int a_next;
  if (n_acc < w) {
    const int k = n_acc;  // slot index of the first rejection (>= 1)
    const int i = ac + k;
    const float sg = sigma[i], c0 = c_0[i];
    const float dotr = s_rej[0], vvr = s_rej[1];
    const float coef = (vvr > 0.f) ? (c0 + 2.0f * sg * dotr / vvr) : 0.f;
    const float* g_k = g_w + (int64_t)k * d;
    float* row = traj + ((int64_t)c * (K + 1) + i + 1) * d;
    for (int blk = tid; blk < nblk; blk += nthreads) {
      const float4 ga = load4(g_a, blk, d, vec);
      const float4 gk = load4(g_k, blk, d, vec);
      float4 y = load4(row, blk, d, vec);
      y.x = fmaf(-(ga.x - gk.x), coef, y.x);
      y.y = fmaf(-(ga.y - gk.y), coef, y.y);
      y.z = fmaf(-(ga.z - gk.z), coef, y.z);
      y.w = fmaf(-(ga.w - gk.w), coef, y.w);
      store4(row, blk, d, vec, y);
    }
    a_next = i + 1;
  } else {
    a_next = ac + w;
  }
  // Model-call reuse: the whole window was accepted, so the next round starts at yhat_b, where the verify call
  // has already evaluated the model (slot w): that value becomes x0a and the chain skips the next draft call.
  // (Every read of x0a by this workgroup lies before the barrier that ended the last group of slots.)
  const bool carried = carry && n_acc == w && a_next < K;
  if (carried) {
    const float* g_e = g_w + (int64_t)w * d;
    for (int blk = tid; blk < nblk; blk += nthreads) store4(x0a + (int64_t)c * d, blk, d, vec, load4(g_e, blk, d, vec));
  }
  if (tid == 0) {
    a[c] = a_next;
    if (carry) carry[c] = carried ? 1 : 0;
    if (prof_counts) {
      atomicAdd((unsigned long long*)&prof_counts[2], (unsigned long long)examined);
      if (n_acc < w) atomicAdd((unsigned long long*)&prof_counts[3], 1ull);
    }
    if (accepted) accepted[c] = n_acc;
    if (rounds) rounds[c] += 1;
    if (win) {
      const int B = gridDim.x;
      const int st = window_next(win[B + c], w, n_acc);
      win[B + c] = st;
      win[c] = window_of(st, L);
    }
    // the round index was advanced at the start of this round
    if (live && a_next < K) atomicAdd(&live[1 + ((live[0] - 1) % kLiveRing)], 1);
    if constexpr (FOLD) if (a_next < K && !carried) {  // this chain's row of the next round's draft call
      const int idx = atomicAdd(&plan.n_rows[0], 1);
      plan.in_off[idx] = ((int64_t)c * (K + 1) + a_next) * d;
      plan.out_off[idx] = (int64_t)c * d;
      plan.row_tau[idx] = plan.tau[a_next];
      plan.row_chain[idx] = c;
      if (plan.row_counts) atomicAdd((unsigned long long*)&plan.row_counts[0], 1ull);
    }
  }
}

// ----------------------------------------------------------------------------
// Draft and accept stage in one, ahead of the draft kernel and the verify call, for chains whose rows the mixture
// denoiser's one-hot certificate covers (gmm_cert.h).  A certified row's model value is c_x' x + c_m' mu_b -- the
// same bits the verify call would store for it -- and a drafted row is a recurrence on the row before it, so a
// workgroup walks its chain's window in registers: it drafts slot k from slot k - 1 (draft_kernel's expression, with
// the noise the accept test of slot k - 1 has just used), certifies it, forms its model value and takes the accept
// test -- the same sums, in the same order, as accept_kernel on stored values, hence the same decisions and the
// same resampled row.  It stops at the first rejection like accept_kernel; what lies behind is neither drafted nor
// read, nothing goes to x0hat, and only the rows the chain keeps go to the trajectory.  A chain commits only if
// every slot up to and including its first rejection (all of them, if none is rejected) passes the certificate; any
// other chain is left with pending[c] = 1 and unchanged state (rows already stored are the drafts draft_kernel stores
// again) and goes through draft_kernel, the verify call and accept_kernel as before: all three take the pending
// chains only.  One coordinate block per thread (d a multiple of 4, d / 4 <= 256).
// ----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void accept_early_kernel(int K, int L, int d, const Key* __restrict__ key_p,
                                                           int32_t* __restrict__ a,
                                                           const float* __restrict__ c_x,
                                                           const float* __restrict__ c_0,
                                                           const float* __restrict__ sigma,
                                                           const int32_t* __restrict__ tau_tab,
                                                           const float* __restrict__ x0a, float* __restrict__ traj,
                                                           int32_t* __restrict__ rounds, int32_t* __restrict__ live,
                                                           int32_t* __restrict__ win, OneHotCert oc,
                                                           int32_t* __restrict__ pending, int light,
                                                           int64_t* __restrict__ prof_counts) {
  // live: [0] round index (advanced at the start of this round), then the ring of chains unfinished after a round,
  // then the ring of chains a round left pending.  light: this kernel is the round (the host has seen rounds without
  // pending chains and launches neither the draft call nor anything behind this kernel): the model value at y_a is
  // formed here like the others, if y_a passes the certificate; a pending chain simply waits for the next full round,
  // and counts as unfinished here because no accept kernel will count it.
  __shared__ float s_part[kAcceptChunk][4][4];   // per slot of the chunk, per wavefront: <D,xi>, |D|^2, <x,mu_b>, |x|^2
  __shared__ float s_r2[kAcceptChunk][4];        // ... |x - s mu_b|^2
  __shared__ float s_s[kAcceptChunk];            // s = <x,mu_b> / |mu_b|^2 of every slot
  __shared__ float s_rej[2];
  __shared__ int s_first, s_fail;

  const int c = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
  const int ac = a[c];
  if (ac >= K || ac < 0) {
    if (tid == 0) pending[c] = 0;
    return;
  }
  const int w = min(win ? win[c] : L, K - ac);
  // is the chain worth a try: a candidate, and a first slot (the noisiest) whose time index does not rule it out
  const int b = oc.chain_comp[c];
  bool go = w > 1 && b >= 0 && b < oc.C;
  float am = 0.f;
  if (go) {
    am = oc.a_min[b];
    go = cert_worth_reading(oc.coef_tau[tau_tab[ac + 1]], am, d);
  }
  auto leave_pending = [&]() {
    if (tid == 0) {
      pending[c] = 1;
      if (live) {
        const int slot = (live[0] - 1) % kLiveRing;
        atomicAdd(&live[1 + kLiveRing + slot], 1);
        if (light) atomicAdd(&live[1 + slot], 1);
      }
    }
  };
  if (!go) {
    leave_pending();
    return;
  }
  const Key key = *key_p;
  const int nblk = d >> 2;
  const bool mine = tid < nblk;
  const float qb = oc.musq[b], bias_b = kCertLog2e * oc.log_w[b];
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  const float4 mv = mine ? load4(oc.means + (int64_t)b * d, tid, d, true) : zero4;
  float* rows = traj + ((int64_t)c * (K + 1) + ac) * d;   // slot k's row: yhat_{a+k}, row k from here
  float4 y = mine ? load4(rows, tid, d, true) : zero4;    // yhat_a = y_a; then the last row drafted
  float4 ga1;                                             // x0a: the model value at y_a
  if (!light) {
    ga1 = mine ? load4(x0a + (int64_t)c * d, tid, d, true) : zero4;
  } else {
    // no draft call in this round: y_a is certified here and its value formed as gmm_certify_kernel would have
    const float4 cf0 = oc.coef_tau[tau_tab[ac]];
    const float p0 = wave_sum((y.x * mv.x + y.y * mv.y) + (y.z * mv.z + y.w * mv.w));
    const float x0 = wave_sum((y.x * y.x + y.y * y.y) + (y.z * y.z + y.w * y.w));
    if (lane == 0) {
      s_part[0][wave][2] = p0;
      s_part[0][wave][3] = x0;
    }
    __syncthreads();
    float ps = 0.f, xs = 0.f;
    for (int q = 0; q < nwaves; ++q) {
      ps += s_part[0][q][2];
      xs += s_part[0][q][3];
    }
    const float s0 = ps / qb;
    const float ex = fmaf(-s0, mv.x, y.x), ey = fmaf(-s0, mv.y, y.y), ez = fmaf(-s0, mv.z, y.z), ew = fmaf(-s0, mv.w, y.w);
    const float r0 = wave_sum((ex * ex + ey * ey) + (ez * ez + ew * ew));
    if (lane == 0) s_r2[0][wave] = r0;
    __syncthreads();
    float rs = 0.f;
    for (int q = 0; q < nwaves; ++q) rs += s_r2[0][q];
    __syncthreads();   // the sums are read; the slots' sums go to the same places
    if (!cert_passes(cf0, s0, rs, xs, am, qb, bias_b, oc.glob, oc.globw)) {   // (the same for every thread)
      leave_pending();
      return;
    }
    ga1 = cert_value(cf0, y, mv);
  }
  float4 xi_d = normal4(key, (uint32_t)c, (uint32_t)(ac + 1), (uint32_t)tid);   // the noise of the next draft step

  auto slot_terms = [&](float4 ga, float4 gk, float4 xi, float& dot, float& vv) {   // as in accept_kernel
    const float dx = ga.x - gk.x, dy = ga.y - gk.y, dz = ga.z - gk.z, dw = ga.w - gk.w;
    dot = fmaf(dx, xi.x, dot);
    dot = fmaf(dy, xi.y, dot);
    dot = fmaf(dz, xi.z, dot);
    dot = fmaf(dw, xi.w, dot);
    vv = fmaf(dx, dx, vv);
    vv = fmaf(dy, dy, vv);
    vv = fmaf(dz, dz, vv);
    vv = fmaf(dw, dw, vv);
  };
  auto draft_step = [&](int i, float4 from, float4 xi) -> float4 {   // yhat_{i+1} from yhat_i: as in draft_kernel
    const float cx = c_x[i], c0 = c_0[i], sg = sigma[i];
    return make_float4(fmaf(sg, xi.x, fmaf(cx, from.x, c0 * ga1.x)), fmaf(sg, xi.y, fmaf(cx, from.y, c0 * ga1.y)),
                       fmaf(sg, xi.z, fmaf(cx, from.z, c0 * ga1.z)), fmaf(sg, xi.w, fmaf(cx, from.w, c0 * ga1.w)));
  };

  int n_acc = w, examined = 0, base = 0;
  float4 xk[kAcceptChunk];
#pragma unroll
  for (int kk = 0; kk < kAcceptChunk; ++kk) xk[kk] = zero4;
  for (; base < w; base += kAcceptChunk) {
    examined = min(w, base + kAcceptChunk) - 1;
    float dot[kAcceptChunk], vv[kAcceptChunk], pp[kAcceptChunk], xx[kAcceptChunk];
#pragma unroll
    for (int kk = 0; kk < kAcceptChunk; ++kk) dot[kk] = vv[kk] = pp[kk] = xx[kk] = 0.f;
    if (mine) {
#pragma unroll
      for (int kk = 0; kk < kAcceptChunk; ++kk) {
        const int k = base + kk;
        if (k >= 1 && k < w) {
          const float4 x = draft_step(ac + k - 1, y, xi_d);   // yhat_{a+k}
          y = x;
          xk[kk] = x;
          const float4 cf = oc.coef_tau[tau_tab[ac + k]];
          const float4 gk = cert_value(cf, x, mv);
          const float4 xi = normal4(key, (uint32_t)c, (uint32_t)(ac + k + 1), (uint32_t)tid);
          xi_d = xi;
          slot_terms(ga1, gk, xi, dot[kk], vv[kk]);
          pp[kk] = (x.x * mv.x + x.y * mv.y) + (x.z * mv.z + x.w * mv.w);
          xx[kk] = (x.x * x.x + x.y * x.y) + (x.z * x.z + x.w * x.w);
        }
      }
    }
#pragma unroll
    for (int kk = 0; kk < kAcceptChunk; ++kk) {
      const float ds = wave_sum(dot[kk]), vs = wave_sum(vv[kk]), ps = wave_sum(pp[kk]), xs = wave_sum(xx[kk]);
      if (lane == 0) {
        s_part[kk][wave][0] = ds;
        s_part[kk][wave][1] = vs;
        s_part[kk][wave][2] = ps;
        s_part[kk][wave][3] = xs;
      }
    }
    __syncthreads();
    if (tid < kAcceptChunk) {
      float p = 0.f;
      for (int q = 0; q < nwaves; ++q) p += s_part[tid][q][2];
      s_s[tid] = p / qb;   // any s is valid: its rounding does not matter
    }
    __syncthreads();
    {
      float r2[kAcceptChunk];
#pragma unroll
      for (int kk = 0; kk < kAcceptChunk; ++kk) {
        const float s = s_s[kk];
        const float ex = fmaf(-s, mv.x, xk[kk].x), ey = fmaf(-s, mv.y, xk[kk].y);
        const float ez = fmaf(-s, mv.z, xk[kk].z), ew = fmaf(-s, mv.w, xk[kk].w);
        r2[kk] = wave_sum((ex * ex + ey * ey) + (ez * ez + ew * ew));
      }
      if (lane == 0) {
#pragma unroll
        for (int kk = 0; kk < kAcceptChunk; ++kk) s_r2[kk][wave] = r2[kk];
      }
    }
    __syncthreads();

    // Alg. 3 accept test (as in accept_kernel) and the certificate, one thread per slot of the chunk
    if (tid < 64) {
      const int k = base + lane;
      const bool valid = lane < kAcceptChunk && k < w;
      float sd = 0.f, sv = 0.f;
      int bit = 1, uncert = 0;
      if (valid && k >= 1) {
        float xs = 0.f, rs = 0.f;
        for (int q = 0; q < nwaves; ++q) {
          sd += s_part[lane][q][0];
          sv += s_part[lane][q][1];
          xs += s_part[lane][q][3];
          rs += s_r2[lane][q];
        }
        const int i = ac + k;
        const float sg = sigma[i], c0 = c_0[i];
        bit = 0;
        if (sg > 0.f) {
          const float vxi = c0 * sd;
          const float v2 = c0 * c0 * sv;
          const float rho = -(vxi / sg + v2 / (2.0f * sg * sg));
          const float logu = logf(uniform1(key, (uint32_t)c, (uint32_t)(i + 1)));
          bit = (logu <= rho) ? 1 : 0;
        }
        uncert = cert_passes(oc.coef_tau[tau_tab[i]], s_s[lane], rs, xs, am, qb, bias_b, oc.glob, oc.globw) ? 0 : 1;
      }
      const unsigned long long inv = ~__ballot(bit);
      const int first = inv ? (__ffsll((long long)inv) - 1) : 64;
      const unsigned long long bad = __ballot(uncert);
      const unsigned long long need = first < 63 ? ((2ull << first) - 1ull) : ~0ull;   // slots up to the first rejection
      if (lane == first) {
        s_rej[0] = sd;
        s_rej[1] = sv;
      }
      if (lane == 0) {
        s_first = first;
        s_fail = (bad & need) ? 1 : 0;
      }
    }
    __syncthreads();
    if (s_fail) {   // a slot that matters is not certified: the chain takes the verify call
      leave_pending();
      return;
    }
    // the rows the chain keeps of this chunk: up to the slot of the first rejection, all of them if there is none
    if (mine) {
#pragma unroll
      for (int kk = 0; kk < kAcceptChunk; ++kk) {
        const int k = base + kk;
        if (k >= 1 && k < w && kk <= s_first) store4(rows + (int64_t)k * d, tid, d, true, xk[kk]);
      }
    }
    if (s_first < 64) {
      n_acc = base + s_first;
      break;
    }
  }

  int a_next;
  if (n_acc < w) {
    const int k = n_acc;  // slot index of the first rejection (>= 1), in the chunk at `base`
    const int i = ac + k;
    const float sg = sigma[i], c0 = c_0[i];
    const float dotr = s_rej[0], vvr = s_rej[1];
    const float coef = (vvr > 0.f) ? (c0 + 2.0f * sg * dotr / vvr) : 0.f;
    if (mine) {
      float4 x = xk[0];
#pragma unroll
      for (int kk = 1; kk < kAcceptChunk; ++kk)
        if (kk == k - base) x = xk[kk];
      const float4 gk = cert_value(oc.coef_tau[tau_tab[i]], x, mv);
      // the drafted yhat_{i+1}, reflected
      float4 yr = draft_step(i, x, normal4(key, (uint32_t)c, (uint32_t)(i + 1), (uint32_t)tid));
      yr.x = fmaf(-(ga1.x - gk.x), coef, yr.x);
      yr.y = fmaf(-(ga1.y - gk.y), coef, yr.y);
      yr.z = fmaf(-(ga1.z - gk.z), coef, yr.z);
      yr.w = fmaf(-(ga1.w - gk.w), coef, yr.w);
      store4(rows + (int64_t)(k + 1) * d, tid, d, true, yr);
    }
    a_next = i + 1;
  } else {
    // the whole window: its last proposal sample yhat_{a+w} is the next round's start
    if (mine) store4(rows + (int64_t)w * d, tid, d, true, draft_step(ac + w - 1, y, xi_d));
    a_next = ac + w;
  }
  if (tid == 0) {
    a[c] = a_next;
    pending[c] = 0;
    if (prof_counts) {
      atomicAdd((unsigned long long*)&prof_counts[1], (unsigned long long)(w - 1));   // the window's rows, as the plan counts them
      atomicAdd((unsigned long long*)&prof_counts[2], (unsigned long long)examined);
      if (n_acc < w) atomicAdd((unsigned long long*)&prof_counts[3], 1ull);
      atomicAdd((unsigned long long*)&prof_counts[4], (unsigned long long)examined);
      atomicAdd((unsigned long long*)&prof_counts[5], 1ull);
      atomicAdd((unsigned long long*)&prof_counts[6], (unsigned long long)(w - 1));
      if (n_acc < w) atomicAdd((unsigned long long*)&prof_counts[7], 1ull);
    }
    if (rounds) rounds[c] += 1;
    if (win) {
      const int B = gridDim.x;
      const int st = window_next(win[B + c], w, n_acc);
      win[B + c] = st;
      win[c] = window_of(st, L);
    }
    // the round index was advanced at the start of this round
    if (live && a_next < K) atomicAdd(&live[1 + ((live[0] - 1) % kLiveRing)], 1);
  }
}

asd_status launch_accept_early(asd_ctx* ctx, float* traj, int32_t* a, int32_t* rounds, int32_t* live, hipStream_t st,
                               bool light) {
  OneHotCert oc;
  if (!model_onehot_cert(ctx, &oc) || ctx->d % 4 != 0 || ctx->d / 4 > 256 || !ctx->pending)
    return ASD_ESTATE;
  ProfScope ps(ctx, ASD_PROF_ACCEPT_EARLY, 0, st);
  const int threads = (int)(ceil_div(ctx->d / 4, 64) * 64);
  hipLaunchKernelGGL(accept_early_kernel, dim3(ctx->B), dim3(threads), 0, st, ctx->K, ctx->L, ctx->d, ctx->key_dev, a,
                     ctx->c_x, ctx->c_0, ctx->sigma, ctx->tau, ctx->x0a, traj, rounds, live, ctx->cur_win, oc, ctx->pending, light ? 1 : 0,
                     prof_counting(ctx) ? ctx->row_counts : nullptr);
  ASD_HIP(hipGetLastError());
  return ASD_OK;
}

asd_status launch_accept(asd_ctx* ctx, float* traj, int32_t* a, const float* x0hat, int x0_slots, int32_t* accepted,
                         float* stats, int32_t* rounds, int32_t* live, hipStream_t st, const int32_t* pending) {
  ProfScope ps(ctx, ASD_PROF_ACCEPT, 0, st);
  const int nblk = (ctx->d + 3) / 4;
  const int threads = (int)std::min<int64_t>(1024, ceil_div(nblk, 64) * 64);
  const PlanOut plan = plan_out(ctx, nullptr);
  int64_t* prof_counts = prof_counting(ctx) ? ctx->row_counts : nullptr;
  int32_t* carry = ctx->reuse_now ? ctx->carry : nullptr;
  if (plan.in_off)
    hipLaunchKernelGGL(accept_kernel<true>, dim3(ctx->B), dim3(threads), 0, st, ctx->K, ctx->L, ctx->d, ctx->key_dev, a,
                       ctx->c_0, ctx->sigma, ctx->x0a, carry, x0hat, x0_slots, traj, accepted, stats, rounds, live,
                       ctx->cur_win, plan, prof_counts, pending);
  else
    hipLaunchKernelGGL(accept_kernel<false>, dim3(ctx->B), dim3(threads), 0, st, ctx->K, ctx->L, ctx->d, ctx->key_dev, a,
                       ctx->c_0, ctx->sigma, ctx->x0a, carry, x0hat, x0_slots, traj, accepted, stats, rounds, live,
                       ctx->cur_win, plan, prof_counts, pending);
  ASD_HIP(hipGetLastError());
  return ASD_OK;
}

// ----------------------------------------------------------------------------
// debug: raw generator words / normals / uniform of one (chain, step)
// ----------------------------------------------------------------------------
__global__ void debug_philox_kernel(Key key, uint32_t chain, uint32_t step, uint32_t stream_id, int nblk,
                                    uint32_t* out) {
  const int blk = blockIdx.x * blockDim.x + threadIdx.x;
  if (blk >= nblk) return;
  const uint4 w = philox4x32_10(make_uint4((uint32_t)blk, step, chain, stream_id), key);
  out[4 * blk + 0] = w.x;
  out[4 * blk + 1] = w.y;
  out[4 * blk + 2] = w.z;
  out[4 * blk + 3] = w.w;
}

__global__ void debug_randoms_kernel(Key key, uint32_t chain, uint32_t step, int d, float* xi, float* u) {
  const int blk = blockIdx.x * blockDim.x + threadIdx.x;
  const int nblk = (d + 3) >> 2;
  if (blk < nblk && xi) store4(xi, blk, d, false, normal4(key, chain, step, (uint32_t)blk));
  if (blk == 0 && u) u[0] = uniform1(key, chain, step);
}

asd_status launch_debug_philox(Key key, uint32_t chain, uint32_t step, uint32_t stream_id, int32_t nblk,
                               uint32_t* out, hipStream_t st) {
  hipLaunchKernelGGL(debug_philox_kernel, dim3((unsigned)ceil_div(nblk, 256)), dim3(256), 0, st, key, chain,
                     step, stream_id, nblk, out);
  ASD_HIP(hipGetLastError());
  return ASD_OK;
}

asd_status launch_debug_randoms(Key key, uint32_t chain, uint32_t step, int32_t d, float* xi, float* u,
                                hipStream_t st) {
  const int nblk = (d + 3) / 4;
  hipLaunchKernelGGL(debug_randoms_kernel, dim3((unsigned)ceil_div(nblk > 0 ? nblk : 1, 256)), dim3(256), 0, st,
                     key, chain, step, d, xi, u);
  ASD_HIP(hipGetLastError());
  return ASD_OK;
}

}  // namespace asd
