// Chain-resident ASD sampler for Gaussian-mixture denoisers that fit in LDS.
//
// For small shapes a round of ASD is a handful of microsecond kernels and the
// sample is bound by launches, not by arithmetic.  Chains never interact, so here
// one workgroup runs the *whole* of Alg. 1 for one chain in a single launch:
// the mixture, the window of proposal samples, the model values and the noise of
// the window live in LDS, and the only HBM traffic is the trajectory rows the
// round produces.  Per round (notation of Alg. 1, x0-prediction form):
//   A. wavefront 0 evaluates x0a = D(y_a, tau_a); meanwhile the other wavefronts
//      generate xi_{a+1..b} and log u_{a+2..b} of the window from the counter
//      (they do not depend on x0a);
//   B. draft: yhat_{i+1} = c_x yhat_i + c_0 x0a + sigma xi_{i+1}, a thread per
//      four coordinates walks the window; rows go to LDS and to the trajectory;
//   C. verify: x0_i = D(yhat_i, tau_i), i = a+1..b-1, one row per wavefront at a
//      time;
//   D. Alg. 3 accept test per slot (a wavefront per slot reduces <D,xi>, |D|^2),
//      Alg. 2 as ballot + trailing ones, reflection of the first rejected row,
//      advance.
// The arithmetic of every step is the one of the stand-alone kernels (same
// formulas, same counters), so the same parity bars apply.  Every wavefront
// leaves the loop when its chain reaches K, which takes at most K rounds.
#include <type_traits>

#include "common.h"
#include "device_util.h"
#include "gmm_state.h"

namespace asd {

namespace {

// Stage timing for development (-DASD_CHAIN_TIMING): thread 0 of chain 0 prints the cycles it spent
// up to each mark, summed over rounds.
#ifdef ASD_CHAIN_TIMING
#define ASD_T_DECL long long t_acc[6] = {0, 0, 0, 0, 0, 0}; long long t_prev = clock64();
#define ASD_T(i) { const long long t_now = clock64(); t_acc[i] += t_now - t_prev; t_prev = t_now; }
#define ASD_T_END if (tid == 0 && c == 0) printf("chain timing: rounds %d cycles loop-top %lld A %lld B %lld C %lld D %lld tail %lld | single-row passes %llu %llu %llu\n", R, t_acc[0], t_acc[1], t_acc[2], t_acc[3], t_acc[4], t_acc[5], g_t2[0], g_t2[1], g_t2[2]);
__device__ unsigned long long g_t2[4];
#define ASD_T2_DECL long long u_prev = clock64();
#define ASD_T2(i) if (R == 1 && blockIdx.x == 0) { const long long u_now = clock64(); if (lane == 0) atomicAdd(&g_t2[i], (unsigned long long)(u_now - u_prev)); u_prev = u_now; }
#else
#define ASD_T_DECL
#define ASD_T(i)
#define ASD_T_END
#define ASD_T2_DECL
#define ASD_T2(i)
#endif

struct ChainLayout {
  int dq, dp, C4, nblk;
  size_t m, q, lw, ps, yh, x0, xi, sch, total;  // offsets in floats
};

__host__ __device__ inline ChainLayout chain_layout(int C, int d, int L, int K) {
  ChainLayout l;
  l.dq = (d + 3) & ~3;   // rows are padded to whole blocks of four coordinates (padding is zero or unused)
  l.dp = l.dq + 4;       // mixture rows: 16 lanes reading one 16-byte column of 16 rows hit 16 bank groups
  l.C4 = (C + 3) & ~3;
  l.nblk = l.dq >> 2;
  l.m = 0;
  l.q = l.m + (size_t)C * l.dp;
  l.lw = l.q + l.C4;
  l.ps = l.lw + l.C4;
  l.yh = l.ps + (size_t)(L + 4) * l.C4;   // logits / softmax weights, a region per group of rows
  l.x0 = l.yh + (size_t)(L + 1) * l.dq;
  l.xi = l.x0 + (size_t)L * l.dq;
  l.sch = l.xi + (size_t)L * l.dq;  // [K][8]: (c_x, c_0, sigma, -, kappa, gamma, cx, cm) of step i
  l.total = l.sch + (size_t)K * 8;
  return l;
}

// D(x, tau) for R consecutive rows held in LDS, by one wavefront (all 64 lanes must call):
//   pass 1: lane = component: logit_k = kappa <x, mu_k> - gamma |mu_k|^2 + log w_k,
//   pass 2: softmax over the C logits,
//   pass 3: lane = coordinate: out_j = cx x_j + cm sum_k p_k mu_k[j].
// LDS delivers 64 lanes x 16 bytes per read instruction whether or not the lanes ask for the same
// address, so the wavefront-uniform operand of each pass (x in pass 1, p in pass 3) is not read per
// use: 64 of its values are fetched once into a register, one per lane, and handed to the FMAs as
// scalars (v_readlane).  The mixture is then the only LDS stream, and it is shared by the R rows.
// The order of the additions is that of the stand-alone row-wise kernel.
template <int R>
__device__ __forceinline__ void gmm_rows_lds(const float* xs, float* out, const float4 (&cf)[R], const float* m_l,
                                             const float* q_l, const float* lw_l, float* ps, int C,
                                             const ChainLayout& l, int d, int lane) {
  const int dq = l.dq, dp = l.dp, C4 = l.C4;
  ASD_T2_DECL
  float mx[R];
#pragma unroll
  for (int r = 0; r < R; ++r) mx[r] = -INFINITY;
  // four groups of 64 components per sweep over x: a coordinate is made scalar once for all of them
  for (int kg = 0; kg < C; kg += 256) {
    const float* mk[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) mk[g] = m_l + min(kg + 64 * g + lane, C - 1) * dp;
    float dot[R][4];
#pragma unroll
    for (int r = 0; r < R; ++r) dot[r][0] = dot[r][1] = dot[r][2] = dot[r][3] = 0.f;
    for (int c64 = 0; c64 < dq; c64 += 64) {
      int xv[R];
#pragma unroll
      for (int r = 0; r < R; ++r) xv[r] = (c64 + lane < dq) ? __float_as_int(xs[r * dq + c64 + lane]) : 0;
      const int nj = min(64, dq - c64);
      auto step = [&](int j) {
        float x[R][4];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int i = 0; i < 4; ++i) x[r][i] = __int_as_float(__builtin_amdgcn_readlane(xv[r], j + i));
        // (groups past C read the last row again and are dropped below: no branch between the reads)
        float4 mv[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) mv[g] = *reinterpret_cast<const float4*>(&mk[g][c64 + j]);
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int r = 0; r < R; ++r)
            dot[r][g] = fmaf(x[r][0], mv[g].x, fmaf(x[r][1], mv[g].y, fmaf(x[r][2], mv[g].z, fmaf(x[r][3], mv[g].w, dot[r][g]))));
      };
      if (nj == 64) {  // a whole chunk: constant lane selects
#pragma unroll
        for (int j = 0; j < 64; j += 4) step(j);
      } else {
        for (int j = 0; j < nj; j += 4) step(j);
      }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int k = kg + 64 * g + lane;
      if (k < C) {
        const float qk = q_l[k], lwk = lw_l[k];
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const float lg = fmaf(cf[r].x, dot[r][g], fmaf(-cf[r].y, qk, lwk));
          ps[r * C4 + k] = lg;
          mx[r] = fmaxf(mx[r], lg);
        }
      }
    }
  }
  ASD_T2(0)
  float sc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const float m = wave_max(mx[r]);
    float sum = 0.f;
    for (int k = lane; k < C4; k += 64) {
      const float p = (k < C) ? expf(ps[r * C4 + k] - m) : 0.f;
      ps[r * C4 + k] = p;
      sum += p;
    }
    sc[r] = cf[r].w / wave_sum(sum);
  }
  ASD_T2(1)
  // (LDS operations of one wavefront complete in order: ps is visible to all its lanes here)
  for (int j0 = 0; j0 < dq; j0 += 64) {
    const int j = j0 + lane;
    const float* mj = m_l + min(j, dq - 1);
    float acc[R][4];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r][0] = acc[r][1] = acc[r][2] = acc[r][3] = 0.f;
    for (int k64 = 0; k64 < C4; k64 += 64) {
      int pv[R];
#pragma unroll
      for (int r = 0; r < R; ++r) pv[r] = (k64 + lane < C4) ? __float_as_int(ps[r * C4 + k64 + lane]) : 0;
      const int nk = min(64, C4 - k64);
      // N components per step: their mixture values are all requested before the first is used.
      // Rows past C do not exist: their weights are 0 and the reads are clamped to the last row.
      auto step = [&](int kk, auto n_tag, auto full_tag) {
        constexpr int N = decltype(n_tag)::value;
        constexpr bool FULL = decltype(full_tag)::value;
        float m[N];
#pragma unroll
        for (int i = 0; i < N; ++i) m[i] = mj[(FULL ? (k64 + kk + i) : min(k64 + kk + i, C - 1)) * dp];
#pragma unroll
        for (int i = 0; i < N; ++i)
#pragma unroll
          for (int r = 0; r < R; ++r)
            acc[r][i & 3] = fmaf(__int_as_float(__builtin_amdgcn_readlane(pv[r], kk + i)), m[i], acc[r][i & 3]);
      };
      using I4 = std::integral_constant<int, 4>;
      using I16 = std::integral_constant<int, 16>;
      if (k64 + 64 <= C) {
#pragma unroll
        for (int kk = 0; kk < 64; kk += 16) step(kk, I16{}, std::true_type{});
      } else {
        for (int kk = 0; kk < nk; kk += 4) step(kk, I4{}, std::false_type{});
      }
    }
    if (j < dq) {
#pragma unroll
      for (int r = 0; r < R; ++r)
        out[r * dq + j] = (j < d) ? fmaf(cf[r].z, xs[r * dq + j], sc[r] * ((acc[r][0] + acc[r][1]) + (acc[r][2] + acc[r][3])))
                                  : 0.f;
    }
  }
  ASD_T2(2)
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for this wavefront's
// global stores to be acknowledged (a microsecond each round for the trajectory rows, which nobody
// in the workgroup reads back from memory).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

__device__ __forceinline__ float4 lds4(const float* row, int blk) {
  return *reinterpret_cast<const float4*>(row + 4 * blk);
}

}  // namespace

template <int RW>
__global__ __launch_bounds__(1024) void gmm_chain_sample_kernel(
    int K, int L, int d, int C, const Key* __restrict__ key_p, const float* __restrict__ c_x,
    const float* __restrict__ c_0, const float* __restrict__ sigma, const int32_t* __restrict__ tau,
    const float4* __restrict__ coef_tau, const float* __restrict__ means, const float* __restrict__ musq,
    const float* __restrict__ log_w, const float* __restrict__ y0, float* __restrict__ traj,
    int32_t* __restrict__ rounds, int32_t* __restrict__ max_rounds) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  __shared__ float s_logu[64], s_dot[64], s_vv[64];
  __shared__ int s_bit[64];
  __shared__ int s_nacc;

  const int c = blockIdx.x;
  const int tid = threadIdx.x, nthreads = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nthreads >> 6;
  const ChainLayout l = chain_layout(C, d, L, K);
  const int dq = l.dq, nblk = l.nblk;
  const bool vec = (d & 3) == 0;
  float* m_l = lds + l.m;
  float* q_l = lds + l.q;
  float* lw_l = lds + l.lw;
  float* ps = lds + l.ps;   // [L + 4][C4]
  float* yh = lds + l.yh;   // [L+1][dq]: yhat_a (= y_a) .. yhat_b
  float* x0 = lds + l.x0;   // [L][dq]:   model value at yhat_{a+s}, s = 0..w-1
  float* xi_l = lds + l.xi; // [L][dq]:   xi_{a+s+1}, the noise of step a+s -> a+s+1
  const Key key = *key_p;
  // The schedule and the denoiser's per-step coefficients: a round would otherwise start with a chain
  // of dependent global loads (tau_a, then its coefficients) and reload the tables step by step.
  const float4* sch = reinterpret_cast<const float4*>(lds + l.sch);
  for (int i = tid; i < K; i += nthreads) {
    float4* e = reinterpret_cast<float4*>(lds + l.sch) + 2 * i;
    e[0] = make_float4(c_x[i], c_0[i], sigma[i], 0.f);
    e[1] = coef_tau[tau[i]];
  }

  for (int t = tid; t < C * l.dp; t += nthreads) {
    const int k = t / l.dp, j = t - k * l.dp;
    m_l[t] = (j < d) ? means[(int64_t)k * d + j] : 0.f;
  }
  for (int t = tid; t < l.C4; t += nthreads) {
    q_l[t] = (t < C) ? musq[t] : 0.f;
    lw_l[t] = (t < C) ? log_w[t] : 0.f;
  }
  {  // y_0 (Alg. 1: given, or drawn from N(0, I))
    float* row0 = traj + (int64_t)c * (K + 1) * d;
    for (int blk = tid; blk < nblk; blk += nthreads) {
      const float4 v = y0 ? load4(y0 + (int64_t)c * d, blk, d, vec) : normal4(key, (uint32_t)c, 0u, (uint32_t)blk);
      store4(row0, blk, d, vec, v);
      *reinterpret_cast<float4*>(yh + 4 * blk) = v;
    }
  }
  __syncthreads();

  int a = 0, R = 0;
  ASD_T_DECL
  while (a < K) {
    ASD_T(0)
    const int w = min(L, K - a);
    // A. x0a on wavefront 0; the window's noise on the others
    if (wave == 0) {
      const float4 cf1[1] = {sch[2 * a + 1]};
      gmm_rows_lds<1>(yh, x0, cf1, m_l, q_l, lw_l, ps, C, l, d, lane);
    }
    if (nw == 1 || wave > 0) {
      const int t0 = (nw == 1) ? tid : tid - 64, nt = (nw == 1) ? 64 : nthreads - 64;
      for (int t = t0; t < w * nblk; t += nt) {
        const int k = t / nblk, blk = t - k * nblk;
        *reinterpret_cast<float4*>(xi_l + (size_t)k * dq + 4 * blk) =
            normal4(key, (uint32_t)c, (uint32_t)(a + k + 1), (uint32_t)blk);
      }
      for (int k = 1 + t0; k < w; k += nt) s_logu[k] = logf(uniform1(key, (uint32_t)c, (uint32_t)(a + k + 1)));
    }
    lds_barrier();
    ASD_T(1)
    // B. draft (proposal loop of Alg. 1)
    for (int blk = tid; blk < nblk; blk += nthreads) {
      float4 y = lds4(yh, blk);
      const float4 g = lds4(x0, blk);
      float* row = traj + ((int64_t)c * (K + 1) + a) * d;
      for (int k = 0; k < w; ++k) {
        const float4 sc = sch[2 * (a + k)];
        const float cx = sc.x, c0 = sc.y, sg = sc.z;
        const float4 xi = lds4(xi_l + (size_t)k * dq, blk);
        y.x = fmaf(sg, xi.x, fmaf(cx, y.x, c0 * g.x));
        y.y = fmaf(sg, xi.y, fmaf(cx, y.y, c0 * g.y));
        y.z = fmaf(sg, xi.z, fmaf(cx, y.z, c0 * g.z));
        y.w = fmaf(sg, xi.w, fmaf(cx, y.w, c0 * g.w));
        row += d;
        store4(row, blk, d, vec, y);
        *reinterpret_cast<float4*>(yh + (size_t)(k + 1) * dq + 4 * blk) = y;
      }
    }
    lds_barrier();
    ASD_T(2)
    // C. verify: target-mean model values at the drafted points (slot 0 reuses x0a)
    // RW rows per wavefront at a time; a group that would run past the window is shifted back to end
    // at its last row (w - 1 >= RW, so it recomputes rows of its neighbour: same values, same addresses)
    if (w - 1 >= RW) {
      for (int k0 = 1 + wave * RW; k0 < w; k0 += nw * RW) {
        const int k = min(k0, w - RW);
        float4 cf[RW];
#pragma unroll
        for (int r = 0; r < RW; ++r) cf[r] = sch[2 * (a + k + r) + 1];
        // (the scratch region follows the unshifted index: a shifted group must not share its neighbour's)
        gmm_rows_lds<RW>(yh + (size_t)k * dq, x0 + (size_t)k * dq, cf, m_l, q_l, lw_l, ps + (size_t)k0 * l.C4, C, l, d,
                         lane);
      }
    } else {
      for (int k = 1 + wave; k < w; k += nw) {
        const float4 cf1[1] = {sch[2 * (a + k) + 1]};
        gmm_rows_lds<1>(yh + (size_t)k * dq, x0 + (size_t)k * dq, cf1, m_l, q_l, lw_l, ps + (size_t)k * l.C4, C, l, d,
                        lane);
      }
    }
    lds_barrier();
    ASD_T(3)
    // D. Alg. 3 accept test, a wavefront per slot
    for (int k = 1 + wave; k < w; k += nw) {
      float dot = 0.f, vv = 0.f;
      for (int blk = lane; blk < nblk; blk += 64) {
        const float4 ga = lds4(x0, blk), gk = lds4(x0 + (size_t)k * dq, blk), xi = lds4(xi_l + (size_t)k * dq, blk);
        const float dx = ga.x - gk.x, dy = ga.y - gk.y, dz = ga.z - gk.z, dw = ga.w - gk.w;
        dot = fmaf(dx, xi.x, dot);
        dot = fmaf(dy, xi.y, dot);
        dot = fmaf(dz, xi.z, dot);
        dot = fmaf(dw, xi.w, dot);
        vv = fmaf(dx, dx, vv);
        vv = fmaf(dy, dy, vv);
        vv = fmaf(dz, dz, vv);
        vv = fmaf(dw, dw, vv);
      }
      dot = wave_sum(dot);
      vv = wave_sum(vv);
      if (lane == 0) {
        const float4 sc = sch[2 * (a + k)];
        const float sg = sc.z, c0 = sc.y;
        int bit = 0;  // sigma == 0 rejects
        if (sg > 0.f) {
          const float vxi = c0 * dot;
          const float v2 = c0 * c0 * vv;
          const float rho = -(vxi / sg + v2 / (2.0f * sg * sg));
          bit = (s_logu[k] <= rho) ? 1 : 0;
        }
        s_bit[k] = bit;
        s_dot[k] = dot;
        s_vv[k] = vv;
      }
    }
    lds_barrier();
    ASD_T(4)
    // Alg. 2: accepted prefix = trailing ones of the ballot (slot 0 is accepted by construction)
    if (wave == 0) {
      const int bit = (lane >= 1 && lane < w) ? s_bit[lane] : 1;
      const unsigned long long inv = ~__ballot(bit);
      const int first = inv ? (__ffsll((long long)inv) - 1) : 64;
      if (lane == 0) s_nacc = min(first, w);
    }
    lds_barrier();
    const int n_acc = s_nacc;
    // reject branch of Alg. 3 (reflection) and the advance rule of Alg. 1
    int a_next, src;  // src: row of yh that is y_{a_next}
    if (n_acc < w) {
      const int k = n_acc, i = a + k;
      const float4 sc = sch[2 * i];
      const float sg = sc.z, c0 = sc.y;
      const float dot = s_dot[k], vv = s_vv[k];
      const float coef = (vv > 0.f) ? (c0 + 2.0f * sg * dot / vv) : 0.f;
      float* row = traj + ((int64_t)c * (K + 1) + i + 1) * d;
      float* yr = yh + (size_t)(k + 1) * dq;
      for (int blk = tid; blk < nblk; blk += nthreads) {
        const float4 ga = lds4(x0, blk), gk = lds4(x0 + (size_t)k * dq, blk);
        float4 y = lds4(yr, blk);
        y.x = fmaf(-(ga.x - gk.x), coef, y.x);
        y.y = fmaf(-(ga.y - gk.y), coef, y.y);
        y.z = fmaf(-(ga.z - gk.z), coef, y.z);
        y.w = fmaf(-(ga.w - gk.w), coef, y.w);
        store4(row, blk, d, vec, y);
        *reinterpret_cast<float4*>(yr + 4 * blk) = y;
      }
      a_next = i + 1;
      src = k + 1;
    } else {
      a_next = a + w;
      src = w;
    }
    // every thread moves the blocks it wrote (or, on full acceptance, rows nobody writes any more)
    for (int blk = tid; blk < nblk; blk += nthreads)
      *reinterpret_cast<float4*>(yh + 4 * blk) = lds4(yh + (size_t)src * dq, blk);
    a = a_next;
    ++R;
    lds_barrier();
    ASD_T(5)
  }
  ASD_T_END
  if (tid == 0) {
    if (rounds) rounds[c] = R;
    atomicMax(max_rounds, R);
  }
}

namespace {

__global__ void set_i32_kernel(int32_t* p, int32_t v) { *p = v; }

// rows a wavefront evaluates together, and wavefronts per workgroup (one per group of verify rows)
#ifndef ASD_CHAIN_RW_SHIFT
#define ASD_CHAIN_RW_SHIFT 0
#endif
inline int chain_rows_per_wave(int L) {
  const int groups16 = (L - 1 + 15) / 16;  // rows per wavefront that keep the group count within 16 wavefronts
  const int rw = groups16 <= 1 ? 1 : (groups16 <= 2 ? 2 : 4);
  return std::min(4, rw << ASD_CHAIN_RW_SHIFT);
}
inline int chain_waves(int L) {
  const int groups = (int)ceil_div(std::max(1, L - 1), chain_rows_per_wave(L));
  return std::min(16, std::max(2, groups));
}
inline size_t chain_lds_bytes(const asd_ctx* ctx) {
  return sizeof(float) * chain_layout(ctx->gmm->C, ctx->d, ctx->L, ctx->K).total;
}

}  // namespace

bool gmm_chain_supported(const asd_ctx* ctx) {
  if (ctx->kind != ASD_DEN_GMM || !ctx->gmm || ctx->L > 64 || ctx->d > 4096) return false;
  return chain_lds_bytes(ctx) + 2048 <= 160 * 1024;
}

asd_status gmm_chain_sample(asd_ctx* ctx, const float* y0, float* traj, int32_t* rounds, hipStream_t st) {
  const GmmState* g = ctx->gmm;
  if (!gmm_chain_supported(ctx)) {
    set_error("chain-resident sampler: the mixture and the window do not fit in LDS");
    return ASD_EUNSUPPORTED;
  }
  const size_t lds_bytes = chain_lds_bytes(ctx);
  const int nw = chain_waves(ctx->L), R = chain_rows_per_wave(ctx->L);
  auto kern = R == 1 ? gmm_chain_sample_kernel<1> : (R == 2 ? gmm_chain_sample_kernel<2> : gmm_chain_sample_kernel<4>);
  static size_t attr_bytes[3] = {0, 0, 0};  // dynamic LDS above the default limit needs the attribute
  size_t& set = attr_bytes[R == 1 ? 0 : (R == 2 ? 1 : 2)];
  if (lds_bytes > set) {
    ASD_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
    set = lds_bytes;
  }
  hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(1), 0, st, ctx->live, 0);
  hipLaunchKernelGGL(kern, dim3(ctx->B), dim3(64 * nw), lds_bytes, st, ctx->K, ctx->L, ctx->d, g->C, ctx->key_dev,
                     ctx->c_x, ctx->c_0, ctx->sigma, ctx->tau, g->coef_tau, g->means, g->musq, g->log_w, y0, traj,
                     rounds, ctx->live);
  ASD_HIP(hipGetLastError());
  ASD_HIP(hipMemcpyAsync(ctx->live_host, ctx->live, sizeof(int32_t), hipMemcpyDeviceToHost, st));
  ASD_HIP(hipStreamSynchronize(st));
  ctx->last_rounds = ctx->live_host[0];
  return ASD_OK;
}

}  // namespace asd
