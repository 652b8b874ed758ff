// Chain-resident ASD sampler for Gaussian-mixture denoisers that fit in LDS.
//
// For small shapes a round of ASD is a handful of microsecond kernels and the
// sample is bound by launches, not by arithmetic.  Chains never interact, so here
// one workgroup runs the *whole* of Alg. 1 for one chain in a single launch:
// the mixture, the schedule, the window of proposal samples, the model values
// and the noise of the window live in LDS, and the only HBM traffic inside the
// loop is the trajectory rows the round produces.  Per round (notation of
// Alg. 1, x0-prediction form):
//   A. xi_{a+1..b} and log u_{a+2..b} of the window from the counter, then
//      x0a = D(y_a, tau_a);
//   B. draft: yhat_{i+1} = c_x yhat_i + c_0 x0a + sigma xi_{i+1}, a thread per
//      four coordinates walks the window; rows go to LDS and to the trajectory;
//   C. verify: x0_i = D(yhat_i, tau_i), i = a+1..b-1, all rows at once;
//   D. Alg. 3 accept test per slot (a wavefront per slot reduces <D,xi>, |D|^2),
//      Alg. 2 as ballot + trailing ones, reflection of the first rejected row,
//      advance.
// The denoiser is two small matrix products around a softmax, done by the whole
// workgroup; the verify rows go through the matrix cores 16 at a time (a window
// of L <= 17 is one tile; the single row of x0a stays on the vector ALUs): v_mfma_f32_16x16x4_f32 takes a 16 x 4 and a 4 x 16 operand straight
// from LDS.  The formulas and the counters are those of the stand-alone kernels,
// so the same parity bars apply.  Every wavefront leaves the loop when its chain
// reaches K, which takes at most K rounds.
#include "common.h"
#include "device_util.h"
#include "gmm_state.h"

namespace asd {

namespace {

typedef float v4f_c __attribute__((ext_vector_type(4)));

// LDS layout, in floats.  Rows that feed the matrix cores (mixture, proposal samples, softmax
// weights) are padded to a multiple of 16 plus 4: a 16-byte operand read by 16 lanes from 16
// consecutive rows then falls into 16 different bank groups.
struct ChainLayout {
  int d16, dp, C16, cp, nblk, tr;
  size_t m, q, lw, ps, part, yh, x0, xi, sch, total;
};

constexpr int kChainSplits = 4;  // most ways the component sum of a tile is split over wavefronts

__host__ __device__ inline ChainLayout chain_layout(int C, int d, int L, int K) {
  ChainLayout l;
  l.d16 = (d + 15) & ~15;
  l.dp = l.d16 + 4;
  l.C16 = (C + 15) & ~15;
  l.cp = l.C16 + 4;
  l.nblk = (d + 3) >> 2;
  l.tr = 16 * ((((L > 1) ? L - 1 : 1) + 15) / 16);  // rows of softmax scratch: whole tiles of 16
  l.m = 0;                                   // [C16][dp] means, rows past C and columns past d zero
  l.q = l.m + (size_t)l.C16 * l.dp;          // [C16] |mu|^2
  l.lw = l.q + l.C16;                        // [C16] log w
  l.ps = l.lw + l.C16;                       // [tr][cp] logits, then softmax weights
  l.part = l.ps + (size_t)l.tr * l.cp;       // [max(16, splits * tr)][dp] partial sums over components
  l.yh = l.part + (size_t)(kChainSplits * l.tr > 16 ? kChainSplits * l.tr : 16) * l.dp;  // [L+1][dp] yhat_a (= y_a) .. yhat_b
  l.x0 = l.yh + (size_t)(L + 1) * l.dp;      // [L][dp] model value at yhat_{a+s}
  l.xi = l.x0 + (size_t)L * l.dp;            // [L][dp] xi_{a+s+1}
  l.sch = l.xi + (size_t)L * l.dp;           // [K][8] (c_x, c_0, sigma, -, kappa, gamma, cx, cm) of step i
  l.total = l.sch + (size_t)K * 8;
  return l;
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

// D(yhat_s, tau_{a+s}) for the n slots s = first .. first+n-1, by the whole workgroup (every thread
// must call; three barriers inside, none at the end).
//
// v_mfma_f32_16x16x4_f32: A is 16 x 4 (lane l holds A[l % 16][l / 16]), B is 4 x 16 (lane l holds
// B[l / 16][l % 16]), D is 16 x 16 (lane l, register r holds D[4 (l / 16) + r][l % 16]).  A lane reads
// four consecutive k of its row at once (16 bytes) and feeds them to four MFMAs; since both operands
// do the same, the pairing of the elements is exact.
//   pass 1: logits = X Mt:  tile (16 rows, 16 components), k = coordinates;
//   pass 2: softmax over the components of a row, a wavefront per row;
//   pass 3: out = cx x + cm softmax(logits) M:  tile (16 rows, 16 coordinates), k = components.
// Rows past the last one repeat it (computed, never stored).
__device__ __forceinline__ void gmm_eval_tiles(int first, int n, int a, const ChainLayout& l, int C, int d,
                                               const float* m_l, const float* q_l, const float* lw_l, float* ps,
                                               float* part, const float* yh, float* x0, const float4* sch,
                                               float* s_sc, int wave, int nw, int lane) {
  const int dp = l.dp, cp = l.cp;
  const int li = lane & 15, kq = lane >> 4;
  const int T = (n + 15) >> 4;
  constexpr float kLog2e = 1.4426950408889634f;  // logits are kept in base-2 units for the hardware exp2
  {
    const int NT = l.C16 >> 4;
    for (int item = wave; item < T * NT; item += nw) {
      const int t = item / NT, nt = item - t * NT;
      const float* xa = yh + (size_t)(first + min(16 * t + li, n - 1)) * dp + 4 * kq;
      const float* mb = m_l + (size_t)(16 * nt + li) * dp + 4 * kq;
      v4f_c acc = {0.f, 0.f, 0.f, 0.f};
      for (int s = 0; s < l.d16; s += 16) {
        const float4 av = *reinterpret_cast<const float4*>(xa + s);
        const float4 bv = *reinterpret_cast<const float4*>(mb + s);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bv.x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, bv.y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.z, bv.z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.w, bv.w, acc, 0, 0, 0);
      }
      const int comp = 16 * nt + li;
      const float qk = q_l[comp], lwk = lw_l[comp];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = 16 * t + 4 * kq + r;
        if (row < n) {
          const float4 cf = sch[2 * (a + first + row) + 1];
          ps[(size_t)row * cp + comp] = kLog2e * fmaf(cf.x, acc[r], fmaf(-cf.y, qk, lwk));
        }
      }
    }
  }
  lds_barrier();
  for (int row = wave; row < n; row += nw) {
    float* pr = ps + (size_t)row * cp;
    float mx = -INFINITY;
    for (int k = lane; k < C; k += 64) mx = fmaxf(mx, pr[k]);
    mx = wave_max(mx);
    float sum = 0.f;
    for (int k = lane; k < l.C16; k += 64) {
      // components past C weigh nothing, nor do weights below 2^-kCertZeroGap of the largest (gmm_cert.h)
      const float p = (k < C && !(pr[k] - mx < -kCertZeroGap)) ? __builtin_amdgcn_exp2f(pr[k] - mx) : 0.f;
      pr[k] = p;
      sum += p;
    }
    sum = wave_sum(sum);
    if (lane == 0) s_sc[row] = sch[2 * (a + first + row) + 1].w / sum;
  }
  lds_barrier();
  {
    // the sum over components of a tile is cut into KS pieces so that every wavefront has a piece;
    // the pieces land in LDS and are added in order
    const int CT = l.d16 >> 4, SS = l.C16 >> 4;
    int KS = 1;
    while (KS < kChainSplits && T * CT * KS * 2 <= nw && SS % (KS * 2) == 0) KS *= 2;
    const int steps = SS / KS;
    for (int item = wave; item < T * CT * KS; item += nw) {
      const int ks = item % KS, tc = item / KS;
      const int t = tc / CT, ct = tc - t * CT;
      const float* pa = ps + (size_t)min(16 * t + li, n - 1) * cp + 4 * kq + 16 * ks * steps;
      const float* mb = m_l + (size_t)(4 * kq + 16 * ks * steps) * dp + 16 * ct + li;
      v4f_c acc = {0.f, 0.f, 0.f, 0.f};
      float4 av = *reinterpret_cast<const float4*>(pa);
      float b0 = mb[0], b1 = mb[dp], b2 = mb[2 * dp], b3 = mb[3 * dp];
      for (int s = 0; s < steps; ++s) {
        // operands of the next step are requested before this step's MFMAs (the last step re-reads its own)
        const int sn = min(s + 1, steps - 1);
        const float4 an = *reinterpret_cast<const float4*>(pa + 16 * sn);
        const float* mr = mb + (size_t)(16 * sn) * dp;
        const float n0 = mr[0], n1 = mr[dp], n2 = mr[2 * dp], n3 = mr[3 * dp];
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, b0, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, b1, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.z, b2, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av.w, b3, acc, 0, 0, 0);
        av = an;
        b0 = n0; b1 = n1; b2 = n2; b3 = n3;
      }
      const int coord = 16 * ct + li;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = 16 * t + 4 * kq + r;
        if (row < n) part[((size_t)ks * l.tr + row) * dp + coord] = acc[r];
      }
    }
    lds_barrier();
    for (int e = wave * 64 + lane; e < n * l.d16; e += nw * 64) {
      const int row = e / l.d16, coord = e - row * l.d16;
      float sum = part[(size_t)row * dp + coord];
      for (int ks = 1; ks < KS; ++ks) sum += part[((size_t)ks * l.tr + row) * dp + coord];
      const int slot = first + row;
      const float cx = sch[2 * (a + slot) + 1].z;
      x0[(size_t)slot * dp + coord] = (coord < d) ? fmaf(cx, yh[(size_t)slot * dp + coord], s_sc[row] * sum) : 0.f;
    }
  }
}

// D(yhat_slot, tau_{a+slot}) for a single slot, by the whole workgroup on the vector ALUs (a 16-row
// matrix-core tile would be 15/16 padding): four lanes share a component in pass 1, the wavefronts
// share the components in pass 3 and their partial sums are added in order.  Every thread must
// call; three barriers inside, none at the end.
__device__ __forceinline__ void gmm_eval_row(int slot, int a, const ChainLayout& l, int C, int d, const float* m_l,
                                             const float* q_l, const float* lw_l, float* ps, float* part,
                                             const float* yh, float* x0, const float4* sch, float* s_sc, int tid,
                                             int nthreads) {
  const int dp = l.dp, d4 = l.d16 >> 2;
  const int lane = tid & 63, wave = tid >> 6, nw = nthreads >> 6;
  const float* xs = yh + (size_t)slot * dp;
  const float4 cf = sch[2 * (a + slot) + 1];
  constexpr float kLog2e = 1.4426950408889634f;
  {
    const int part4 = tid & 3;
    for (int comp = tid >> 2; comp < l.C16; comp += nthreads >> 2) {
      const float* mk = m_l + (size_t)comp * dp;
      float dot = 0.f;
      for (int b = part4; b < d4; b += 4) {
        const float4 xv = *reinterpret_cast<const float4*>(xs + 4 * b);
        const float4 mv = *reinterpret_cast<const float4*>(mk + 4 * b);
        dot = fmaf(xv.x, mv.x, fmaf(xv.y, mv.y, fmaf(xv.z, mv.z, fmaf(xv.w, mv.w, dot))));
      }
      // sum over the four lanes of the quad (C16 is a multiple of 16 and the workgroup of 64: whole quads loop together)
      dot += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(dot), 0xB1, 0xf, 0xf, true));
      dot += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(dot), 0x4E, 0xf, 0xf, true));
      if (part4 == 0) ps[comp] = kLog2e * fmaf(cf.x, dot, fmaf(-cf.y, q_l[comp], lw_l[comp]));
    }
  }
  lds_barrier();
  if (wave == 0) {
    float mx = -INFINITY;
    for (int k = lane; k < C; k += 64) mx = fmaxf(mx, ps[k]);
    mx = wave_max(mx);
    float sum = 0.f;
    for (int k = lane; k < l.C16; k += 64) {
      const float p = (k < C && !(ps[k] - mx < -kCertZeroGap)) ? __builtin_amdgcn_exp2f(ps[k] - mx) : 0.f;
      ps[k] = p;
      sum += p;
    }
    sum = wave_sum(sum);
    if (lane == 0) s_sc[0] = cf.w / sum;
  }
  lds_barrier();
  {
    // wavefront g takes the component quads g, g + nw, ...
    for (int j = lane; j < l.d16; j += 64) {
      float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
      for (int k = 4 * wave; k < l.C16; k += 4 * nw) {
        const float4 p = *reinterpret_cast<const float4*>(ps + k);
        const float* mk = m_l + (size_t)k * dp + j;
        a0 = fmaf(p.x, mk[0], a0);
        a1 = fmaf(p.y, mk[dp], a1);
        a2 = fmaf(p.z, mk[2 * dp], a2);
        a3 = fmaf(p.w, mk[3 * dp], a3);
      }
      part[(size_t)wave * dp + j] = (a0 + a1) + (a2 + a3);
    }
  }
  lds_barrier();
  for (int j = tid; j < l.d16; j += nthreads) {
    float sum = part[j];
    for (int g = 1; g < nw; ++g) sum += part[(size_t)g * dp + j];
    x0[(size_t)slot * dp + j] = (j < d) ? fmaf(cf.z, xs[j], s_sc[0] * sum) : 0.f;
  }
}

}  // namespace

__global__ __launch_bounds__(1024) void gmm_chain_sample_kernel(
    int K, int L, int d, int C, const Key* __restrict__ key_p, const float* __restrict__ c_x,
    const float* __restrict__ c_0, const float* __restrict__ sigma, const int32_t* __restrict__ tau,
    const float4* __restrict__ coef_tau, const float* __restrict__ means, const float* __restrict__ musq,
    const float* __restrict__ log_w, const float* __restrict__ y0, float* __restrict__ traj,
    int32_t* __restrict__ rounds, unsigned long long* __restrict__ max_rounds, uint32_t launch_id,
    int adaptive) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  __shared__ float s_logu[64], s_dot[64], s_vv[64], s_sc[64];
  __shared__ int s_bit[64];
  __shared__ int s_nacc;

  const int c = blockIdx.x;
  const int tid = threadIdx.x, nthreads = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nthreads >> 6;
  const ChainLayout l = chain_layout(C, d, L, K);
  const int dp = l.dp, nblk = l.nblk;
  const bool vec = (d & 3) == 0;
  float* m_l = lds + l.m;
  float* q_l = lds + l.q;
  float* lw_l = lds + l.lw;
  float* ps = lds + l.ps;
  float* part = lds + l.part;
  float* yh = lds + l.yh;
  float* x0 = lds + l.x0;
  float* xi_l = lds + l.xi;
  const Key key = *key_p;
  // The schedule and the denoiser's per-step coefficients: a round would otherwise start with a chain
  // of dependent global loads (tau_a, then its coefficients) and reload the tables step by step.
  const float4* sch = reinterpret_cast<const float4*>(lds + l.sch);
  for (int i = tid; i < K; i += nthreads) {
    float4* e = reinterpret_cast<float4*>(lds + l.sch) + 2 * i;
    e[0] = make_float4(c_x[i], c_0[i], sigma[i], 0.f);
    e[1] = coef_tau[tau[i]];
  }
  for (int t = tid; t < l.C16 * dp; t += nthreads) {
    const int k = t / dp, j = t - k * dp;
    m_l[t] = (k < C && j < d) ? means[(int64_t)k * d + j] : 0.f;
  }
  for (int t = tid; t < l.C16; t += nthreads) {
    q_l[t] = (t < C) ? musq[t] : 0.f;
    lw_l[t] = (t < C) ? log_w[t] : 0.f;
  }
  // everything between the softmax scratch and the schedule starts as zero: the padding of the rows is
  // multiplied (by zero mixture entries) on the matrix cores and must be finite
  for (size_t t = l.ps + tid; t < l.sch; t += nthreads) lds[t] = 0.f;
  lds_barrier();
  {  // y_0 (Alg. 1: given, or drawn from N(0, I))
    float* row0 = traj + (int64_t)c * (K + 1) * d;
    for (int blk = tid; blk < nblk; blk += nthreads) {
      const float4 v = y0 ? load4(y0 + (int64_t)c * d, blk, d, vec) : normal4(key, (uint32_t)c, 0u, (uint32_t)blk);
      store4(row0, blk, d, vec, v);
      *reinterpret_cast<float4*>(yh + 4 * blk) = v;
    }
  }
  lds_barrier();

  int a = 0, R = 0;
  int wstate = 4 * L;  // window controller (device_util.h); without it every window is L
  while (a < K) {
    const int w = min(adaptive ? window_of(wstate, L) : L, K - a);
    // A. the window's noise, then x0a
    for (int t = tid; t < w * nblk; t += nthreads) {
      const int k = t / nblk, blk = t - k * nblk;
      *reinterpret_cast<float4*>(xi_l + (size_t)k * dp + 4 * blk) =
          normal4(key, (uint32_t)c, (uint32_t)(a + k + 1), (uint32_t)blk);
    }
    for (int k = 1 + tid; k < w; k += nthreads) s_logu[k] = logf(uniform1(key, (uint32_t)c, (uint32_t)(a + k + 1)));
    gmm_eval_row(0, a, l, C, d, m_l, q_l, lw_l, ps, part, yh, x0, sch, s_sc, tid, nthreads);
    lds_barrier();
    // B. draft (proposal loop of Alg. 1)
    for (int blk = tid; blk < nblk; blk += nthreads) {
      float4 y = lds4(yh, blk);
      const float4 g = lds4(x0, blk);
      float* row = traj + ((int64_t)c * (K + 1) + a) * d;
      // four steps at a time: their table entries and noise are all requested before the first is
      // used, so the LDS latency is paid once per four steps of the recurrence
      for (int k0 = 0; k0 < w; k0 += 4) {
        float4 sc[4], xi[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int k = min(k0 + u, w - 1);
          sc[u] = sch[2 * (a + k)];
          xi[u] = lds4(xi_l + (size_t)k * dp, blk);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (k0 + u < w) {
            const float cx = sc[u].x, c0 = sc[u].y, sg = sc[u].z;
            y.x = fmaf(sg, xi[u].x, fmaf(cx, y.x, c0 * g.x));
            y.y = fmaf(sg, xi[u].y, fmaf(cx, y.y, c0 * g.y));
            y.z = fmaf(sg, xi[u].z, fmaf(cx, y.z, c0 * g.z));
            y.w = fmaf(sg, xi[u].w, fmaf(cx, y.w, c0 * g.w));
            row += d;
            store4(row, blk, d, vec, y);
            *reinterpret_cast<float4*>(yh + (size_t)(k0 + u + 1) * dp + 4 * blk) = y;
          }
        }
      }
    }
    lds_barrier();
    // C. verify: target-mean model values at the drafted points (slot 0 reuses x0a)
    if (w > 1) gmm_eval_tiles(1, w - 1, a, l, C, d, m_l, q_l, lw_l, ps, part, yh, x0, sch, s_sc, wave, nw, lane);
    lds_barrier();
    // D. Alg. 3 accept test, a wavefront per slot
    for (int k = 1 + wave; k < w; k += nw) {
      float dot = 0.f, vv = 0.f;
      for (int blk = lane; blk < nblk; blk += 64) {
        const float4 ga = lds4(x0, blk), gk = lds4(x0 + (size_t)k * dp, blk), xi = lds4(xi_l + (size_t)k * dp, blk);
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
      float* yr = yh + (size_t)(k + 1) * dp;
      for (int blk = tid; blk < nblk; blk += nthreads) {
        const float4 ga = lds4(x0, blk), gk = lds4(x0 + (size_t)k * dp, blk);
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
      *reinterpret_cast<float4*>(yh + 4 * blk) = lds4(yh + (size_t)src * dp, blk);
    wstate = window_next(wstate, w, n_acc);
    a = a_next;
    ++R;
    lds_barrier();
  }
  if (tid == 0) {
    if (rounds) rounds[c] = R;
    // (launch id, rounds) packed so that the maximum needs no reset between samples
    atomicMax(max_rounds, ((unsigned long long)launch_id << 32) | (unsigned)R);
  }
}

namespace {

// wavefronts per workgroup: enough for the tiles of the logits pass, within 4..16
inline int chain_waves(const asd_ctx* ctx) {
  const ChainLayout l = chain_layout(ctx->gmm->C, ctx->d, ctx->L, ctx->K);
  const int items = (l.C16 / 16) * (l.tr / 16);
  return items >= 16 ? 16 : (items >= 8 ? 8 : 4);
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
    set_error("chain-resident sampler: the mixture, the window and the schedule do not fit in LDS");
    return ASD_EUNSUPPORTED;
  }
  const size_t lds_bytes = chain_lds_bytes(ctx);
  const int nw = chain_waves(ctx);
  static size_t attr_bytes = 0;  // dynamic LDS above the default limit needs the attribute
  if (lds_bytes > attr_bytes) {
    ASD_HIP(hipFuncSetAttribute((const void*)gmm_chain_sample_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_bytes));
    attr_bytes = lds_bytes;
  }
  hipLaunchKernelGGL(gmm_chain_sample_kernel, dim3(ctx->B), dim3(64 * nw), lds_bytes, st, ctx->K, ctx->L, ctx->d,
                     g->C, ctx->key_dev, ctx->c_x, ctx->c_0, ctx->sigma, ctx->tau, g->coef_tau, g->means, g->musq,
                     g->log_w, y0, traj, rounds, ctx->chain_max, ++ctx->chain_launches, ctx->adaptive ? 1 : 0);
  ASD_HIP(hipGetLastError());
  ASD_HIP(hipMemcpyAsync(ctx->live_host, ctx->chain_max, sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
  ASD_HIP(hipStreamSynchronize(st));
  ctx->last_rounds = ctx->live_host[0];  // low word: the largest round count of this launch
  return ASD_OK;
}

}  // namespace asd
