// Residual-MLP denoiser (stand-in for the paper's trained networks; the
// diffusion-policy and image-shaped workloads):
//   in  = [ bf16(x) ; temb[tau] ]                    (d + E)
//   h   = W_in in + b_in
//   h  += SiLU( W_l bf16(h) + b_l )                  l = 0..n_blocks-1
//   out = W_out bf16(h) + b_out,  D = clamp(out, -clip, clip)   interpreted as E[x_0 | x]
// Every matrix product takes bf16 inputs and accumulates in fp32 on the matrix
// cores; bias, SiLU and the residual stream are fp32 and are fused into the
// GEMM epilogues, which also emit the bf16 copy of h the next product reads.
//
// Activation precision (act_terms).  1: an activation enters a product as one bf16 number, bf16(h) above.
// 2: as the sum of two, hi = bf16(h), lo = bf16(h - hi) -- 16 significant bits -- held as two planes of the
// same matrix; the GEMM multiplies the weights with both planes into one accumulator.  Why it exists: a
// random-weight residual network amplifies the 2^-9 relative rounding of one-term activations to ~2e-3 of
// its output scale, whatever the accumulation order, so two correct implementations of the one-term
// network differ by that much (0.03-0.05 on outputs clipped to [-1, 1] when the unclipped scale is ~17);
// with two terms the same figure is ~4e-6 of the output scale.
#include "common.h"
#include "gemm_bf16.h"
#include "gemm_bf16_pipe.h"

namespace asd {

// Verify call, K % 64 == 0: the direct-to-LDS pipeline.  A CU moves about 30 bytes per clock from
// L2 into LDS whatever the kernel does, so the tile is as large as the problem allows: 128 x 256
// (MFMA-bound fraction of the loop ~60%) when that still gives every CU a tile, else 128 x 128.
typedef PipeCfg16<128, 256, 3, 2, 4> MlpPipeWide;
typedef PipeCfg16<128, 128, 4, 2, 4> MlpPipeSquare;
// Draft call (one row per chain): the weights are streamed once for a handful of rows.  64 x 64 tiles
// with 7 slabs (56 KB of weights) in flight each, and K split so that there are at least as many
// workgroups as CUs: ~14 MB of the weight stream in flight, which is what HBM latency asks for.
typedef PipeCfg16<64, 64, 8, 2, 2> MlpPipeSkinny;
// The same three roles with a two-plane A operand (act_terms = 2).  A stage holds both planes of the A slab, so
// 128 x 128 output tiles load as many bytes per MFMA as 128 x 256 tiles do with one plane.
typedef PipeCfg16<128, 128, 3, 2, 4, 2> MlpPipe2;
typedef PipeCfg16<64, 64, 6, 2, 2, 2> MlpPipeSkinny2;
constexpr int kMaxSplits = 8;

struct SplitScratch {
  float* part = nullptr;   // [kMaxSplits][rows][max N] fp32 partial tiles
  int rows = 0;            // rows the scratch was sized for (one per chain)
  bool small_verify = false;  // verify calls may be far below their row bound (windows from the controller)
};
// Verify calls of at most this many rows go to the 64 x 64 tiles of the draft call: a few row tiles
// against a whole weight matrix is a weight stream again, not a 128 x 256-tile problem.
constexpr int kSmallVerifyRows = 256;

// Both operands have row pitch ld = padded(K) (see pitch_of).  a_plane > 0: A has a second plane that many
// elements behind the first (two-term activations).
template <class Epi>
static hipError_t mlp_gemm(int call, const int* n_dev, int n, int N, int K, int64_t ld, const uint16_t* A,
                           int64_t a_plane, const uint16_t* Wt, Epi e, hipStream_t st, const SplitScratch& sc) {
  // K is rounded up to the slab size: columns K .. ld-1 of both operands are zero (pitch_of leaves
  // room for it), so the extra products vanish.
  const int Kp = (int)(ceil_div(K, 64) * 64);
  const bool two = a_plane > 0;
  if (call == 0) {
    const int64_t tiles = ceil_div(n, MlpPipeSkinny::BM) * ceil_div(N, MlpPipeSkinny::BN);
    int splits = 1;
    // only a weight matrix that takes several microseconds to stream repays the second launch
    if (n <= sc.rows && (int64_t)N * Kp * 2 >= (8 << 20))
      while (splits < kMaxSplits && tiles * splits < 256 && (Kp / 64) % (2 * splits) == 0) splits *= 2;
    return two ? launch_gemm_bf16_nt_pipe<MlpPipeSkinny2, 0>(n_dev, n, N, Kp, A, ld, a_plane, Wt, ld, e, st, splits, sc.part)
               : launch_gemm_bf16_nt_pipe<MlpPipeSkinny, 0>(n_dev, n, N, Kp, A, ld, 0, Wt, ld, e, st, splits, sc.part);
  }
  {
    const int64_t wide_tiles = ceil_div(n, 128) * ceil_div(N, 256);
    int m_lo = -1;
    if (sc.small_verify && n > kSmallVerifyRows && (int64_t)N * Kp * 2 >= (8 << 20)) {
      // both shapes are queued; the row count in device memory decides which one does the work
      hipError_t e0 =
          two ? launch_gemm_bf16_nt_pipe<MlpPipeSkinny2, 1>(n_dev, kSmallVerifyRows, N, Kp, A, ld, a_plane, Wt, ld, e, st, 1,
                                                            nullptr, -1, kSmallVerifyRows)
              : launch_gemm_bf16_nt_pipe<MlpPipeSkinny, 1>(n_dev, kSmallVerifyRows, N, Kp, A, ld, 0, Wt, ld, e, st, 1,
                                                           nullptr, -1, kSmallVerifyRows);
      if (e0 != hipSuccess) return e0;
      m_lo = kSmallVerifyRows;
    }
    if (two) return launch_gemm_bf16_nt_pipe<MlpPipe2, 1>(n_dev, n, N, Kp, A, ld, a_plane, Wt, ld, e, st, 1, nullptr, m_lo);
    return wide_tiles >= 192 ? launch_gemm_bf16_nt_pipe<MlpPipeWide, 1>(n_dev, n, N, Kp, A, ld, 0, Wt, ld, e, st, 1, nullptr, m_lo)
                             : launch_gemm_bf16_nt_pipe<MlpPipeSquare, 1>(n_dev, n, N, Kp, A, ld, 0, Wt, ld, e, st, 1, nullptr,
                                                                          m_lo);
  }
}

// Row pitch (elements) of every bf16 matrix the GEMMs read: K plus 64 elements (128 bytes).
// With the natural pitch (a power of two times 2 bytes for the widths used here) the rows a
// workgroup streams in parallel all start on the same few HBM channels; the odd pitch spreads them.
static inline int64_t pitch_of(int K) { return (int64_t)K + 64; }

struct MlpState {
  int width = 0, n_blocks = 0, E = 0, in_dim = 0;
  int64_t ld_in = 0, ld_h = 0;   // padded pitches of [*, in_dim] and [*, width] bf16 matrices
  uint16_t* wp_in = nullptr;     // padded copies of the caller's weights
  uint16_t* wp_blk = nullptr;
  uint16_t* wp_out = nullptr;
  float out_clip = 0.f;
  float2* eps_coef = nullptr;    // [n_tau] (1/sqrt(abar), sqrt(1-abar)/sqrt(abar)) when the network predicts the noise
  const uint16_t* w_in = nullptr;
  const uint16_t* w_blk = nullptr;
  const uint16_t* w_out = nullptr;
  const float* b_in = nullptr;
  const float* b_blk = nullptr;
  const float* b_out = nullptr;
  const uint16_t* temb = nullptr;
  int act_terms = 1;          // bf16 terms an activation enters a product with (1 or 2)
  uint16_t* in_bf = nullptr;  // [act_terms][rows_max, ld_in]: the planes of a matrix lie in_plane elements apart
  float* h = nullptr;         // [rows_max, width]
  uint16_t* hb[2] = {nullptr, nullptr};   // [act_terms][rows_max, ld_h] each, planes h_plane apart
  int64_t in_plane = 0, h_plane = 0;      // 0 when act_terms == 1
  SplitScratch split;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
// lo term of a two-term activation: bf16(v - float(hi)) (the difference is exact in fp32)
__device__ __forceinline__ uint16_t bf16_lo(float v, uint16_t hi) { return f32_to_bf16_rne(v - bf16_to_f32(hi)); }

// in_bf[n] = [ bf16(x_n) ; temb[tau_n] ], eight elements per thread; in_plane > 0: the lo terms of x (zero for
// the time embedding, which is bf16 data) go to the second plane
__global__ void mlp_pack_kernel(const int* __restrict__ n_dev, int n_rows, int d, int E, const float* __restrict__ in_base,
                                const int64_t* __restrict__ in_off, const int32_t* __restrict__ tau,
                                const uint16_t* __restrict__ temb, uint16_t* __restrict__ in_bf, int64_t ld_in,
                                int64_t in_plane) {
  const int n = blockIdx.x;
  const int q = blockIdx.y * blockDim.x + threadIdx.x;  // group of 8 elements
  const int in_dim = d + E;
  if (q * 8 >= in_dim || n >= min(*n_dev, n_rows)) return;
  uint4 o, l = make_uint4(0u, 0u, 0u, 0u);
  if (q * 8 < d) {
    const float* x = in_base + in_off[n] + q * 8;
    const float4 lo = *reinterpret_cast<const float4*>(x);
    const float4 hi = *reinterpret_cast<const float4*>(x + 4);
    const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    uint16_t h[8], r[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      h[k] = f32_to_bf16_rne(v[k]);
      r[k] = bf16_lo(v[k], h[k]);
    }
    o = make_uint4((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16),
                   (uint32_t)h[4] | ((uint32_t)h[5] << 16), (uint32_t)h[6] | ((uint32_t)h[7] << 16));
    l = make_uint4((uint32_t)r[0] | ((uint32_t)r[1] << 16), (uint32_t)r[2] | ((uint32_t)r[3] << 16),
                   (uint32_t)r[4] | ((uint32_t)r[5] << 16), (uint32_t)r[6] | ((uint32_t)r[7] << 16));
  } else {
    o = *reinterpret_cast<const uint4*>(temb + (int64_t)tau[n] * E + (q * 8 - d));
  }
  *reinterpret_cast<uint4*>(in_bf + (int64_t)n * ld_in + q * 8) = o;
  if (in_plane) *reinterpret_cast<uint4*>(in_bf + in_plane + (int64_t)n * ld_in + q * 8) = l;
}

// SiLU with the hardware exp2 and reciprocal: relative error ~1e-6, inside what the re-rounding of the
// activations leaves of the value (2^-9 with one bf16 term, 2^-17 with two).
__device__ __forceinline__ float silu(float z) {
  return z * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}

// hi and (lo_plane > 0) lo terms of four activations, to p and p + lo_plane
__device__ __forceinline__ void store_act4(uint16_t* p, int64_t lo_plane, float4 v) {
  const uint16_t h0 = f32_to_bf16_rne(v.x), h1 = f32_to_bf16_rne(v.y), h2 = f32_to_bf16_rne(v.z), h3 = f32_to_bf16_rne(v.w);
  *reinterpret_cast<uint2*>(p) = make_uint2((uint32_t)h0 | ((uint32_t)h1 << 16), (uint32_t)h2 | ((uint32_t)h3 << 16));
  if (lo_plane)
    *reinterpret_cast<uint2*>(p + lo_plane) =
        make_uint2((uint32_t)bf16_lo(v.x, h0) | ((uint32_t)bf16_lo(v.y, h1) << 16),
                   (uint32_t)bf16_lo(v.z, h2) | ((uint32_t)bf16_lo(v.w, h3) << 16));
}
__device__ __forceinline__ float4 load_bias4(const float* bias, int n) {
  return bias ? *reinterpret_cast<const float4*>(bias + n) : make_float4(0.f, 0.f, 0.f, 0.f);
}

struct InEpi {  // h = acc + b; hb = bf16 terms of h
  float* h;
  uint16_t* hb;
  const float* bias;
  int64_t ld, ldb;  // pitch of h (fp32) and of hb (bf16)
  int64_t lo_plane; // > 0: offset of hb's second plane (two-term activations)
  static constexpr bool kLoads = false;
  // four consecutive columns n..n+3 (n % 4 == 0) of row m
  __device__ __forceinline__ float4 load4(int, int) const { return make_float4(0.f, 0.f, 0.f, 0.f); }
  __device__ __forceinline__ void store4(int m, int n, float4 a, float4) const {
    const float4 b = load_bias4(bias, n);
    const float4 v = make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w);
    *reinterpret_cast<float4*>(h + (int64_t)m * ld + n) = v;
    store_act4(hb + (int64_t)m * ldb + n, lo_plane, v);
  }
};

struct BlockEpi {  // h += SiLU(acc + b); hb_next = bf16 terms of h
  float* h;
  uint16_t* hb_next;
  const float* bias;
  int64_t ld, ldb;
  int64_t lo_plane;
  static constexpr bool kLoads = true;
  __device__ __forceinline__ float4 load4(int m, int n) const {
    return *reinterpret_cast<const float4*>(h + (int64_t)m * ld + n);
  }
  __device__ __forceinline__ void store4(int m, int n, float4 a, float4 p) const {
    const float4 b = load_bias4(bias, n);
    float* hp = h + (int64_t)m * ld + n;
    const float4 v = make_float4(p.x + silu(a.x + b.x), p.y + silu(a.y + b.y), p.z + silu(a.z + b.z),
                                 p.w + silu(a.w + b.w));
    *reinterpret_cast<float4*>(hp) = v;
    store_act4(hb_next + (int64_t)m * ldb + n, lo_plane, v);
  }
};

struct OutEpi {  // out[out_off[m] + n] = acc + b, as x_0 (or converted from a noise estimate), clipped
  float* out_base;
  const int64_t* out_off;
  const float* bias;
  float clip;  // 0: none
  // noise-predicting networks: x_0 = x / sqrt(abar) - out * sqrt(1 - abar) / sqrt(abar), x = the row evaluated
  const float2* eps_coef;  // NULL: the network predicts x_0
  const int32_t* tau;
  const float* in_base;
  const int64_t* in_off;
  static constexpr bool kLoads = false;
  __device__ __forceinline__ float4 load4(int, int) const { return make_float4(0.f, 0.f, 0.f, 0.f); }
  __device__ __forceinline__ void store4(int m, int n, float4 a, float4) const {
    const float4 b = load_bias4(bias, n);
    float4 v = make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w);
    if (eps_coef) {
      const float2 ec = eps_coef[tau[m]];
      const float4 x = *reinterpret_cast<const float4*>(in_base + in_off[m] + n);
      v.x = fmaf(x.x, ec.x, -v.x * ec.y);
      v.y = fmaf(x.y, ec.x, -v.y * ec.y);
      v.z = fmaf(x.z, ec.x, -v.z * ec.y);
      v.w = fmaf(x.w, ec.x, -v.w * ec.y);
    }
    if (clip > 0.f) {
      v.x = fminf(fmaxf(v.x, -clip), clip);
      v.y = fminf(fmaxf(v.y, -clip), clip);
      v.z = fminf(fmaxf(v.z, -clip), clip);
      v.w = fminf(fmaxf(v.w, -clip), clip);
    }
    *reinterpret_cast<float4*>(out_base + out_off[m] + n) = v;
  }
};

asd_status mlp_create(asd_ctx* ctx, const asd_denoiser& den) {
  MlpState* s = new (std::nothrow) MlpState();
  if (!s) return ASD_ENOMEM;
  ctx->mlp = s;
  s->width = den.width;
  s->n_blocks = den.n_blocks;
  s->E = den.temb_dim;
  s->out_clip = den.out_clip;
  s->act_terms = den.act_terms;
  if (den.predict_eps) {
    std::vector<float2> ec((size_t)ctx->n_tau);
    for (int t = 0; t < ctx->n_tau; ++t) {
      const double ab = den.abar[t];
      ec[t] = make_float2((float)(1.0 / sqrt(ab)), (float)(sqrt(1.0 - ab) / sqrt(ab)));
    }
    ASD_HIP(hipMalloc(&s->eps_coef, sizeof(float2) * ec.size()));
    ASD_HIP(hipMemcpy(s->eps_coef, ec.data(), sizeof(float2) * ec.size(), hipMemcpyHostToDevice));
  }
  s->in_dim = ctx->d + den.temb_dim;
  s->w_in = (const uint16_t*)den.w_in;
  s->w_blk = (const uint16_t*)den.w_blk;
  s->w_out = (const uint16_t*)den.w_out;
  s->b_in = den.b_in;
  s->b_blk = den.b_blk;
  s->b_out = den.b_out;
  s->temb = (const uint16_t*)den.temb;
  const size_t rows = (size_t)ctx->n_rows_max;
  ctx->model_macs_per_row = (double)s->in_dim * s->width + (double)s->n_blocks * s->width * s->width +
                            (double)s->width * ctx->d;
  s->ld_in = pitch_of(s->in_dim);
  s->ld_h = pitch_of(s->width);
  const size_t Wd = (size_t)s->width, nb = (size_t)s->n_blocks, dd = (size_t)ctx->d;
  const size_t planes = (size_t)s->act_terms;
  if (planes > 1) {
    s->in_plane = (int64_t)rows * s->ld_in;
    s->h_plane = (int64_t)rows * s->ld_h;
  }
  ASD_HIP(hipMalloc(&s->in_bf, sizeof(uint16_t) * planes * rows * s->ld_in));
  ASD_HIP(hipMalloc(&s->h, sizeof(float) * rows * s->width));
  ASD_HIP(hipMalloc(&s->hb[0], sizeof(uint16_t) * planes * rows * s->ld_h));
  ASD_HIP(hipMalloc(&s->hb[1], sizeof(uint16_t) * planes * rows * s->ld_h));
  ASD_HIP(hipMemset(s->in_bf, 0, sizeof(uint16_t) * planes * rows * s->ld_in));
  ASD_HIP(hipMemset(s->hb[0], 0, sizeof(uint16_t) * planes * rows * s->ld_h));
  ASD_HIP(hipMemset(s->hb[1], 0, sizeof(uint16_t) * planes * rows * s->ld_h));
  // padded copies of the weights (one-time; the caller's arrays are not read again)
  ASD_HIP(hipMalloc(&s->wp_in, sizeof(uint16_t) * Wd * s->ld_in));
  ASD_HIP(hipMalloc(&s->wp_out, sizeof(uint16_t) * dd * s->ld_h));
  ASD_HIP(hipMemset(s->wp_in, 0, sizeof(uint16_t) * Wd * s->ld_in));
  ASD_HIP(hipMemset(s->wp_out, 0, sizeof(uint16_t) * dd * s->ld_h));
  ASD_HIP(hipMemcpy2D(s->wp_in, 2 * s->ld_in, s->w_in, 2 * (size_t)s->in_dim, 2 * (size_t)s->in_dim, Wd,
                      hipMemcpyDeviceToDevice));
  ASD_HIP(hipMemcpy2D(s->wp_out, 2 * s->ld_h, s->w_out, 2 * Wd, 2 * Wd, dd, hipMemcpyDeviceToDevice));
  if (nb) {
    ASD_HIP(hipMalloc(&s->wp_blk, sizeof(uint16_t) * nb * Wd * s->ld_h));
    ASD_HIP(hipMemset(s->wp_blk, 0, sizeof(uint16_t) * nb * Wd * s->ld_h));
    ASD_HIP(hipMemcpy2D(s->wp_blk, 2 * s->ld_h, s->w_blk, 2 * Wd, 2 * Wd, nb * Wd, hipMemcpyDeviceToDevice));
  }
  {
    const size_t max_n = std::max(Wd, dd);
    s->split.rows = ctx->B;
    ASD_HIP(hipMalloc(&s->split.part, sizeof(float) * kMaxSplits * (size_t)ctx->B * max_n));
  }
  ASD_HIP(hipDeviceSynchronize());
  return ASD_OK;
}

void mlp_destroy(asd_ctx* ctx) {
  MlpState* s = ctx->mlp;
  if (!s) return;
  (void)hipFree(s->in_bf);
  (void)hipFree(s->h);
  (void)hipFree(s->hb[0]);
  (void)hipFree(s->hb[1]);
  (void)hipFree(s->wp_in);
  (void)hipFree(s->wp_blk);
  (void)hipFree(s->wp_out);
  (void)hipFree(s->eps_coef);
  (void)hipFree(s->split.part);
  delete s;
  ctx->mlp = nullptr;
}

asd_status mlp_eval(asd_ctx* ctx, const RowPlan& rows, hipStream_t st) {
  MlpState* s = ctx->mlp;
  const int n = rows.n, d = ctx->d, W = s->width;
  s->split.small_verify = ctx->cur_win != nullptr;
  {
    ProfScope ps(ctx, ASD_PROF_MLP_PACK, rows.call, st);
    const int groups = s->in_dim / 8;
    const int threads = groups >= 256 ? 256 : 64;
    dim3 grid((unsigned)n, (unsigned)ceil_div(groups, threads));
    hipLaunchKernelGGL(mlp_pack_kernel, grid, dim3(threads), 0, st, rows.n_dev, n, d, s->E, rows.in_base, rows.in_off,
                       rows.tau, s->temb, s->in_bf, s->ld_in, s->in_plane);
    ASD_HIP(hipGetLastError());
  }
  {
    ProfScope ps(ctx, ASD_PROF_MLP_GEMM_IN, rows.call, st);
    ASD_HIP(mlp_gemm(rows.call, rows.n_dev, n, W, s->in_dim, s->ld_in, s->in_bf, s->in_plane, s->wp_in,
                     InEpi{s->h, s->hb[0], s->b_in, W, s->ld_h, s->h_plane}, st, s->split));
  }
  int cur = 0;
  for (int l = 0; l < s->n_blocks; ++l) {
    ProfScope ps(ctx, ASD_PROF_MLP_GEMM_BLK, rows.call, st);
    const BlockEpi e{s->h, s->hb[cur ^ 1], s->b_blk ? s->b_blk + (size_t)l * W : nullptr, W, s->ld_h, s->h_plane};
    ASD_HIP(mlp_gemm(rows.call, rows.n_dev, n, W, W, s->ld_h, s->hb[cur], s->h_plane,
                     s->wp_blk + (size_t)l * W * s->ld_h, e, st, s->split));
    cur ^= 1;
  }
  {
    ProfScope ps(ctx, ASD_PROF_MLP_GEMM_OUT, rows.call, st);
    const OutEpi e{rows.out_base, rows.out_off, s->b_out, s->out_clip, s->eps_coef, rows.tau, rows.in_base, rows.in_off};
    ASD_HIP(mlp_gemm(rows.call, rows.n_dev, n, d, W, s->ld_h, s->hb[cur], s->h_plane, s->wp_out, e, st, s->split));
  }
  return ASD_OK;
}

}  // namespace asd
