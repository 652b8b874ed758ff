// Residual-MLP denoiser (stand-in for the paper's trained networks; the
// diffusion-policy and image-shaped workloads):
//   in  = [ bf16(x) ; temb[tau] ]                    (d + E)
//   h   = W_in in + b_in
//   h  += SiLU( W_l bf16(h) + b_l )                  l = 0..n_blocks-1
//   out = W_out bf16(h) + b_out,  D = clamp(out, -clip, clip)   interpreted as E[x_0 | x]
// Every matrix product takes bf16 inputs and accumulates in fp32 on the matrix
// cores; bias, SiLU and the residual stream are fp32 and are fused into the
// GEMM epilogues, which also emit the bf16 copy of h the next product reads.
#include "common.h"
#include "gemm_bf16.h"

namespace asd {

struct MlpState {
  int width = 0, n_blocks = 0, E = 0, in_dim = 0;
  float out_clip = 0.f;
  const uint16_t* w_in = nullptr;
  const uint16_t* w_blk = nullptr;
  const uint16_t* w_out = nullptr;
  const float* b_in = nullptr;
  const float* b_blk = nullptr;
  const float* b_out = nullptr;
  const uint16_t* temb = nullptr;
  uint16_t* in_bf = nullptr;  // [rows_max, in_dim]
  float* h = nullptr;         // [rows_max, width]
  uint16_t* hb[2] = {nullptr, nullptr};
};

// in_bf[n] = [ bf16(x_n) ; temb[tau_n] ], eight elements per thread
__global__ void mlp_pack_kernel(const int* __restrict__ n_dev, int n_rows, int d, int E, const float* __restrict__ in_base,
                                const int64_t* __restrict__ in_off, const int32_t* __restrict__ tau,
                                const uint16_t* __restrict__ temb, uint16_t* __restrict__ in_bf) {
  const int n = blockIdx.x;
  const int q = blockIdx.y * blockDim.x + threadIdx.x;  // group of 8 elements
  const int in_dim = d + E;
  if (q * 8 >= in_dim || n >= min(*n_dev, n_rows)) return;
  uint4 o;
  if (q * 8 < d) {
    const float* x = in_base + in_off[n] + q * 8;
    const float4 lo = *reinterpret_cast<const float4*>(x);
    const float4 hi = *reinterpret_cast<const float4*>(x + 4);
    o.x = (uint32_t)f32_to_bf16_rne(lo.x) | ((uint32_t)f32_to_bf16_rne(lo.y) << 16);
    o.y = (uint32_t)f32_to_bf16_rne(lo.z) | ((uint32_t)f32_to_bf16_rne(lo.w) << 16);
    o.z = (uint32_t)f32_to_bf16_rne(hi.x) | ((uint32_t)f32_to_bf16_rne(hi.y) << 16);
    o.w = (uint32_t)f32_to_bf16_rne(hi.z) | ((uint32_t)f32_to_bf16_rne(hi.w) << 16);
  } else {
    o = *reinterpret_cast<const uint4*>(temb + (int64_t)tau[n] * E + (q * 8 - d));
  }
  *reinterpret_cast<uint4*>(in_bf + (int64_t)n * in_dim + q * 8) = o;
}

__device__ __forceinline__ float silu(float z) { return z / (1.0f + expf(-z)); }

struct InEpi {  // h = acc + b; hb = bf16(h)
  float* h;
  uint16_t* hb;
  const float* bias;
  int64_t ld;
  __device__ __forceinline__ void operator()(int m, int n, float acc) const {
    const float v = acc + (bias ? bias[n] : 0.f);
    h[(int64_t)m * ld + n] = v;
    hb[(int64_t)m * ld + n] = f32_to_bf16_rne(v);
  }
};

struct BlockEpi {  // h += SiLU(acc + b); hb_next = bf16(h)
  float* h;
  uint16_t* hb_next;
  const float* bias;
  int64_t ld;
  __device__ __forceinline__ void operator()(int m, int n, float acc) const {
    const int64_t o = (int64_t)m * ld + n;
    const float v = h[o] + silu(acc + (bias ? bias[n] : 0.f));
    h[o] = v;
    hb_next[o] = f32_to_bf16_rne(v);
  }
};

struct OutEpi {  // out[out_off[m] + n] = acc + b
  float* out_base;
  const int64_t* out_off;
  const float* bias;
  float clip;  // 0: none
  __device__ __forceinline__ void operator()(int m, int n, float acc) const {
    float v = acc + (bias ? bias[n] : 0.f);
    if (clip > 0.f) v = fminf(fmaxf(v, -clip), clip);
    out_base[out_off[m] + n] = v;
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
  ASD_HIP(hipMalloc(&s->in_bf, sizeof(uint16_t) * rows * s->in_dim));
  ASD_HIP(hipMalloc(&s->h, sizeof(float) * rows * s->width));
  ASD_HIP(hipMalloc(&s->hb[0], sizeof(uint16_t) * rows * s->width));
  ASD_HIP(hipMalloc(&s->hb[1], sizeof(uint16_t) * rows * s->width));
  return ASD_OK;
}

void mlp_destroy(asd_ctx* ctx) {
  MlpState* s = ctx->mlp;
  if (!s) return;
  (void)hipFree(s->in_bf);
  (void)hipFree(s->h);
  (void)hipFree(s->hb[0]);
  (void)hipFree(s->hb[1]);
  delete s;
  ctx->mlp = nullptr;
}

asd_status mlp_eval(asd_ctx* ctx, const RowPlan& rows, hipStream_t st) {
  MlpState* s = ctx->mlp;
  const int n = rows.n, d = ctx->d, W = s->width;
  {
    ProfScope ps(ctx, ASD_PROF_MLP_PACK, rows.call, st);
    const int groups = s->in_dim / 8;
    const int threads = groups >= 256 ? 256 : 64;
    dim3 grid((unsigned)n, (unsigned)ceil_div(groups, threads));
    hipLaunchKernelGGL(mlp_pack_kernel, grid, dim3(threads), 0, st, rows.n_dev, n, d, s->E, rows.in_base, rows.in_off,
                       rows.tau, s->temb, s->in_bf);
    ASD_HIP(hipGetLastError());
  }
  {
    ProfScope ps(ctx, ASD_PROF_MLP_GEMM_IN, rows.call, st);
    const InEpi e{s->h, s->hb[0], s->b_in, W};
    ASD_HIP(rows.call ? launch_gemm_bf16_nt<1>(rows.n_dev, n, W, s->in_dim, s->in_bf, s->in_dim, s->w_in, s->in_dim, e, st)
                      : launch_gemm_bf16_nt<0>(rows.n_dev, n, W, s->in_dim, s->in_bf, s->in_dim, s->w_in, s->in_dim, e, st));
  }
  int cur = 0;
  for (int l = 0; l < s->n_blocks; ++l) {
    ProfScope ps(ctx, ASD_PROF_MLP_GEMM_BLK, rows.call, st);
    const BlockEpi e{s->h, s->hb[cur ^ 1], s->b_blk ? s->b_blk + (size_t)l * W : nullptr, W};
    const uint16_t* wl = s->w_blk + (size_t)l * W * W;
    ASD_HIP(rows.call ? launch_gemm_bf16_nt<1>(rows.n_dev, n, W, W, s->hb[cur], W, wl, W, e, st)
                      : launch_gemm_bf16_nt<0>(rows.n_dev, n, W, W, s->hb[cur], W, wl, W, e, st));
    cur ^= 1;
  }
  {
    ProfScope ps(ctx, ASD_PROF_MLP_GEMM_OUT, rows.call, st);
    const OutEpi e{rows.out_base, rows.out_off, s->b_out, s->out_clip};
    ASD_HIP(rows.call ? launch_gemm_bf16_nt<1>(rows.n_dev, n, d, W, s->hb[cur], W, s->w_out, W, e, st)
                      : launch_gemm_bf16_nt<0>(rows.n_dev, n, d, W, s->hb[cur], W, s->w_out, W, e, st));
  }
  return ASD_OK;
}

}  // namespace asd
