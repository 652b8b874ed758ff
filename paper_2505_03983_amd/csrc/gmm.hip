// Gaussian-mixture posterior-mean denoiser  D(x, tau) = E[x_0 | x_tau = x]
// for data  sum_k w_k N(mu_k, s2 I)  (the mean function m(t, y) of Eq. sl-defn
// for that law): the "model call" of Alg. 1 in the analytic workloads.
//
// (DDPM coordinates; the same four coefficients per time index express the SL mean function, see gmm_create)
// With ab = abar[tau], V = ab*s2 + 1 - ab:
//   logit_k = (sqrt(ab)/V) <x, mu_k> - (ab/(2V)) |mu_k|^2 + log w_k     (|x|^2 cancels)
//   r       = softmax(logit)
//   D       = (sqrt(ab) s2 / V) x + (1 - ab s2 / V) sum_k r_k mu_k
// i.e. single-head attention with keys = values = the component means.
//
// Two paths:
//  * row-wise kernel (one wavefront per row) for small or oddly shaped
//    problems, where a launch is latency-bound anyway;
//  * matrix-core path for large aligned problems: logits = X M^T (MFMA GEMM
//    with the affine map fused in the epilogue) materialised in HBM
//    [rows, C] -- at 288 GB of HBM the 1 GB of logits of the largest workload
//    costs ~4% of the GEMM time to write and re-read, and keeps both GEMMs at
//    full tile efficiency with head dimension d = 1024 -- then P M (second
//    MFMA GEMM against the pre-transposed means) with the softmax fused into
//    its operand load and the final affine combination into its epilogue.
//    By default on the 16-bit matrix pipes with split operands (gemm_split3.h;
//    two fp16 or three bf16 terms, fp32 accuracy), else on the fp32 pipe
//    (gemm_f32.h).
//
// The verify call of the split path leaves out the matrix work whose result is
// an exact zero, bit-identically (sections below, in this order of the call):
//  0. certificate: row tiles whose rows are provably one-hot on the component their chain's draft-call row sat on
//     are written in closed form and skip everything else;
//  1. screening: an int8 product with a rigorous error bound finds the tiles
//     of logits that cannot hold a softmax weight other than 0.0f;
//  2. the first GEMM computes the other tiles only (list form of the kernel);
//  3. row maxima and live column groups once per row tile; rows with a single
//     non-zero weight are written in closed form;
//  4. the second GEMM visits the live K slabs of the remaining row tiles.
#include "common.h"
#include "device_util.h"
#include "gemm_bf16_pipe.h"
#include "gemm_i8_stream.h"
#include "gemm_f32.h"
#include "gemm_split3.h"
#include "gemm_split2_big.h"
#include "gmm_state.h"
#include "gmm_cert.h"

namespace asd {

// verify call: tens of thousands of rows.  Measured on workload 5 (share of the fp32 MFMA peak, logits /
// combine GEMM): 128x128x16 74 / 76%, 128x128x32 71 / 71%, 256x128x16 60 / 56%, 256x128x32 61 / 42%.
typedef GemmCfg<128, 128, 16> GmmTile;
typedef GemmCfg<64, 64, 32> GmmTileSkinny;                    // draft call: one row per chain, fill the chip
// verify call on the bf16 matrix pipe with three-way split operands (fp32 accuracy; shapes that are multiples of 16 only)
typedef Split3Cfg<128, 128, 2, 2> GmmTileSplit;
// draft call on the same pipe: half-height tiles, four wavefronts of 32 x 64, K slabs of 32
typedef Split3Cfg<64, 128, 2, 2, 32> GmmTileSplitSkinny;
// d and C multiples of 32: both GEMMs of both calls with two fp16 terms per operand and three products, K slabs of 32;
// one image of an operand serves the full and the half-height tiling.  (Otherwise: the verify call on the two bf16
// tilings above, the draft call on the fp32 pipe.)
typedef Split3Cfg<128, 128, 2, 2, 32, 2> GmmTile2;
typedef Split3Cfg<64, 128, 2, 2, 32, 2> GmmTile2Skinny;
// ... and verify calls of at least kBigRows rows, where every tile is wanted, on 256 x 256 tiles (gemm_split2_big.h):
// the same terms in the same order per element, so the same bits; 64-column groups of partial maxima as the others
constexpr int kBigRows = 16384;
static_assert(Split2BigCfg::WN == GmmTile2::WN && Split2BigCfg::BM % 128 == 0, "partial maxima and row flags");
static_assert(GmmTile2::BN == GmmTileSplit::BN && GmmTile2::WGN == GmmTileSplit::WGN && GmmTile2::BM == GmmTileSplit::BM &&
              GmmTile2::B_STAGE == GmmTile2Skinny::B_STAGE && GmmTile2::BK == GmmTile2Skinny::BK,
              "the tilings lay rows, row maxima and images out alike");

// (kappa, gamma, cx, cm) of a row
__device__ __forceinline__ float4 row_coef(const float4* coef_tau, const int32_t* tau, int n) {
  return coef_tau[tau[n]];
}

// ---------------------------------------------------------------------------
// preparation kernels
// ---------------------------------------------------------------------------
__global__ void gmm_prep_kernel(int C, int d, const float* __restrict__ means, float* __restrict__ means_t,
                                float* __restrict__ musq) {
  const int k = blockIdx.x;
  float s = 0.f;
  for (int j = threadIdx.x; j < d; j += blockDim.x) {
    const float m = means[(int64_t)k * d + j];
    means_t[(int64_t)j * C + k] = m;
    s = fmaf(m, m, s);
  }
  __shared__ float red[256];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) musq[k] = red[0];
}

// Largest |v[i]| as the bits of a float (non-negative floats order like their bit patterns); *out = 0 on entry.
__global__ __launch_bounds__(256) void gmm_absmax_kernel(const float* __restrict__ v, int64_t n, uint32_t* __restrict__ out) {
  float mx = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) mx = fmaxf(mx, fabsf(v[i]));
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) atomicMax(out, __float_as_uint(mx));
}

// The power of two that brings a largest magnitude mx into [2^14, 2^15): fp16's largest finite number is 65504, and
// the larger the scaled values, the less of their second terms falls below fp16's normal range.  1 for 0, inf, NaN.
__host__ __device__ __forceinline__ float fp16_scale(float mx) {
  if (!(mx > 0.f) || !(mx < 3.0e38f)) return 1.f;
  int e;
  (void)frexpf(mx, &e);   // mx = f 2^e, f in [0.5, 1)
  return ldexpf(1.f, max(-100, min(100, 15 - e)));
}

// The means as the two fp16 terms of the split carry them: out = (m1 + m2) / scale with m1 = the nearest fp16 of
// scale * v, m2 = the nearest fp16 of scale * v - m1 (both differences and the sum are exact in fp32).  A row of
// softmax weights (1, 0, 0, ...) gets exactly this from the second GEMM on fp16 terms.
__global__ __launch_bounds__(256) void gmm_means22_kernel(const float* __restrict__ v, int64_t n, float scale,
                                                          float* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float x = scale * v[i];
  const float m1 = (float)(_Float16)x;
  const float m2 = (float)(_Float16)(x - m1);
  out[i] = (m1 + m2) / scale;
}

// a_scale[m] = fp16_scale(largest |x| of row m), for the rows a split-operand GEMM with fp16 terms will read: one
// wavefront per row.  skip_tile (or NULL): row tiles of 128 rows nobody reads.
__global__ __launch_bounds__(256) void gmm_row_scale_kernel(const int* __restrict__ n_dev, int n_max, int d,
                                                            const float* __restrict__ in_base,
                                                            const int64_t* __restrict__ in_off,
                                                            float* __restrict__ a_scale,
                                                            const uint8_t* __restrict__ skip_tile) {
  const int lane = threadIdx.x & 63, m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= min(*n_dev, n_max)) return;
  if (skip_tile && skip_tile[m / 128]) return;
  const float* x = in_base + in_off[m];
  float mx = 0.f;
  if ((d & 3) == 0) {
    const float4* x4 = reinterpret_cast<const float4*>(x);
    for (int j = lane; j < d / 4; j += 64) {
      const float4 v = x4[j];
      mx = fmaxf(fmaxf(mx, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    }
  } else {
    for (int j = lane; j < d; j += 64) mx = fmaxf(mx, fabsf(x[j]));
  }
  mx = wave_max(mx);
  if (lane == 0) a_scale[m] = fp16_scale(mx);
}

// ---------------------------------------------------------------------------
// row-wise path: 4 wavefronts per workgroup, one row per wavefront per pass
// LDS per wavefront: x[d] then p[C]
// ---------------------------------------------------------------------------
constexpr float kZeroGapNat = kCertZeroGap * 0.6931471805599453f;   // the zero gap in the natural-log units of these kernels
__global__ __launch_bounds__(256) void gmm_rowwise_kernel(const int* __restrict__ n_dev, int nrows_max, int d, int C, const float* __restrict__ in_base,
                                                          const int64_t* __restrict__ in_off,
                                                          float* __restrict__ out_base,
                                                          const int64_t* __restrict__ out_off,
                                                          const int32_t* __restrict__ tau,
                                                          const float4* __restrict__ coef_tau,
                                                          const float* __restrict__ means,
                                                          const float* __restrict__ musq,
                                                          const float* __restrict__ log_w) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  float* xs = lds + (size_t)wave * (d + C);
  float* ps = xs + d;
  const int nrows = min(*n_dev, nrows_max);
  for (int base = blockIdx.x * 4; base < nrows; base += gridDim.x * 4) {
    const int n = base + wave;
    const bool active = n < nrows;
    float4 cf = make_float4(0.f, 0.f, 0.f, 0.f);
    const float* x = nullptr;
    if (active) {
      cf = row_coef(coef_tau, tau, n);
      x = in_base + in_off[n];
      for (int j = lane; j < d; j += 64) xs[j] = x[j];
    }
    __syncthreads();
    float mx = -INFINITY;
    if (active) {
      for (int k = lane; k < C; k += 64) {
        const float* mu = means + (int64_t)k * d;
        float dot = 0.f;
        for (int j = 0; j < d; ++j) dot = fmaf(xs[j], mu[j], dot);
        const float lg = fmaf(cf.x, dot, fmaf(-cf.y, musq[k], log_w[k]));
        ps[k] = lg;
        mx = fmaxf(mx, lg);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float sum = 0.f;
    if (active) {
      for (int k = lane; k < C; k += 64) {
        const float p = (ps[k] - mx < -kZeroGapNat) ? 0.f : expf(ps[k] - mx);
        ps[k] = p;
        sum += p;
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    __syncthreads();
    if (active) {
      const float inv = 1.0f / sum;
      float* out = out_base + out_off[n];
      for (int j = lane; j < d; j += 64) {
        float acc = 0.f;
        for (int k = 0; k < C; ++k) acc = fmaf(ps[k], means[(int64_t)k * d + j], acc);
        out[j] = fmaf(cf.z, xs[j], cf.w * (acc * inv));
      }
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// row-wise path with the mixture in LDS (d % 4 == 0 and C*(d+4) floats fit): the workgroup copies
// the means (rows padded by 4 floats, so that 16 lanes reading the same 16-byte column of 16
// different rows hit 16 different bank groups), |mu|^2 and log w into LDS, then each wavefront
// serves rows from it.  No cross-lane traffic inside the loops:
//   pass 1: lane = component: <x, mu_k> over d from LDS (x is a broadcast read),
//   pass 2: softmax over the C logits (two wavefront reductions),
//   pass 3: lane = coordinate: sum_k p_k mu_k[j] (p is a broadcast read).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gmm_rowwise_lds_kernel(const int* __restrict__ n_dev, int nrows_max, int d,
                                                              int C, int rows_per_wave,
                                                              const float* __restrict__ in_base,
                                                              const int64_t* __restrict__ in_off,
                                                              float* __restrict__ out_base,
                                                              const int64_t* __restrict__ out_off,
                                                              const int32_t* __restrict__ tau,
                                                              const float4* __restrict__ coef_tau,
                                                              const float* __restrict__ means,
                                                              const float* __restrict__ musq,
                                                              const float* __restrict__ log_w) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int d4 = d >> 2, dp = d + 4, C4 = (C + 3) & ~3;
  const int nrows = min(*n_dev, nrows_max);
  if (blockIdx.x * 4 * rows_per_wave >= nrows) return;
  float* m_l = lds;                          // [C][dp]
  float* q_l = m_l + (size_t)C * dp;         // [C]
  float* lw_l = q_l + C4;                    // [C]
  float* ps = lw_l + C4 + (size_t)wave * C4; // [4][C4] logits, then softmax weights
  float* xs = lw_l + C4 + 4 * (size_t)C4 + (size_t)wave * d;  // [4][d]
  {
    const float4* Mg = reinterpret_cast<const float4*>(means);
    for (int t = threadIdx.x; t < C * d4; t += 256) {
      const int k = t / d4, c = t - k * d4;
      *reinterpret_cast<float4*>(&m_l[k * dp + 4 * c]) = Mg[t];
    }
    for (int t = threadIdx.x; t < C; t += 256) {
      q_l[t] = musq[t];
      lw_l[t] = log_w[t];
    }
  }
  __syncthreads();
  for (int it = 0; it < rows_per_wave; ++it) {
    const int n = (blockIdx.x * rows_per_wave + it) * 4 + wave;
    if (n >= nrows) break;  // uniform per wavefront; no workgroup barrier below
    const float4 cf = coef_tau[tau[n]];
    const float* x = in_base + in_off[n];
    for (int j = lane; j < d; j += 64) xs[j] = x[j];
    // (LDS operations of one wavefront complete in order: xs is visible to all its lanes below)
    float mx = -INFINITY;
    for (int k = lane; k < C; k += 64) {
      const float* mk = m_l + k * dp;
      float dot = 0.f;
#pragma unroll 4
      for (int c = 0; c < d4; ++c) {
        const float4 xv = *reinterpret_cast<const float4*>(&xs[4 * c]);
        const float4 mv = *reinterpret_cast<const float4*>(&mk[4 * c]);
        dot = fmaf(xv.x, mv.x, fmaf(xv.y, mv.y, fmaf(xv.z, mv.z, fmaf(xv.w, mv.w, dot))));
      }
      const float lg = fmaf(cf.x, dot, fmaf(-cf.y, q_l[k], lw_l[k]));
      ps[k] = lg;
      mx = fmaxf(mx, lg);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float sum = 0.f;
    for (int k = lane; k < C4; k += 64) {
      const float p = (k < C && !(ps[k] - mx < -kZeroGapNat)) ? expf(ps[k] - mx) : 0.f;
      ps[k] = p;
      sum += p;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    const float sc = cf.w / sum;
    float* out = out_base + out_off[n];
    for (int j = lane; j < d; j += 64) {
      float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
      const float* mj = m_l + j;
#pragma unroll 2
      for (int k = 0; k < C4; k += 4) {
        const float4 p = *reinterpret_cast<const float4*>(&ps[k]);
        // rows past C do not exist: their weights are 0 and the reads are clamped to the last row
        a0 = fmaf(p.x, mj[min(k + 0, C - 1) * dp], a0);
        a1 = fmaf(p.y, mj[min(k + 1, C - 1) * dp], a1);
        a2 = fmaf(p.z, mj[min(k + 2, C - 1) * dp], a2);
        a3 = fmaf(p.w, mj[min(k + 3, C - 1) * dp], a3);
      }
      out[j] = fmaf(cf.z, xs[j], sc * ((a0 + a1) + (a2 + a3)));
    }
  }
}

// ---------------------------------------------------------------------------
// matrix-core path
// ---------------------------------------------------------------------------
// GEMM 1: logits.  The epilogue applies the affine map, stores the logits and
// the maximum of each row over the columns the wavefront owns
// (pmax[row][WGN*column_tile + wn]); the softmax normalisation is finished
// inside GEMM 2, so the logits are written once and read once.
struct LogitOp {
  static constexpr bool kSplitK = false;
  static constexpr bool kSparseK = false;
  static constexpr bool kTileList = true;
  static constexpr bool kRowTileSkip = true;
  float* logits;
  int64_t ld;
  float* pmax;
  int np;  // partial maxima per row = (wavefronts across a tile) * (number of column tiles)
  const float4* coef_tau;
  const int32_t* tau;
  const float* musq;
  const float* log_w;
  // NULL, or the lists of tiles the screening pass below wants computed (see the list form of the kernel for the
  // layout).  The tiles left out hold only logits more than CombineOp::kZeroGap below the maxima of their rows; the
  // screening pass has set their partial maxima to -inf, which the second GEMM reads as "all weights zero, skip",
  // and the logits themselves are never read.
  const uint32_t* tile_list = nullptr;
  const int32_t* tile_count = nullptr;
  int list_cap = 0;
  // NULL, or [row tiles of kSkipTile rows]: 1 = nobody will read this tile's logits (the one-hot certificate below
  // has written its rows)
  const uint8_t* skip_tile = nullptr;
  // Operand scales of the fp16-term kernels (powers of two; 1 elsewhere): row m of A is multiplied by a_scale[m]
  // (NULL: 1) on its way into the split, B's image holds b_scale B, and the epilogue takes both out again (exactly)
  const float* a_scale = nullptr;
  float b_scale = 1.f;
  static constexpr int kMaxPasses = 8;
  float asc[kMaxPasses];
  static constexpr int kSkipTile = 128;
  __device__ __forceinline__ bool skip_row_tile(int m0) const { return skip_tile && skip_tile[m0 / kSkipTile] != 0; }
  template <int BM>   // a taller tile (gemm_split2_big.h): every flag of its rows m0 .. min(m0 + BM, M) - 1
  __device__ __forceinline__ bool skip_rows(int m0, int M) const {
    if (!skip_tile) return false;
    for (int m = m0; m < min(m0 + BM, M); m += kSkipTile)
      if (!skip_tile[m / kSkipTile]) return false;
    return true;
  }
  static constexpr float kLog2e = 1.4426950408889634f;  // logits are stored in base-2 units for the exp2 of GEMM 2
  // s_row[8 r + 1], [8 r + 2]: log2(e) kappa, log2(e) gamma of tile row r
  template <class Cfg>
  __device__ __forceinline__ void init(int m0, int M, int lrow, int lkq, float* s_row) {
    static_assert(Cfg::RA <= kMaxPasses, "loader passes");
#pragma unroll
    for (int p = 0; p < Cfg::RA; ++p) {
      const int r = lrow + Cfg::RPP * p;
      const int m = min(m0 + r, M - 1);
      asc[p] = a_scale ? a_scale[m] : 1.f;
      if (lkq != 0) continue;
      const float4 cf = coef_tau[tau[m]];
      s_row[8 * r + 1] = (kLog2e * cf.x) / (asc[p] * b_scale);   // (a division by a power of two: exact)
      s_row[8 * r + 2] = kLog2e * cf.y;
    }
  }
  __device__ __forceinline__ float4 load_a(float4 v, int p) const {
    const float s = asc[p];
    return make_float4(s * v.x, s * v.y, s * v.z, s * v.w);
  }
  template <class Cfg>
  __device__ __forceinline__ void finish(int, int, float*) {}
  template <class Cfg>
  __device__ __forceinline__ void epilogue(const v16f (&acc)[Cfg::MI][Cfg::NJ], const Frag<Cfg>& fr, int m0, int n0,
                                           int M, int N, const float* s_row) const {
    constexpr int MI = Cfg::MI, NJ = Cfg::NJ;
    float bias[NJ], q[NJ];
    bool nok[NJ];
    int n[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int nn = n0 + fr.col(j);
      nok[j] = nn < N;
      n[j] = nok[j] ? nn : N - 1;
      bias[j] = kLog2e * log_w[n[j]];
      q[j] = musq[n[j]];
    }
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int ml = fr.row(i, r);
        const int m = m0 + ml;
        const bool mok = m < M;
        const float c1 = s_row[8 * ml + 1], c2 = s_row[8 * ml + 2];
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const float v = fmaf(c1, acc[i][j][r], fmaf(-c2, q[j], bias[j]));
          if (nok[j]) {
            mx = fmaxf(mx, v);
            if (mok) logits[(int64_t)m * ld + n[j]] = v;
          }
        }
        // maximum over the 32 lanes of the half-wave: four DPP steps inside each row of 16 lanes, then one
        // cross-lane exchange between the two rows (a full butterfly of shuffles costs five LDS round trips)
        mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mx), 0xB1, 0xf, 0xf, true)));
        mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mx), 0x4E, 0xf, 0xf, true)));
        mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mx), 0x141, 0xf, 0xf, true)));
        mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mx), 0x140, 0xf, 0xf, true)));
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        if (mok && fr.l32 == 0) pmax[(int64_t)m * np + Cfg::WGN * fr.tile_n + fr.wn] = mx;
      }
    }
  }
};

// GEMM 2: out = c_x' x + c_m' (softmax(logits) M).  The A operand is turned
// into exp(logit - rowmax) on its way into LDS; the row sums are accumulated on
// the side and divided out in the epilogue.
struct CombineOp {
  static constexpr bool kSplitK = true;
  static constexpr bool kSparseK = true;
  static constexpr bool kTileList = false;
  const float* pmax;
  int np;
  int gcols;  // logits columns behind one partial maximum (sub-tile width of the first GEMM), 0: unknown
  // Weights below 2^-kZeroGap of the row's largest are zero by definition (gmm_cert.h): load_a gives 0.0f for a logit
  // below lo = row maximum - kZeroGap.  Sparse K: column group q (the columns behind pmax[.][q]) is dead for a row when
  // its largest logit lies below the same lo (the same fp32 expression, so "left out" and "computed" agree bit for
  // bit): every product of the group is then an exact zero.
  static constexpr float kZeroGap = 40.0f;
  static_assert(kZeroGap == kCertZeroGap, "the certificate proves weights zero by this gap");
  // NULL, or what gmm_rowmax_kernel made of pmax once for all the column tiles of a row tile: the row maxima [rows]
  // and the live flag of every column group [row tiles of kRowmaxTile rows][np]
  const float* rmax_pre = nullptr;
  const uint8_t* live_pre = nullptr;
  static constexpr int kRowmaxTile = 128;
  // NULL, or [row tiles of kRowmaxTile rows]: 1 = every row of the tile has one weight of 1.0 and zeros, and
  // gmm_onehot_kernel writes its results in closed form (below): the tile's workgroups have nothing to do
  const uint8_t* onehot_tile = nullptr;
  static constexpr bool kRowTileSkip = true;
  __device__ __forceinline__ bool skip_row_tile(int m0) const { return onehot_tile && onehot_tile[m0 / kRowmaxTile] != 0; }
  // A taller tile (gemm_split2_big.h) is skipped when every flag of its rows is set; when only some are, the rows
  // behind them are computed along (on whatever their logits hold) and not stored (the epilogue's per-row flag).
  template <int BM>
  __device__ __forceinline__ bool skip_rows(int m0, int M) const {
    if (!onehot_tile) return false;
    for (int m = m0; m < min(m0 + BM, M); m += kRowmaxTile)
      if (!onehot_tile[m / kRowmaxTile]) return false;
    return true;
  }
  __host__ __device__ __forceinline__ int groups() const { return np; }
  __host__ __device__ __forceinline__ int group_cols() const { return gcols; }
  template <class Cfg>
  __device__ __forceinline__ void mark_live(int m0, int M, int lrow, int lkq, uint8_t* flags) const {
    if (live_pre) {
      static_assert(Cfg::BM * 2 == kRowmaxTile || Cfg::BM % kRowmaxTile == 0, "row tiles of the precomputed flags");
      const uint8_t* src = live_pre + (int64_t)(m0 / kRowmaxTile) * np;   // (a half-height tile takes its parent's flags)
      if constexpr (Cfg::BM <= kRowmaxTile) {
        for (int q = lrow * Cfg::KQ + lkq; q < np; q += Cfg::THREADS) flags[q] = src[q];
      } else {   // a taller tile: what any of its row tiles wants, those written in closed form aside
        for (int q = lrow * Cfg::KQ + lkq; q < np; q += Cfg::THREADS) {
          uint8_t f = 0;
          for (int s = 0; s < Cfg::BM / kRowmaxTile && m0 + s * kRowmaxTile < M; ++s)
            if (!(onehot_tile && onehot_tile[m0 / kRowmaxTile + s])) f |= src[(int64_t)s * np + q];
          flags[q] = f;
        }
      }
      return;
    }
#pragma unroll
    for (int p = 0; p < Cfg::RA; ++p) {
      const int m = min(m0 + lrow + Cfg::RPP * p, M - 1);
      const float lo = rmax[p] - kZeroGap;
      for (int q = lkq; q < np; q += Cfg::KQ)
        if (pmax[(int64_t)m * np + q] >= lo) flags[q] = 1;
    }
  }
  const float* in_base;
  const int64_t* in_off;
  float* out_base;
  const int64_t* out_off;
  const float4* coef_tau;
  const int32_t* tau;
  unsigned long long* work = nullptr;   // NULL, or DEV [2]: += K slabs this workgroup visits, += K slabs there are
  __device__ __forceinline__ void note_slabs(int visited, int all, int tid) const {
    if (work && tid == 0) {
      atomicAdd(&work[0], (unsigned long long)visited);
      atomicAdd(&work[1], (unsigned long long)all);
    }
  }
  static constexpr int kMaxPasses = 8;
  float rmax[kMaxPasses];
  float rsum[kMaxPasses];
  // Operand scales of the fp16-term kernels (powers of two; 1 elsewhere): the weights -- at most 1 -- go into the
  // split times a_scale, B's image holds b_scale B, and the epilogue takes both out again (exactly).  The row sums
  // are those of the unscaled weights.
  float a_scale = 1.f, b_scale = 1.f;
  // s_row[8 r ..]: row sum, c_x', c_m' / (a_scale b_scale), 1 = do not store, in_off (8 bytes), out_off (8 bytes) of tile row r
  template <class Cfg>
  __device__ __forceinline__ void init(int m0, int M, int lrow, int lkq, float* s_row) {
    static_assert(Cfg::RA <= kMaxPasses, "loader passes");
#pragma unroll
    for (int p = 0; p < Cfg::RA; ++p) {
      const int r = lrow + Cfg::RPP * p;
      const int m = min(m0 + r, M - 1);
      float mx = -INFINITY;
      if (rmax_pre) {
        mx = rmax_pre[m];
      } else {
        for (int q = lkq; q < np; q += Cfg::KQ) mx = fmaxf(mx, pmax[(int64_t)m * np + q]);
#pragma unroll
        for (int o = 1; o < Cfg::KQ; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));  // the KQ lanes of a row are adjacent
      }
      rmax[p] = mx;
      rsum[p] = 0.f;
      if (lkq == 0) {
        const float4 cf = coef_tau[tau[m]];
        s_row[8 * r + 1] = cf.z;
        s_row[8 * r + 2] = cf.w / (a_scale * b_scale);   // (a division by a power of two: exact)
        s_row[8 * r + 3] = (onehot_tile && onehot_tile[m / kRowmaxTile]) ? 1.f : 0.f;   // written in closed form: not ours
        *reinterpret_cast<int64_t*>(&s_row[8 * r + 4]) = in_off[m];
        *reinterpret_cast<int64_t*>(&s_row[8 * r + 6]) = out_off[m];
      }
    }
  }
  // logits are in base-2 units: p = 2^(l - rowmax) <= 1
  __device__ __forceinline__ float4 load_a(float4 v, int p) {
    const float mx = rmax[p], lo = mx - kZeroGap;
    float4 e = make_float4(v.x < lo ? 0.f : __builtin_amdgcn_exp2f(v.x - mx), v.y < lo ? 0.f : __builtin_amdgcn_exp2f(v.y - mx),
                           v.z < lo ? 0.f : __builtin_amdgcn_exp2f(v.z - mx), v.w < lo ? 0.f : __builtin_amdgcn_exp2f(v.w - mx));
    rsum[p] += (e.x + e.y) + (e.z + e.w);
    return make_float4(a_scale * e.x, a_scale * e.y, a_scale * e.z, a_scale * e.w);
  }
  template <class Cfg>
  __device__ __forceinline__ void finish(int lrow, int lkq, float* s_row) {
#pragma unroll
    for (int p = 0; p < Cfg::RA; ++p) {
      float s = rsum[p];
#pragma unroll
      for (int o = 1; o < Cfg::KQ; o <<= 1) s += __shfl_xor(s, o, 64);
      if (lkq == 0) s_row[8 * (lrow + Cfg::RPP * p)] = s;
    }
  }
  // split K: the partial tile and (from the workgroups of column tile 0) the partial row sums, for combine_finish_kernel
  template <class Cfg>
  __device__ __forceinline__ void store_partial(const v16f (&acc)[Cfg::MI][Cfg::NJ], const Frag<Cfg>& fr, int m0,
                                                int n0, int M, int M_max, int N, const float* s_row, float* part,
                                                int z, int splits) const {
    float* tile = part + (size_t)z * M_max * N;
    float* psum = part + (size_t)splits * M_max * N + (size_t)z * M_max;
#pragma unroll
    for (int i = 0; i < Cfg::MI; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int ml = fr.row(i, r), m = m0 + ml;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < Cfg::NJ; ++j) {
          const int n = n0 + fr.col(j);
          if (n < N) tile[(size_t)m * N + n] = acc[i][j][r];
        }
        if (n0 == 0 && fr.wn == 0 && fr.l32 == 0) psum[m] = s_row[8 * ml];
      }
  }
  template <class Cfg>
  __device__ __forceinline__ void epilogue(const v16f (&acc)[Cfg::MI][Cfg::NJ], const Frag<Cfg>& fr, int m0, int n0,
                                           int M, int N, const float* s_row) const {
    constexpr int NJ = Cfg::NJ, RB = 8;   // rows per batch: all of a batch's reads of x are issued before its stores
#pragma unroll
    for (int i = 0; i < Cfg::MI; ++i) {
#pragma unroll
      for (int r0 = 0; r0 < 16; r0 += RB) {
        float xv[RB][NJ];
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) {
          const int ml = fr.row(i, r0 + rr);
          const float* x = in_base + *reinterpret_cast<const int64_t*>(&s_row[8 * ml + 4]);
#pragma unroll
          for (int j = 0; j < NJ; ++j) {
            const int n = n0 + fr.col(j);
            xv[rr][j] = (m0 + ml < M && n < N) ? x[n] : 0.f;
          }
        }
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) {
          const int ml = fr.row(i, r0 + rr);
          if (m0 + ml >= M || s_row[8 * ml + 3] != 0.f) continue;
          const float cz = s_row[8 * ml + 1];
          const float scale = s_row[8 * ml + 2] / s_row[8 * ml];
          float* o = out_base + *reinterpret_cast<const int64_t*>(&s_row[8 * ml + 6]);
#pragma unroll
          for (int j = 0; j < NJ; ++j) {
            const int n = n0 + fr.col(j);
            if (n < N) o[n] = fmaf(cz, xv[rr][j], scale * acc[i][j][r0 + rr]);
          }
        }
      }
    }
  }
};

// Between the two GEMMs of a verify call: the maximum of every row over its partial maxima, and for every row
// tile the column groups that are live for one of its rows (CombineOp::mark_live's rule) -- once, instead of by
// each of the second GEMM's workgroups that share the row tile (d / 128 of them, each scanning 32 KB).
//
// One-hot rows (onehot != NULL; needs np <= 64 and column groups of 64).  Once a posterior has collapsed a row has
// exactly one logit within kZeroGap of its maximum -- the maximum itself.  Its weights are then 2^0 = 1.0 for that
// component b and exact zeros elsewhere, the row sum is 1.0, and the second GEMM's result for it is known bit for bit:
// the terms of mu_b times the terms of 1.0, added in an order in which every partial sum is exact, all other products
// zeros -- mu_b itself from three bf16 terms, (m1 + m2) / scale from two fp16 terms (gmm_means22_kernel) -- so
// out = fma(c_x', x, c_m' mu_b)  with that mu_b needs no GEMM.  A row's few live groups are scanned for
// that (rows with more than two live groups are not candidates): onehot[row] = b or -1, and onehot_tile[row tile] =
// 1 when all its rows qualify -- the second GEMM then skips the tile and gmm_onehot_kernel writes it.
// The component b of a one-hot row, or -1: called by a whole wavefront with the row's partial maxima p[np] (np <= 64,
// groups of 64 columns), its maximum mx and its logits.
__device__ __forceinline__ int onehot_component(const float* __restrict__ p, int np, float mx,
                                                const float* __restrict__ row_logits, int lane) {
  const float thr = mx - CombineOp::kZeroGap;
  unsigned long long groups = __ballot(lane < np && p[min(lane, np - 1)] >= thr);
  if (__popcll(groups) > 2) return -1;
  int count = 0, b = -1;
  while (groups) {
    const int g = __ffsll((long long)groups) - 1;
    groups &= groups - 1;
    const float v = row_logits[g * 64 + lane];
    count += __popcll(__ballot(v >= thr));
    const unsigned long long at_max = __ballot(v == mx);
    if (at_max) b = g * 64 + __ffsll((long long)at_max) - 1;
  }
  return count == 1 ? b : -1;
}

__global__ __launch_bounds__(256) void gmm_rowmax_kernel(const int* __restrict__ n_dev, int n_max, int np,
                                                         const float* __restrict__ pmax, float* __restrict__ rmax,
                                                         uint8_t* __restrict__ glive,
                                                         const float* __restrict__ logits, int64_t ldl, int gcols,
                                                         int32_t* __restrict__ onehot, uint8_t* __restrict__ onehot_tile,
                                                         const uint8_t* __restrict__ cert_tile,
                                                         unsigned long long* __restrict__ counts) {
  // counts (or NULL): [5] += row tiles found one-hot.  cert_tile (or NULL): row tiles already known to be one-hot
  // (gmm_certify_kernel); their logits do not exist.
  extern __shared__ int s_any[];   // [np], then one flag: every row so far is one-hot
  constexpr int BM = CombineOp::kRowmaxTile, RW = 4;
  const int n = min(*n_dev, n_max);
  const int m0 = blockIdx.x * BM;
  if (m0 >= n) return;
  if (cert_tile && cert_tile[blockIdx.x]) return;
  const bool want_onehot = onehot && np <= 64 && gcols == 64;
  for (int q = threadIdx.x; q < np; q += 256) s_any[q] = 0;
  if (threadIdx.x == 0) s_any[np] = want_onehot ? 1 : 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int r0 = RW * wave; r0 < BM && m0 + r0 < n; r0 += 4 * RW) {
    const float* p[RW];
    float mx[RW];
#pragma unroll
    for (int k = 0; k < RW; ++k) {   // rows past the end repeat the last one
      p[k] = pmax + (int64_t)min(m0 + r0 + k, n - 1) * np;
      mx[k] = -INFINITY;
    }
    for (int q = lane; q < np; q += 64)
#pragma unroll
      for (int k = 0; k < RW; ++k) mx[k] = fmaxf(mx[k], p[k][q]);
#pragma unroll
    for (int k = 0; k < RW; ++k) {
      mx[k] = wave_max(mx[k]);
      if (lane == 0 && m0 + r0 + k < n) rmax[m0 + r0 + k] = mx[k];
    }
    for (int q = lane; q < np; q += 64) {
      bool any = false;
#pragma unroll
      for (int k = 0; k < RW; ++k) any = any || (p[k][q] >= mx[k] - CombineOp::kZeroGap);
      if (any) s_any[q] = 1;
    }
    if (want_onehot) {
#pragma unroll
      for (int k = 0; k < RW; ++k) {
        const int row = m0 + r0 + k;
        if (row >= n) continue;   // the same for the whole wavefront
        const int b = onehot_component(p[k], np, mx[k], logits + (int64_t)row * ldl, lane);
        if (lane == 0) {
          onehot[row] = b;
          if (b < 0) s_any[np] = 0;
        }
      }
    }
  }
  __syncthreads();
  for (int q = threadIdx.x; q < np; q += 256) glive[(int64_t)blockIdx.x * np + q] = (uint8_t)s_any[q];
  if (onehot_tile && threadIdx.x == 0) {
    onehot_tile[blockIdx.x] = (uint8_t)s_any[np];
    if (counts && s_any[np]) atomicAdd(&counts[5], 1ull);
  }
}

// The same for a call of few rows (the draft call: one row per chain), where a workgroup per 128 rows would be eight
// workgroups: one wavefront per row for the maxima and the one-hot components (no live groups: that call's second
// GEMM does not skip slabs), then one small workgroup per row tile for the tile flags.
__global__ __launch_bounds__(256) void gmm_rowmax_rows_kernel(const int* __restrict__ n_dev, int n_max, int np,
                                                              const float* __restrict__ pmax, float* __restrict__ rmax,
                                                              const float* __restrict__ logits, int64_t ldl,
                                                              int32_t* __restrict__ onehot,
                                                              const int32_t* __restrict__ chain,
                                                              int32_t* __restrict__ chain_comp,
                                                              const uint8_t* __restrict__ cert_tile) {
  // chain, chain_comp (or NULL): the component of a one-hot row (or -1) is also kept per chain, as the candidate of
  // the one-hot certificate (gmm_certify_kernel).  cert_tile (or NULL): row tiles it has certified in this call --
  // their rows have no logits, and their chains' candidates stand.
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= min(*n_dev, n_max)) return;
  if (cert_tile && cert_tile[row / CombineOp::kRowmaxTile]) return;
  const float* p = pmax + (int64_t)row * np;
  float mx = -INFINITY;
  for (int q = lane; q < np; q += 64) mx = fmaxf(mx, p[q]);
  mx = wave_max(mx);
  if (lane == 0) rmax[row] = mx;
  if (onehot) {
    const int b = onehot_component(p, np, mx, logits + (int64_t)row * ldl, lane);
    if (lane == 0) {
      onehot[row] = b;
      if (chain && chain_comp) chain_comp[chain[row]] = b;
    }
  }
}
__global__ __launch_bounds__(CombineOp::kRowmaxTile) void gmm_onehot_tiles_kernel(const int* __restrict__ n_dev, int n_max,
                                                                                 const int32_t* __restrict__ onehot,
                                                                                 uint8_t* __restrict__ onehot_tile) {
  const int n = min(*n_dev, n_max), m = blockIdx.x * CombineOp::kRowmaxTile + threadIdx.x;
  if (blockIdx.x * CombineOp::kRowmaxTile >= n) return;
  const int bad = __syncthreads_or(m < n && onehot[m] < 0);
  if (threadIdx.x == 0) onehot_tile[blockIdx.x] = bad ? 0 : 1;
}

// The rows of the one-hot tiles, in closed form (see gmm_rowmax_kernel): kOnehotRows rows per workgroup, four of them
// in flight at a time.  (A workgroup per row was 65 k workgroups at cfg 5's verify call: 14 us of dispatch even when
// every one of them leaves at once, which is the common case.)
constexpr int kOnehotRows = 8;
static_assert(CombineOp::kRowmaxTile % kOnehotRows == 0, "a workgroup's rows lie in one row tile");
__global__ __launch_bounds__(256) void gmm_onehot_kernel(const int* __restrict__ n_dev, int n_max, int d,
                                                         const int32_t* __restrict__ onehot,
                                                         const uint8_t* __restrict__ onehot_tile,
                                                         const float* __restrict__ means,
                                                         const float* __restrict__ in_base,
                                                         const int64_t* __restrict__ in_off,
                                                         float* __restrict__ out_base,
                                                         const int64_t* __restrict__ out_off,
                                                         const float4* __restrict__ coef_tau,
                                                         const int32_t* __restrict__ tau,
                                                         const uint8_t* __restrict__ cert_tile) {
  // cert_tile (or NULL): one-hot row tiles whose rows gmm_certify_kernel has written already
  const int n = min(*n_dev, n_max), m0 = blockIdx.x * kOnehotRows;
  if (m0 >= n) return;
  const int tile = m0 / CombineOp::kRowmaxTile;
  if (!onehot_tile[tile]) return;
  if (cert_tile && cert_tile[tile]) return;
  constexpr int U = 4;
  for (int r0 = 0; r0 < kOnehotRows && m0 + r0 < n; r0 += U) {
    float4 cf[U];
    const float4* x[U];
    const float4* mu[U];
    float4* o[U];
    bool live[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int m = min(m0 + r0 + u, n - 1);
      live[u] = m0 + r0 + u < n;
      cf[u] = coef_tau[tau[m]];
      x[u] = reinterpret_cast<const float4*>(in_base + in_off[m]);
      mu[u] = reinterpret_cast<const float4*>(means + (int64_t)onehot[m] * d);
      o[u] = reinterpret_cast<float4*>(out_base + out_off[m]);
    }
    for (int j = threadIdx.x; j < d / 4; j += 256) {
      float4 xv[U], mv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        xv[u] = x[u][j];
        mv[u] = mu[u][j];
      }
      // what the second GEMM's epilogue computes with acc = mu_b (+0.0: the accumulator never holds a negative zero)
      // and scale = c_m' / 1.0
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (live[u])
          o[u][j] = make_float4(fmaf(cf[u].z, xv[u].x, __fmul_rn(cf[u].w, mv[u].x + 0.f)),
                                fmaf(cf[u].z, xv[u].y, __fmul_rn(cf[u].w, mv[u].y + 0.f)),
                                fmaf(cf[u].z, xv[u].z, __fmul_rn(cf[u].w, mv[u].z + 0.f)),
                                fmaf(cf[u].z, xv[u].w, __fmul_rn(cf[u].w, mv[u].w + 0.f)));
    }
  }
}

// ---------------------------------------------------------------------------
// One-hot certificate of a model call.
//
// Late in a chain a row lies so close to s mu_b -- b the component the chain's last draft-call row was found one-hot
// on -- that the distance from mu_b to its nearest other mean alone proves every other softmax weight an exact zero,
// with no product against the other means.  For a row x, a candidate b (any guess is safe: a wrong one fails the
// test) and any s >= 0, with e = x - s mu_b, D_n = mu_n - mu_b, a_n = |D_n|:
//   logit_n - logit_b  =  kappa' <x, D_n> - gamma' (|mu_n|^2 - |mu_b|^2) + log2 w_n - log2 w_b,
//   <x, D_n>  =  s <mu_b, D_n> + <e, D_n>  <=  s (|mu_n|^2 - |mu_b|^2 - a_n^2) / 2 + |e| a_n        (Cauchy-Schwarz).
// With A = kappa' s, B = kappa' |e| the part that depends on a_n is the parabola  f(a) = -(A/2) a^2 + B a, which
// falls beyond its vertex B / A: if the nearest neighbour of mu_b is at least that far, a_min(b) >= B / A, then
// f(a_n) <= f(a_min(b)) for every n.  What is left, (A/2 - gamma') (|mu_n|^2 - |mu_b|^2) + log2 w_n - log2 w_b, is
// small (A/2 = gamma' at s = sqrt(abar)) and is bounded with the extremes of |mu|^2 and log2 w over the mixture.  So
//   logit_n - logit_b  <=  f(a_min(b)) + (A/2 - gamma') (q* - |mu_b|^2) + max log2 w - log2 w_b      for all n != b,
// q* = max or min |mu|^2 by the sign of the factor: four numbers per row -- s = <x, mu_b> / |mu_b|^2, which makes |e|
// least, |e|, |x| -- and one table, a_min, of C floats.  A row passes when the bound stays below
// -(kZeroGap + margin).  The exact path would then find logit b the row's maximum and nothing else within kZeroGap of
// it, so onehot[row] = b is what gmm_rowmax_kernel would have written and out = fma(c_x', x, c_m' mu_b) what
// gmm_onehot_kernel would have: the kernel writes both at once, from the registers the row was tested in.  A row tile
// (kCertTile rows) whose rows all passed is certified: it skips the screening pass, both GEMMs and the row maxima.
// In any other tile the normal path runs over all rows and overwrites what the passing rows wrote, with the same bits.
//
// Margin.  A computed logit is fl(c1 acc + fl(-c2 musq[n] + bias[n])), acc the split-operand sum: three of the nine
// products of pieces are dropped (3 * 2^-24 sum |x_k mu_k| at most) and 6 d products are added in fp32 in some order
// (6 d 2^-24 sum |x_k mu_k| at most), so for d <= 2048 |acc - <x, mu_n>| <= 2^-10 |x| |mu_n|.  Two logits are
// compared: c1 2^-9 |x| max |mu| covers the sums.  musq[] is an fp32 sum of squares (within 2^-13 of |mu|^2, which
// the geometry above is about): (c2 + |A/2 - c2|) 2^-12 max |mu|^2.  1e-5 of the terms' magnitudes covers the
// roundings of the affine map and of the bound's own evaluation here (a few 2^-24 each).
// ---------------------------------------------------------------------------
constexpr int kCertTile = CombineOp::kRowmaxTile;   // rows per certified tile = rows per one-hot flag

// a_min[b] = a lower bound of the distance from mu_b to the nearest other mean: one thread per pair (b, n), double
// sums from LDS tiles of 16 + 16 means, then a minimum per b (positive floats order like their bit patterns).
// a_min must hold +inf (0x7f800000) on entry.
__global__ __launch_bounds__(256) void gmm_cert_amin_kernel(int C, int d, const float* __restrict__ means,
                                                            int32_t* __restrict__ a_min) {
  __shared__ float s_b[16][65], s_n[16][65];
  const int tb = threadIdx.x >> 4, tn = threadIdx.x & 15;
  const int b0 = blockIdx.y * 16, n0 = blockIdx.x * 16;
  double dist = 0.0;
  for (int k0 = 0; k0 < d; k0 += 64) {
    for (int i = threadIdx.x; i < 16 * 64; i += 256) {
      const int r = i >> 6, k = i & 63;
      const bool kin = k0 + k < d;
      s_b[r][k] = (kin && b0 + r < C) ? means[(int64_t)(b0 + r) * d + k0 + k] : 0.f;
      s_n[r][k] = (kin && n0 + r < C) ? means[(int64_t)(n0 + r) * d + k0 + k] : 0.f;
    }
    __syncthreads();
    for (int k = 0; k < 64; ++k) {
      const double df = (double)s_n[tn][k] - (double)s_b[tb][k];   // the difference of two floats: exact
      dist = fma(df, df, dist);
    }
    __syncthreads();
  }
  const int b = b0 + tb, n = n0 + tn;
  if (b >= C || n >= C || b == n) return;
  // (the double sum is off by d 2^-53 of itself at most; rounded down, then one part in a million off)
  const float a = __double2float_rd(sqrt(dist)) * (1.f - 1e-6f);
  atomicMin(&a_min[b], __float_as_int(fmaxf(a, 0.f)));
}

// One wavefront per row, four rows per workgroup; V float4 per lane hold the row (d <= 256 V) and as many mu_b.
// chain_comp[chain[row]]: the candidate component of the row (< 0: none).  means: as the second GEMM carries them
// (gmm_means22_kernel; the caller's own where that GEMM takes them whole): what a one-hot row's result is made of.
// glob = (largest |mu_n|, largest and smallest musq, -), globw = (largest log2 w_n, largest |log2 w_n|, -, -).  Rows of a tile count themselves through
// tile_cnt[tile] (finished in the low half, passed in the high half); the workgroup that brings the tile to its
// full count writes cert_tile (always) and onehot_tile = 1 (if certified) and clears the counter for the next call.
// counts (or NULL): [5] += one-hot row tiles, [6] += certified row tiles (verify call only: count_tiles).
template <int V>
__global__ __launch_bounds__(256) void gmm_certify_kernel(const int* __restrict__ n_dev, int n_max, int d, int C,
                                                          const float* __restrict__ in_base,
                                                          const int64_t* __restrict__ in_off,
                                                          float* __restrict__ out_base,
                                                          const int64_t* __restrict__ out_off,
                                                          const int32_t* __restrict__ tau,
                                                          const float4* __restrict__ coef_tau,
                                                          const int32_t* __restrict__ chain,
                                                          const int32_t* __restrict__ chain_comp,
                                                          const float* __restrict__ means,
                                                          const float* __restrict__ musq,
                                                          const float* __restrict__ log_w,
                                                          const float* __restrict__ a_min, float4 glob, float4 globw,
                                                          int32_t* __restrict__ onehot,
                                                          uint8_t* __restrict__ onehot_tile,
                                                          uint8_t* __restrict__ cert_tile,
                                                          int32_t* __restrict__ tile_cnt,
                                                          unsigned long long* __restrict__ counts) {
  static_assert(kCertTile % 4 == 0, "whole workgroups per row tile");
  __shared__ int s_pass[4];
  const int n = min(*n_dev, n_max), m0 = blockIdx.x * 4;
  if (m0 >= n) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = m0 + wave;
  bool pass = false;
  if (m < n) {   // the same for the whole wavefront
    int b = chain_comp[chain[m]];
    if (b >= C) b = -1;
    float4 cf = make_float4(0.f, 0.f, 0.f, 0.f);
    float am = 0.f;
    if (b >= 0) {
      cf = coef_tau[tau[m]];
      am = a_min[b];
      if (!cert_worth_reading(cf, am, d)) b = -1;
    }
    if (b >= 0) {
      const float4* x = reinterpret_cast<const float4*>(in_base + in_off[m]);
      const float4* mu = reinterpret_cast<const float4*>(means + (int64_t)b * d);
      float4 xv[V], mv[V];
      float p = 0.f, xx = 0.f;
#pragma unroll
      for (int i = 0; i < V; ++i) {
        const int j = lane + 64 * i;
        const bool in = j < d / 4;
        xv[i] = in ? x[j] : make_float4(0.f, 0.f, 0.f, 0.f);
        mv[i] = in ? mu[j] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
      const float qb = musq[b], bias_b = LogitOp::kLog2e * log_w[b];
#pragma unroll
      for (int i = 0; i < V; ++i) {
        p += (xv[i].x * mv[i].x + xv[i].y * mv[i].y) + (xv[i].z * mv[i].z + xv[i].w * mv[i].w);
        xx += (xv[i].x * xv[i].x + xv[i].y * xv[i].y) + (xv[i].z * xv[i].z + xv[i].w * xv[i].w);
      }
      p = wave_sum(p);
      xx = wave_sum(xx);
      const float s = p / qb;   // any s is valid: its rounding does not matter
      float r2 = 0.f;
#pragma unroll
      for (int i = 0; i < V; ++i) {
        const float ex = fmaf(-s, mv[i].x, xv[i].x), ey = fmaf(-s, mv[i].y, xv[i].y);
        const float ez = fmaf(-s, mv[i].z, xv[i].z), ew = fmaf(-s, mv[i].w, xv[i].w);
        r2 += (ex * ex + ey * ey) + (ez * ez + ew * ew);
      }
      r2 = wave_sum(r2);
      pass = cert_passes(cf, s, r2, xx, am, qb, bias_b, glob, globw);
      if (pass) {
        float4* o = reinterpret_cast<float4*>(out_base + out_off[m]);
#pragma unroll
        for (int i = 0; i < V; ++i) {
          const int j = lane + 64 * i;
          if (j < d / 4) o[j] = cert_value(cf, xv[i], mv[i]);
        }
        if (lane == 0) onehot[m] = b;
      }
    }
  }
  if (lane == 0) s_pass[wave] = pass ? 1 : 0;
  __syncthreads();   // the rows of all four wavefronts before the workgroup's count
  if (threadIdx.x == 0) {
    const int tile = m0 / kCertTile;
    const int rows = min(4, n - m0), rows_tile = min(kCertTile, n - tile * kCertTile);
    const int add = rows + ((s_pass[0] + s_pass[1] + s_pass[2] + s_pass[3]) << 16);
    // (no fence: within this kernel only the counter passes between workgroups; the flags and the rows are read by
    // later kernels.  A device-wide release per workgroup would write the L2 back sixteen thousand times.)
    const int seen = atomicAdd(&tile_cnt[tile], add) + add;
    if ((seen & 0xffff) == rows_tile) {   // the tile is complete
      const bool all = (seen >> 16) == rows_tile;
      tile_cnt[tile] = 0;
      cert_tile[tile] = all ? 1 : 0;
      if (all) {
        onehot_tile[tile] = 1;
        if (counts) {
          atomicAdd(&counts[5], 1ull);
          atomicAdd(&counts[6], 1ull);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Screening of the verify call's logits.
//
// Once the noise is low a posterior sits on one or two components: every other softmax weight is 0.0f (below
// 2^-kZeroGap of the largest: CombineOp), and the exact logits GEMM spends its time on numbers that only have to be
// "far below the row maximum".  An int8 GEMM (a twelfth of the matrix time, exact int32 sums) says which tiles
// those are, rigorously.  A row x is quantised with its own scale, the means with one scale per group of kGroup
// components:  x ~ sx qx,  mu ~ sg qm  (q = the nearest integer in [-127, 127], s = max |.| / 127), so
//   |sx sg <qx, qm> - <x, mu>|  <=  (sg / 2) |x|_1 + (sx / 2) |mu^|_1,      mu^ = sg qm,
// from  x_k mu_k - x^_k mu^_k = x_k (mu_k - mu^_k) + mu^_k (x_k - x^_k).  The GEMM keeps, for every row and group,
// only the largest integer sum I (gemm_i8_stream.h).  The exact logit of component n is
// kappa' <x, mu_n> - gamma' |mu_n|^2 + log2 w_n  with kappa', gamma' >= 0, so with e = kappa' (the bound above, with
// the group's largest |mu^|_1) + a rounding allowance every logit of the group lies below
//   U = kappa' sx sg I - gamma' min |mu|^2 + max log2 w + e
// and the one at the largest sum lies above
//   L = kappa' sx sg I - gamma' max |mu|^2 + min log2 w - e      (min, max over the group).
// A 128 x 128 tile is dead when, for each of its rows, the U of its groups are all more than kZeroGap below the
// largest L of the row.  Dead tiles are left out by the exact GEMM and, through their -inf partial maxima, by the
// second GEMM; the result is bit-identical to computing everything, because the skipped weights are exact zeros
// there too.  (kScreenFp32 covers what the exact GEMM's own fp32 sums may be off by: below 2^-13 sum |x_k mu_k| <=
// 2^-13 127 sg |x|_1 for d <= 2048, i.e. 3% of the first term.  The spread of |mu|^2 inside a group loosens the
// test by gamma' (max - min), a few percent of the gap between two components' logits at any noise level.)
//
// The pass costs a fraction of the exact GEMM but is pure overhead while the posteriors are broad, so it only
// runs when it is likely to pay: the draft call of the same round (one row per chain, the noisiest row of each
// window) counts the column groups its rows keep alive, and the verify call is screened when that is less than
// a quarter of them.
// ---------------------------------------------------------------------------
typedef PipeCfg16<256, 128, 3, 4, 2> ScreenTile;   // 256 components x 128 rows; a wavefront owns 64 x 64
constexpr int kGroup = ScreenTile::WM;             // components per group = rows of a wavefront's sub-tile
static_assert(GmmTileSplit::BN % kGroup == 0, "whole groups per tile of the exact GEMM");
constexpr float kScreenFp32 = 1.05f;    // see above
constexpr float kScreenRound = 1.001f;  // the quantiser divides in fp32: a value may land 127 * 2^-23 steps off the nearest
constexpr int kScreenWgs = 256;         // resident workgroups of the screening GEMM: one per CU
constexpr int kResidentWgs = 512;       // workgroups of the list form of the exact GEMM: two per CU
// screen when the draft rows keep less than this share of their groups alive (timed at workload 5, where an unscreened
// call runs on the tall tiles: 0.25, 0.4, 0.6, 0.85 give 55.0, 54.4, 54.7, 55.8 ms per sample)
constexpr float kScreenDense = 0.4f;

__device__ __forceinline__ int quant8(float v, float inv_s) { return max(-127, min(127, (int)rintf(v * inv_s))); }

// means -> int8, one workgroup per group of kGroup components: qm [C, d], and per group
//   grp[2 g] = (sg, largest |mu^|_1, min |mu|^2, max |mu|^2),  grp[2 g + 1] = (min log2 w, max log2 w, -, -)
__global__ __launch_bounds__(256) void gmm_screen_quant_means_kernel(int C, int d, const float* __restrict__ means,
                                                                     const float* __restrict__ musq,
                                                                     const float* __restrict__ log_w,
                                                                     int8_t* __restrict__ qm, float4* __restrict__ grp) {
  __shared__ float s_red[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int k0 = blockIdx.x * kGroup, k1 = min(C, k0 + kGroup);
  float mx = 0.f;
  for (int64_t i = (int64_t)k0 * d + threadIdx.x; i < (int64_t)k1 * d; i += 256) mx = fmaxf(mx, fabsf(means[i]));
  mx = wave_max(mx);
  if (lane == 0) s_red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
  __syncthreads();
  const float s = mx > 0.f ? mx / 127.f : 1.f, inv = 1.f / s;
  float l1max = 0.f;   // per wavefront: components wave, wave + 4, ...
  for (int k = k0 + wave; k < k1; k += 4) {
    float a = 0.f;
    for (int j = lane; j < d; j += 64) {
      const int q = quant8(means[(int64_t)k * d + j], inv);
      qm[(int64_t)k * d + j] = (int8_t)q;
      a += fabsf((float)q);
    }
    l1max = fmaxf(l1max, wave_sum(a));   // an integer below 2^24: exact
  }
  if (lane == 0) s_red[wave] = l1max;
  __syncthreads();
  if (threadIdx.x == 0) {
    l1max = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    float qlo = INFINITY, qhi = -INFINITY, blo = INFINITY, bhi = -INFINITY;
    for (int k = k0; k < k1; ++k) {
      qlo = fminf(qlo, musq[k]);
      qhi = fmaxf(qhi, musq[k]);
      const float b = LogitOp::kLog2e * log_w[k];
      blo = fminf(blo, b);
      bhi = fmaxf(bhi, b);
    }
    grp[2 * blockIdx.x] = make_float4(s, s * l1max * (1.f + 1e-6f), qlo, qhi);
    grp[2 * blockIdx.x + 1] = make_float4(blo, bhi, 0.f, 0.f);
  }
}

// rows of the plan -> int8 [n, d]; per row (scale, 1-norm); one wavefront per row (d <= 2048: a row in registers).
// The row's largest magnitude is at hand: a_scale[m] = its fp16 scale for the exact GEMM's split (gmm_row_scale_kernel),
// also when the screening pass is switched off (*on == 0: nothing is packed).
__global__ __launch_bounds__(256) void gmm_screen_pack_kernel(const int* __restrict__ n_dev, int n_max, int d,
                                                              const float* __restrict__ in_base,
                                                              const int64_t* __restrict__ in_off,
                                                              const int32_t* __restrict__ on,
                                                              int8_t* __restrict__ xq, float2* __restrict__ xs,
                                                              float* __restrict__ a_scale,
                                                              int32_t* __restrict__ tile_count,
                                                              const uint8_t* __restrict__ cert_tile,
                                                              int32_t* __restrict__ live_tiles) {
  // cert_tile, live_tiles (or NULL): row tiles of kCertTile rows that need no screening (gmm_certify_kernel) are not
  // packed, and the others are listed for the screening GEMM: live_tiles[0] = how many, then their indices in order
  const int n = min(*n_dev, n_max);
  const int lane = threadIdx.x & 63;
  if (blockIdx.x == 0) {
    // list lengths (the decision kernel appends) and tickets of the exact GEMM
    for (int i = threadIdx.x; i < kTicketInts; i += 256) tile_count[i] = 0;
    if (live_tiles && threadIdx.x < 64) {
      const int nt = (n + kCertTile - 1) / kCertTile;
      int base = 0;
      for (int t0 = 0; t0 < nt; t0 += 64) {
        const int tt = t0 + lane;
        const bool live = tt < nt && !cert_tile[tt];
        const unsigned long long mask = __ballot(live);
        if (live) live_tiles[1 + base + __popcll(mask & ((1ull << lane) - 1ull))] = tt;
        base += __popcll(mask);
      }
      if (lane == 0) live_tiles[0] = base;
    }
  }
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= n) return;
  if (cert_tile && cert_tile[m / kCertTile]) return;
  const bool pack = *on != 0;
  const float4* x = reinterpret_cast<const float4*>(in_base + in_off[m]);
  constexpr int kMaxV = 2048 / 4 / 64;
  float4 v[kMaxV];
  float mx = 0.f, a = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxV; ++i) {
    const int j = lane + 64 * i;
    v[i] = j < d / 4 ? x[j] : make_float4(0.f, 0.f, 0.f, 0.f);
    mx = fmaxf(fmaxf(mx, fmaxf(fabsf(v[i].x), fabsf(v[i].y))), fmaxf(fabsf(v[i].z), fabsf(v[i].w)));
    a += (fabsf(v[i].x) + fabsf(v[i].y)) + (fabsf(v[i].z) + fabsf(v[i].w));
  }
  mx = wave_max(mx);
  if (lane == 0 && a_scale) a_scale[m] = fp16_scale(mx);
  if (!pack) return;
  a = wave_sum(a);
  const float s = mx > 0.f ? mx / 127.f : 1.f, inv = 1.f / s;
  uint32_t* o = reinterpret_cast<uint32_t*>(xq + (int64_t)m * d);
#pragma unroll
  for (int i = 0; i < kMaxV; ++i) {
    const int j = lane + 64 * i;
    if (j < d / 4)
      o[j] = (uint32_t)(quant8(v[i].x, inv) & 0xff) | ((uint32_t)(quant8(v[i].y, inv) & 0xff) << 8) |
             ((uint32_t)(quant8(v[i].z, inv) & 0xff) << 16) | ((uint32_t)(quant8(v[i].w, inv) & 0xff) << 24);
  }
  if (lane == 0) xs[m] = make_float2(s, a * (1.f + 1e-5f));   // (the 1-norm's own fp32 rounding)
}

// One workgroup per row tile of the exact GEMM: the bounds U, L above from the largest integer sums imax[row][group]
// -> the tiles of this row tile that the exact GEMM has to compute, appended to the lists (list t % 8 for column tile
// t), and -inf into the partial maxima of the others (pmax[row][np], gpt of them per column tile).  The two halves of
// the tile's rows are judged separately: a column tile that only one half needs is listed as a half tile (halves != 0;
// see gemm_split3.h) -- with every chain's rows in a block of 64 a half holds one chain -- and the other half's logits
// of that tile are set to -inf here: the second GEMM visits a column group for all rows of its row tile, and those rows'
// weights there must come out as the zeros they are.  Not screened (*on == 0): every tile, whole.  spt: groups per column tile.  counts (or NULL), in half tiles: [0] += to compute, [1] += all, [4] +=
// all of screened launches.
__global__ __launch_bounds__(256) void gmm_screen_decide_kernel(const int* __restrict__ n_dev, int n_max, int nps, int ntn,
                                                                int spt, const int32_t* __restrict__ imax,
                                                                const float2* __restrict__ xs,
                                                                const float4* __restrict__ grp,
                                                                const float4* __restrict__ coef_tau,
                                                                const int32_t* __restrict__ tau,
                                                                const int32_t* __restrict__ on,
                                                                uint32_t* __restrict__ tile_list,
                                                                int32_t* __restrict__ tile_count, int list_cap,
                                                                float* __restrict__ pmax, int np, int gpt, int halves,
                                                                float* __restrict__ logits, int64_t ldl,
                                                                const uint8_t* __restrict__ cert_tile,
                                                                int dense_elsewhere,
                                                                unsigned long long* __restrict__ counts) {
  // dense_elsewhere: a call that is not screened (*on == 0) has its tiles computed by another kernel (the tall-tile
  // form, which runs on the same switch): nothing is listed for it, the tiles are only counted.
  extern __shared__ int s_flag[];   // [2][ntn]: upper, lower half of the rows
  constexpr int BM = GmmTileSplit::BM, RW = 4;   // rows a wavefront works on at a time (their loads overlap)
  const int n = min(*n_dev, n_max);
  const int m0 = blockIdx.x * BM;
  if (m0 >= n) return;
  const bool screened = *on != 0;
  if (cert_tile && cert_tile[blockIdx.x]) {   // certified one-hot (gmm_certify_kernel): no tile of logits is wanted
    if (counts && threadIdx.x == 0) atomicAdd(&counts[1], (unsigned long long)(2 * ntn));   // (not among the screened)
    return;
  }
  const bool lower_exists = m0 + BM / 2 < n;
  for (int t = threadIdx.x; t < 2 * ntn; t += 256) s_flag[t] = screened ? 0 : ((t < ntn || lower_exists) ? 1 : 0);
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (screened) {
    for (int r0 = RW * wave; r0 < BM && m0 + r0 < n; r0 += 4 * RW) {   // (r0 .. r0 + RW - 1 lie in one half)
      int* flag = s_flag + (r0 < BM / 2 ? 0 : ntn);
      float c1s[RW], c2[RW], ea[RW], eb[RW], lo[RW];
      const int32_t* im[RW];
#pragma unroll
      for (int k = 0; k < RW; ++k) {   // rows past the end repeat the last one: the same flags again
        const int m = min(m0 + r0 + k, n - 1);
        im[k] = imax + (int64_t)m * nps;
        const float2 rc = xs[m];
        const float4 cf = coef_tau[tau[m]];
        const float c1 = LogitOp::kLog2e * cf.x;
        c1s[k] = c1 * rc.x;
        c2[k] = LogitOp::kLog2e * cf.y;
        ea[k] = 0.5f * kScreenRound * kScreenFp32 * c1 * rc.y;   // times sg
        eb[k] = 0.5f * kScreenRound * c1 * rc.x;                 // times the group's largest |mu^|_1
        lo[k] = -INFINITY;
      }
      // (base, e): kappa' sx sg I, and how far an exact logit may lie from what the bounds say -- the quantisation and
      // an allowance for the roundings of these few operations and of the exact GEMM's affine map
      auto bounds = [&](int k, int p, float4 g1, float& base, float& e) {
        base = c1s[k] * g1.x * (float)im[k][p];
        e = fmaf(ea[k], g1.x, fmaf(eb[k], g1.y, 0.5f)) + 1e-6f * (fabsf(base) + c2[k] * g1.w);
      };
      for (int p = lane; p < nps; p += 64) {
        const float4 g1 = grp[2 * p], g2 = grp[2 * p + 1];
#pragma unroll
        for (int k = 0; k < RW; ++k) {
          float base, e;
          bounds(k, p, g1, base, e);
          lo[k] = fmaxf(lo[k], base - c2[k] * g1.w + g2.x - e);
        }
      }
#pragma unroll
      for (int k = 0; k < RW; ++k) lo[k] = wave_max(lo[k]) - CombineOp::kZeroGap;
      for (int p = lane; p < nps; p += 64) {
        const float4 g1 = grp[2 * p], g2 = grp[2 * p + 1];
        bool any = false;
#pragma unroll
        for (int k = 0; k < RW; ++k) {
          float base, e;
          bounds(k, p, g1, base, e);
          any = any || (base - c2[k] * g1.z + g2.y + e >= lo[k]);
        }
        if (any) flag[p / spt] = 1;
      }
    }
    __syncthreads();
  }
  int mine = 0;
  for (int t = threadIdx.x; t < ntn; t += 256) {
    const int up = s_flag[t], low = s_flag[ntn + t];
    if (!up && !low) continue;
    mine += up + low;
    if (dense_elsewhere && !screened) continue;
    uint32_t e = (uint32_t)(blockIdx.x * ntn + t);
    if (halves && up != low) e |= kListHalf | (low ? kListLower : 0u);
    const int pos = atomicAdd(&tile_count[t % 8], 1);
    if (pos < list_cap) tile_list[(int64_t)(t % 8) * list_cap + pos] = e;
  }
  if (screened && halves) {   // the half of a half tile that is not computed: logits of -inf (16-byte pieces)
    for (int t = 0; t < ntn; ++t) {
      const int up = s_flag[t], low = s_flag[ntn + t];
      if (up == low) continue;   // the same for the whole workgroup
      const int r_first = up ? BM / 2 : 0, r_end = min(r_first + BM / 2, n - m0);
      constexpr int kPieces = GmmTileSplit::BN / 4;
      for (int i = threadIdx.x; i < (r_end - r_first) * kPieces; i += 256)
        *reinterpret_cast<float4*>(logits + (int64_t)(m0 + r_first + i / kPieces) * ldl + (int64_t)t * GmmTileSplit::BN +
                                   4 * (i % kPieces)) = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    }
  }
  if (screened) {   // what is left out: nothing will write those partial maxima
    const int rows = min(BM, n - m0);
    for (int i = threadIdx.x; i < rows * np; i += 256) {
      const int r = i / np, t = (i % np) / gpt;
      const bool computed = halves ? s_flag[(r < BM / 2 ? 0 : ntn) + t] != 0 : (s_flag[t] | s_flag[ntn + t]) != 0;
      if (!computed) pmax[(int64_t)m0 * np + i] = -INFINITY;
    }
  }
  if (counts) {
    const int total = (int)wave_sum((float)mine);   // this wavefront's share; at most a few thousand: exact in fp32
    if (lane == 0 && total) atomicAdd(&counts[0], (unsigned long long)total);
    if (threadIdx.x == 0) {
      atomicAdd(&counts[1], (unsigned long long)(2 * ntn));
      if (screened) atomicAdd(&counts[4], (unsigned long long)(2 * ntn));
    }
  }
}

// After the draft call's logits: the share of column groups its rows keep alive -> on[0].  One wavefront per row;
// acc[0] collects the count, acc[1] the workgroups that are done: the last one decides and clears both.
constexpr int kRegimeBlocks = 64;
__global__ __launch_bounds__(256) void gmm_regime_kernel(const int* __restrict__ n_dev, int n_max, int np,
                                                         const float* __restrict__ pmax, int32_t* __restrict__ on,
                                                         int32_t* __restrict__ acc,
                                                         const uint8_t* __restrict__ cert_tile) {
  // cert_tile (or NULL): row tiles certified one-hot; their rows have no logits and keep one group alive each
  const int n = min(*n_dev, n_max);
  if (n <= 0) return;   // every workgroup alike: nothing is counted, the verdict stands
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float alive = 0.f;
  for (int m = blockIdx.x * 4 + wave; m < n; m += 4 * gridDim.x) {
    if (cert_tile && cert_tile[m / kCertTile]) {
      alive += 1.f;
      continue;
    }
    const float* p = pmax + (int64_t)m * np;
    float mx = -INFINITY;
    for (int q = lane; q < np; q += 64) mx = fmaxf(mx, p[q]);
    mx = wave_max(mx) - CombineOp::kZeroGap;
    float c = 0.f;
    for (int q = lane; q < np; q += 64) c += p[q] >= mx ? 1.f : 0.f;
    alive += wave_sum(c);
  }
  if (lane == 0 && alive > 0.f) atomicAdd(&acc[0], (int32_t)alive);
  __syncthreads();   // the four additions above come before this workgroup's ticket
  if (threadIdx.x == 0) {
    __threadfence();
    if (atomicAdd(&acc[1], 1) == (int32_t)gridDim.x - 1) {
      __threadfence();
      const int32_t tot = atomicAdd(&acc[0], 0);
      on[0] = (float)tot < kScreenDense * (float)n * (float)np ? 1 : 0;
      acc[0] = 0;
      acc[1] = 0;
    }
  }
}

// Finish of a split-K second GEMM: one workgroup per row adds the partial tiles and row sums in split order and
// applies  out = c_x' x + c_m' acc / sum.
__global__ __launch_bounds__(256) void combine_finish_kernel(const int* __restrict__ M_dev, int M_max, int N, int splits,
                                                             const float* __restrict__ part,
                                                             const float* __restrict__ in_base,
                                                             const int64_t* __restrict__ in_off,
                                                             float* __restrict__ out_base,
                                                             const int64_t* __restrict__ out_off,
                                                             const float4* __restrict__ coef_tau,
                                                             const int32_t* __restrict__ tau,
                                                             const uint8_t* __restrict__ onehot_tile, float acc_scale) {
  // acc_scale: what the partial tiles are scaled by (the operand scales of the fp16-term kernels; 1 otherwise)
  const int M = min(*M_dev, M_max);
  const int m = blockIdx.x;
  if (m >= M) return;
  if (onehot_tile && onehot_tile[m / CombineOp::kRowmaxTile]) return;   // written in closed form; no partials exist
  const float* psum = part + (size_t)splits * M_max * N;
  float sum = 0.f;
  for (int z = 0; z < splits; ++z) sum += psum[(size_t)z * M_max + m];
  const float4 cf = coef_tau[tau[m]];
  const float scale = (cf.w / acc_scale) / sum;
  const float* x = in_base + in_off[m];
  float* o = out_base + out_off[m];
  for (int n = threadIdx.x; n < N; n += 256) {
    float a = 0.f;
    for (int z = 0; z < splits; ++z) a += part[((size_t)z * M_max + m) * N + n];
    o[n] = fmaf(cf.z, x[n], scale * a);
  }
}

// ---------------------------------------------------------------------------
// host
// ---------------------------------------------------------------------------
asd_status gmm_create(asd_ctx* ctx, const asd_denoiser& den) {
  GmmState* g = new (std::nothrow) GmmState();
  if (!g) return ASD_ENOMEM;
  ctx->gmm = g;
  g->C = den.C;
  g->var = den.var;
  g->means = den.means;
  g->log_w = den.log_w;
  const int d = ctx->d, C = den.C;
  ctx->model_macs_per_row = 2.0 * C * d;
  ASD_HIP(hipMalloc(&g->means_t, sizeof(float) * (size_t)d * C));
  ASD_HIP(hipMalloc(&g->musq, sizeof(float) * (size_t)C));
  ASD_HIP(hipMalloc(&g->coef_tau, sizeof(float4) * (size_t)ctx->n_tau));
  // per-time-index coefficients, in double on the host
  float4* h = new (std::nothrow) float4[ctx->n_tau];
  if (!h) return ASD_ENOMEM;
  for (int t = 0; t < ctx->n_tau; ++t) {
    const double s2 = (double)den.var;
    if (den.abar) {
      const double ab = den.abar[t];
      const double V = ab * s2 + 1.0 - ab;
      h[t].x = (float)(sqrt(ab) / V);
      h[t].y = (float)(ab / (2.0 * V));
      h[t].z = (float)(sqrt(ab) * s2 / V);
      h[t].w = (float)(1.0 - ab * s2 / V);
    } else {
      // Stochastic-localization coordinates (Eq. sl-defn): y ~ N(t mu_k, (t^2 s2 + t) I) under component
      // k, E[x* | y, k] = mu_k + s2 (y - t mu_k) / (t s2 + 1).  The |y|^2 term drops out of the softmax.
      const double tt = den.sl_time[t];
      const double W1 = tt * s2 + 1.0;
      h[t].x = (float)(1.0 / W1);
      h[t].y = (float)(tt / (2.0 * W1));
      h[t].z = (float)(s2 / W1);
      h[t].w = (float)(1.0 / W1);
    }
  }
  hipError_t e = hipMemcpy(g->coef_tau, h, sizeof(float4) * (size_t)ctx->n_tau, hipMemcpyHostToDevice);
  delete[] h;
  ASD_HIP(e);
  hipLaunchKernelGGL(gmm_prep_kernel, dim3(C), dim3(256), 0, 0, C, d, g->means, g->means_t, g->musq);
  ASD_HIP(hipGetLastError());
  ASD_HIP(hipDeviceSynchronize());

  g->rowwise_lds = sizeof(float) * 4 * (size_t)(d + C);
  const bool aligned = (d % 4 == 0) && (C % 4 == 0);
  const bool big = (double)ctx->n_rows_max * C * d >= (double)(1 << 26);
  const bool rowwise_ok = g->rowwise_lds <= 64 * 1024;
  g->use_mfma = aligned && (big || !rowwise_ok);
  if (!g->use_mfma && !rowwise_ok) {
    set_error("GMM denoiser: C=%d, d=%d needs d %% 4 == 0 and C %% 4 == 0 at this size", C, d);
    return ASD_EUNSUPPORTED;
  }
  if (!g->use_mfma && d % 4 == 0) {
    const size_t C4 = ((size_t)C + 3) & ~(size_t)3;
    const size_t bytes = sizeof(float) * ((size_t)C * (d + 4) + 2 * C4 + 4 * C4 + 4 * (size_t)d);
    if (bytes <= 150 * 1024) {
      g->lds_rowwise_bytes = bytes;
      ASD_HIP(hipFuncSetAttribute((const void*)gmm_rowwise_lds_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  160 * 1024));
    }
  }
  if (g->use_mfma && d % 16 == 0 && C % 16 == 0) {
    if (d % GmmTile2::BK == 0 && C % GmmTile2::BK == 0) {
      // fp16 terms for both calls: the means times b_scale (a power of two that brings the largest |mu| into fp16's
      // upper range), one image per GEMM for both tilings, and the means as their two fp16 terms carry them
      uint32_t* mx_dev = nullptr;
      uint32_t mx_bits = 0;
      ASD_HIP(hipMalloc(&mx_dev, sizeof(uint32_t)));
      ASD_HIP(hipMemset(mx_dev, 0, sizeof(uint32_t)));
      hipLaunchKernelGGL(gmm_absmax_kernel, dim3(256), dim3(256), 0, 0, g->means, (int64_t)C * d, mx_dev);
      hipError_t e1 = hipGetLastError();
      hipError_t e2 = hipMemcpy(&mx_bits, mx_dev, sizeof(uint32_t), hipMemcpyDeviceToHost);
      (void)hipFree(mx_dev);
      ASD_HIP(e1);
      ASD_HIP(e2);
      g->b_scale = fp16_scale(__builtin_bit_cast(float, mx_bits));
      ASD_HIP(hipMalloc(&g->means_img2, split3_image_bytes<GmmTile2>(C, d)));
      ASD_HIP(hipMalloc(&g->means_t_img2, split3_image_bytes<GmmTile2>(d, C)));
      ASD_HIP(launch_split3_pack_b<GmmTile2>(g->means, d, C, d, g->means_img2, 0, g->b_scale));
      ASD_HIP(launch_split3_pack_b<GmmTile2>(g->means_t, C, d, C, g->means_t_img2, 0, g->b_scale));
      ASD_HIP(hipMalloc(&g->a_scale, sizeof(float) * (size_t)ctx->n_rows_max));
      ASD_HIP(hipMalloc(&g->means22, sizeof(float) * (size_t)C * d));
      hipLaunchKernelGGL(gmm_means22_kernel, dim3((unsigned)ceil_div((int64_t)C * d, 256)), dim3(256), 0, 0, g->means,
                         (int64_t)C * d, g->b_scale, g->means22);
      ASD_HIP(hipGetLastError());
      g->two_ok = g->split_draft_ok = true;
      if (ctx->n_rows_max >= kBigRows) {   // enough rows for 256 x 256 tiles to fill the chip
        ASD_HIP(hipMalloc(&g->means_img_big, split3_image_bytes<Split2BigCfg>(C, d)));
        ASD_HIP(hipMalloc(&g->means_t_img_big, split3_image_bytes<Split2BigCfg>(d, C)));
        ASD_HIP(launch_split3_pack_b<Split2BigCfg>(g->means, d, C, d, g->means_img_big, 0, g->b_scale));
        ASD_HIP(launch_split3_pack_b<Split2BigCfg>(g->means_t, C, d, C, g->means_t_img_big, 0, g->b_scale));
        g->big_ok = true;
      }
    } else {   // the verify call only, on three bf16 terms
      ASD_HIP(hipMalloc(&g->means_img, split3_image_bytes<GmmTileSplit>(C, d)));
      ASD_HIP(hipMalloc(&g->means_t_img, split3_image_bytes<GmmTileSplit>(d, C)));
      ASD_HIP(launch_split3_pack_b<GmmTileSplit>(g->means, d, C, d, g->means_img, 0));
      ASD_HIP(launch_split3_pack_b<GmmTileSplit>(g->means_t, C, d, C, g->means_t_img, 0));
    }
    ASD_HIP(hipDeviceSynchronize());
    g->split_ok = g->use_split = true;
    const int np_v = GmmTileSplit::WGN * (int)ceil_div(C, GmmTileSplit::BN);   // partial maxima per row, verify call
    ASD_HIP(hipMalloc(&g->rmax, sizeof(float) * (size_t)ctx->n_rows_max));
    ASD_HIP(hipMalloc(&g->glive, (size_t)ceil_div(ctx->n_rows_max, CombineOp::kRowmaxTile) * np_v));
    ASD_HIP(hipMalloc(&g->onehot, sizeof(int32_t) * (size_t)ctx->n_rows_max));
    ASD_HIP(hipMalloc(&g->onehot_tile, (size_t)ceil_div(ctx->n_rows_max, CombineOp::kRowmaxTile)));
    ASD_HIP(hipMalloc(&g->work_counts, 8 * sizeof(unsigned long long)));
    ASD_HIP(hipMemset(g->work_counts, 0, 8 * sizeof(unsigned long long)));
    // screening pass of the verify call: full tiles only, and the second GEMM must be able to skip what it leaves out
    if (d % 128 == 0 && C % ScreenTile::BM == 0 && C % GmmTileSplit::BN == 0 && d <= 2048 && g->two_ok &&
        split3_sparse_fits<GmmTile2>(C, np_v, GmmTile2::WN)) {
      g->nps = C / kGroup;
      const int64_t row_tiles = ceil_div(ctx->n_rows_max, GmmTileSplit::BM);
      ASD_HIP(hipMalloc(&g->means_q, (size_t)C * d));
      ASD_HIP(hipMalloc(&g->means_grp, sizeof(float4) * 2 * (size_t)g->nps));
      ASD_HIP(hipMalloc(&g->xq, (size_t)ctx->n_rows_max * d));
      ASD_HIP(hipMalloc(&g->xs, sizeof(float2) * (size_t)ctx->n_rows_max));
      ASD_HIP(hipMalloc(&g->imax, sizeof(int32_t) * (size_t)ctx->n_rows_max * g->nps));
      g->list_cap = (int)(row_tiles * ceil_div(C / GmmTileSplit::BN, 8));
      ASD_HIP(hipMalloc(&g->tile_list, sizeof(uint32_t) * 8 * (size_t)g->list_cap));
      ASD_HIP(hipMalloc(&g->tile_count, kTicketInts * sizeof(int32_t)));
      ASD_HIP(hipMemset(g->tile_count, 0, kTicketInts * sizeof(int32_t)));
      ASD_HIP(hipMalloc(&g->screen_on, 4 * sizeof(int32_t)));
      const int32_t on[4] = {1, 1, 0, 0};   // verdict, the constant 1, the regime kernel's two accumulators
      ASD_HIP(hipMemcpy(g->screen_on, on, sizeof(on), hipMemcpyHostToDevice));
      hipLaunchKernelGGL(gmm_screen_quant_means_kernel, dim3((unsigned)g->nps), dim3(256), 0, 0, C, d, g->means, g->musq,
                         g->log_w, g->means_q, g->means_grp);
      ASD_HIP(hipGetLastError());
      ASD_HIP(hipDeviceSynchronize());
      g->screen_ok = true;
      // one-hot certificate: needs the one-hot closed form (64 groups of 64 columns at most)
      static_assert(ScreenTile::BN == kCertTile && GmmTileSplit::BM == kCertTile, "one row tile for every stage");
      if (np_v <= 64 && GmmTileSplit::WN == 64 && d % 4 == 0) {
        float* h_q = new (std::nothrow) float[2 * (size_t)C];
        if (!h_q) return ASD_ENOMEM;
        hipError_t e1 = hipMemcpy(h_q, g->musq, sizeof(float) * (size_t)C, hipMemcpyDeviceToHost);
        hipError_t e2 = hipMemcpy(h_q + C, g->log_w, sizeof(float) * (size_t)C, hipMemcpyDeviceToHost);
        float qmax = 0.f, qmin = INFINITY, bmax = -INFINITY, babs = 0.f;
        for (int k = 0; k < C; ++k) {
          qmax = fmaxf(qmax, h_q[k]);
          qmin = fminf(qmin, h_q[k]);
          const float bias = LogitOp::kLog2e * h_q[C + k];   // as the kernels form it
          bmax = fmaxf(bmax, bias);
          babs = fmaxf(babs, fabsf(bias));
        }
        delete[] h_q;
        ASD_HIP(e1);
        ASD_HIP(e2);
        // (musq is an fp32 sum of d squares: 1e-3 covers its rounding many times over)
        const float mumax = sqrtf(qmax) * 1.001f;
        g->cert_glob = make_float4(mumax, qmax, qmin, 0.f);
        g->cert_globw = make_float4(bmax, babs, 0.f, 0.f);
        ASD_HIP(hipMalloc(&g->cert_amin, sizeof(float) * (size_t)C));
        ASD_HIP(hipMemset(g->cert_amin, 0, sizeof(float) * (size_t)C));
        {
          int32_t* h_inf = new (std::nothrow) int32_t[C];
          if (!h_inf) return ASD_ENOMEM;
          for (int k = 0; k < C; ++k) h_inf[k] = 0x7f800000;
          hipError_t e3 = hipMemcpy(g->cert_amin, h_inf, sizeof(int32_t) * (size_t)C, hipMemcpyHostToDevice);
          delete[] h_inf;
          ASD_HIP(e3);
        }
        ASD_HIP(hipMalloc(&g->chain_comp, sizeof(int32_t) * (size_t)ctx->B));
        ASD_HIP(hipMemset(g->chain_comp, 0xff, sizeof(int32_t) * (size_t)ctx->B));   // -1: no candidate yet
        ASD_HIP(hipMalloc(&g->cert_tile, (size_t)row_tiles));
        ASD_HIP(hipMemset(g->cert_tile, 0, (size_t)row_tiles));
        ASD_HIP(hipMalloc(&g->cert_cnt, sizeof(int32_t) * (size_t)row_tiles));
        ASD_HIP(hipMemset(g->cert_cnt, 0, sizeof(int32_t) * (size_t)row_tiles));
        ASD_HIP(hipMalloc(&g->live_tiles, sizeof(int32_t) * (1 + (size_t)row_tiles)));
        ASD_HIP(hipMemset(g->live_tiles, 0, sizeof(int32_t) * (1 + (size_t)row_tiles)));
        hipLaunchKernelGGL(gmm_cert_amin_kernel, dim3((unsigned)ceil_div(C, 16), (unsigned)ceil_div(C, 16)), dim3(256), 0,
                           0, C, d, g->means, reinterpret_cast<int32_t*>(g->cert_amin));
        ASD_HIP(hipGetLastError());
        ASD_HIP(hipDeviceSynchronize());
        g->cert_ok = std::isfinite(mumax) && std::isfinite(babs);
      }
    }
  }
  if (g->use_mfma) {
    g->np = 2 * (int)ceil_div(C, GmmTileSkinny::BN);  // room for the finest of the tilings
    // split K for the second GEMM of the draft call (one row per chain): few output tiles, long K
    const int64_t tiles = ceil_div(ctx->B, GmmTileSkinny::BM) * ceil_div(d, GmmTileSkinny::BN);
    if (C % GmmTileSkinny::BK == 0) {
      const int slabs = C / GmmTileSkinny::BK;
      for (int sp = 4; sp >= 2; sp /= 2)   // up to ~4 workgroups per CU, at least 16 slabs each (8 splits measured no better)
        if (tiles * sp <= 1024 && slabs % sp == 0 && slabs / sp >= 16) {
          g->draft_splits = sp;
          break;
        }
    }
    if (g->draft_splits > 1)
      ASD_HIP(hipMalloc(&g->part, sizeof(float) * gemm_f32_splitk_floats(g->draft_splits, ctx->B, d)));
    ASD_HIP(hipMalloc(&g->logits, sizeof(float) * (size_t)ctx->n_rows_max * C));
    ASD_HIP(hipMalloc(&g->pmax, sizeof(float) * (size_t)ctx->n_rows_max * g->np));
  }
  return ASD_OK;
}

// The screened verify call works on 128 x 128 tiles of (rows, components) and can leave out a tile only if all its
// rows agree that its components are irrelevant.  Rows of one chain do (its window sits on one component once the
// posterior has collapsed); with each chain's rows starting at a multiple of 64 a tile holds two chains, not three.
// Only when the filling cannot overflow the plan: windows of at most L - 1 rows (+ 1 with reuse) fit L = 64 m.
bool gmm_onehot_cert(const asd_ctx* ctx, OneHotCert* out) {
  const GmmState* g = ctx->gmm;
  // the conditions under which the verify call certifies rows itself (gmm_eval) and carries the means as two fp16
  // terms: only then is a certified row's value what that call would have stored
  if (!g || !g->use_mfma || !g->use_split || !g->two_ok || !g->screen_ok || g->screen_mode == 0 || !g->sparse_combine ||
      !g->cert_ok || !g->cert_on || !g->means22 || !g->chain_comp || !g->cert_amin)
    return false;
  out->chain_comp = g->chain_comp;
  out->means = g->means22;
  out->musq = g->musq;
  out->log_w = g->log_w;
  out->a_min = g->cert_amin;
  out->coef_tau = g->coef_tau;
  out->glob = g->cert_glob;
  out->globw = g->cert_globw;
  out->C = g->C;
  return true;
}

int gmm_row_block(const asd_ctx* ctx) {
  const GmmState* g = ctx->gmm;
  const bool screening = g && g->use_split && g->screen_ok && g->screen_mode != 0 && g->sparse_combine;
  return (screening && ctx->L % 64 == 0) ? 64 : 0;
}

void gmm_destroy(asd_ctx* ctx) {
  GmmState* g = ctx->gmm;
  if (!g) return;
  (void)hipFree(g->means_t);
  (void)hipFree(g->means_img);
  (void)hipFree(g->means_t_img);
  (void)hipFree(g->means_img_s);
  (void)hipFree(g->means_t_img_s);
  (void)hipFree(g->means_img2);
  (void)hipFree(g->means_t_img2);
  (void)hipFree(g->means_img_big);
  (void)hipFree(g->means_t_img_big);
  (void)hipFree(g->means22);
  (void)hipFree(g->a_scale);
  (void)hipFree(g->musq);
  (void)hipFree(g->coef_tau);
  (void)hipFree(g->part);
  (void)hipFree(g->logits);
  (void)hipFree(g->pmax);
  (void)hipFree(g->means_q);
  (void)hipFree(g->means_grp);
  (void)hipFree(g->xq);
  (void)hipFree(g->xs);
  (void)hipFree(g->imax);
  (void)hipFree(g->tile_list);
  (void)hipFree(g->tile_count);
  (void)hipFree(g->screen_on);
  (void)hipFree(g->work_counts);
  (void)hipFree(g->rmax);
  (void)hipFree(g->glive);
  (void)hipFree(g->onehot);
  (void)hipFree(g->onehot_tile);
  (void)hipFree(g->cert_amin);
  (void)hipFree(g->chain_comp);
  (void)hipFree(g->cert_tile);
  (void)hipFree(g->cert_cnt);
  (void)hipFree(g->live_tiles);
  delete g;
  ctx->gmm = nullptr;
}

asd_status gmm_eval(asd_ctx* ctx, const RowPlan& rows, hipStream_t st) {
  GmmState* g = ctx->gmm;
  const int d = ctx->d, C = g->C, n = rows.n;
  if (!g->use_mfma && g->lds_rowwise_bytes) {
    ProfScope ps(ctx, ASD_PROF_GMM_ROWWISE, rows.call, st);
    // one row per wavefront while that still gives fewer workgroups than CUs, else four
    const int rpw = n > 4 * 256 ? 4 : 1;
    hipLaunchKernelGGL(gmm_rowwise_lds_kernel, dim3((unsigned)ceil_div(n, 4 * rpw)), dim3(256),
                       g->lds_rowwise_bytes, st, rows.n_dev, n, d, C, rpw, rows.in_base, rows.in_off, rows.out_base,
                       rows.out_off, rows.tau, g->coef_tau, g->means, g->musq, g->log_w);
    ASD_HIP(hipGetLastError());
    return ASD_OK;
  }
  if (!g->use_mfma) {
    ProfScope ps(ctx, ASD_PROF_GMM_ROWWISE, rows.call, st);
    const int blocks = (int)std::min<int64_t>(ceil_div(n, 4), 4096);
    hipLaunchKernelGGL(gmm_rowwise_kernel, dim3(blocks), dim3(256), g->rowwise_lds, st, rows.n_dev, n, d, C, rows.in_base,
                       rows.in_off, rows.out_base, rows.out_off, rows.tau, g->coef_tau, g->means, g->musq,
                       g->log_w);
    ASD_HIP(hipGetLastError());
    return ASD_OK;
  }
  // partial row maxima per row: one per wavefront column of the tiling in use
  const bool split = g->use_split && (rows.call == 1 || g->split_draft_ok);
  static_assert(GmmTileSplit::BN == GmmTileSplitSkinny::BN && GmmTileSplit::WGN == GmmTileSplitSkinny::WGN,
                "the two split tilings lay the row maxima out alike");
  const int np = split ? GmmTileSplit::WGN * (int)ceil_div(C, GmmTileSplit::BN)
                       : 2 * (int)ceil_div(C, rows.call ? GmmTile::BN : GmmTileSkinny::BN);
  // K split of the draft call's second GEMM (few output tiles, long K); both of its tilings use slabs of 32
  static_assert(GmmTileSplitSkinny::BK == GmmTileSkinny::BK, "one split plan for both");
  const int splits = (!rows.call && g->draft_splits > 1 && n <= ctx->B) ? g->draft_splits : 1;
  RowSrc X{rows.in_base, rows.in_off, 0};
  LogitOp op1{g->logits, C, g->pmax, np, g->coef_tau, rows.tau, g->musq, g->log_w};
  // the verify call of the split path may be screened; only when the second GEMM skips what the first leaves out
  const bool screen = split && rows.call == 1 && g->screen_ok && g->screen_mode != 0 && g->sparse_combine;
  // ... and rows may be certified one-hot before anything else (the plan says which chain a row belongs to): in the
  // verify call, and in the draft call of a context whose verify calls are
  // (not in a verify call behind the early accept kernel: a chain is in that call because one of its rows failed this
  // very test, so no row tile of it -- two chains' blocks -- can pass whole)
  const bool cert = split && g->screen_ok && g->screen_mode != 0 && g->sparse_combine && g->cert_ok && g->cert_on &&
                    rows.chain != nullptr && (rows.call == 1 || g->split_draft_ok) && !(rows.call == 1 && ctx->early_now);
  const uint8_t* cert_tile = cert ? g->cert_tile : nullptr;
  // the screening pass's switch in device memory: this round's verdict of the draft call, or the constant 1
  const int32_t* on = screen ? g->screen_on + (g->screen_mode == 2 ? 1 : 0) : nullptr;
  // launches in which every tile is wanted -- a verify call of many rows that is not screened, by this round's verdict
  // or at all -- take the 256 x 256 tiles; both forms of a GEMM are queued then and the switch picks one
  const bool big = split && g->two_ok && g->big_ok && g->big_on && rows.call == 1 && n >= kBigRows;
  if (cert) {
    ProfScope ps(ctx, ASD_PROF_GMM_CERT, rows.call, st);
    auto kern = d <= 1024 ? gmm_certify_kernel<4> : gmm_certify_kernel<8>;
    hipLaunchKernelGGL(kern, dim3((unsigned)ceil_div(n, 4)), dim3(256), 0, st, rows.n_dev, n, d, C, rows.in_base,
                       rows.in_off, rows.out_base, rows.out_off, rows.tau, g->coef_tau, rows.chain, g->chain_comp,
                       g->means22, g->musq, g->log_w, g->cert_amin, g->cert_glob, g->cert_globw, g->onehot, g->onehot_tile,
                       g->cert_tile, g->cert_cnt, (prof_counting(ctx) && rows.call == 1) ? g->work_counts : nullptr);
    ASD_HIP(hipGetLastError());
    op1.skip_tile = cert_tile;
  }
  if (screen) {
    ProfScope ps(ctx, ASD_PROF_GMM_SCREEN, rows.call, st);
    const int ntn = C / GmmTileSplit::BN;
    hipLaunchKernelGGL(gmm_screen_pack_kernel, dim3((unsigned)ceil_div(n, 4)), dim3(256), 0, st, rows.n_dev, n, d,
                       rows.in_base, rows.in_off, on, g->xq, g->xs, g->a_scale, g->tile_count, cert_tile,
                       cert ? g->live_tiles : (int32_t*)nullptr);
    ASD_HIP(hipGetLastError());
    // int8 operands, handed over as 16-bit units (two k each): the means as the kernel's rows, the call's rows as its columns
    ASD_HIP(launch_gemm_i8_colmax_stream<ScreenTile>(C, rows.n_dev, n, d / 2, reinterpret_cast<const uint16_t*>(g->means_q),
                                                     d / 2, reinterpret_cast<const uint16_t*>(g->xq), d / 2, on,
                                                     cert ? g->live_tiles : (const int32_t*)nullptr, g->imax, g->nps,
                                                     kScreenWgs, st));
    hipLaunchKernelGGL(gmm_screen_decide_kernel, dim3((unsigned)ceil_div(n, GmmTileSplit::BM)), dim3(256),
                       sizeof(int) * 2 * ntn, st, rows.n_dev, n, g->nps, ntn, GmmTileSplit::BN / kGroup, g->imax,
                       g->xs, g->means_grp, g->coef_tau, rows.tau, on, g->tile_list, g->tile_count, g->list_cap,
                       g->pmax, np, GmmTileSplit::WGN, g->split_draft_ok ? 1 : 0, g->logits, (int64_t)C, cert_tile,
                       big ? 1 : 0, prof_counting(ctx) ? g->work_counts : nullptr);
    ASD_HIP(hipGetLastError());
    op1.tile_list = g->tile_list;
    op1.tile_count = g->tile_count;
    op1.list_cap = g->list_cap;
  }
  const bool two = split && g->two_ok;   // fp16 terms (both calls), else three bf16 terms (verify call only)
  {
    ProfScope ps(ctx, ASD_PROF_GMM_LOGITS, rows.call, st);
    if (two) {   // every row has its scale first: from the screening pass's quantiser, else from a kernel of its own
      if (!screen) {
        hipLaunchKernelGGL(gmm_row_scale_kernel, dim3((unsigned)ceil_div(n, 4)), dim3(256), 0, st, rows.n_dev, n, d,
                           rows.in_base, rows.in_off, g->a_scale, cert_tile);
        ASD_HIP(hipGetLastError());
      }
      op1.a_scale = g->a_scale;
      op1.b_scale = g->b_scale;
    }
    if (screen) {
      // resident workgroups draw the tiles (and half tiles, on the draft call's tiling) the screening pass listed;
      // a call it was switched off for lists nothing when the tall tiles take it
      ASD_HIP(launch_gemm_split3_nt_list<GmmTile2, GmmTile2Skinny, 1>(rows.n_dev, n, C, d, X, g->means_img2, g->means_img2,
                                                                       op1, kResidentWgs, st));
      if (big) ASD_HIP(launch_gemm_split2_big<false>(rows.n_dev, n, C, d, X, g->means_img_big, op1, st, false, on, 0));
    } else if (big) {
      ASD_HIP(launch_gemm_split2_big<false>(rows.n_dev, n, C, d, X, g->means_img_big, op1, st, false, nullptr, 0));
    } else if (two) {
      ASD_HIP(rows.call ? launch_gemm_split3_nt<GmmTile2, 1, false>(rows.n_dev, n, C, d, X, g->means_img2, op1, st)
                        : launch_gemm_split3_nt<GmmTile2Skinny, 0, false>(rows.n_dev, n, C, d, X, g->means_img2, op1, st));
    } else if (split) {
      ASD_HIP(launch_gemm_split3_nt<GmmTileSplit, 1, false>(rows.n_dev, n, C, d, X, g->means_img, op1, st));
    } else {
      ASD_HIP(rows.call ? launch_gemm_f32_nt<GmmTile, 1>(rows.n_dev, n, C, d, X, g->means, d, op1, st)
                        : launch_gemm_f32_nt<GmmTileSkinny, 0>(rows.n_dev, n, C, d, X, g->means, d, op1, st));
    }
  }
  if (rows.call == 0 && g->screen_ok && g->screen_mode == 1) {   // this round's verify call: screen or not
    hipLaunchKernelGGL(gmm_regime_kernel, dim3(kRegimeBlocks), dim3(256), 0, st, rows.n_dev, n, np, g->pmax,
                       g->screen_on, g->screen_on + 2, cert_tile);
    ASD_HIP(hipGetLastError());
  }
  RowSrc P{g->logits, nullptr, C};
  // columns behind one partial row maximum: the first GEMM's wavefront sub-tile width (the last group may be short)
  const int gcols = split ? GmmTileSplit::WN : (rows.call ? GmmTile::WN : GmmTileSkinny::WN);
  CombineOp op2{g->pmax, np, gcols, nullptr, nullptr, nullptr, rows.in_base, rows.in_off, rows.out_base, rows.out_off, g->coef_tau,
                rows.tau, (prof_counting(ctx) && rows.call == 1 && split) ? g->work_counts + 2 : nullptr, {}, {}};
  // between the GEMMs: row maxima and live groups once per row tile; one-hot rows (the draft call's rows -- one per
  // chain -- are one-hot too once the posteriors have collapsed)
  if (split) {
    ProfScope ps(ctx, ASD_PROF_GMM_SOFTMAX, rows.call, st);
    // one-hot rows in closed form: with the sparse second GEMM only (the same switch), whole float4 rows
    const bool onehot = g->sparse_combine && d % 4 == 0 && np <= 64 && gcols == 64;
    if (rows.call == 1) {
      hipLaunchKernelGGL(gmm_rowmax_kernel, dim3((unsigned)ceil_div(n, CombineOp::kRowmaxTile)), dim3(256),
                         sizeof(int) * (np + 1), st, rows.n_dev, n, np, g->pmax, g->rmax, g->glive, g->logits, (int64_t)C,
                         gcols, onehot ? g->onehot : (int32_t*)nullptr, onehot ? g->onehot_tile : (uint8_t*)nullptr,
                         cert_tile, prof_counting(ctx) ? g->work_counts : nullptr);
    } else {
      hipLaunchKernelGGL(gmm_rowmax_rows_kernel, dim3((unsigned)ceil_div(n, 4)), dim3(256), 0, st, rows.n_dev, n, np,
                         g->pmax, g->rmax, g->logits, (int64_t)C, onehot ? g->onehot : (int32_t*)nullptr, rows.chain,
                         (onehot && g->cert_ok) ? g->chain_comp : (int32_t*)nullptr, cert_tile);
      if (onehot)
        hipLaunchKernelGGL(gmm_onehot_tiles_kernel, dim3((unsigned)ceil_div(n, CombineOp::kRowmaxTile)),
                           dim3(CombineOp::kRowmaxTile), 0, st, rows.n_dev, n, g->onehot, g->onehot_tile);
    }
    ASD_HIP(hipGetLastError());
    if (onehot) {
      hipLaunchKernelGGL(gmm_onehot_kernel, dim3((unsigned)ceil_div(n, kOnehotRows)), dim3(256), 0, st, rows.n_dev, n, d, g->onehot,
                         g->onehot_tile, two ? g->means22 : g->means, rows.in_base, rows.in_off, rows.out_base,
                         rows.out_off, g->coef_tau, rows.tau, cert_tile);
      ASD_HIP(hipGetLastError());
      op2.onehot_tile = g->onehot_tile;
    }
    op2.rmax_pre = g->rmax;
    if (rows.call == 1) op2.live_pre = g->glive;
  }
  {
    ProfScope ps(ctx, ASD_PROF_GMM_COMBINE, rows.call, st);
    if (two) {
      op2.a_scale = 32768.f;   // the weights are at most 1: 2^15 is the largest power of two fp16 can take them at
      op2.b_scale = g->b_scale;
      if (rows.call == 0) {
        ASD_HIP(launch_gemm_split3_nt<GmmTile2Skinny, 0, false>(rows.n_dev, n, d, C, P, g->means_t_img2, op2, st, splits,
                                                                 g->part));
      } else {
        // (with the tall tiles queued as well: the small ones when this call was screened, the tall ones when not)
        if (!big || screen)
          ASD_HIP(launch_gemm_split3_nt<GmmTile2, 1, true>(rows.n_dev, n, d, C, P, g->means_t_img2, op2, st, 1, nullptr,
                                                           g->sparse_combine, big ? on : nullptr, 1));
        if (big)
          ASD_HIP(launch_gemm_split2_big<true>(rows.n_dev, n, d, C, P, g->means_t_img_big, op2, st, g->sparse_combine,
                                               screen ? on : nullptr, 0));
      }
    } else if (split)
      ASD_HIP(launch_gemm_split3_nt<GmmTileSplit, 1, true>(rows.n_dev, n, d, C, P, g->means_t_img, op2, st, 1, nullptr,
                                                           g->sparse_combine));
    else
      ASD_HIP(rows.call ? launch_gemm_f32_nt<GmmTile, 1>(rows.n_dev, n, d, C, P, g->means_t, C, op2, st)
                        : launch_gemm_f32_nt<GmmTileSkinny, 0>(rows.n_dev, n, d, C, P, g->means_t, C, op2, st, splits,
                                                                g->part));
    if (splits > 1) {
      hipLaunchKernelGGL(combine_finish_kernel, dim3((unsigned)n), dim3(256), 0, st, rows.n_dev, ctx->B, d, splits,
                         g->part, rows.in_base, rows.in_off, rows.out_base, rows.out_off, g->coef_tau, rows.tau,
                         op2.onehot_tile, op2.a_scale * op2.b_scale);
      ASD_HIP(hipGetLastError());
    }
  }
  return ASD_OK;
}

}  // namespace asd
