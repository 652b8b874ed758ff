// bf16 x bf16 -> fp32 "NT" GEMM on the gfx950 matrix cores:
//   acc[m][n] = sum_k A[m][k] * W[n][k],  A [M, K] and W [N, K] row-major bf16,
// handed to an epilogue functor (bias / SiLU / residual / scatter fused there).
//
// Tiling (Cfg16): a workgroup of 4 wavefronts (2 x 2) owns a BM x BN tile, each
// wavefront a (BM/2) x (BN/2) quadrant as MI x NJ blocks of
// v_mfma_f32_32x32x16_bf16.  K slabs of BK are staged through double-buffered
// LDS with register prefetch of the next slab; inside a slab the fragments of
// the next 16 k are fetched while the MFMAs of the current 16 issue.  Each lane
// feeds 8 consecutive k of its row per MFMA (one 128-bit LDS read); half-wave
// h takes k = 16*group + 8*h .. +7 for both operands, so the pairing of A and
// W elements is exact whatever order the unit sums them in.
// LDS rows are BK + 8 elements (BK*2 + 16 bytes) apart: 16 B aligned, and eight
// consecutive rows start in eight different groups of four banks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace asd {

typedef float v16f_b __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

template <int BM_, int BN_, int BK_>
struct GemmCfg16 {
  static constexpr int BM = BM_, BN = BN_, BK = BK_;
  static constexpr int THREADS = 256;
  static constexpr int LDSS = BK + 8;          // LDS row stride in bf16 elements
  static constexpr int KQ = BK / 8;            // loader threads per row (one 16-byte load each)
  static constexpr int RPP = THREADS / KQ;
  static constexpr int RA = BM / RPP, RB = BN / RPP;
  static constexpr int MI = BM / 64, NJ = BN / 64;
  static constexpr int KS = BK / 16;
  static constexpr size_t LDS_BYTES = sizeof(uint16_t) * 2 * (BM + BN) * LDSS;
  static_assert(BM % 64 == 0 && BN % 64 == 0 && BK % 16 == 0 && BM % RPP == 0 && BN % RPP == 0, "tile shape");
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Epilogue functor: `prev = epi.load(m, n)` then `epi.store(m, n, acc, prev)` for every in-range
// element.  The loads of a whole 32-row block are issued before its first store, so a functor that
// reads and rewrites the same array (the residual stream) costs one memory round trip per block,
// not one per element.
template <int MI, int NJ, int BM, int BN, class Epi>
__device__ __forceinline__ void bf16_epilogue(const v16f_b (&acc)[MI][NJ], int m0, int n0, int wm, int wn, int l32,
                                              int half, int M, int N, const Epi& epi) {
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    float prev[16][NJ];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int n = n0 + wn * (BN / 2) + j * 32 + l32;
        prev[r][j] = (Epi::kLoads && m < M && n < N) ? epi.load(m, n) : 0.f;
      }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
      if (m < M) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int n = n0 + wn * (BN / 2) + j * 32 + l32;
          if (n < N) epi.store(m, n, acc[i][j][r], prev[r][j]);
        }
      }
    }
  }
}

// Requirements (checked by the host): K % 8 == 0, rows 16 B aligned.
// KTAIL: K is not a multiple of BK.  CALL: distinct symbols for the two model calls.
template <class Cfg, class Epi, bool KTAIL, int CALL>
__global__ __launch_bounds__(256) void gemm_bf16_nt_kernel(const int* __restrict__ M_dev, int M_max, int N, int K,
                                                           const uint16_t* __restrict__ A, int64_t lda,
                                                           const uint16_t* __restrict__ W, int64_t ldw, Epi epi) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, LDSS = Cfg::LDSS;
  constexpr int KQ = Cfg::KQ, RPP = Cfg::RPP, RA = Cfg::RA, RB = Cfg::RB, MI = Cfg::MI, NJ = Cfg::NJ, KS = Cfg::KS;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds16[];
  uint16_t* As = lds16;                    // [2][BM * LDSS]
  uint16_t* Ws = lds16 + 2 * BM * LDSS;    // [2][BN * LDSS]

  // the row count lives on the device (compacted row plan); the grid covers M_max
  const int M = M_dev ? min(*M_dev, M_max) : M_max;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  if (m0 >= M) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, half = lane >> 5;

  const int lrow = tid / KQ, lkq = tid % KQ;
  const uint16_t* ap[RA];
  const uint16_t* wp[RB];
#pragma unroll
  for (int p = 0; p < RA; ++p) ap[p] = A + (int64_t)min(m0 + lrow + RPP * p, M - 1) * lda + lkq * 8;
#pragma unroll
  for (int p = 0; p < RB; ++p) wp[p] = W + (int64_t)min(n0 + lrow + RPP * p, N - 1) * ldw + lkq * 8;
  const int nk = (K + BK - 1) / BK;

  uint4 ra[RA], rw[RB];
  auto gload = [&](int kt) {
    const bool ok = !KTAIL || (kt * BK + lkq * 8 < K);
#pragma unroll
    for (int p = 0; p < RA; ++p)
      ra[p] = ok ? *reinterpret_cast<const uint4*>(ap[p] + kt * BK) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int p = 0; p < RB; ++p)
      rw[p] = ok ? *reinterpret_cast<const uint4*>(wp[p] + kt * BK) : make_uint4(0u, 0u, 0u, 0u);
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int p = 0; p < RA; ++p)
      *reinterpret_cast<uint4*>(&As[buf * BM * LDSS + (lrow + RPP * p) * LDSS + lkq * 8]) = ra[p];
#pragma unroll
    for (int p = 0; p < RB; ++p)
      *reinterpret_cast<uint4*>(&Ws[buf * BN * LDSS + (lrow + RPP * p) * LDSS + lkq * 8]) = rw[p];
  };

  v16f_b acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  gload(0);
  sstore(0);
  __syncthreads();

  const int a_lane = (wm * (BM / 2) + l32) * LDSS + half * 8;
  const int w_lane = (wn * (BN / 2) + l32) * LDSS + half * 8;

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) gload(kt + 1);
    const uint16_t* Ac = As + cur * BM * LDSS + a_lane;
    const uint16_t* Wc = Ws + cur * BN * LDSS + w_lane;
    v8bf af[2][MI], wf[2][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i) af[0][i] = *reinterpret_cast<const v8bf*>(Ac + i * 32 * LDSS);
#pragma unroll
    for (int j = 0; j < NJ; ++j) wf[0][j] = *reinterpret_cast<const v8bf*>(Wc + j * 32 * LDSS);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = ks & 1;
      if (ks + 1 < KS) {
#pragma unroll
        for (int i = 0; i < MI; ++i) af[c ^ 1][i] = *reinterpret_cast<const v8bf*>(Ac + i * 32 * LDSS + (ks + 1) * 16);
#pragma unroll
        for (int j = 0; j < NJ; ++j) wf[c ^ 1][j] = *reinterpret_cast<const v8bf*>(Wc + j * 32 * LDSS + (ks + 1) * 16);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[c][i], wf[c][j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) sstore(cur ^ 1);
    __syncthreads();
  }

  // register r of block (i, j) is C[row][col] with
  //   row = m0 + wm*BM/2 + i*32 + 8*(r/4) + 4*half + r%4,  col = n0 + wn*BN/2 + j*32 + l32
  bf16_epilogue<MI, NJ, BM, BN>(acc, m0, n0, wm, wn, l32, half, M, N, epi);
}

template <class Cfg, int CALL, class Epi>
inline hipError_t launch_gemm_bf16_nt(const int* M_dev, int M, int N, int K, const uint16_t* A, int64_t lda,
                                      const uint16_t* W, int64_t ldw, Epi epi, hipStream_t st) {
  dim3 grid((unsigned)((N + Cfg::BN - 1) / Cfg::BN), (unsigned)((M + Cfg::BM - 1) / Cfg::BM));
  if (K % Cfg::BK == 0) {
    auto kern = gemm_bf16_nt_kernel<Cfg, Epi, false, CALL>;
    static bool attr_set = false;  // dynamic LDS above the default limit needs the attribute once per kernel
    if (!attr_set && Cfg::LDS_BYTES > 48 * 1024) {
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)Cfg::LDS_BYTES);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(Cfg::THREADS), Cfg::LDS_BYTES, st, M_dev, M, N, K, A, lda, W, ldw, epi);
  } else {
    auto kern = gemm_bf16_nt_kernel<Cfg, Epi, true, CALL>;
    static bool attr_set = false;
    if (!attr_set && Cfg::LDS_BYTES > 48 * 1024) {
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)Cfg::LDS_BYTES);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(Cfg::THREADS), Cfg::LDS_BYTES, st, M_dev, M, N, K, A, lda, W, ldw, epi);
  }
  return hipGetLastError();
}

}  // namespace asd
