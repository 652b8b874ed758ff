// bf16 x bf16 -> fp32 "NT" GEMM on the gfx950 matrix cores:
//   acc[m][n] = sum_k A[m][k] * W[n][k],  A [M, K] and W [N, K] row-major bf16,
// handed to an epilogue functor (bias / SiLU / residual / scatter fused there).
//
// Same structure as the fp32 kernel: 128 x 128 workgroup tile, 4 wavefronts of
// 64 x 64 (2 x 2 blocks of v_mfma_f32_32x32x16_bf16), K slabs of 32 staged
// through double-buffered LDS with register prefetch.  Each lane feeds 8
// consecutive k of its row per MFMA (one 128-bit LDS read); half-wave h takes
// k = 16*group + 8*h .. +7 for both operands, so the pairing of A and W
// elements is exact whatever order the unit sums them in.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace asd {

typedef float v16f_b __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

namespace gemm16 {
constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDSS = BK + 8;  // row stride in bf16 elements (80 B)
constexpr int THREADS = 256;
}  // namespace gemm16

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Requirements (checked by the host): K % 8 == 0, rows 16 B aligned.
// CALL only gives the draft-call and verify-call launches distinct symbols in profiles.
template <class Epi, int CALL>
__global__ __launch_bounds__(gemm16::THREADS, 2) void gemm_bf16_nt_kernel(const int* __restrict__ M_dev, int M_max,
                                                                          int N, int K,
                                                                          const uint16_t* __restrict__ A,
                                                                          int64_t lda,
                                                                          const uint16_t* __restrict__ W,
                                                                          int64_t ldw, Epi epi) {
  using namespace gemm16;
  __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * LDSS];
  __shared__ __attribute__((aligned(16))) uint16_t Ws[2][BN * LDSS];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, half = lane >> 5;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  // the row count lives on the device (compacted row plan); the grid covers M_max
  const int M = M_dev ? min(*M_dev, M_max) : M_max;
  if (m0 >= M) return;

  const int lrow = tid >> 2, lkq = tid & 3;
  const uint16_t* ap[2];
  const uint16_t* wp[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int ra = min(m0 + lrow + 64 * i, M - 1);
    const int rw = min(n0 + lrow + 64 * i, N - 1);
    ap[i] = A + (int64_t)ra * lda + lkq * 8;
    wp[i] = W + (int64_t)rw * ldw + lkq * 8;
  }
  const int nk = (K + BK - 1) / BK;

  uint4 ra[2], rw[2];
  auto gload = [&](int kt) {
    const bool ok = kt * BK + lkq * 8 < K;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      ra[i] = ok ? *reinterpret_cast<const uint4*>(ap[i] + kt * BK) : make_uint4(0u, 0u, 0u, 0u);
      rw[i] = ok ? *reinterpret_cast<const uint4*>(wp[i] + kt * BK) : make_uint4(0u, 0u, 0u, 0u);
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      *reinterpret_cast<uint4*>(&As[buf][(lrow + 64 * i) * LDSS + lkq * 8]) = ra[i];
      *reinterpret_cast<uint4*>(&Ws[buf][(lrow + 64 * i) * LDSS + lkq * 8]) = rw[i];
    }
  };

  v16f_b acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  gload(0);
  sstore(0);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) gload(kt + 1);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      v8bf af[2], wf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = *reinterpret_cast<const v8bf*>(&As[cur][(wm * 64 + i * 32 + l32) * LDSS + ks * 16 + half * 8]);
        wf[i] = *reinterpret_cast<const v8bf*>(&Ws[cur][(wn * 64 + i * 32 + l32) * LDSS + ks * 16 + half * 8]);
      }
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[0], wf[0], acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[0], wf[1], acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[1], wf[0], acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[1], wf[1], acc[1][1], 0, 0, 0);
    }
    if (kt + 1 < nk) sstore(cur ^ 1);
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
      if (m < M) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int n = n0 + wn * 64 + j * 32 + l32;
          if (n < N) epi(m, n, acc[i][j][r]);
        }
      }
    }
  }
}

template <int CALL, class Epi>
inline hipError_t launch_gemm_bf16_nt(const int* M_dev, int M, int N, int K, const uint16_t* A, int64_t lda, const uint16_t* W,
                                      int64_t ldw, Epi epi, hipStream_t st) {
  using namespace gemm16;
  dim3 grid((unsigned)((N + BN - 1) / BN), (unsigned)((M + BM - 1) / BM));
  hipLaunchKernelGGL((gemm_bf16_nt_kernel<Epi, CALL>), grid, dim3(THREADS), 0, st, M_dev, M, N, K, A, lda,
                     W, ldw, epi);
  return hipGetLastError();
}

}  // namespace asd
