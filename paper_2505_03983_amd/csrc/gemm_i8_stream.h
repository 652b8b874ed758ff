// int8 x int8 -> int32 "NT" product  acc[m][n] = sum_k A[m][k] * W[n][k]  whose only output is, for every column n
// and every block of WM rows, the largest entry:  out[n][block] = max over the block's rows m of acc[m][n].
// For short K: a stream of tiles through one resident pipeline.
//
// (What it is for: A = a fixed matrix of quantised keys, W = quantised queries, a runtime number of them; the
// caller wants to know which blocks of keys can matter to which query, not the products themselves.)
//
// With K = 1024 a 256 x 128 tile is 8 slabs of 128 k -- about 4 us of matrix work.  One tile per workgroup, a
// pipeline fills (a memory latency), runs those 8 slabs and drains into its epilogue, with one workgroup per CU
// and nothing to cover either end.  Here a workgroup stays resident and walks its tiles as one sequence of slabs:
// the loads of the next tile's first slabs are issued under the last slabs of the current one and land during its
// epilogue, which works on the accumulators alone -- and is short: the rows of A sit in the register index of the
// MFMA result, so the maximum over a block of rows is a chain of integer v_max in each lane, one exchange between
// the two half-waves, and one store per column.  No loads, so nothing in it waits for the prefetches in flight.
//
// Tiles: workgroup w takes tiles w, w + G, w + 2 G, ... of the tile grid, row tile (of A) fastest.  With G a
// multiple of the number of row tiles a workgroup keeps its rows of A -- they stay in the caches -- and walks along
// the columns; the workgroups of one XCD (w mod 8) share row tiles modulo 8.
//
// Data movement, LDS layout, swizzle and the hand-over between slabs are those of gemm_bf16_pipe.h with two int8 in
// the place of one bf16: a row's slab is 128 bytes = 128 k, a lane's 16-byte chunk feeds one
// v_mfma_i32_32x32x32_i8 (twice the multiply-adds of the bf16 instruction in the same time), and the sums are exact.
// A and W are handed over as arrays of 16-bit units: K16, lda and ldw count pairs of int8.
// Waits: loads return in order, so "at most n operations outstanding" means all loads but the youngest n have
// landed; the epilogue's stores in flight only make such a wait longer, never shorter.
//
// Requirements (checked by the launcher): K16 % 64 == 0, rows of A a multiple of BM, lda and ldw multiples of 8.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_bf16_pipe.h"

namespace asd {

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_i8_colmax_stream_kernel(int Ma, const int* __restrict__ N_dev,
                                                                             int N_max, int K16,
                                                                             const uint16_t* __restrict__ A, int64_t lda,
                                                                             const uint16_t* __restrict__ W, int64_t ldw,
                                                                             const int32_t* __restrict__ on,
                                                                             const int32_t* __restrict__ live_cols,
                                                                             int32_t* __restrict__ out, int nsub) {
  static_assert(Cfg::PLANES == 1, "one plane");
  constexpr int BM = Cfg::BM, BN = Cfg::BN, STAGES = Cfg::STAGES, MI = Cfg::MI, NJ = Cfg::NJ, NW = Cfg::NW;
  constexpr int AR = Cfg::AR, WM = Cfg::WM, WN = Cfg::WN;
  constexpr int A_LOADS = Cfg::A_LOADS, W_LOADS = Cfg::W_LOADS, LPS = Cfg::LPS, STAGE_BYTES = Cfg::STAGE_BYTES;
  extern __shared__ __attribute__((aligned(16))) uint8_t ldsb[];

  if (on && *on == 0) return;   // the caller's switch, in device memory
  const int N = min(N_dev ? *N_dev : N_max, N_max);
  // live_cols (or NULL): [0] = how many column tiles of W are wanted, then their indices (each below ceil(N / BN))
  const int ntn_all = (N + BN - 1) / BN;
  const int ntm = Ma / BM, ntn = live_cols ? max(0, min(live_cols[0], ntn_all)) : ntn_all;
  const int total = ntm * ntn;
  if ((int)blockIdx.x >= total) return;
  const int n_my = (total - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;   // tiles of this workgroup
  const int nk = K16 / 64;          // slabs per tile
  const int F = n_my * nk;          // slabs of this workgroup

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / Cfg::WGN, wn = wave % Cfg::WGN;
  const int l32 = lane & 31, half = lane >> 5;
  const int lr = lane >> 3;

  // ---- the issue stream: the next slab to issue is slab kt_i of this workgroup's tile number ti_i
  const uint16_t* ap[A_LOADS];
  const uint16_t* wp[W_LOADS];
  auto point_at = [&](int tile) {   // loader addresses of slab 0 of a tile
    const int m0 = (tile % ntm) * BM, n0 = (live_cols ? max(0, min(live_cols[1 + tile / ntm], ntn_all - 1)) : tile / ntm) * BN;
#pragma unroll
    for (int p = 0; p < A_LOADS; ++p) {
      const int row = (wave + NW * p) * 8 + lr;
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      ap[p] = A + (int64_t)(m0 + row) * lda + chunk * 8;
    }
#pragma unroll
    for (int p = 0; p < W_LOADS; ++p) {
      const int row = (wave + NW * p) * 8 + lr;
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      wp[p] = W + (int64_t)min(n0 + row, N - 1) * ldw + chunk * 8;
    }
  };
  auto issue = [&](int kt, int stage, int first, int count) {   // wave-loads first .. first+count-1 of a slab
    uint8_t* sb = ldsb + stage * STAGE_BYTES;
#pragma unroll
    for (int q = 0; q < LPS; ++q) {
      if (q < first || q >= first + count) continue;
      if (q < A_LOADS)
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(ap[q < A_LOADS ? q : 0] + (int64_t)kt * 64),
                                         (lds_ptr_t)(sb + (wave + NW * q) * 1024), 16, 0, 0);
      else
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(wp[q >= A_LOADS ? q - A_LOADS : 0] + (int64_t)kt * 64),
                                         (lds_ptr_t)(sb + AR * 128 + (wave + NW * (q - A_LOADS)) * 1024), 16, 0, 0);
    }
  };

  v16i_b acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  constexpr int G = MI * NJ;                         // MFMAs per group of 32 k
  constexpr int H1 = (G + 1) / 2, H2 = G - H1;       // MFMAs of the last group before / after the hand-over
  constexpr int RD = MI + NJ, SLOTS = (RD + 1) / 2, RLAST = RD - 2 * (SLOTS - 1);
  constexpr int REM = G > SLOTS ? G - SLOTS : 0;
  constexpr int LA = Cfg::LA, LB = Cfg::loads_in_group(3) - LA;

  // prologue: slabs 0 .. STAGES-2 of the stream
  int ti_i = 0, kt_i = 0;
  point_at((int)blockIdx.x);
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < F) {
      issue(kt_i, s, 0, LPS);
      if (++kt_i == nk) {
        kt_i = 0;
        ++ti_i;
        if (ti_i < n_my) point_at((int)blockIdx.x + ti_i * (int)gridDim.x);
      }
    }

  const int sw = (l32 >> 1) & 7;
  const int a_row = (wm * WM + l32) * 128;
  const int w_row = AR * 128 + (wn * WN + l32) * 128;
  int cp[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) cp[ks] = ((ks * 2 + half) ^ sw) * 16;
  v4i_b af[2][MI], wf[2][NJ];
  auto read_frags = [&](const uint8_t* sb, int ks, int buf) {
#pragma unroll
    for (int i = 0; i < MI; ++i) af[buf][i] = *reinterpret_cast<const v4i_b*>(sb + a_row + i * 32 * 128 + cp[ks]);
#pragma unroll
    for (int j = 0; j < NJ; ++j) wf[buf][j] = *reinterpret_cast<const v4i_b*>(sb + w_row + j * 32 * 128 + cp[ks]);
  };
  auto mma = [&](int buf, int first, int count) {
#pragma unroll
    for (int q = 0; q < G; ++q)
      if (q >= first && q < first + count)
        acc[q / NJ][q % NJ] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[buf][q / NJ], wf[buf][q % NJ], acc[q / NJ][q % NJ], 0, 0, 0);
  };

  wait_vmcnt_slabs<LPS, 0>(min(STAGES - 2, F - 1));   // slab 0 landed
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  read_frags(ldsb, 0, 0);

  int kt_c = 0, ti_c = 0;   // of the slab being multiplied: its index within its tile, the tile's number
  for (int f = 0; f < F; ++f) {
    const uint8_t* sb = ldsb + (f % STAGES) * STAGE_BYTES;
    const bool more = f + STAGES - 1 < F;   // uniform: slab f+STAGES-1 exists and is fetched during this slab
    const int nst = (f + STAGES - 1) % STAGES;
    const int kt_n = kt_i;                   // its index within its tile (the loader addresses point at that tile)
#pragma unroll
    for (int ks = 0; ks < 3; ++ks) {
      constexpr int L0 = Cfg::loads_in_group(0);
      read_frags(sb, ks + 1, (ks + 1) & 1);
      if (more) issue(kt_n, nst, Cfg::loads_before_group(ks), Cfg::loads_in_group(ks));
      mma(ks & 1, 0, G);
      sched_pairs<0x100, SLOTS - 1, 2>();
      sched_pairs<0x100, 1, RLAST>();
      sched_pairs<0x010, (L0 < REM ? L0 : REM), 1>();
      sched_mfma<REM - (L0 < REM ? L0 : REM)>();
    }
    if (more) issue(kt_n, nst, Cfg::loads_before_group(3), LB);
    mma(1, 0, H1);
    sched_pairs<0x010, (LB < H1 ? LB : H1), 1>();
    sched_mfma<H1 - (LB < H1 ? LB : H1)>();
    if (f + 1 < F) {
      // this wavefront's loads of slab f+1 must have landed; younger ones may stay in flight
      if (more) wait_vmcnt_slabs<LPS, LPS - LA>(STAGES - 3);
      else wait_vmcnt_slabs<LPS, 0>(F - 2 - f);
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();   // after it nobody reads slab f's stage again: the last group's fragments are in registers
      asm volatile("" ::: "memory");
      read_frags(ldsb + ((f + 1) % STAGES) * STAGE_BYTES, 0, 0);
    }
    if (more) issue(kt_n, nst, Cfg::loads_before_group(3) + LB, LA);
    mma(1, H1, H2);
    sched_pairs<0x100, (SLOTS - 1 < H2 ? SLOTS - 1 : H2), 2>();
    if (more) {   // the issue stream moves on; a new tile gets its addresses
      if (++kt_i == nk) {
        kt_i = 0;
        ++ti_i;
        if (ti_i < n_my) point_at((int)blockIdx.x + ti_i * (int)gridDim.x);
      }
    }
    if (++kt_c == nk) {   // the tile is complete: reduce it, clear the accumulators
      const int tile = (int)blockIdx.x + ti_c * (int)gridDim.x;
      const int m0 = (tile % ntm) * BM, n0 = (live_cols ? max(0, min(live_cols[1 + tile / ntm], ntn_all - 1)) : tile / ntm) * BN;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        // entry r of block i is row 32 i + 8 (r / 4) + 4 half + r % 4 of the wavefront's rows, column 32 j + l32
        int mx = acc[0][j][0];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = max(mx, acc[i][j][r]);
        mx = max(mx, __shfl_xor(mx, 32, 64));   // the other half-wave holds the other rows of the same column
        const int n = n0 + wn * WN + j * 32 + l32;
        if (half == 0 && n < N) out[(int64_t)n * nsub + (m0 + wm * WM) / WM] = mx;
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
      kt_c = 0;
      ++ti_c;
    }
  }
}

// wgs: resident workgroups (one per CU; a multiple of Ma / BM keeps each on one row tile of A).
// out [N, nsub] with nsub >= Ma / WM.
template <class Cfg>
inline hipError_t launch_gemm_i8_colmax_stream(int Ma, const int* N_dev, int N_max, int K16, const uint16_t* A,
                                               int64_t lda, const uint16_t* W, int64_t ldw, const int32_t* on,
                                               const int32_t* live_cols, int32_t* out, int nsub, int wgs,
                                               hipStream_t st) {
  if (K16 <= 0 || K16 % 64 != 0 || Ma <= 0 || Ma % Cfg::BM != 0 || lda % 8 != 0 || ldw % 8 != 0 || wgs <= 0 ||
      nsub < Ma / Cfg::WM)
    return hipErrorInvalidValue;
  auto kern = gemm_i8_colmax_stream_kernel<Cfg>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cfg::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(Cfg::THREADS), Cfg::LDS_BYTES, st, Ma, N_dev, N_max, K16, A, lda, W, ldw,
                     on, live_cols, out, nsub);
  return hipGetLastError();
}

}  // namespace asd
