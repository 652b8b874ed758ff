// fp32 "NT" GEMM on the gfx950 matrix cores:  acc[m][n] = sum_k f(A[m][k]) * B[n][k]
// with both operands K-contiguous.  What happens to the A operand on its way
// into LDS (f) and to the accumulators at the end is supplied by an `Op`.
//
// Tiling (Cfg): a workgroup of 4 wavefronts (2 x 2) owns a BM x BN tile; each
// wavefront a (BM/2) x (BN/2) quadrant as MI x NJ blocks of
// v_mfma_f32_32x32x2_f32.  K is consumed in slabs of BK, staged through LDS
// with register prefetch of the next slab (double-buffered LDS, one barrier
// per slab); inside a slab the LDS fragments of the next group of 8 k values
// are fetched while the MFMAs of the current group issue.
//
// Operand layout of the 32x32x2 instruction: lane l supplies A[row l%32][k l/32]
// and B[col l%32][k l/32]; it receives 16 results, register r holding
// C[8*(r/4) + 4*(l/32) + r%4][l%32].  The order in which k values are fed is
// free as long as A and B agree, so each lane reads four consecutive k of its
// row with one 128-bit LDS load and the four values go to four MFMAs: in MFMA
// t of a group, half-wave h feeds k = 8*group + 4*h + t.
//
// LDS rows are BK + 4 floats apart: 16 B aligned for the 128-bit reads, and
// eight consecutive rows then start in eight different groups of four banks.
//
// Tile order: blockIdx.x = column tile (fastest), blockIdx.y = row tile.  Workgroups go to the 8 XCDs
// round-robin by linear id, so an XCD keeps a fixed set of column tiles (its share of B stays in its
// L2) and streams the row tiles of A.  An XCD-aware order over 8 x 8 super-tiles was measured: it cut
// the L2 fills of the second GEMM by 40% but raised those of the first and was ~3% slower overall --
// these kernels are bound by the matrix pipe, not by L2 fills -- so the plain order stays.
//
// The number of rows M is read from device memory (the row plan of a model
// call is compacted on the device, so the host does not know it): the grid is
// sized for M_max and workgroups past M exit at once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace asd {

typedef float v16f __attribute__((ext_vector_type(16)));

// Rows of the A operand: dense (base + m*ld) or gathered (base + off[m]).
struct RowSrc {
  const float* base;
  const int64_t* off;
  int64_t ld;
  __device__ __forceinline__ const float* row(int m) const {
    return off ? base + off[m] : base + (int64_t)m * ld;
  }
};

template <int BM_, int BN_, int BK_>
struct GemmCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_;
  static constexpr int THREADS = 256;
  static constexpr int LDSS = BK + 4;          // LDS row stride in floats
  static constexpr int KQ = BK / 4;            // loader threads per row (one float4 each)
  static constexpr int RPP = THREADS / KQ;     // rows covered by one loader pass
  static constexpr int RA = BM / RPP;          // loader passes over the A tile
  static constexpr int RB = BN / RPP;          // loader passes over the B tile
  static constexpr int WGN = 2, WM = BM / 2, WN = BN / 2;   // 2 x 2 wavefronts and their sub-tile
  static constexpr int MI = BM / 64, NJ = BN / 64;  // 32x32 blocks per wavefront
  static constexpr int KS = BK / 8;            // groups of 8 k per slab
  static constexpr size_t LDS_BYTES = sizeof(float) * (2 * (BM + BN) * LDSS + 8 * BM);
  static_assert(BM % 64 == 0 && BN % 64 == 0 && BK % 8 == 0 && BM % RPP == 0 && BN % RPP == 0, "tile shape");
};

// Position of a lane's accumulators inside the workgroup tile (wavefront (wm, wn) owns a WM x WN sub-tile).
template <class Cfg>
struct Frag {
  int wm, wn, l32, half;
  int tile_n;  // column-tile index of the workgroup
  __device__ __forceinline__ int row(int i, int r) const {
    return wm * Cfg::WM + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
  }
  __device__ __forceinline__ int col(int j) const { return wn * Cfg::WN + j * 32 + l32; }
};

// Op interface (all __device__, templated on Cfg where the tile shape matters):
//   void   init<Cfg>(int m0, int M, int lrow, int lkq, float* s_row)  once, before the K loop (a barrier follows
//                                                          before the epilogue); loader rows lrow + p*RPP
//   float4 load_a(float4 v, int p)                        transform of loader pass p's 4 values (not called on padding)
//   void   finish<Cfg>(int lrow, int lkq, float* s_row)   after the K loop, before a barrier
//   void   epilogue<Cfg>(acc, frag, m0, n0, M, N, s_row)  writes the results
// s_row: 8 floats of LDS per tile row, the Op's own (per-row coefficients and addresses are parked there by
// the loader threads, so that the epilogue -- whose loads the compiler may not move above its stores -- has
// no chain of dependent global loads per row).
// KTAIL: K is not a multiple of BK (the last slab is zero-padded).
// Split K (gridDim.z > 1, Ops with kSplitK only): workgroup z of a tile contracts the z-th share of the slabs and hands
// its accumulators to op.store_partial (fp32 partial tiles in scratch) instead of the epilogue; a finishing kernel of
// the Op's owner adds the partials in z order.  For products with few output tiles and a long K (the second GEMM of
// the mixture denoiser on one row per chain: 256 tiles, K = 4096).
// Requirements (checked by the host launcher): K % 4 == 0, rows 16 B aligned.
// CALL only gives the draft-call and verify-call launches distinct symbols in profiles.
template <class Cfg, class Op, bool KTAIL, int CALL>
__global__ __launch_bounds__(256) void gemm_f32_nt_kernel(const int* __restrict__ M_dev, int M_max, int N, int K,
                                                          RowSrc A, const float* __restrict__ Bm, int64_t ldb,
                                                          Op op, float* __restrict__ part) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, LDSS = Cfg::LDSS;
  constexpr int KQ = Cfg::KQ, RPP = Cfg::RPP, RA = Cfg::RA, RB = Cfg::RB, MI = Cfg::MI, NJ = Cfg::NJ, KS = Cfg::KS;
  extern __shared__ __attribute__((aligned(16))) float lds[];
  float* As = lds;                       // [2][BM * LDSS]
  float* Bs = lds + 2 * BM * LDSS;       // [2][BN * LDSS]
  float* s_row = Bs + 2 * BN * LDSS;     // [8 * BM]

  const int M = M_dev ? min(*M_dev, M_max) : M_max;
  const int tile_n = blockIdx.x;
  const int m0 = blockIdx.y * BM, n0 = tile_n * BN;
  if (m0 >= M) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const Frag<Cfg> fr{wave >> 1, wave & 1, lane & 31, lane >> 5, tile_n};

  const int lrow = tid / KQ, lkq = tid % KQ;
  const float* ap[RA];
  const float* bp[RB];
#pragma unroll
  for (int p = 0; p < RA; ++p) ap[p] = A.row(min(m0 + lrow + RPP * p, M - 1)) + lkq * 4;
#pragma unroll
  for (int p = 0; p < RB; ++p) bp[p] = Bm + (int64_t)min(n0 + lrow + RPP * p, N - 1) * ldb + lkq * 4;
  op.template init<Cfg>(m0, M, lrow, lkq, s_row);
  const int nk_all = (K + BK - 1) / BK;
  const int splits = gridDim.z;
  const int nk = nk_all / splits;                 // slabs of this workgroup (the host makes it divide)
  const int kb = blockIdx.z * nk;                 // its first slab

  float4 ra[RA], rb[RB];
  auto gload = [&](int kt) {
    const bool ok = !KTAIL || (kt * BK + lkq * 4 < K);
#pragma unroll
    for (int p = 0; p < RA; ++p)
      ra[p] = ok ? op.load_a(*reinterpret_cast<const float4*>(ap[p] + kt * BK), p) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int p = 0; p < RB; ++p)
      rb[p] = ok ? *reinterpret_cast<const float4*>(bp[p] + kt * BK) : make_float4(0.f, 0.f, 0.f, 0.f);
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int p = 0; p < RA; ++p)
      *reinterpret_cast<float4*>(&As[buf * BM * LDSS + (lrow + RPP * p) * LDSS + lkq * 4]) = ra[p];
#pragma unroll
    for (int p = 0; p < RB; ++p)
      *reinterpret_cast<float4*>(&Bs[buf * BN * LDSS + (lrow + RPP * p) * LDSS + lkq * 4]) = rb[p];
  };

  v16f acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  gload(kb);
  sstore(0);
  __syncthreads();

  const int a_lane = (fr.wm * (BM / 2) + fr.l32) * LDSS + fr.half * 4;
  const int b_lane = (fr.wn * (BN / 2) + fr.l32) * LDSS + fr.half * 4;

  static_assert(KS % 2 == 0, "the first fragments of a slab go to fragment buffer 0");
  float4 af[2][MI], bf[2][NJ];
  auto read_frags = [&](const float* Ac, const float* Bc, int ks, int buf) {
#pragma unroll
    for (int i = 0; i < MI; ++i) af[buf][i] = *reinterpret_cast<const float4*>(Ac + i * 32 * LDSS + ks * 8);
#pragma unroll
    for (int j = 0; j < NJ; ++j) bf[buf][j] = *reinterpret_cast<const float4*>(Bc + j * 32 * LDSS + ks * 8);
  };
  auto mma = [&](int c, int t) {  // the MI x NJ MFMAs that consume element t of the fragments in buffer c
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const float av = t == 0 ? af[c][i].x : t == 1 ? af[c][i].y : t == 2 ? af[c][i].z : af[c][i].w;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const float bv = t == 0 ? bf[c][j].x : t == 1 ? bf[c][j].y : t == 2 ? bf[c][j].z : bf[c][j].w;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
      }
    }
  };
  read_frags(As + a_lane, Bs + b_lane, 0, 0);

  // Per slab: the global loads of the next slab are issued first; its LDS buffer is free for the whole
  // slab (everybody left it at the previous barrier), so the store into it, the barrier and the first
  // fragment reads of the next slab all sit in the middle of the last group of MFMAs -- whose
  // fragments are in registers by then -- and their latency is covered by this wavefront's own MFMAs.
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < nk;
    if (more) gload(kb + kt + 1);
    const float* Ac = As + cur * BM * LDSS + a_lane;
    const float* Bc = Bs + cur * BN * LDSS + b_lane;
    // While it has fragments to feed, a wavefront outranks its SIMD neighbours that are between slabs:
    // the matrix pipe is the resource to keep busy.
    __builtin_amdgcn_s_setprio(2);
#pragma unroll
    for (int ks = 0; ks < KS - 1; ++ks) {
      read_frags(Ac, Bc, ks + 1, (ks + 1) & 1);
#pragma unroll
      for (int t = 0; t < 4; ++t) mma(ks & 1, t);
    }
    mma((KS - 1) & 1, 0);
    mma((KS - 1) & 1, 1);
    if (more) {
      sstore(cur ^ 1);
      __syncthreads();
      read_frags(As + (cur ^ 1) * BM * LDSS + a_lane, Bs + (cur ^ 1) * BN * LDSS + b_lane, 0, 0);
    }
    mma((KS - 1) & 1, 2);
    mma((KS - 1) & 1, 3);
    __builtin_amdgcn_s_setprio(0);
  }
  __syncthreads();   // every wavefront is done with the operand buffers (the Op may reuse LDS)

  op.template finish<Cfg>(lrow, lkq, s_row);
  __syncthreads();
  if constexpr (Op::kSplitK) {
    if (splits > 1) {
      op.template store_partial<Cfg>(acc, fr, m0, n0, M, M_max, N, s_row, part, (int)blockIdx.z, splits);
      return;
    }
  }
  op.template epilogue<Cfg>(acc, fr, m0, n0, M, N, s_row);
}

// Floats of scratch a split-K launch needs: the partial tiles, then the Op's per-row partials ([splits][M_max]).
inline size_t gemm_f32_splitk_floats(int splits, int M_max, int N) { return (size_t)splits * M_max * ((size_t)N + 1); }

template <class Cfg, int CALL, class Op>
inline hipError_t launch_gemm_f32_nt(const int* M_dev, int M_max, int N, int K, RowSrc A, const float* Bm,
                                     int64_t ldb, Op op, hipStream_t st, int splits = 1, float* part = nullptr) {
  if (splits < 1 || (splits > 1 && (!Op::kSplitK || !part || K % Cfg::BK != 0 || (K / Cfg::BK) % splits != 0)))
    return hipErrorInvalidValue;
  dim3 grid((unsigned)((N + Cfg::BN - 1) / Cfg::BN), (unsigned)((M_max + Cfg::BM - 1) / Cfg::BM), (unsigned)splits);
  if (K % Cfg::BK == 0) {
    auto kern = gemm_f32_nt_kernel<Cfg, Op, false, CALL>;
    static bool attr_set = false;   // dynamic LDS above 64 KB needs the attribute once per kernel
    if (!attr_set && Cfg::LDS_BYTES > 48 * 1024) {
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)Cfg::LDS_BYTES);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(Cfg::THREADS), Cfg::LDS_BYTES, st, M_dev, M_max, N, K, A, Bm, ldb, op, part);
  } else {
    auto kern = gemm_f32_nt_kernel<Cfg, Op, true, CALL>;
    static bool attr_set = false;
    if (!attr_set && Cfg::LDS_BYTES > 48 * 1024) {
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)Cfg::LDS_BYTES);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(Cfg::THREADS), Cfg::LDS_BYTES, st, M_dev, M_max, N, K, A, Bm, ldb, op, part);
  }
  return hipGetLastError();
}

}  // namespace asd
