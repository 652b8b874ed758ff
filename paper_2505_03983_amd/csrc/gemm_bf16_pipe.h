// bf16 x bf16 -> fp32 "NT" GEMM for gfx950 with a multi-stage, direct-to-LDS
// pipeline:  acc[m][n] = sum_k A[m][k] * W[n][k],  A [M, K], W [N, K] bf16.
//
// Why a second kernel: one bf16 MFMA does 16x the work of an fp32 one per
// cycle, so a K slab is consumed in a few hundred cycles -- far less than the
// latency of the global loads that fetch the next one.  Here the loads of
// STAGES-1 slabs are kept in flight: global_load_lds_dwordx4 moves 16 bytes per
// lane from HBM/L2 straight into LDS (no VGPR staging, no ds_write), completion
// is tracked with s_waitcnt vmcnt, and one barrier per slab hands a landed
// stage to the MFMA loop while the stage just consumed is refilled.
//
// LDS layout of a stage: A rows then W rows, each row = one slab of 64 bf16 =
// 8 chunks of 16 bytes, unpadded (a wave's direct load writes 64 consecutive
// chunks = 8 rows).  LDS serves 256 bytes per clock (64 banks), i.e. 16 lanes
// of a 128-bit read at a time; to keep the fragment reads (16 consecutive rows,
// same chunk) free of bank conflicts, chunk c of row r is stored at chunk slot
// c ^ ((r >> 1) & 7): a row pair shares a key and differs in the 128-byte half,
// so 16 rows land in 16 different 16-byte slots of a 256-byte line.  The
// permutation is applied on the global side (lane L of a wave-load fetches
// the chunk that belongs in slot L), which still reads whole 128-byte row
// segments.  A lane feeds k = 16*ks + 8*half .. +7 of its row to MFMA ks, for
// both operands, so the pairing of elements is exact.
//
// Requirements (checked by the host): K % 64 == 0, lda and ldw multiples of 8,
// 16-byte aligned bases.  M comes from device memory (compacted row plan).
//
// Two-plane A operand (PLANES = 2): A is given as the sum of two bf16 matrices of the same shape, a_plane
// elements apart (activations kept to 16 significant bits as hi + lo, see mlp.hip).  A stage then holds
// the slab of both planes above the W slab and every (A fragment, W fragment) pair is multiplied twice,
// once per plane, into the same accumulator: the weights are loaded once for both.
//
// Split K (gridDim.z > 1): for a handful of rows the kernel is a stream of the weight matrix, and HBM
// only delivers its bandwidth with ~16 MB in flight -- more workgroups than the output has tiles.  The
// z-th workgroup of a tile contracts the z-th share of K and leaves its fp32 partial tile in scratch;
// splitk_finish_kernel then adds the partials in z order and runs the epilogue.  (Finishing inside the
// GEMM, by whichever workgroup of a tile arrives last, was measured: the device-scope fences it needs
// write back and invalidate an XCD's whole L2 and cost more than the second launch.)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_bf16.h"

namespace asd {

// BM x BN workgroup tile, STAGES LDS stages, WGM x WGN wavefronts (each owns a (BM/WGM) x (BN/WGN) sub-tile).
// Eight wavefronts (two per SIMD) let one wavefront's MFMAs run while its SIMD neighbour waits on the
// address unit: a direct-to-LDS load of 1 KB occupies the CU's single address path for ~16 cycles and
// the issuing wavefront stalls until it is accepted.
template <int BM_, int BN_, int STAGES_, int WGM_ = 2, int WGN_ = 4, int PLANES_ = 1>
struct PipeCfg16 {
  static constexpr int BM = BM_, BN = BN_, STAGES = STAGES_, BK = 64, WGM = WGM_, WGN = WGN_, PLANES = PLANES_;
  static constexpr int NW = WGM * WGN, THREADS = 64 * NW;
  static constexpr int WM = BM / WGM, WN = BN / WGN;          // wavefront sub-tile
  static constexpr int MI = WM / 32, NJ = WN / 32;
  static constexpr int AR = PLANES * BM;                      // A rows of a stage: the tile's rows of every plane
  static constexpr int A_LOADS = AR / 8 / NW, W_LOADS = BN / 8 / NW;  // wave-loads (8 rows each) per wavefront per slab
  static constexpr int LPS = A_LOADS + W_LOADS;
  static constexpr int STAGE_BYTES = (AR + BN) * 128;
  static constexpr size_t LDS_BYTES = (size_t)STAGES * STAGE_BYTES;
  static_assert(PLANES == 1 || PLANES == 2, "A operand planes");
  static_assert(WM % 32 == 0 && WN % 32 == 0 && STAGES >= 3 && STAGES <= 8, "tile shape");
  static_assert(AR % (8 * NW) == 0 && BN % (8 * NW) == 0, "wave-loads must divide evenly among the wavefronts");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS of a CU");
  static_assert(LPS * (STAGES - 1) <= 63, "vmcnt range");
  // loads of the next slab issued inside MFMA group g (0..3), and those of group 3 issued after the hand-over
  static constexpr int loads_in_group(int g) { return LPS / 4 + (g < LPS % 4 ? 1 : 0); }
  static constexpr int loads_before_group(int g) { return g == 0 ? 0 : loads_before_group(g - 1) + loads_in_group(g - 1); }
  static constexpr int LA = loads_in_group(3) > 0 ? 1 : 0;
};

// Wait until at most `slabs` * LPS + EXTRA of this wavefront's loads are outstanding (slabs in 0..6).
template <int LPS, int EXTRA>
__device__ __forceinline__ void wait_vmcnt_slabs(int slabs) {
  switch (slabs) {
    case 0: wait_vmcnt<EXTRA>(); break;
    case 1: wait_vmcnt<(1 * LPS + EXTRA <= 63 ? 1 * LPS + EXTRA : 63)>(); break;
    case 2: wait_vmcnt<(2 * LPS + EXTRA <= 63 ? 2 * LPS + EXTRA : 63)>(); break;
    case 3: wait_vmcnt<(3 * LPS + EXTRA <= 63 ? 3 * LPS + EXTRA : 63)>(); break;
    case 4: wait_vmcnt<(4 * LPS + EXTRA <= 63 ? 4 * LPS + EXTRA : 63)>(); break;
    case 5: wait_vmcnt<(5 * LPS + EXTRA <= 63 ? 5 * LPS + EXTRA : 63)>(); break;
    default: wait_vmcnt<(6 * LPS + EXTRA <= 63 ? 6 * LPS + EXTRA : 63)>(); break;
  }
}

template <class Cfg, class Epi, int CALL>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_bf16_nt_pipe_kernel(const int* __restrict__ M_dev, int M_max,
                                                                         int N, int K,
                                                                         const uint16_t* __restrict__ A, int64_t lda,
                                                                         int64_t a_plane,
                                                                         const uint16_t* __restrict__ W, int64_t ldw,
                                                                         Epi epi, float* __restrict__ part, int m_lo,
                                                                         int m_hi) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, STAGES = Cfg::STAGES, MI = Cfg::MI, NJ = Cfg::NJ, NW = Cfg::NW;
  constexpr int AR = Cfg::AR, PL = Cfg::PLANES, AI = PL * MI;   // AI: A fragments per k group (all planes)
  constexpr int WM = Cfg::WM, WN = Cfg::WN;
  constexpr int A_LOADS = Cfg::A_LOADS, W_LOADS = Cfg::W_LOADS, LPS = Cfg::LPS, STAGE_BYTES = Cfg::STAGE_BYTES;
  extern __shared__ __attribute__((aligned(16))) uint8_t ldsb[];

  const int M_all = M_dev ? *M_dev : M_max;   // the gate below looks at the true row count
  const int M = min(M_all, M_max);
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  // (m_lo, m_hi]: the row counts this launch serves -- the caller may queue several tile shapes for one
  // product and let the row count, known on the device only, pick the one that runs
  if (m0 >= M || M_all <= m_lo || M_all > m_hi) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: LDS bases of the direct loads stay scalar
  const int wm = wave / Cfg::WGN, wn = wave % Cfg::WGN;
  const int l32 = lane & 31, half = lane >> 5;

  const int splits = gridDim.z;
  const int nk = K / 64 / splits;                       // slabs of this workgroup's share of K
  const int64_t k0 = (int64_t)blockIdx.z * nk * 64;

  // loader: wave-load q covers rows 8q..8q+7; lane L fills chunk slot L of that 1 KB block
  const int lr = lane >> 3;
  const uint16_t* ap[A_LOADS];
  const uint16_t* wp[W_LOADS];
#pragma unroll
  for (int p = 0; p < A_LOADS; ++p) {
    const int srow = (wave + NW * p) * 8 + lr;               // row inside the stage: plane * BM + row inside the tile
    const int plane = srow / BM, row = srow - plane * BM;    // (a wave-load's eight rows lie in one plane: BM % 8 == 0)
    const int chunk = (lane & 7) ^ ((srow >> 1) & 7);        // global chunk that belongs in slot (lane & 7)
    ap[p] = A + plane * a_plane + (int64_t)min(m0 + row, M - 1) * lda + chunk * 8 + k0;
  }
#pragma unroll
  for (int p = 0; p < W_LOADS; ++p) {
    const int row = (wave + NW * p) * 8 + lr;
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    wp[p] = W + (int64_t)min(n0 + row, N - 1) * ldw + chunk * 8 + k0;
  }
  // wave-loads first .. first+count-1 (A loads, then W loads) of slab kt into `stage`
  auto issue = [&](int kt, int stage, int first, int count) {
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

  v16f_b acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- software pipeline, rotated so that everything that is not an MFMA runs in the shadow of MFMAs:
  //   prologue : loads of slabs 0..STAGES-2 in flight, slab 0 landed, its first fragments read
  //   slab kt  : four groups of 16 k.  Each group issues its MFMAs with the next group's fragment reads
  //              (two behind each of the first MFMAs) and its share of the direct loads of slab
  //              kt+STAGES-1 (one behind each following MFMA; that slab's stage was released by the
  //              barrier of the previous iteration) slotted in.
  //              Half-way through group 3 the wavefront waits for its loads of slab kt+1, meets the
  //              others at the barrier (after which nobody reads slab kt's stage again: group 3's
  //              fragments are already in registers) and reads the first fragments of slab kt+1 --
  //              while the rest of group 3 executes.
  constexpr int G = AI * NJ;                         // MFMAs per group
  constexpr int H1 = (G + 1) / 2, H2 = G - H1;       // MFMAs of group 3 before / after the hand-over
  constexpr int RD = AI + NJ, SLOTS = (RD + 1) / 2, RLAST = RD - 2 * (SLOTS - 1);
  constexpr int REM = G > SLOTS ? G - SLOTS : 0;     // MFMAs of a group left after the read slots
  constexpr int LA = Cfg::LA, LB = Cfg::loads_in_group(3) - LA;
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < nk) issue(s, s, 0, LPS);

  const int sw = (l32 >> 1) & 7;  // swizzle key of this lane's rows (tile offsets are multiples of 16)
  const int a_row = (wm * WM + l32) * 128;
  const int w_row = AR * 128 + (wn * WN + l32) * 128;
  int cp[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) cp[ks] = ((ks * 2 + half) ^ sw) * 16;

  v8bf af[2][AI], wf[2][NJ];
  auto read_frags = [&](const uint8_t* sb, int ks, int buf) {
#pragma unroll
    for (int i = 0; i < AI; ++i)   // fragment i: plane i / MI, 32-row block i % MI
      af[buf][i] = *reinterpret_cast<const v8bf*>(sb + (i / MI) * (BM * 128) + a_row + (i % MI) * 32 * 128 + cp[ks]);
#pragma unroll
    for (int j = 0; j < NJ; ++j) wf[buf][j] = *reinterpret_cast<const v8bf*>(sb + w_row + j * 32 * 128 + cp[ks]);
  };
  auto mma = [&](int buf, int first, int count) {  // MFMAs first .. first+count-1 of a group, row-major over (i, j)
#pragma unroll
    for (int q = 0; q < G; ++q)
      if (q >= first && q < first + count)
        acc[(q / NJ) % MI][q % NJ] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][q / NJ], wf[buf][q % NJ],
                                                                             acc[(q / NJ) % MI][q % NJ], 0, 0, 0);
  };

  wait_vmcnt_slabs<LPS, 0>(min(STAGES - 2, nk - 1));   // slab 0 landed; the other prologue slabs may be in flight
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  read_frags(ldsb, 0, 0);

  for (int kt = 0; kt < nk; ++kt) {
    const uint8_t* sb = ldsb + (kt % STAGES) * STAGE_BYTES;
    const bool more = kt + STAGES - 1 < nk;  // uniform: slab kt+STAGES-1 exists and is fetched during this slab
    const int nxt = kt + STAGES - 1, nst = (kt + STAGES - 1) % STAGES;
#pragma unroll
    for (int ks = 0; ks < 3; ++ks) {
      constexpr int L0 = Cfg::loads_in_group(0);  // groups 0..2 may differ by one load; hints use the larger count
      read_frags(sb, ks + 1, (ks + 1) & 1);
      if (more) issue(nxt, nst, Cfg::loads_before_group(ks), Cfg::loads_in_group(ks));
      mma(ks & 1, 0, G);
      sched_pairs<0x100, SLOTS - 1, 2>();
      sched_pairs<0x100, 1, RLAST>();
      sched_pairs<0x010, (L0 < REM ? L0 : REM), 1>();
      sched_mfma<REM - (L0 < REM ? L0 : REM)>();
    }
    // group 3, first part
    if (more) issue(nxt, nst, Cfg::loads_before_group(3), LB);
    mma(1, 0, H1);
    sched_pairs<0x010, (LB < H1 ? LB : H1), 1>();
    sched_mfma<H1 - (LB < H1 ? LB : H1)>();
    if (kt + 1 < nk) {
      // This wavefront's loads of slab kt+1 must have landed.  Younger loads that may stay in flight:
      // whole slabs kt+2 .. and, if slab kt+STAGES-1 exists, the LPS-LA loads of it issued so far.
      if (more) wait_vmcnt_slabs<LPS, LPS - LA>(STAGES - 3);
      else wait_vmcnt_slabs<LPS, 0>(nk - 2 - kt);
      // A bare barrier: __syncthreads() would add a fence that waits for *all* outstanding loads.
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      read_frags(ldsb + ((kt + 1) % STAGES) * STAGE_BYTES, 0, 0);
    }
    if (more) issue(nxt, nst, Cfg::loads_before_group(3) + LB, LA);
    mma(1, H1, H2);
    sched_pairs<0x100, (SLOTS - 1 < H2 ? SLOTS - 1 : H2), 2>();
  }

  // Epilogue through LDS (the pipeline stages are free now): each wavefront parks its WM x WN fp32
  // sub-tile in its own LDS region, then walks it row by row with 16-byte accesses, so global traffic
  // is row-contiguous and the code is a short loop rather than 16*MI*NJ unrolled scalar stores.
  static_assert((size_t)BM * BN * 4 <= Cfg::LDS_BYTES, "epilogue staging must fit in the pipeline's LDS");
  __builtin_amdgcn_s_barrier();  // every wavefront is done reading the last stage
  float* stage = reinterpret_cast<float*>(ldsb) + wave * (WM * WN);
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        stage[(i * 32 + 8 * (r >> 2) + 4 * half + (r & 3)) * WN + j * 32 + l32] = acc[i][j][r];
  // the region is private to this wavefront: LDS operations of one wavefront complete in order
  constexpr int LPR = WN / 4;        // lanes per row (one float4 each)
  constexpr int RPI = 64 / LPR;      // rows per iteration
  const int lrow = lane / LPR, lcol = (lane % LPR) * 4;
  // The residual stream is read and rewritten in place: all reads of a batch of rows are issued
  // before its first write, so a batch costs one memory round trip.
  constexpr int ITERS = WM / RPI, BATCH = ITERS < 8 ? ITERS : 8;
  static_assert(ITERS % BATCH == 0, "epilogue batching");
  const int n = n0 + wn * WN + lcol;
  if (splits > 1) {
    for (int it = 0; it < ITERS; ++it) {
      const int row = it * RPI + lrow;
      const int m = m0 + wm * WM + row;
      if (m < M && n < N)
        *reinterpret_cast<float4*>(part + ((int64_t)blockIdx.z * M_max + m) * N + n) =
            *reinterpret_cast<const float4*>(&stage[row * WN + lcol]);
    }
    return;
  }
  for (int it0 = 0; it0 < ITERS; it0 += BATCH) {
    float4 v[BATCH], prev[BATCH];
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
      const int row = (it0 + b) * RPI + lrow;
      const int m = m0 + wm * WM + row;
      v[b] = *reinterpret_cast<const float4*>(&stage[row * WN + lcol]);
      prev[b] = (Epi::kLoads && m < M && n < N) ? epi.load4(m, n) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
      const int m = m0 + wm * WM + (it0 + b) * RPI + lrow;
      if (m < M && n < N) epi.store4(m, n, v[b], prev[b]);
    }
  }
}

// One thread per four columns of a row: partials added in z order, then the epilogue.
template <class Epi>
__global__ __launch_bounds__(256) void splitk_finish_kernel(const int* __restrict__ M_dev, int M_max, int N, int splits,
                                                            const float* __restrict__ part, Epi epi, int m_lo,
                                                            int m_hi) {
  const int M_all = M_dev ? *M_dev : M_max;
  const int M = min(M_all, M_max);
  const int m = blockIdx.y;
  const int n = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (m >= M || n >= N || M_all <= m_lo || M_all > m_hi) return;
  const float4 prev = Epi::kLoads ? epi.load4(m, n) : make_float4(0.f, 0.f, 0.f, 0.f);
  float4 v = *reinterpret_cast<const float4*>(part + (int64_t)m * N + n);
  for (int z = 1; z < splits; ++z) {
    const float4 q = *reinterpret_cast<const float4*>(part + ((int64_t)z * M_max + m) * N + n);
    v.x += q.x; v.y += q.y; v.z += q.z; v.w += q.w;
  }
  epi.store4(m, n, v, prev);
}

// splits > 1 needs (K / 64) % splits == 0 and `part` of splits * M * N floats.
template <class Cfg, int CALL, class Epi>
inline hipError_t launch_gemm_bf16_nt_pipe(const int* M_dev, int M, int N, int K, const uint16_t* A, int64_t lda,
                                           int64_t a_plane, const uint16_t* W, int64_t ldw, Epi epi, hipStream_t st,
                                           int splits = 1, float* part = nullptr, int m_lo = -1,
                                           int m_hi = 0x7fffffff) {
  if (splits < 1 || (K / 64) % splits != 0 || (splits > 1 && !part)) return hipErrorInvalidValue;
  dim3 grid((unsigned)((N + Cfg::BN - 1) / Cfg::BN), (unsigned)((M + Cfg::BM - 1) / Cfg::BM), (unsigned)splits);
  auto kern = gemm_bf16_nt_pipe_kernel<Cfg, Epi, CALL>;
  static bool attr_set = false;  // dynamic LDS above the default limit needs the attribute once per kernel
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)Cfg::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(Cfg::THREADS), Cfg::LDS_BYTES, st, M_dev, M, N, K, A, lda, a_plane, W, ldw, epi,
                     part, m_lo, m_hi);
  if (splits > 1)
    hipLaunchKernelGGL(splitk_finish_kernel<Epi>, dim3((unsigned)((N / 4 + 255) / 256), (unsigned)M), dim3(256), 0, st,
                       M_dev, M, N, splits, part, epi, m_lo, m_hi);
  return hipGetLastError();
}

}  // namespace asd
