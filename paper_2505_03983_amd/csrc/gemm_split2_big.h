// The two-fp16-term GEMM of gemm_split3.h on a 256 x 256 tile, for launches in which (nearly) every tile is wanted.
//
// With three products per element pair the 128 x 128 kernel moves as much as it multiplies: per K slab of 32 a CU
// needs 125 bytes per clock from its LDS and 43 from L2 to keep the matrix pipes busy, which is what those paths give
// at best, and the three do not overlap well.  Operand traffic per product falls with the tile: a workgroup of eight
// wavefronts, each owning 128 x 64 of a 256 x 256 tile, needs 83 and 21 bytes per clock.  What stood in the way was
// registers -- two planes per operand double the fragments -- so this kernel streams them: per group of 16 k a
// wavefront holds one plane of A and one of B at a time and takes the three plane pairs in the order
//   a1 b1,  a1 b2,  a2 b1
// reading b2 under the first eight MFMAs, a2 under the second and the next group's a1, b1 under the third (a1's
// registers are free by then; b1 has a second buffer).  Global loads: B -- an image that stays in the caches -- one
// slab ahead in a single register slot (a slab is 48 MFMAs = 1536 cycles per wavefront), A -- which streams from
// memory -- two slabs ahead in two.  Same terms, same order of accumulation per output element as gemm_split3.h's
// tile: the results are bit-identical to it.
//
// Requirements (checked by the launcher): K % 32 == 0, B's image packed for this tiling (BN = 256), rows of A 16-byte
// aligned.  One workgroup per CU (136 KB of LDS).  No K split, no tile lists.
#pragma once
#include "gemm_split3.h"

namespace asd {

typedef Split3Cfg<256, 256, 2, 4, 32, 2> Split2BigCfg;

// run_if (or NULL): the kernel runs only if *run_if == run_val (a switch in device memory, so that one captured
// graph can hold this kernel and the small-tile one for the same GEMM).
template <class Op, bool ROWS_PER_XCD>
__global__ __launch_bounds__(512, 1) void gemm_split2_big_kernel(const int* __restrict__ M_dev, int M_max, int N, int K,
                                                                 RowSrc A, const uint8_t* __restrict__ Bimg, Op op,
                                                                 int sparse, const int32_t* __restrict__ run_if,
                                                                 int run_val) {
  typedef Split2BigCfg Cfg;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, MI = Cfg::MI, NJ = Cfg::NJ, BK = Cfg::BK, RB = Cfg::RB;
  constexpr int RA = Cfg::RA, RPP = Cfg::RPP, A_PLANE = Cfg::A_PLANE, B_PLANE = Cfg::B_PLANE;
  constexpr int A_STAGE = Cfg::A_STAGE, B_STAGE = Cfg::B_STAGE, B_LOADS = Cfg::B_LOADS;
  static_assert(Cfg::PLANES == 2 && Cfg::NG == 2 && MI == 4 && NJ == 2, "written for this shape");
  constexpr int kUnits = (BM / 128) * (BN / 128);
  if (run_if && *run_if != run_val) return;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_all[];
  uint8_t* lds_a = lds_all;                                   // [2 stages][2 planes][BM rows][RB bytes]
  uint8_t* lds_b = lds_all + 2 * A_STAGE;                     // [2 stages][2 planes][BN rows][RB bytes]
  float* s_row = reinterpret_cast<float*>(lds_all + 2 * (A_STAGE + B_STAGE));   // [8 * BM], the Op's
  uint16_t* s_list = reinterpret_cast<uint16_t*>(s_row + 8 * BM);                // sparse K: [K / BK] live slabs, in order

  const int M = M_dev ? min(*M_dev, M_max) : M_max;
  int tile_n = blockIdx.x, tile_m = blockIdx.y;
  if (ROWS_PER_XCD) {   // all column tiles of a row tile on one XCD (see gemm_split3.h; grid.y is a multiple of 8)
    const unsigned ntn = gridDim.x, lin = blockIdx.x + ntn * blockIdx.y;
    const unsigned G = lin / (8 * ntn), r = lin % (8 * ntn);
    tile_m = (int)(8 * G + r % 8);
    tile_n = (int)(r / 8);
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  if (m0 >= M) return;
  if constexpr (Op::kRowTileSkip) {
    if (op.template skip_rows<BM>(m0, M)) return;   // every row of the tile is somebody else's
  }
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const Frag<Cfg> fr{wave / Cfg::WGN, wave % Cfg::WGN, lane & 31, lane >> 5, tile_n};
  const int nk_all = K / BK;
  int nk = nk_all;

  const int lrow = tid / Cfg::KQ, lkq = tid % Cfg::KQ;
  const float* ap[RA];
  int a_dst[RA];
#pragma unroll
  for (int p = 0; p < RA; ++p) {
    const int r = lrow + RPP * p;
    ap[p] = A.row(min(m0 + r, M - 1)) + lkq * 8;
    a_dst[p] = r * RB + Cfg::slot(r, lkq) * 16;
  }
  op.template init<Cfg>(m0, M, lrow, lkq, s_row);
  bool listed = false;
  if constexpr (Op::kSparseK) {
    if (sparse) {   // as in gemm_split3.h: the Op's live column groups -> a list of slabs in LDS
      const int ng = op.groups(), spg = op.group_cols() / BK;
      uint8_t* flags = reinterpret_cast<uint8_t*>(s_list) + ((2 * nk_all + 15) & ~15);
      int* s_cnt = reinterpret_cast<int*>(flags + ((ng + 15) & ~15));
      for (int g = tid; g < ng; g += Cfg::THREADS) flags[g] = 0;
      __syncthreads();
      op.template mark_live<Cfg>(m0, M, lrow, lkq, flags);
      __syncthreads();
      if (wave == 0) {
        int count = 0;
        for (int g0 = 0; g0 < ng; g0 += 64) {
          const int g = g0 + lane;
          const bool live = g < ng && flags[g] != 0;
          const unsigned long long mask = __ballot(live);
          const int pos = count + __popcll(mask & ((1ull << lane) - 1ull));
          if (live)
            for (int t = 0; t < spg; ++t) s_list[pos * spg + t] = (uint16_t)(g * spg + t);
          count += __popcll(mask);
        }
        if (lane == 0) *s_cnt = count * spg;
      }
      __syncthreads();
      nk = __builtin_amdgcn_readfirstlane(*s_cnt);
      if (nk == 0) nk = nk_all;   // nothing live (rows of NaN): walk everything rather than an unwritten list
      listed = nk < nk_all;
    }
    op.note_slabs(kUnits * nk, kUnits * nk_all, tid);   // in slabs of a 128 x 128 tile, like the small kernel's
  }
  const uint8_t* bsrc = Bimg + (int64_t)tile_n * nk_all * B_STAGE + tid * 16;
  auto slab_of = [&](int kt) -> int64_t {
    if constexpr (Op::kSparseK) {   // read in either case (the list's room is always there): a branch here would cut
      const int sl = __builtin_amdgcn_readfirstlane((int)s_list[kt]);   // the slab's code into scheduling regions
      return (int64_t)(listed ? sl : kt);
    }
    return (int64_t)kt;
  };
  float4 ra[2][RA][2];
  u32x4 rb[B_LOADS];
  auto gload_a = [&](int kt, int slot) {
    const int64_t sl = slab_of(kt);
#pragma unroll
    for (int p = 0; p < RA; ++p) {
      ra[slot][p][0] = *reinterpret_cast<const float4*>(ap[p] + sl * BK);
      ra[slot][p][1] = *reinterpret_cast<const float4*>(ap[p] + sl * BK + 4);
    }
  };
  auto gload_b = [&](int kt) {
    const int64_t sl = slab_of(kt);
#pragma unroll
    for (int q = 0; q < B_LOADS; ++q) rb[q] = *reinterpret_cast<const u32x4*>(bsrc + sl * B_STAGE + q * 16 * Cfg::THREADS);
  };
  auto sstore = [&](int stage, int slot) {   // register slot -> LDS stage `stage`
    uint8_t* sa = lds_a + stage * A_STAGE;
    uint8_t* sb = lds_b + stage * B_STAGE + tid * 16;
#pragma unroll
    for (int q = 0; q < B_LOADS; ++q) *reinterpret_cast<u32x4*>(sb + q * 16 * Cfg::THREADS) = rb[q];
#pragma unroll
    for (int p = 0; p < RA; ++p) {
      const float4 v0 = op.load_a(ra[slot][p][0], p), v1 = op.load_a(ra[slot][p][1], p);
      const float x[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
      u32x4 p1, p2;
      split2_pack(x, p1, p2);
      *reinterpret_cast<u32x4*>(sa + a_dst[p]) = p1;
      *reinterpret_cast<u32x4*>(sa + A_PLANE + a_dst[p]) = p2;
    }
  };

  v16f acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  int f_off[2];
#pragma unroll
  for (int g = 0; g < 2; ++g) f_off[g] = fr.l32 * RB + Cfg::slot(fr.l32, 2 * g + fr.half) * 16;
  const uint8_t* fa = lds_a + fr.wm * Cfg::WM * RB;
  const uint8_t* fb = lds_b + fr.wn * Cfg::WN * RB;
  v8h a1[MI], a2[MI], b1[2][NJ], b2[NJ];
  auto read_a = [&](int stage, int plane, int g, v8h (&dst)[MI]) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
      dst[i] = *reinterpret_cast<const v8h*>(fa + stage * A_STAGE + plane * A_PLANE + i * 32 * RB + f_off[g]);
  };
  auto read_b = [&](int stage, int plane, int g, v8h (&dst)[NJ]) {
#pragma unroll
    for (int j = 0; j < NJ; ++j)
      dst[j] = *reinterpret_cast<const v8h*>(fb + stage * B_STAGE + plane * B_PLANE + j * 32 * RB + f_off[g]);
  };
  auto mma = [&](const v8h (&a)[MI], const v8h (&b)[NJ]) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
  };
  auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

  // ---- prologue: slab 0 in stage 0; A of slabs 1 and 2 and B of slab 1 on their way.  Slab k's A waits in register
  // slot k & 1.
  gload_a(0, 0);
  gload_b(0);
  if (nk > 1) gload_a(1, 1);
  sstore(0, 0);
  if (nk > 1) gload_b(1);
  if (nk > 2) gload_a(2, 0);
  lds_barrier();
  read_a(0, 0, 0, a1);
  read_b(0, 0, 0, b1[0]);
  // One slab (LDS stage par): two groups of three plane pairs.  The slab after it goes from the registers into the
  // other stage under the first group, and the loads that refill them are issued right behind; the barrier sits in
  // front of the last eight MFMAs, under which the next slab's first fragments arrive.
  // steady: slabs kt + 1 .. kt + 3 exist -- no branches, so that the slab is one scheduling region and the interleaving
  // asked for below holds: three VALU instructions of the split behind each of the first sixteen MFMAs, in the first
  // GEMM also the stores into the other stage and B's loads behind the next eight and A's loads behind the eight after.
  // (An MFMA holds its pipe for 32 cycles in which the wavefront can issue half a dozen other instructions for
  // nothing; clumped behind the MFMAs they cost their full time.  Measured on 65536 x 4096 x 1024: first GEMM 1.84 ->
  // 1.80 ms, second 1.64 -> 1.53 ms, most of the latter from the single region.)
  auto slab = [&](int kt, auto par_c, auto steady_c) {
    constexpr int par = decltype(par_c)::value, npar = par ^ 1;
    constexpr bool steady = decltype(steady_c)::value;
    const bool more = steady || kt + 1 < nk;
    __builtin_amdgcn_s_setprio(1);
    // group 0
    read_b(par, 1, 0, b2);
    mma(a1, b1[0]);
    read_a(par, 1, 0, a2);
    mma(a1, b2);
    // (stage npar: its last readers passed the barrier of the slab before; slab kt + 1 sits in A slot (kt + 1) & 1)
    if (more) sstore(npar, npar);
    if (steady || kt + 2 < nk) gload_b(kt + 2);
    read_a(par, 0, 1, a1);
    read_b(par, 0, 1, b1[1]);
    mma(a2, b1[0]);
    if (steady || kt + 3 < nk) gload_a(kt + 3, npar);   // the slot sstore has just emptied
    // group 1
    read_b(par, 1, 1, b2);
    mma(a1, b1[1]);
    if constexpr (steady) {
      sched_pairs<0x002, 16, 3>();
      if constexpr (!Op::kSparseK) {   // (the second GEMM, with four times the VALU work in load_a, ran slower with these)
        sched_pairs<0x200, 8, 1>();
        sched_pairs<0x020, 8, 1>();
      }
    }
    read_a(par, 1, 1, a2);
    mma(a1, b2);
    if (more) {
      lds_barrier();
      read_a(npar, 0, 0, a1);
      read_b(npar, 0, 0, b1[0]);
    }
    mma(a2, b1[1]);
    __builtin_amdgcn_s_setprio(0);
  };
  typedef std::integral_constant<int, 0> I0;
  typedef std::integral_constant<int, 1> I1;
  typedef std::integral_constant<bool, true> Steady;
  typedef std::integral_constant<bool, false> Tail;
  int kt = 0;
  for (; kt + 4 < nk; kt += 2) {
    slab(kt, I0(), Steady());
    slab(kt + 1, I1(), Steady());
  }
  for (; kt < nk; kt += 2) {
    slab(kt, I0(), Tail());
    if (kt + 1 < nk) slab(kt + 1, I1(), Tail());
  }
  __syncthreads();   // every wavefront is done with the operand stages

  op.template finish<Cfg>(lrow, lkq, s_row);
  __syncthreads();
  op.template epilogue<Cfg>(acc, fr, m0, n0, M, N, s_row);
}

// LDS of a launch: the stages, the Op's rows and, for a sparse second GEMM, the slab list.
template <class Op>
inline size_t split2_big_lds(int K, const Op& op, bool sparse) {
  size_t lds = Split2BigCfg::LDS_BYTES;
  if constexpr (Op::kSparseK) {
    (void)sparse;   // the list's room also when nothing is listed: the kernel reads it without asking
    lds += (size_t)((2 * (K / Split2BigCfg::BK) + 15) & ~15) + (size_t)((op.groups() + 15) & ~15) + 16;
  }
  return lds;
}

template <bool ROWS_PER_XCD, class Op>
inline hipError_t launch_gemm_split2_big(const int* M_dev, int M_max, int N, int K, RowSrc A, const uint8_t* Bimg, Op op,
                                         hipStream_t st, bool sparse, const int32_t* run_if, int run_val) {
  typedef Split2BigCfg Cfg;
  if (K <= 0 || K % Cfg::BK != 0) return hipErrorInvalidValue;
  if constexpr (Op::kSparseK) {
    sparse = sparse && op.group_cols() > 0 && op.group_cols() % Cfg::BK == 0 && K % op.group_cols() == 0 && K / Cfg::BK <= 65535;
  } else {
    sparse = false;
  }
  const size_t lds = split2_big_lds(K, op, sparse);
  if (lds > 160 * 1024) return hipErrorInvalidValue;
  unsigned mt = (unsigned)((M_max + Cfg::BM - 1) / Cfg::BM);
  if (ROWS_PER_XCD) mt = (mt + 7) / 8 * 8;
  dim3 grid((unsigned)((N + Cfg::BN - 1) / Cfg::BN), mt, 1);
  auto kern = gemm_split2_big_kernel<Op, ROWS_PER_XCD>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(Cfg::THREADS), lds, st, M_dev, M_max, N, K, A, Bimg, op, sparse ? 1 : 0, run_if, run_val);
  return hipGetLastError();
}

}  // namespace asd
