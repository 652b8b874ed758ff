// fp32 "NT" GEMM on the gfx950 16-bit matrix cores:  acc[m][n] = sum_k f(A[m][k]) * B[n][k]
// with every fp32 operand split into 16-bit terms, in two forms (Split3Cfg::PLANES).
//
// Three bf16 terms, six products.  An fp32 number has a 24-bit significand; cut into three runs of 8 bits it is the
// exact sum x = x1 + x2 + x3 of three bf16 numbers (bf16 has fp32's exponent range, so nothing overflows; the
// cut is by truncation: x1 = the top 16 bits of x, x2 = the top 16 bits of x - x1, x3 = the rest).
// A product of two bf16 numbers is exact in fp32, and the matrix cores accumulate in fp32, so
//   a*b ~= a1*b1 + (a1*b2 + a2*b1) + (a2*b2 + a1*b3 + a3*b1)
// leaves out a2*b3 + a3*b2 + a3*b3: with |x2| < 2^-7 |x1| and |x3| < 2^-15 |x1| that is below 2^-21 |a||b|
// always and 2^-23 |a||b| on average -- a few units of the rounding of one fp32 multiply-add (2^-24), and
// small against the rounding that accumulating K = 10^3 terms in fp32 brings with it either way.  Six bf16 MFMAs
// replace one fp32 MFMA of the same shape, on a pipe that is 16x as fast on paper.  (Splitting into bf16 terms for
// higher-precision products is an old, published device -- e.g. Henry, Tang, Heinecke 2019; the arrangement here is
// this file's.)
//
// Two fp16 terms, three products.  fp16 has an 11-bit significand: x1 = the nearest fp16 of x and x2 = the nearest
// fp16 of x - x1 (exact in fp32) carry 22 bits, |x - x1 - x2| <= 2^-22 |x|, and
//   a*b ~= a1*b1 + a1*b2 + a2*b1
// leaves out a2*b2 and what the terms miss of a and of b: at most 3 * 2^-22 |a||b|, 2^-23 on average -- the same
// accuracy from half the matrix instructions.  fp16 lacks the range, so the caller scales each operand by a power of
// two (exact) that brings its largest magnitude into [2^14, 2^15) -- per row of A through the Op's load_a, once for B
// (split3_pack_b_kernel's scale) -- and the Op's epilogue takes the scales out again.  A second term then leaves
// fp16's normal range only where the element is below 2^-10 of the largest one: an absolute error of 2^-39 of that.
//
// Either way the loop moves as much as it multiplies.  Per 128 x 128 x 32 slab with fp16 terms a workgroup has 768
// cycles of MFMA per SIMD, 96 KB through LDS and 32 KB from L2, and on this chip the three overlap little: a full
// launch keeps the matrix pipes busy in ~40% of the cycles (three bf16 terms: ~62%, at a power-managed ~1.8 GHz).
//
// Dataflow per K slab (BK = 16: one MFMA group; 32: two), written for three planes -- two are the same with a plane less:
//  * B is constant across calls: it is split once (split3_pack_b_kernel) into an *image* of what a
//    workgroup's LDS stage holds -- per column tile and slab: three planes of BN rows x 32 bytes,
//    chunk-swizzled -- so a thread copies three 16-byte pieces (one per plane) at fixed offsets:
//    no address arithmetic, no conversion.
//  * A arrives as fp32 (rows gathered through RowSrc, transformed by the Op's load_a): each thread
//    owns 8 consecutive k of one row, splits them (~5 VALU operations per element) and stores three
//    16-byte chunks, one per plane.
//  * Both operands are loaded two slabs ahead into registers and stored into LDS one slab ahead, under the
//    first half of the MFMAs of a slab; half-way the wavefront meets the others at the barrier and
//    reads the fragments of the next slab under the second half.  (Direct-to-LDS loads would spare the
//    registers of B, but the compiler then waits for *every* load in flight before each use of a
//    loaded register -- it counts the two kinds of load as returning out of order -- which drains the
//    prefetch once per slab.)
//  * Two LDS stages of 3 (BM + BN) 32 bytes; with 128 x 128 tiles and four wavefronts two workgroups
//    share a CU, and the epilogue, the prologue and the barrier waits of one are covered by the
//    MFMAs of the other.  Chunk c (0/1) of row r sits in slot c ^ ((r >> 3) & 1) of its 32-byte row:
//    16 consecutive rows reading the same chunk then cover all 64 banks once.
//  * MFMA v_mfma_f32_32x32x16_bf16: lane l feeds k = 8 (l / 32) .. + 7 of row l % 32, for A and B
//    alike, so the pairing of elements is exact; per slab a wavefront reads 3 (MI + NJ) fragments
//    and issues 6 MI NJ MFMAs -- twice the MFMAs per fragment of a plain bf16 GEMM.
//
// Requirements (checked by the host): K % 16 == 0, rows of A 16-byte aligned.  Rows of the image past
// N are zero.  M is read from device memory; workgroups past it exit at once.
//
// Sparse K (Ops with kSparseK, no K split).  When load_a maps whole stretches of A to exactly 0.0f -- the
// second GEMM of the mixture denoiser, whose A operand is 2^(logit - row maximum): once a posterior has
// narrowed to a few components every other weight is 0.0f (the Op's load_a cuts them off) -- the slabs of K in which
// every row of the tile is zero contribute nothing, bit for bit, and are not visited.  The Op marks the
// groups of columns that are live for some row of the tile (mark_live, from data the producer of A
// left behind); one wavefront compacts them into a list of slabs in LDS and the K loop walks that list.
// The result equals the dense loop's exactly: the skipped products and row-sum terms are zeros.
//
// Two forms of the kernel share the tile code (split3_tile): one workgroup per tile of the grid, and -- for an Op that
// carries lists of the tiles that are wanted at all -- resident workgroups that draw tiles (or half tiles, on a
// second tiling of half the rows) from those lists by ticket; see gemm_split3_nt_list_kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "gemm_bf16.h"
#include "gemm_f32.h"

namespace asd {

// BK: K slab, 16 (one MFMA group) or 32 (two).  The large tile with BK = 16 lets two workgroups share a CU; small
// tiles for few rows take BK = 32, so that a slab carries enough MFMAs to cover the load -> LDS -> fragment
// chain of the next one even with few wavefronts per SIMD.
// PLANES: 3 = three bf16 terms per operand and six products, 2 = two fp16 terms and three products (see above).
template <int BM_, int BN_, int WGM_ = 2, int WGN_ = 2, int BK_ = 16, int PLANES_ = 3>
struct Split3Cfg {
  static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_, BK = BK_, STAGES = 2, PLANES = PLANES_;
  static constexpr int NPROD = PLANES == 3 ? 6 : 3;   // MFMAs per block of the tile and MFMA group
  static constexpr int NG = BK / 16;             // MFMA groups (k = 16) per slab
  static constexpr int RB = 2 * BK;              // bytes of a row of a plane in LDS
  static constexpr int NW = WGM * WGN, THREADS = 64 * NW;
  static constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NJ = WN / 32;
  static constexpr int KQ = BK / 8;              // loader threads per row of A (8 k each)
  static constexpr int RPP = THREADS / KQ;       // rows covered by one loader pass
  static constexpr int RA = BM / RPP;            // loader passes over the A tile
  static constexpr int A_PLANE = BM * RB, B_PLANE = BN * RB;      // bytes of one plane of a slab
  static constexpr int A_STAGE = PLANES * A_PLANE, B_STAGE = PLANES * B_PLANE;
  static constexpr int B_LOADS = B_STAGE / (16 * THREADS);        // 16-byte pieces of a slab's B image per thread
  static constexpr size_t LDS_BYTES = (size_t)STAGES * (A_STAGE + B_STAGE) + sizeof(float) * 8 * BM;
  static_assert(BK == 16 || BK == 32, "K slab");
  static_assert(PLANES == 2 || PLANES == 3, "terms per operand");
  static_assert(WM % 32 == 0 && WN % 32 == 0 && RA >= 1 && BM % RPP == 0 && B_STAGE % (16 * THREADS) == 0, "tile shape");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
  // 16-byte slot of chunk c of row r inside the row: 16 consecutive rows reading one chunk cover all 64 banks once
  __host__ __device__ static constexpr int slot(int r, int c) { return BK == 16 ? (c ^ ((r >> 3) & 1)) : (c ^ ((r >> 2) & 3)); }
};

// Bytes of the B image for an [N, K] operand.
template <class Cfg>
inline size_t split3_image_bytes(int N, int K) {
  return (size_t)((N + Cfg::BN - 1) / Cfg::BN) * (size_t)(K / Cfg::BK) * Cfg::B_STAGE;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));   // A / B operand of v_mfma_f32_32x32x16_f16

// x[0..7] -> three planes of 8 bf16 each (element 0 in the low half of word 0)
__device__ __forceinline__ void split3_pack(const float (&x)[8], u32x4& p1, u32x4& p2, u32x4& p3) {
  uint32_t w1[4], w2[4], w3[4];
  constexpr uint32_t kHiHalves = 0x07060302u;   // v_perm_b32: {S0[31:16], S1[31:16]}
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float xa = x[2 * j], xb = x[2 * j + 1];
    const uint32_t ua = __float_as_uint(xa), ub = __float_as_uint(xb);
    w1[j] = __builtin_amdgcn_perm(ub, ua, kHiHalves);
    const float ra = xa - __uint_as_float(ua & 0xffff0000u), rb = xb - __uint_as_float(ub & 0xffff0000u);
    const uint32_t va = __float_as_uint(ra), vb = __float_as_uint(rb);
    w2[j] = __builtin_amdgcn_perm(vb, va, kHiHalves);
    const float ta = ra - __uint_as_float(va & 0xffff0000u), tb = rb - __uint_as_float(vb & 0xffff0000u);
    w3[j] = __builtin_amdgcn_perm(__float_as_uint(tb), __float_as_uint(ta), kHiHalves);
  }
  p1 = u32x4{w1[0], w1[1], w1[2], w1[3]};
  p2 = u32x4{w2[0], w2[1], w2[2], w2[3]};
  p3 = u32x4{w3[0], w3[1], w3[2], w3[3]};
}

// x[0..7] -> two planes of 8 fp16 each: x1 = the nearest fp16, x2 = the nearest fp16 of x - x1 (that difference is
// exact in fp32).  The caller has scaled x into fp16's range (see the header).
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void split2_pack(const float (&x)[8], u32x4& p1, u32x4& p2) {
  uint32_t w1[4], w2[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float xa = x[2 * j], xb = x[2 * j + 1];
    const f16x2 h = {(_Float16)xa, (_Float16)xb};
    const f16x2 l = {(_Float16)(xa - (float)h.x), (_Float16)(xb - (float)h.y)};
    w1[j] = __builtin_bit_cast(uint32_t, h);
    w2[j] = __builtin_bit_cast(uint32_t, l);
  }
  p1 = u32x4{w1[0], w1[1], w1[2], w1[3]};
  p2 = u32x4{w2[0], w2[1], w2[2], w2[3]};
}
template <int PLANES>
__device__ __forceinline__ void split_pack(const float (&x)[8], u32x4 (&p)[3]) {
  if constexpr (PLANES == 3) split3_pack(x, p[0], p[1], p[2]);
  else split2_pack(x, p[0], p[1]);
}

// B [N, K] fp32 (row stride ldb), times `scale` (a power of two; 1 for three bf16 terms) -> image.  One thread per
// (row of the padded tile grid, chunk of 8 k).
template <class Cfg>
__global__ __launch_bounds__(256) void split3_pack_b_kernel(const float* __restrict__ B, int64_t ldb, int N, int K,
                                                            uint8_t* __restrict__ img, float scale) {
  const int kc = K / 8;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t n_pad = (int64_t)((N + Cfg::BN - 1) / Cfg::BN) * Cfg::BN;
  if (idx >= n_pad * kc) return;
  const int n = (int)(idx / kc), c8 = (int)(idx % kc);
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = n < N ? scale * B[(int64_t)n * ldb + c8 * 8 + e] : 0.f;
  u32x4 p[3];
  split_pack<Cfg::PLANES>(x, p);
  const int tn = n / Cfg::BN, r = n % Cfg::BN, ks = c8 / Cfg::KQ, c = c8 % Cfg::KQ;
  uint8_t* dst = img + ((int64_t)tn * (K / Cfg::BK) + ks) * Cfg::B_STAGE + r * Cfg::RB + Cfg::slot(r, c) * 16;
#pragma unroll
  for (int pl = 0; pl < Cfg::PLANES; ++pl) *reinterpret_cast<u32x4*>(dst + pl * Cfg::B_PLANE) = p[pl];
}

template <class Cfg>
inline hipError_t launch_split3_pack_b(const float* B, int64_t ldb, int N, int K, uint8_t* img, hipStream_t st,
                                       float scale = 1.f) {
  const int64_t n_pad = (int64_t)((N + Cfg::BN - 1) / Cfg::BN) * Cfg::BN;
  const int64_t threads = n_pad * (K / 8);
  hipLaunchKernelGGL(split3_pack_b_kernel<Cfg>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, B, ldb, N, K,
                     img, scale);
  return hipGetLastError();
}

// The Op interface is that of gemm_f32.h (init / load_a / finish / epilogue); load_a is applied when
// the values are split, not when they are loaded.  An Op with kTileList may carry lists of the output tiles
// that are wanted (tile_list, tile_count, list_cap: in device memory); see the list form of the kernel.  An Op with
// kRowTileSkip may declare the rows of a tile somebody else's business (skip_row_tile).
//
// Tile order.  Workgroups go to the 8 XCDs round-robin by linear id (x fastest).  ROWS_PER_XCD = false: blockIdx.x
// = column tile, so an XCD keeps a fixed set of column tiles (its share of B stays in its L2) and every XCD
// streams all of A.  ROWS_PER_XCD = true, for an A that is large and a B that is re-read anyway (the second
// GEMM of the mixture denoiser: A = 1 GB of logits, 8 column tiles): all column tiles of a row tile run on one
// XCD, back to back, so a tile of A crosses the fabric once instead of once per XCD.
// One output tile (tile_m, tile_n) by the calling workgroup.
template <class Cfg, class Op>
__device__ __forceinline__ void split3_tile(int M, int M_max, int N, int K, const RowSrc& A,
                                            const uint8_t* __restrict__ Bimg, Op& op, float* __restrict__ part,
                                            int sparse, int tile_m, int tile_n) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, MI = Cfg::MI, NJ = Cfg::NJ, BK = Cfg::BK, NG = Cfg::NG, RB = Cfg::RB;
  constexpr int RA = Cfg::RA, RPP = Cfg::RPP, A_PLANE = Cfg::A_PLANE, B_PLANE = Cfg::B_PLANE;
  constexpr int A_STAGE = Cfg::A_STAGE, B_STAGE = Cfg::B_STAGE, B_LOADS = Cfg::B_LOADS, PLANES = Cfg::PLANES;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_all[];
  uint8_t* lds_a = lds_all;                                   // [2 stages][PLANES][BM rows][RB bytes]
  uint8_t* lds_b = lds_all + 2 * A_STAGE;                     // [2 stages][PLANES][BN rows][RB bytes]
  float* s_row = reinterpret_cast<float*>(lds_all + 2 * (A_STAGE + B_STAGE));   // [8 * BM], the Op's
  uint16_t* s_list = reinterpret_cast<uint16_t*>(s_row + 8 * BM);                // sparse K: [K / BK] live slabs, in order

  const int m0 = tile_m * BM, n0 = tile_n * BN;
  if (m0 >= M) return;
  if constexpr (Op::kRowTileSkip) {
    if (op.skip_row_tile(m0)) return;   // the same for the whole workgroup: someone else writes these rows
  }

  // (opaque to the optimiser: when this is called in a loop over tiles, everything derived from the thread index
  // below would otherwise be hoisted out of that loop and held in registers across it, which the K loop has none
  // to spare for)
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const Frag<Cfg> fr{wave / Cfg::WGN, wave % Cfg::WGN, lane & 31, lane >> 5, tile_n};
  const int splits = gridDim.z;                  // K split: this workgroup contracts slabs kb .. kb + nk - 1
  const int nk_all = K / BK, kb = blockIdx.z * (nk_all / splits);
  int nk = nk_all / splits;

  // ---- loaders.  A: thread = (row lrow + RPP p, chunk lkq of 8 k).  B: thread t copies bytes 16 t + 16 THREADS q
  // of a slab's image.  Slab j waits in register slot j & 1 and goes to LDS stage j & 1.
  const int lrow = tid / Cfg::KQ, lkq = tid % Cfg::KQ;
  const float* ap[RA];
  int a_dst[RA];
#pragma unroll
  for (int p = 0; p < RA; ++p) {
    const int r = lrow + RPP * p;
    ap[p] = A.row(min(m0 + r, M - 1)) + lkq * 8 + (int64_t)kb * BK;
    a_dst[p] = r * RB + Cfg::slot(r, lkq) * 16;
  }
  op.template init<Cfg>(m0, M, lrow, lkq, s_row);
  bool listed = false;   // the K loop walks s_list instead of slabs kb, kb + 1, ...
  if constexpr (Op::kSparseK) {
    if (sparse && splits == 1) {
      // flags of the Op's column groups (bytes, in the LDS of the list's tail), then the list itself
      const int ng = op.groups(), spg = op.group_cols() / BK;   // slabs per group (host: group_cols % BK == 0, K % group_cols == 0)
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
      nk = __builtin_amdgcn_readfirstlane(*s_cnt);   // the same for every lane: keep the K loop's control flow scalar
      // everything live: walk the slabs in order, without the list.  Nothing live -- rows of NaN, whose comparisons
      // all fail: the same, so that the loop's first loads never index with a list that was not written
      if (nk == 0) nk = nk_all;
      listed = nk < nk_all;
    }
  }
  if constexpr (Op::kSparseK) op.note_slabs(nk, nk_all / splits, tid);
  const uint8_t* bsrc = Bimg + ((int64_t)tile_n * nk_all + kb) * B_STAGE + tid * 16;
  // slab visited in step kt of the K loop, relative to kb (a list is only built when kb = 0)
  auto slab_of = [&](int kt) -> int64_t {
    if constexpr (Op::kSparseK) return listed ? (int64_t)__builtin_amdgcn_readfirstlane((int)s_list[kt]) : (int64_t)kt;
    return (int64_t)kt;
  };
  float4 ra[2][RA][2];
  u32x4 rb[2][B_LOADS];
  auto gload = [&](int kt, auto slot) {
    const int64_t sl = slab_of(kt);
#pragma unroll
    for (int p = 0; p < RA; ++p) {
      ra[slot][p][0] = *reinterpret_cast<const float4*>(ap[p] + sl * BK);
      ra[slot][p][1] = *reinterpret_cast<const float4*>(ap[p] + sl * BK + 4);
    }
#pragma unroll
    for (int q = 0; q < B_LOADS; ++q)
      rb[slot][q] = *reinterpret_cast<const u32x4*>(bsrc + sl * B_STAGE + q * 16 * Cfg::THREADS);
  };
  auto sstore = [&](auto slot) {   // register slot `slot` -> LDS stage `slot`
    uint8_t* sa = lds_a + slot * A_STAGE;
    uint8_t* sb = lds_b + slot * B_STAGE + tid * 16;
#pragma unroll
    for (int q = 0; q < B_LOADS; ++q) *reinterpret_cast<u32x4*>(sb + q * 16 * Cfg::THREADS) = rb[slot][q];
#pragma unroll
    for (int p = 0; p < RA; ++p) {
      const float4 v0 = op.load_a(ra[slot][p][0], p), v1 = op.load_a(ra[slot][p][1], p);
      const float x[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
      u32x4 pp[3];
      split_pack<PLANES>(x, pp);
#pragma unroll
      for (int pl = 0; pl < PLANES; ++pl) *reinterpret_cast<u32x4*>(sa + pl * A_PLANE + a_dst[p]) = pp[pl];
    }
  };

  v16f acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- fragments (tile and sub-tile offsets are multiples of 32 rows, so the swizzle key depends on l32 only)
  int f_off[NG];   // group g: chunk 2 g + half of this lane's rows
#pragma unroll
  for (int g = 0; g < NG; ++g) f_off[g] = fr.l32 * RB + Cfg::slot(fr.l32, 2 * g + fr.half) * 16;
  const uint8_t* fa = lds_a + fr.wm * Cfg::WM * RB;
  const uint8_t* fb = lds_b + fr.wn * Cfg::WN * RB;
  v8bf af[2][PLANES][MI], bf[2][PLANES][NJ];   // (fp16 terms travel in the same 16-byte type)
  auto read_frags = [&](auto stage, auto g, auto buf) {   // group g of LDS stage `stage` -> fragment buffer `buf`
#pragma unroll
    for (int pl = 0; pl < PLANES; ++pl) {
#pragma unroll
      for (int i = 0; i < MI; ++i)
        af[buf][pl][i] = *reinterpret_cast<const v8bf*>(fa + stage * A_STAGE + pl * A_PLANE + i * 32 * RB + f_off[g]);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        bf[buf][pl][j] = *reinterpret_cast<const v8bf*>(fb + stage * B_STAGE + pl * B_PLANE + j * 32 * RB + f_off[g]);
    }
  };
  constexpr int G = MI * NJ, NM = Cfg::NPROD * G;     // MFMAs per plane pair and per group
  auto mma = [&](auto buf, int first, int count) {   // MFMAs first .. first+count-1 of a group
    // pairs of terms, largest products first; with two terms the first three are all
    constexpr int pa[6] = {0, 0, 1, 1, 0, 2};
    constexpr int pb[6] = {0, 1, 0, 1, 2, 0};
#pragma unroll
    for (int q = 0; q < NM; ++q)
      if (q >= first && q < first + count) {
        const int pr = q / G, i = (q % G) / NJ, j = q % NJ;
        if constexpr (PLANES == 3)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][pa[pr]][i], bf[buf][pb[pr]][j], acc[i][j], 0, 0, 0);
        else
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, af[buf][pa[pr]][i]),
                                                             __builtin_bit_cast(v8h, bf[buf][pb[pr]][j]), acc[i][j], 0, 0, 0);
      }
  };
  // this wavefront's LDS stores have completed; then meet the others (no fence: global loads stay in flight)
  auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

  typedef std::integral_constant<int, 0> I0;
  typedef std::integral_constant<int, 1> I1;
  // ---- prologue: slab 0 into stage 0, slab 1 on its way into registers
  gload(0, I0());
  if (nk > 1) gload(1, I1());
  sstore(I0());
  lds_barrier();
  read_frags(I0(), I0(), I0());

  // One slab, par = kt & 1 (its LDS stage and register slot).  Fragment buffers: with one group per slab the
  // buffer of a slab is its parity; with two, group g sits in buffer g (buffer 0 is free again once group 0 has
  // issued, which is before the hand-over).  steady: slabs kt+1 and kt+2 exist -- no branches, so that the
  // interleaving below holds (a scheduling group does not cross a branch).
  auto slab = [&](int kt, auto par, auto npar, auto steady) {
    const bool l2 = steady || kt + 2 < nk, s1 = steady || kt + 1 < nk;
    typedef std::integral_constant<int, (NG == 1 ? decltype(par)::value : NG - 1)> LastBuf;   // buffer of the last group
    typedef std::integral_constant<int, (NG == 1 ? decltype(npar)::value : 0)> NextBuf;       // of group 0 of the next slab
    __builtin_amdgcn_s_setprio(2);
    if (l2) gload(kt + 2, par);     // slot par held slab kt, which went to LDS during slab kt-1
    if constexpr (NG == 2) {
      read_frags(par, I1(), I1());
      mma(I0(), 0, NM);
    }
    mma(LastBuf(), 0, NM / 2);
    if (s1) sstore(npar);           // stage npar: its last readers (slab kt-1) passed the barrier of slab kt-1
    if (steady && NG == 1) {
      // first half: a load behind each of the first MFMAs, then the copy and the split spread over the rest
      constexpr int NL = B_LOADS + 2 * RA, NV = NM / 2 - NL;
      sched_pairs<0x020, NL, 1>();
      sched_pairs<0x002, NV, (44 * RA + NV - 1) / NV>();
    }
    if (s1) {
      lds_barrier();
      read_frags(npar, I0(), NextBuf());
    }
    mma(LastBuf(), NM / 2, NM - NM / 2);
    if (steady && NG == 1) sched_pairs<0x100, NM - NM / 2, (PLANES * (MI + NJ) + NM - NM / 2 - 1) / (NM - NM / 2)>();
    __builtin_amdgcn_s_setprio(0);
  };
  typedef std::integral_constant<bool, true> Steady;
  typedef std::integral_constant<bool, false> Tail;
  int kt = 0;
  for (; kt + 3 < nk; kt += 2) {
    slab(kt, I0(), I1(), Steady());
    slab(kt + 1, I1(), I0(), Steady());
  }
  for (; kt < nk; kt += 2) {
    slab(kt, I0(), I1(), Tail());
    if (kt + 1 < nk) slab(kt + 1, I1(), I0(), Tail());
  }
  __syncthreads();   // every wavefront is done with the operand stages

  op.template finish<Cfg>(lrow, lkq, s_row);
  __syncthreads();
  if constexpr (Op::kSplitK) {
    if (splits > 1) {   // partial tile and row sums to scratch; the Op's owner finishes (as for gemm_f32.h)
      op.template store_partial<Cfg>(acc, fr, m0, n0, M, M_max, N, s_row, part, (int)blockIdx.z, splits);
      return;
    }
  }
  op.template epilogue<Cfg>(acc, fr, m0, n0, M, N, s_row);
}

// Grid: (column tiles, row tiles, K splits), one tile per workgroup.
template <class Cfg, class Op, int CALL, bool ROWS_PER_XCD>
__global__ __launch_bounds__(Cfg::THREADS, 2) void gemm_split3_nt_kernel(const int* __restrict__ M_dev, int M_max,
                                                                         int N, int K, RowSrc A,
                                                                         const uint8_t* __restrict__ Bimg, Op op,
                                                                         float* __restrict__ part, int sparse,
                                                                         const int32_t* __restrict__ run_if, int run_val) {
  // run_if (or NULL): the kernel runs only if *run_if == run_val -- a switch in device memory, so that one captured
  // graph can hold two forms of a GEMM and the device picks one
  if (run_if && *run_if != run_val) return;
  const int M = M_dev ? min(*M_dev, M_max) : M_max;
  int tile_n = blockIdx.x, tile_m = blockIdx.y;
  if (ROWS_PER_XCD) {
    // linear id = 8 ntn G + r: XCD r % 8 takes row tile 8 G + r % 8, column tile r / 8 (grid.y is a multiple of 8)
    const unsigned ntn = gridDim.x, lin = blockIdx.x + ntn * blockIdx.y;
    const unsigned G = lin / (8 * ntn), r = lin % (8 * ntn);
    tile_m = (int)(8 * G + r % 8);
    tile_n = (int)(r / 8);
  }
  split3_tile<Cfg, Op>(M, M_max, N, K, A, Bimg, op, part, sparse, tile_m, tile_n);
}

// The list form, for an Op with kTileList that carries lists of the wanted tiles: tile_list = 8 lists of list_cap
// entries, tile_count[q] = length of list q, and a ticket counter per list at tile_count[kTicketBase + kTicketStride *
// q], zero at launch (each on a cache line of its own: read-modify-write operations on one line are served one after
// the other, some 60 ns each).  Any number of workgroups (a multiple of 8) stay resident and draw tiles by ticket.
// The lists are by column tile modulo 8 and workgroup w starts on list w % 8 -- its XCD's, so an XCD keeps to its
// share of B, as in the grid order -- and moves on to the next list when one has run dry, so the launch ends evenly.
// Nothing is launched for the tiles that are not wanted, which matters when those are nearly all.
// An entry is  row tile * column tiles + column tile  of Cfg's tile grid; with kListHalf set it names only the upper
// (kListLower clear) or lower half of that tile's rows, which is then computed as a tile of CfgH (half the rows, the
// same columns, its own image of B): when the rows of a half have nothing in common with the other half's, one of
// them usually needs the tile and the other does not.
constexpr int kTicketBase = 32, kTicketStride = 32, kTicketInts = kTicketBase + 8 * kTicketStride;
constexpr uint32_t kListHalf = 1u << 31, kListLower = 1u << 30, kListIndex = kListLower - 1;
template <class Cfg, class CfgH, class Op, int CALL>
__global__ __launch_bounds__(Cfg::THREADS, 2) void gemm_split3_nt_list_kernel(const int* __restrict__ M_dev, int M_max,
                                                                              int N, int K, RowSrc A,
                                                                              const uint8_t* __restrict__ Bimg,
                                                                              const uint8_t* __restrict__ BimgH, Op op) {
  static_assert(CfgH::BM * 2 == Cfg::BM && CfgH::BN == Cfg::BN && CfgH::THREADS == Cfg::THREADS, "half tiles");
  constexpr size_t kLds = Cfg::LDS_BYTES > CfgH::LDS_BYTES ? Cfg::LDS_BYTES : CfgH::LDS_BYTES;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_all[];
  int* s_ticket = reinterpret_cast<int*>(lds_all + kLds);   // the launcher adds 16 bytes for it
  const int M = M_dev ? min(*M_dev, M_max) : M_max;
  const int ntn = (N + Cfg::BN - 1) / Cfg::BN;
  int lists_done = 0;   // thread 0: lists this workgroup has found dry
  auto draw = [&]() -> int {   // thread 0: the next tile (index into tile_list), or -1
    while (lists_done < 8) {
      const int q = (blockIdx.x + lists_done) % 8;
      const int count = min(op.tile_count[q], op.list_cap);
      int32_t* ticket = const_cast<int32_t*>(op.tile_count) + kTicketBase + kTicketStride * q;
      // a look before the draw: a dry list then costs a load, not a place in the line's queue
      if (__hip_atomic_load(ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < count) {
        const int i = atomicAdd(ticket, 1);
        if (i < count) return q * op.list_cap + i;
      }
      ++lists_done;
    }
    return -1;
  };
  if (threadIdx.x == 0) *s_ticket = draw();
  __syncthreads();
  for (;;) {
    const int cur = __builtin_amdgcn_readfirstlane(*s_ticket);
    if (cur < 0) break;
    __syncthreads();   // everyone has read the ticket
    // the next ticket is drawn now and published at the end of this tile: its latency hides under the tile
    int nxt = -1;
    if (threadIdx.x == 0) nxt = draw();
    const uint32_t e = (uint32_t)__builtin_amdgcn_readfirstlane((int)op.tile_list[cur]);
    const int tile_m = (int)((e & kListIndex) / (uint32_t)ntn), tile_n = (int)((e & kListIndex) % (uint32_t)ntn);
    if (e & kListHalf)
      split3_tile<CfgH, Op>(M, M_max, N, K, A, BimgH, op, nullptr, 0, 2 * tile_m + ((e & kListLower) ? 1 : 0), tile_n);
    else
      split3_tile<Cfg, Op>(M, M_max, N, K, A, Bimg, op, nullptr, 0, tile_m, tile_n);
    if (threadIdx.x == 0) *s_ticket = nxt;
    __syncthreads();   // the ticket is visible; the next tile reuses the stages and the Op's rows
  }
}

// Whether a launch with `sparse` set walks a slab list (else it stays dense): the list must fit beside the stages.
template <class Cfg>
inline bool split3_sparse_fits(int K, int groups, int group_cols) {
  if (group_cols <= 0 || group_cols % Cfg::BK != 0 || K % group_cols != 0 || K / Cfg::BK > 65535) return false;
  const size_t lds = Cfg::LDS_BYTES + (size_t)((2 * (K / Cfg::BK) + 15) & ~15) + (size_t)((groups + 15) & ~15) + 16;
  return lds <= 80 * 1024;   // two workgroups per CU
}

// splits > 1 (Ops with kSplitK, not with ROWS_PER_XCD): `part` = gemm_f32_splitk_floats(splits, M_max, N) floats.
// sparse: let an Op with kSparseK skip the slabs of K it marks dead (needs K / BK <= 65535, the Op's column groups a
// multiple of BK wide and K a multiple of them; otherwise the loop stays dense).
template <class Cfg, int CALL, bool ROWS_PER_XCD, class Op>
inline hipError_t launch_gemm_split3_nt(const int* M_dev, int M_max, int N, int K, RowSrc A, const uint8_t* Bimg,
                                        Op op, hipStream_t st, int splits = 1, float* part = nullptr, bool sparse = false,
                                        const int32_t* run_if = nullptr, int run_val = 0) {
  if (K % Cfg::BK != 0 || K <= 0 || splits < 1) return hipErrorInvalidValue;
  size_t lds = Cfg::LDS_BYTES;
  if constexpr (Op::kSparseK) {
    sparse = sparse && splits == 1 && split3_sparse_fits<Cfg>(K, op.groups(), op.group_cols());
    // list of slabs (2 bytes each), a flag byte per column group, the count
    if (sparse) lds += (size_t)((2 * (K / Cfg::BK) + 15) & ~15) + (size_t)((op.groups() + 15) & ~15) + 16;
  } else {
    sparse = false;
  }
  if (splits > 1 && (!Op::kSplitK || ROWS_PER_XCD || !part || (K / Cfg::BK) % splits != 0)) return hipErrorInvalidValue;
  unsigned mt = (unsigned)((M_max + Cfg::BM - 1) / Cfg::BM);
  if (ROWS_PER_XCD) mt = (mt + 7) / 8 * 8;
  dim3 grid((unsigned)((N + Cfg::BN - 1) / Cfg::BN), mt, (unsigned)splits);
  auto kern = gemm_split3_nt_kernel<Cfg, Op, CALL, ROWS_PER_XCD>;
  static bool attr_set = false;   // dynamic LDS above the default limit needs the attribute once per kernel
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(Cfg::THREADS), lds, st, M_dev, M_max, N, K, A, Bimg, op, part, sparse ? 1 : 0, run_if,
                     run_val);
  return hipGetLastError();
}

// The list form: `wgs` resident workgroups (a multiple of 8), the Op carries the lists.  BimgH: B's image for CfgH, or
// NULL if no entry of the lists names a half tile.
template <class Cfg, class CfgH, int CALL, class Op>
inline hipError_t launch_gemm_split3_nt_list(const int* M_dev, int M_max, int N, int K, RowSrc A, const uint8_t* Bimg,
                                             const uint8_t* BimgH, Op op, int wgs, hipStream_t st) {
  static_assert(Op::kTileList && !Op::kSparseK, "an Op with tile lists and a dense K loop");
  if (K <= 0 || K % Cfg::BK != 0 || K % CfgH::BK != 0 || wgs <= 0 || wgs % 8 != 0) return hipErrorInvalidValue;
  auto kern = gemm_split3_nt_list_kernel<Cfg, CfgH, Op, CALL>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const size_t lds = (Cfg::LDS_BYTES > CfgH::LDS_BYTES ? Cfg::LDS_BYTES : CfgH::LDS_BYTES) + 16;
  static_assert((Cfg::LDS_BYTES > CfgH::LDS_BYTES ? Cfg::LDS_BYTES : CfgH::LDS_BYTES) + 16 <= 80 * 1024, "two workgroups per CU");
  hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(Cfg::THREADS), lds, st, M_dev, M_max, N, K, A, Bimg, BimgH, op);
  return hipGetLastError();
}

}  // namespace asd
