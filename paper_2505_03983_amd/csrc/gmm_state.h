// State of the Gaussian-mixture denoiser (owned by gmm.hip; read by the chain-resident sampler).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace asd {

struct GmmState {
  int C = 0;
  float var = 0.f;
  const float* means = nullptr;  // caller's [C, d]
  const float* log_w = nullptr;  // caller's [C]
  float* means_t = nullptr;      // [d, C]
  float* musq = nullptr;         // [C]
  float4* coef_tau = nullptr;    // [n_tau]: (kappa, gamma, cx, cm)
  float* logits = nullptr;       // [rows_max, C] (matrix-core path only)
  float* pmax = nullptr;         // [rows_max, np] partial row maxima of the logits
  int np = 0;
  float* rmax = nullptr;         // [rows_max] row maxima of the verify call's logits (split-operand path)
  uint8_t* glive = nullptr;      // [row tiles][np] column groups that are live for a row of the tile
  int32_t* onehot = nullptr;     // [rows_max] the one component with a non-zero weight, or -1
  uint8_t* onehot_tile = nullptr;  // [row tiles] every row of the tile is one-hot: written in closed form, no GEMM
  float* part = nullptr;         // split-K scratch of the draft call's second GEMM: [splits][chains][d] tiles, [splits][chains] sums
  int draft_splits = 1;
  bool use_mfma = false;
  // split-bf16 verify GEMMs (gemm_split3.h): the means, split and laid out as LDS images, for both GEMMs
  uint8_t* means_img = nullptr;    // B of the logits GEMM  ([C, d])
  uint8_t* means_t_img = nullptr;  // B of the combine GEMM ([d, C])
  uint8_t* means_img_s = nullptr;  // the same two for the draft call's tiling (K slabs of 32)
  uint8_t* means_t_img_s = nullptr;
  // Both GEMMs on two fp16 terms per operand (d and C multiples of 32; then the images above do not exist): the means
  // times b_scale as one image per GEMM for both tilings, the scale of every row of a call's first GEMM, and the
  // means as two fp16 terms carry them (what the closed form of a one-hot row must use)
  uint8_t* means_img2 = nullptr;
  uint8_t* means_t_img2 = nullptr;
  float b_scale = 1.f;
  float* a_scale = nullptr;        // [rows_max]
  float* means22 = nullptr;        // [C, d]
  bool two_ok = false;
  // ... and for verify calls of many rows the same two images for 256 x 256 tiles (gemm_split2_big.h): launches in
  // which every tile is wanted take those
  uint8_t* means_img_big = nullptr;
  uint8_t* means_t_img_big = nullptr;
  bool big_ok = false;
  bool big_on = true;              // the switch (asd_use_tall_tiles)
  bool split_draft_ok = false;     // d and C are multiples of 32: the draft call can take the split kernels too
  bool split_ok = false;           // the shape allows them
  bool use_split = false;          // ... and they are switched on (asd_use_split_gemm)
  // DEV [8], summed over the verify calls while profiling: tiles of logits computed / there were (calls that went
  // through the screening launches), K slabs the second GEMM's workgroups visited / there were, tiles of the calls
  // that were screened, row tiles of the second GEMM written in closed form (one-hot rows), row tiles that the
  // certificate below proved one-hot before any matrix work
  unsigned long long* work_counts = nullptr;
  bool sparse_combine = true;      // the second split GEMM of the verify call skips slabs of exact zeros (gemm_split3.h)
  // Screening of the verify call's logits GEMM (gmm.hip): an int8 GEMM finds the tiles whose softmax weights are
  // all exactly zero; the exact GEMM skips them.
  bool screen_ok = false;          // the shape allows it (and the buffers below exist)
  int screen_mode = 1;             // 0: off, 1: when the draft call of the round found its posteriors collapsed, 2: always
  int8_t* means_q = nullptr;       // [C, d] quantised means, one scale per group of components
  float4* means_grp = nullptr;     // [2 nps] per group: scale, largest 1-norm, range of |mu|^2; range of log2 w
  int8_t* xq = nullptr;            // [rows_max, d] the call's rows, quantised
  float2* xs = nullptr;            // [rows_max]: scale, 1-norm
  int32_t* imax = nullptr;         // [rows_max, nps] largest integer sum per row and group
  int nps = 0;                     // groups of components
  uint32_t* tile_list = nullptr;   // [8][list_cap] tiles of logits to compute, by column tile modulo 8
  int32_t* tile_count = nullptr;   // the lists' lengths and the tickets drawn from each (layout: gemm_split3.h)
  int list_cap = 0;
  int32_t* screen_on = nullptr;    // DEV [4]: the draft call's verdict for this round; the constant 1; two accumulators
  // One-hot certificate (gmm.hip): rows proven one-hot from the distance of a mean to its nearest neighbour and the
  // component the chain's last draft-call row sat on, written in closed form at once; row tiles of such rows skip the
  // rest of the call.
  bool cert_ok = false;            // the shape allows it (and the buffers below exist)
  bool cert_on = true;             // the switch (asd_use_onehot_certificate)
  float* cert_amin = nullptr;      // [C]: lower bounds of the distance from mu_b to the nearest other mean
  float4 cert_glob = {0.f, 0.f, 0.f, 0.f};   // largest |mu_n|, largest and smallest musq
  float4 cert_globw = {0.f, 0.f, 0.f, 0.f};  // largest log2 w_n, largest |log2 w_n|
  int32_t* chain_comp = nullptr;   // [chains]: component of the chain's last one-hot draft-call row, or -1
  uint8_t* cert_tile = nullptr;    // [row tiles]: 1 = certified in this call
  int32_t* cert_cnt = nullptr;     // [row tiles]: rows of the tile that have finished / passed (zero between calls)
  int32_t* live_tiles = nullptr;   // [1 + row tiles]: number of row tiles that are not certified, then their indices
  size_t rowwise_lds = 0;
  size_t lds_rowwise_bytes = 0;  // > 0: the mixture fits in LDS and d % 4 == 0 (gmm_rowwise_lds_kernel)
};

}  // namespace asd
