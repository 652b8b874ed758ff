// State of the Gaussian-mixture denoiser (owned by gmm.hip; read by the chain-resident sampler).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

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
  bool use_mfma = false;
  size_t rowwise_lds = 0;
  size_t lds_rowwise_bytes = 0;  // > 0: the mixture fits in LDS and d % 4 == 0 (gmm_rowwise_lds_kernel)
};

}  // namespace asd
