// The arithmetic of the one-hot certificate of the mixture denoiser, for the two kernels that apply it: the model
// call's own (gmm_certify_kernel: every row of a call) and the accept kernel's (rows it is about to examine, whose
// model values it then forms itself).  The derivation is at gmm_certify_kernel.
#pragma once
#include <hip/hip_runtime.h>

namespace asd {

constexpr float kCertLog2e = 1.4426950408889634f;   // the logits' unit (LogitOp::kLog2e)
// Softmax weights more than this many base-2 units below their row's largest are taken as exactly zero, in every
// kernel of the mixture denoiser: a row's result moves by less than 2 C 2^-40 max |mu| for it (C <= 4096: 2^-27, a
// tenth of what fp32 rounding does to it), and everything that can be shown to lie that far down -- most of both
// GEMMs once a posterior has begun to narrow -- need not be computed at all.
constexpr float kCertZeroGap = 40.0f;               // = CombineOp::kZeroGap

// What a kernel outside the denoiser needs to certify rows and to write their model values in closed form.
struct OneHotCert {
  const int32_t* chain_comp = nullptr;   // [chains]: candidate component of a chain, or negative (NULL: not available)
  const float* means = nullptr;          // [C][d]: the means as the second GEMM carries them
  const float* musq = nullptr;           // [C]
  const float* log_w = nullptr;          // [C]
  const float* a_min = nullptr;          // [C]: distance to the nearest other mean (a lower bound)
  const float4* coef_tau = nullptr;      // [n_tau]: kappa, gamma, c_x', c_m' of a time index
  float4 glob, globw;                    // max |mu|, max and min |mu|^2; max log2 w, max |log2 w|
  int C = 0;
};

// A look before a row is read.  Under the mixture a row at this time index has s = 2 gamma / kappa and
// |e|^2 = d / (kappa / s) to within a few percent (the noise of d coordinates); if the test would fail even with
// four fifths of that |e| and nothing of its smaller terms, the row is not worth its 4 d bytes.  (Only a guess that
// saves work: a row it turns away takes the exact path.)
__device__ __forceinline__ bool cert_worth_reading(float4 cf, float am, int d) {
  if (cf.x > 0.f && cf.y > 0.f) {
    const float s0 = 2.f * cf.y / cf.x, e0 = 0.8f * sqrtf((float)d * s0 / cf.x);
    const float A0 = kCertLog2e * cf.x * s0, B0 = kCertLog2e * cf.x * e0;
    if (!(am * A0 >= B0 && am * (B0 - 0.5f * A0 * am) + kCertZeroGap < 0.f)) return false;
  }
  return true;
}

// The test proper.  s: the factor in e = x - s mu_b (any value is valid); r2 = |e|^2 and xx = |x|^2 as fp32 sums;
// am = a_min[b], qb = |mu_b|^2 (musq), bias_b = log2 w_b.
__device__ __forceinline__ bool cert_passes(float4 cf, float s, float r2, float xx, float am, float qb, float bias_b,
                                            float4 glob, float4 globw) {
  // upper bounds of the two norms (their fp32 sums are off by a few 2^-24 d of themselves at most); `means` holds
  // the means as the second GEMM carries them, within 2^-21 max |mu| of the true ones in norm, and |e| is about
  // the true mu_b
  const float e_up = fmaf(fabsf(s) * glob.x, 0x1p-21f, sqrtf(r2) * (1.f + 0x1p-10f)), x_up = sqrtf(xx) * (1.f + 0x1p-10f);
  const float c1 = kCertLog2e * cf.x, c2 = kCertLog2e * cf.y;
  const float A = c1 * s, B = c1 * e_up, half = 0.5f * A;
  const float f = am * (B - half * am);                 // the parabola at the nearest neighbour ...
  const bool beyond = am * A >= B;                      // ... which must lie beyond its vertex
  const float dq = half - c2;
  const float qterm = dq * ((dq >= 0.f ? glob.y : glob.z) - qb);
  const float bterm = globw.x - bias_b;
  const float mag = (am * B + half * am * am) + fabsf(qterm) + (globw.y + fabsf(bias_b)) + c2 * glob.y;
  const float margin = fmaf(c1 * x_up * glob.x, 0x1p-9f + 1e-5f,
                            fmaf((c2 + fabsf(dq)) * glob.y, 0x1p-12f, fmaf(1e-5f, mag, 1.f)));
  // (a NaN or an infinity anywhere above fails these comparisons)
  return s >= 0.f && c1 >= 0.f && c2 >= 0.f && beyond && mag < 1e30f && margin < 1e30f &&
         (f + qterm + bterm) + (kCertZeroGap + margin) < 0.f;
}

// A certified row's model value: what the second GEMM's epilogue computes with acc = mu_b (+0.0: the accumulator
// never holds a negative zero) and scale = c_m' / 1.0.
__device__ __forceinline__ float4 cert_value(float4 cf, float4 x, float4 mu) {
  return make_float4(fmaf(cf.z, x.x, __fmul_rn(cf.w, mu.x + 0.f)), fmaf(cf.z, x.y, __fmul_rn(cf.w, mu.y + 0.f)),
                     fmaf(cf.z, x.z, __fmul_rn(cf.w, mu.z + 0.f)), fmaf(cf.z, x.w, __fmul_rn(cf.w, mu.w + 0.f)));
}

}  // namespace asd
