// Small device-side helpers shared by the round kernels and the chain-resident sampler.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace asd {

// ----------------------------------------------------------------------------
// helpers: a row of d floats is handled in blocks of four coordinates, one
// Philox call per block.  d need not be a multiple of four.
// ----------------------------------------------------------------------------
__device__ __forceinline__ float4 load4(const float* p, int blk, int d, bool vec) {
  if (vec) return reinterpret_cast<const float4*>(p)[blk];
  float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
  const int j = blk * 4;
  if (j + 0 < d) r.x = p[j + 0];
  if (j + 1 < d) r.y = p[j + 1];
  if (j + 2 < d) r.z = p[j + 2];
  if (j + 3 < d) r.w = p[j + 3];
  return r;
}

__device__ __forceinline__ void store4(float* p, int blk, int d, bool vec, float4 v) {
  if (vec) {
    reinterpret_cast<float4*>(p)[blk] = v;
    return;
  }
  const int j = blk * 4;
  if (j + 0 < d) p[j + 0] = v.x;
  if (j + 1 < d) p[j + 1] = v.y;
  if (j + 2 < d) p[j + 2] = v.z;
  if (j + 3 < d) p[j + 3] = v.w;
}

// Sum over the 64 lanes of a wavefront, returned in every lane.  Four DPP steps reduce each row of
// 16 lanes (swap inside pairs, swap pairs, mirror the half row, mirror the row); the four row totals
// are then read out as scalars.  (A butterfly of ds_bpermute-based shuffles costs an LDS round trip
// per step.)
__device__ __forceinline__ float wave_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, true));   // quad_perm [2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, true));  // row_half_mirror
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, true));  // row_mirror
  const int b = __float_as_int(v);
  return (__int_as_float(__builtin_amdgcn_readlane(b, 0)) + __int_as_float(__builtin_amdgcn_readlane(b, 16))) +
         (__int_as_float(__builtin_amdgcn_readlane(b, 32)) + __int_as_float(__builtin_amdgcn_readlane(b, 48)));
}

// Maximum over the 64 lanes of a wavefront, returned in every lane (same data movement as wave_sum).
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, true)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, true)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, true)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, true)));
  const int b = __float_as_int(v);
  return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 0)), __int_as_float(__builtin_amdgcn_readlane(b, 16))),
               fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 32)), __int_as_float(__builtin_amdgcn_readlane(b, 48))));
}

// ----------------------------------------------------------------------------
// Window controller (an extension: Alg. 1 takes the speculation length as a fixed input).  The next
// window may depend on the chain's past only, which leaves every step's law intact.  It follows a
// running mean of the accepted run length in integers: state <- state - state/4 + obs, obs = n_acc, or
// 2 w when the whole window of w was accepted (the run was cut by the window); the window asked for is
// 3/4 of that mean (state / 4), within [min(4, L), L].  win[c] = window, win[B + c] = state.
// ----------------------------------------------------------------------------
__device__ __forceinline__ int window_of(int state, int L) { return max(min(4, L), min(L, (3 * state) >> 4)); }
__device__ __forceinline__ int window_next(int state, int w_used, int n_acc) {
  return state - (state >> 2) + (n_acc == w_used ? 2 * w_used : n_acc);
}

}  // namespace asd
