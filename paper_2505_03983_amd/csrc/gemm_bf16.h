// Shared pieces of the bf16 x bf16 -> fp32 GEMMs on the gfx950 matrix cores (the kernels are in
// gemm_bf16_pipe.h and gemm_split3.h): the MFMA operand / accumulator vector types, the fp32 -> bf16
// rounding, and the pointer types and wait of the direct-to-LDS loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace asd {

typedef float v16f_b __attribute__((ext_vector_type(16)));   // accumulator of v_mfma_f32_32x32x16_bf16
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));      // its A / B operand: 8 consecutive k of a row
typedef int v16i_b __attribute__((ext_vector_type(16)));      // accumulator of v_mfma_i32_32x32x32_i8
typedef int v4i_b __attribute__((ext_vector_type(4)));        // its A / B operand: 16 consecutive k of a row, one byte each

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Scheduling hints for an MFMA loop.
// `pairs` times {one MFMA, then `per` instructions of class `mask`}
template <int MASK, int PAIRS, int PER>
__device__ __forceinline__ void sched_pairs() {
  if constexpr (PAIRS > 0) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(MASK, PER, 0);
    sched_pairs<MASK, PAIRS - 1, PER>();
  }
}
template <int COUNT>
__device__ __forceinline__ void sched_mfma() {
  if constexpr (COUNT > 0) __builtin_amdgcn_sched_group_barrier(0x008, COUNT, 0);
}

// round to nearest even (finite inputs)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

}  // namespace asd
