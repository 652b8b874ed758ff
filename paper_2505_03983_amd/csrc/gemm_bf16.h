// Shared pieces of the bf16 x bf16 -> fp32 GEMM on the gfx950 matrix cores (the kernel itself is in
// gemm_bf16_pipe.h): the MFMA operand / accumulator vector types and the fp32 -> bf16 rounding.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace asd {

typedef float v16f_b __attribute__((ext_vector_type(16)));   // accumulator of v_mfma_f32_32x32x16_bf16
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));      // its A / B operand: 8 consecutive k of a row

// round to nearest even (finite inputs)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

}  // namespace asd
