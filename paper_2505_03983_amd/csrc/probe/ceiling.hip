// What the matrix pipe of the chip at hand sustains: a register-only MFMA loop (no memory traffic at
// all), timed over a stated duration, with operands that are either random (zero-mean, like real
// data) or constant.  The two differ by almost 2x on this chip: the dense rate with random operands
// is set by the power limit, not by the issue rate, so it -- not the data-sheet peak -- is the
// ceiling a real GEMM can approach.  A measurement probe for the benchmark harness, built into a
// library of its own (libasd_probe.so); the sampling library neither contains nor calls it.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include <new>

#include "../../../include/asd_probe.h"

namespace asd_probe {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));      // A / B operand of v_mfma_f32_32x32x16_bf16
typedef _Float16 v8h __attribute__((ext_vector_type(8)));     // A / B operand of v_mfma_f32_32x32x16_f16

static thread_local char g_err[256] = "";
static void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

typedef uint32_t cu32x4 __attribute__((ext_vector_type(4)));
typedef float cv16f __attribute__((ext_vector_type(16)));

// 24 MFMAs per iteration on four accumulators, six A and six B fragments in rotation.  HALF: fp16 operands, else bf16.
template <bool HALF>
__device__ __forceinline__ cv16f mfma16(cu32x4 a, cu32x4 b, cv16f c) {
  if constexpr (HALF) return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
  else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}
template <bool HALF>
__global__ __launch_bounds__(256, 2) void ceiling_16bit_kernel(float* __restrict__ out, const cu32x4* __restrict__ in,
                                                               int iters) {
  cv16f acc[4];
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  cu32x4 a[6], b[6];
  for (int i = 0; i < 6; ++i) {
    a[i] = in[(threadIdx.x + 256 * i) & 4095];
    b[i] = in[(threadIdx.x + 256 * i + 2048) & 4095];
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 6; ++u) {
      acc[0] = mfma16<HALF>(a[u], b[(u + 1) % 6], acc[0]);
      acc[1] = mfma16<HALF>(a[u], b[(u + 2) % 6], acc[1]);
      acc[2] = mfma16<HALF>(a[(u + 3) % 6], b[u], acc[2]);
      acc[3] = mfma16<HALF>(a[(u + 4) % 6], b[u], acc[3]);
    }
  }
  float s = 0.f;
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256, 2) void ceiling_f32_kernel(float* __restrict__ out, const cu32x4* __restrict__ in,
                                                             int iters) {
  cv16f acc[4];
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  float a[6], b[6];
  for (int i = 0; i < 6; ++i) {
    // a bf16 pair read as one fp32: random sign, exponent near 1, random 23-bit significand
    a[i] = __uint_as_float(in[(threadIdx.x + 256 * i) & 4095].x);
    b[i] = __uint_as_float(in[(threadIdx.x + 256 * i + 2048) & 4095].y);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 6; ++u) {
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[(u + 1) % 6], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[(u + 2) % 6], acc[1], 0, 0, 0);
      acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[(u + 3) % 6], b[u], acc[2], 0, 0, 0);
      acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[(u + 4) % 6], b[u], acc[3], 0, 0, 0);
    }
  }
  float s = 0.f;
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace asd_probe

using namespace asd_probe;

extern "C" const char* asd_probe_last_error(void) { return g_err; }

extern "C" int32_t asd_probe_mfma_ceiling(int32_t dtype, int32_t random_data, int32_t ms_target, double* tflops) {
  if (!tflops || ms_target < 1 || ms_target > 5000 || dtype < 0 || dtype > 2) {
    set_error("asd_probe_mfma_ceiling: tflops is NULL, ms_target outside [1, 5000] or dtype not 0 (fp32), 1 (bf16), 2 (fp16)");
    return -1;
  }
  const bool bf16 = dtype != 0, half = dtype == 2;   // (bf16: a 16-bit operand type)
  constexpr int kWgs = 512, kWords = 4096 * 4, kBatch = 8;
  float* out = nullptr;
  cu32x4* in = nullptr;
  uint32_t* h = new (std::nothrow) uint32_t[kWords];
  if (!h) return -3;
  uint64_t s = 0x9E3779B97F4A7C15ull;   // splitmix64
  auto next = [&]() {
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return (uint32_t)((z ^ (z >> 31)) >> 16);
  };
  for (int i = 0; i < kWords; ++i) {
    uint32_t w = 0;
    for (int hlf = 0; hlf < 2; ++hlf) {
      const uint32_t r = next();
      // |value| in [0.25, 4): bf16 = 1 + 8 + 7 bits, fp16 = 1 + 5 + 10
      const uint32_t sign = r & 1u, e = (half ? 13u : 125u) + ((r >> 1) & 3u), m = (r >> 3) & (half ? 1023u : 127u);
      const uint32_t one = half ? 0x3c00u : 0x3f80u;
      w |= (random_data ? ((sign << 15) | (e << (half ? 10 : 7)) | m) : one) << (16 * hlf);
    }
    h[i] = w;
  }
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&]() {
    delete[] h;
    (void)hipFree(out);
    (void)hipFree(in);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
#define CEIL_HIP(x)                                                            \
  do {                                                                         \
    hipError_t e__ = (x);                                                      \
    if (e__ != hipSuccess) {                                                   \
      set_error("%s failed: %s", #x, hipGetErrorString(e__));                  \
      cleanup();                                                               \
      return -3;                                                      \
    }                                                                          \
  } while (0)
  CEIL_HIP(hipMalloc(&out, sizeof(float) * kWgs * 256));
  CEIL_HIP(hipMalloc(&in, sizeof(uint32_t) * kWords));
  CEIL_HIP(hipMemcpy(in, h, sizeof(uint32_t) * kWords, hipMemcpyHostToDevice));
  CEIL_HIP(hipEventCreate(&e0));
  CEIL_HIP(hipEventCreate(&e1));
  // launches of ~5 ms each (at the data-sheet rate); the rate of the second half of the run is reported
  const int iters = bf16 ? 4000 : 250;
  const double flop_per_launch = (double)kWgs * 4 * iters * 24 * (32.0 * 32 * (bf16 ? 16 : 2) * 2);
  double total_ms = 0.0, last = 0.0;
  int launches_timed = 0;
  for (int phase = 0; phase < 2; ++phase) {
    double phase_ms = 0.0;
    int n = 0;
    while (phase_ms < 0.5 * ms_target) {
      CEIL_HIP(hipEventRecord(e0, 0));
      for (int l = 0; l < kBatch; ++l) {   // back to back: host round trips between launches let the chip recover
        if (half) hipLaunchKernelGGL(ceiling_16bit_kernel<true>, dim3(kWgs), dim3(256), 0, 0, out, in, iters);
        else if (bf16) hipLaunchKernelGGL(ceiling_16bit_kernel<false>, dim3(kWgs), dim3(256), 0, 0, out, in, iters);
        else hipLaunchKernelGGL(ceiling_f32_kernel, dim3(kWgs), dim3(256), 0, 0, out, in, iters);
      }
      CEIL_HIP(hipGetLastError());
      CEIL_HIP(hipEventRecord(e1, 0));
      CEIL_HIP(hipEventSynchronize(e1));
      float ms = 0.f;
      CEIL_HIP(hipEventElapsedTime(&ms, e0, e1));
      phase_ms += ms;
      n += kBatch;
    }
    total_ms += phase_ms;
    last = phase_ms;
    launches_timed = n;
  }
#undef CEIL_HIP
  (void)total_ms;
  *tflops = flop_per_launch * launches_timed / (last * 1e-3) / 1e12;
  cleanup();
  return 0;
}
