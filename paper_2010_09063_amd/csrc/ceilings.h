// Measured reference points for the roofline figures: what a plain copy, a register-only fp32 MFMA loop and an
// empty launch reach on the GPU the library runs on.  Not part of the step.
#pragma once
#include <hip/hip_runtime.h>

typedef float ceil_f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void ceiling_copy_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst, long n) {
  const long stride = (long)gridDim.x * blockDim.x;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// four independent 32x32 accumulator tiles per wave, operands in registers: nothing but v_mfma_f32_32x32x2_f32
__global__ __launch_bounds__(256) void ceiling_mfma_kernel(float *__restrict__ out, int iters, float a, float b) {
  ceil_f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  const float av = a + threadIdx.x, bv = b;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[(long)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ void ceiling_empty_kernel() {}
