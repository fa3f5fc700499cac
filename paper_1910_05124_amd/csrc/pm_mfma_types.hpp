// Operand and accumulator vector types of the bf16 matrix instructions (v_mfma_f32_32x32x16_bf16) and of
// the LDS transpose load, shared by the GEMM, convolution and attention kernels.
#pragma once
#include <cstdint>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 pm_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float pm_f32x16;
typedef short pm_v4s __attribute__((ext_vector_type(4)));

__device__ __forceinline__ pm_bf16x8 pm_at_zero8() {
  union { pm_bf16x8 v; uint32_t w[4]; } u;
  u.w[0] = u.w[1] = u.w[2] = u.w[3] = 0u;
  return u.v;
}
