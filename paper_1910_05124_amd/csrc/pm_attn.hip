// MFMA attention core: kernels and their launchers (see pm_attn_api.hpp for why this is a separate
// translation unit).
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>

#include "pm_attn_mfma.hpp"

void pm_attn_mfma_fwd(hipStream_t st, int B, int S, int H, const bf16_t* q, const bf16_t* k, const bf16_t* v,
                             bf16_t* o, float* lse) {
  const int qblocks = (S + 127) / 128;
  hipLaunchKernelGGL(pm_attn_mfma_fwd_kernel, dim3(B * H * qblocks), dim3(256), 0, st, q, k, v, o, lse, S, H, B * H, 0.125f);
}
void pm_attn_mfma_bwd(hipStream_t st, int B, int S, int H, const bf16_t* q, const bf16_t* k, const bf16_t* v,
                             const bf16_t* o, const bf16_t* dO, const float* lse, bf16_t* dq, bf16_t* dk, bf16_t* dv) {
  const int qblocks = (S + 127) / 128;
  hipLaunchKernelGGL(pm_attn_mfma_dq_kernel, dim3(B * H * qblocks), dim3(256), 0, st, q, k, v, o, dO, lse, dq, S, H, B * H,
                     0.125f);
  hipLaunchKernelGGL(pm_attn_mfma_dkv_kernel, dim3(B * H * qblocks), dim3(256), 0, st, q, k, v, o, dO, lse, dk, dv, S, H,
                     B * H, 0.125f);
}
