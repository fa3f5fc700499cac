// Entry points of the MFMA attention core (kernels in pm_attn.hip, a translation unit of its own: it is
// compiled with accumulators of the matrix instructions kept in ordinary vector registers, which suits
// these kernels (the softmax arithmetic works on the accumulators between two products) and not the
// 256 x 256-tile GEMM, whose accumulators fill the second register file).
#pragma once
#include <hip/hip_runtime.h>

#include "pm_common.hpp"

inline bool pm_attn_mfma_fits(int S, int dh) { return dh == 64 && S >= 32 && (S % 32) == 0; }

// q, k, v, o, dO, dq, dk, dv: [B * S, H * 64] bf16, row b * S + s; lse: [B, H, S] fp32 (natural-log units)
void pm_attn_mfma_fwd(hipStream_t st, int B, int S, int H, const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* o,
                      float* lse);
void pm_attn_mfma_bwd(hipStream_t st, int B, int S, int H, const bf16_t* q, const bf16_t* k, const bf16_t* v,
                      const bf16_t* o, const bf16_t* dO, const float* lse, bf16_t* dq, bf16_t* dk, bf16_t* dv);
