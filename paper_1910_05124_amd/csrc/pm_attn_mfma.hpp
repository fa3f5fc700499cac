// Causal attention core on bf16 MFMA (v_mfma_f32_32x32x16_bf16), head size 64, gfx950.
//
// The attention core carries no weights (so no stale / corrected weight enters it); it is on the
// path of the fine-grained Transformer stages because q, k, v come from three weight units and o
// feeds a fourth.  q, k, v, o and their gradients are [tokens, H * 64] bf16, row t = b * S + s.
//
// One scheme serves the forward and both backward kernels.  A wave owns 32 rows of one index
// (queries in the forward and the dQ kernel, keys in the dK/dV kernel) and streams 32-row tiles of
// the other index through LDS.  Every score-like product is computed TRANSPOSED, streamed index on
// the MFMA rows and owned index on the MFMA columns: the 32 x 32 fp32 result then has the owned row
// in the lane (column l % 32) and 16 streamed entries per lane in registers, so
//   * row statistics of the owned index (running max / sum, log-sum-exp, D) are per-lane scalars,
//   * the result, rounded to bf16, IS the B operand (k = streamed index, column = owned index) of
//     the second product, whose A operand is a transposed tile of the streamed matrix read with the
//     LDS transpose load.  No cross-lane movement of probabilities.
// For the in-lane hand-over the streamed tile's rows are permuted on the way into the first MFMA:
// MFMA row m holds streamed row perm(m) (bits 2 and 3 of m swapped), which makes accumulator value
// v of lane group g = l / 32 the streamed row 16 (v / 8) + 8 g + v % 8, i.e. values 8 s .. 8 s + 7 are
// exactly the k-slots of lane group g in k-step s of the second MFMA.
//
// Probabilities are recomputed in the backward from q, k and the stored log-sum-exp of the scaled
// scores; D_i = sum_c dO[i, c] O[i, c].  Two backward kernels (dQ; dK and dV) so that every output
// has one owner and no atomics are needed.
#pragma once
#include "pm_attn_api.hpp"
#include "pm_common.hpp"
#include "pm_mfma_types.hpp"

constexpr int PM_AT_ST = 72;          // LDS row stride (elements) of a [32][64] tile: 144 B, 16-byte aligned rows

__device__ __forceinline__ int pm_at_perm(int m) { return (m & 0x13) | ((m & 4) << 1) | ((m & 8) >> 1); }

// A fragment, contraction index contiguous: tile row `row`, contraction indices kb + 8 * (lane / 32) .. + 7
__device__ __forceinline__ pm_bf16x8 pm_at_frag(const bf16_t* s, int row, int kb, int lane) {
  return *reinterpret_cast<const pm_bf16x8*>(s + row * PM_AT_ST + kb + (lane >> 5) * 8);
}
// A fragment of the transposed tile: MFMA row = tile column r32 + lane % 32, contraction = tile rows
// kb + 8 * (lane / 32) .. + 7 (LDS transpose load; lane mapping as in the GEMM's row-contiguous operands)
__device__ __forceinline__ pm_bf16x8 pm_at_frag_tr(const bf16_t* s, int r32, int kb, int lane) {
  const int g = lane >> 4, q = lane & 15;
  const bf16_t* p = s + (kb + 8 * (g >> 1) + (q >> 2)) * PM_AT_ST + r32 + 16 * (g & 1) + 4 * (q & 3);
  typedef pm_v4s __attribute__((address_space(3))) * lds_v4s;
  const pm_v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
  const pm_v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 4 * PM_AT_ST));
  union { pm_bf16x8 v; pm_v4s h[2]; } u;
  u.h[0] = lo;
  u.h[1] = hi;
  return u.v;
}
__device__ __forceinline__ pm_bf16x8 pm_at_pack8(const float* x) {
  union { pm_bf16x8 v; uint32_t w[4]; } u;
#pragma unroll
  for (int e = 0; e < 4; ++e) u.w[e] = pm_pack_bf16(x[2 * e], x[2 * e + 1]);
  return u.v;
}
// result tile [64 x 32] held as two accumulators (MFMA rows = head dimension, column = owned row):
// store transposed into out[row0 + lane % 32][0..63] (bf16), 4 consecutive head-dimension entries at a time
__device__ __forceinline__ void pm_at_store_t(bf16_t* out_row, const pm_f32x16* acc, float mul, int lane) {
  const int g = lane >> 5;
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      uint2 w;
      w.x = pm_pack_bf16(acc[dt][4 * a] * mul, acc[dt][4 * a + 1] * mul);
      w.y = pm_pack_bf16(acc[dt][4 * a + 2] * mul, acc[dt][4 * a + 3] * mul);
      *reinterpret_cast<uint2*>(out_row + dt * 32 + 8 * a + 4 * g) = w;
    }
}

// ---------------------------------------------------------------------------------------------
// forward: block = 4 waves x 32 queries of one (sequence, head); key / value tiles of 32 rows
// double-buffered in LDS (one barrier per tile).
// ---------------------------------------------------------------------------------------------
// (register budget of four waves per SIMD: two values spill, and the fourth wave is worth more - 26.2 -> 24.7 us on
// 16 x 512 tokens, 16 heads; the dQ kernel would spill 34 and is left at three)
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void pm_attn_mfma_fwd_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                               const bf16_t* __restrict__ v, bf16_t* __restrict__ o,
                                                               float* __restrict__ lse, int S, int H, int BH, float scale) {
  __shared__ __attribute__((aligned(16))) bf16_t sK[2][32 * PM_AT_ST];
  __shared__ __attribute__((aligned(16))) bf16_t sV[2][32 * PM_AT_ST];
  const int qblocks = (S + 127) / 128;
  const int bh = blockIdx.x % BH, qb = qblocks - 1 - blockIdx.x / BH;      // long blocks first
  const int b = bh / H, h = bh % H, d = H * 64;
  const int64_t base = (int64_t)b * S * d + (int64_t)h * 64;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, ql = lane & 31, g = lane >> 5;
  const int q0 = qb * 128 + wave * 32;
  const bool active = q0 < S;
  const int my_last = q0 >> 5;
  const int n_tiles = (S < qb * 128 + 128 ? S : qb * 128 + 128) >> 5;

  pm_bf16x8 fq[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    fq[kk] = active ? *reinterpret_cast<const pm_bf16x8*>(q + base + (int64_t)(q0 + ql) * d + kk * 16 + 8 * g) : pm_at_zero8();
  pm_f32x16 acc[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[dt][e] = 0.f;
  float m = -3.0e38f, lsum = 0.f;

  const int lrow = threadIdx.x >> 3, lcol = (threadIdx.x & 7) * 8;       // loader: 32 rows x 8 pieces of 16 bytes
  // Two register sets: while tile jt is consumed from LDS, tile jt + 1 (loaded an iteration earlier) waits
  // in one set for its LDS store at the end of the iteration and tile jt + 2 is being loaded into the other,
  // so a load has more than a whole iteration to arrive.
  uint4 rk0, rv0, rk1 = make_uint4(0, 0, 0, 0), rv1 = rk1;
  auto gload = [&](int t, uint4& rk, uint4& rv) __attribute__((always_inline)) {
    rk = *reinterpret_cast<const uint4*>(k + base + (int64_t)(t * 32 + lrow) * d + lcol);
    rv = *reinterpret_cast<const uint4*>(v + base + (int64_t)(t * 32 + lrow) * d + lcol);
  };
  auto sstore = [&](int buf, const uint4& rk, const uint4& rv) __attribute__((always_inline)) {
    *reinterpret_cast<uint4*>(&sK[buf][lrow * PM_AT_ST + lcol]) = rk;
    *reinterpret_cast<uint4*>(&sV[buf][lrow * PM_AT_ST + lcol]) = rv;
  };
  gload(0, rk0, rv0);
  sstore(0, rk0, rv0);
  if (1 < n_tiles) gload(1, rk1, rv1);
  __syncthreads();
  const int prow = pm_at_perm(ql);
  const float c2 = scale * 1.44269504f;            // scores in base-2 units: exp(x) = exp2(x log2 e)
  auto tile = [&](int jt, int cur) __attribute__((always_inline)) {
    if (active && jt <= my_last) {
      pm_f32x16 s;
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag(sK[cur], prow, kk * 16, lane), fq[kk], s, 0, 0, 0);
      float p[16], mx = -3.0e38f;
#pragma unroll
      for (int e = 0; e < 16; ++e) p[e] = s[e] * c2;
      if (jt == my_last) {                        // the diagonal tile (uniform over the wave): causal mask
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int kidx = jt * 32 + 16 * (e >> 3) + 8 * g + (e & 7);
          if (kidx > q0 + ql) p[e] = -3.0e38f;
        }
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, p[e]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mn = fmaxf(m, mx);            // finite: key jt * 32 <= query for every tile visited
      const float corr = __builtin_amdgcn_exp2f(m - mn);
      float ps = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        p[e] = __builtin_amdgcn_exp2f(p[e] - mn);              // masked entries: exp2(-huge) = 0
        ps += p[e];
      }
      lsum = lsum * corr + ps;
      if (__builtin_amdgcn_ballot_w64(mn != m) != 0) {      // some row's maximum moved (rare after the first tiles)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[dt][e] *= corr;
      }
      m = mn;
      const pm_bf16x8 pb0 = pm_at_pack8(p), pb1 = pm_at_pack8(p + 8);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag_tr(sV[cur], dt * 32, 0, lane), pb0, acc[dt], 0, 0, 0);
        acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag_tr(sV[cur], dt * 32, 16, lane), pb1, acc[dt], 0, 0, 0);
      }
    }
  };
  // steady part: the loads are unconditional, so the compiler counts outstanding loads exactly and the
  // wait before an LDS store covers only the older register set (a load under a condition would force a
  // wait for everything in flight, the fresh loads included)
  int jt = 0;
  for (; jt + 3 < n_tiles; jt += 2) {
    gload(jt + 2, rk0, rv0);
    tile(jt, 0);
    sstore(1, rk1, rv1);
    __syncthreads();
    gload(jt + 3, rk1, rv1);
    tile(jt + 1, 1);
    sstore(0, rk0, rv0);
    __syncthreads();
  }
  for (; jt < n_tiles; jt += 2) {           // the last one to three tiles
    if (jt + 2 < n_tiles) gload(jt + 2, rk0, rv0);
    tile(jt, 0);
    if (jt + 1 < n_tiles) sstore(1, rk1, rv1);
    __syncthreads();
    if (jt + 1 < n_tiles) {
      tile(jt + 1, 1);
      if (jt + 2 < n_tiles) sstore(0, rk0, rv0);
      __syncthreads();
    }
  }
  if (active) {
    lsum += __shfl_xor(lsum, 32, 64);
    pm_at_store_t(o + base + (int64_t)(q0 + ql) * d, acc, 1.f / lsum, lane);
    if (g == 0) lse[((int64_t)b * H + h) * S + q0 + ql] = m * 0.693147181f + __logf(lsum);   // m is in base-2 units
  }
}

// ---------------------------------------------------------------------------------------------
// backward, dQ: block = 4 waves x 32 queries; streams key / value tiles.
//   S^T = K Q^T, dP^T = V dO^T, dS^T = P^T (dP^T - D) / sqrt(dh), dQ^T += K^T dS^T
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pm_attn_mfma_dq_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                              const bf16_t* __restrict__ v, const bf16_t* __restrict__ o,
                                                              const bf16_t* __restrict__ dO, const float* __restrict__ lse,
                                                              bf16_t* __restrict__ dq, int S, int H, int BH, float scale) {
  __shared__ __attribute__((aligned(16))) bf16_t sK[2][32 * PM_AT_ST];
  __shared__ __attribute__((aligned(16))) bf16_t sV[2][32 * PM_AT_ST];
  const int qblocks = (S + 127) / 128;
  const int bh = blockIdx.x % BH, qb = qblocks - 1 - blockIdx.x / BH;
  const int b = bh / H, h = bh % H, d = H * 64;
  const int64_t base = (int64_t)b * S * d + (int64_t)h * 64;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, ql = lane & 31, g = lane >> 5;
  const int q0 = qb * 128 + wave * 32;
  const bool active = q0 < S;
  const int my_last = q0 >> 5;
  const int n_tiles = (S < qb * 128 + 128 ? S : qb * 128 + 128) >> 5;

  pm_bf16x8 fq[4], fdo[4];
  float Dq = 0.f, lq = 0.f;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    fq[kk] = pm_at_zero8();
    fdo[kk] = pm_at_zero8();
  }
  if (active) {
    const int64_t ro = base + (int64_t)(q0 + ql) * d;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      fq[kk] = *reinterpret_cast<const pm_bf16x8*>(q + ro + kk * 16 + 8 * g);
      fdo[kk] = *reinterpret_cast<const pm_bf16x8*>(dO + ro + kk * 16 + 8 * g);
      float a[8], c[8];
      pm_ld8(dO + ro + kk * 16 + 8 * g, a);
      pm_ld8(o + ro + kk * 16 + 8 * g, c);
#pragma unroll
      for (int e = 0; e < 8; ++e) Dq += a[e] * c[e];
    }
    Dq += __shfl_xor(Dq, 32, 64);
    lq = lse[((int64_t)b * H + h) * S + q0 + ql];
  }
  pm_f32x16 acc[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[dt][e] = 0.f;

  const int lrow = threadIdx.x >> 3, lcol = (threadIdx.x & 7) * 8;
  // two register sets as in the forward kernel: a tile is loaded two iterations before its use
  uint4 rk0, rv0, rk1 = make_uint4(0, 0, 0, 0), rv1 = rk1;
  auto gload = [&](int t, uint4& rk, uint4& rv) __attribute__((always_inline)) {
    rk = *reinterpret_cast<const uint4*>(k + base + (int64_t)(t * 32 + lrow) * d + lcol);
    rv = *reinterpret_cast<const uint4*>(v + base + (int64_t)(t * 32 + lrow) * d + lcol);
  };
  auto sstore = [&](int buf, const uint4& rk, const uint4& rv) __attribute__((always_inline)) {
    *reinterpret_cast<uint4*>(&sK[buf][lrow * PM_AT_ST + lcol]) = rk;
    *reinterpret_cast<uint4*>(&sV[buf][lrow * PM_AT_ST + lcol]) = rv;
  };
  gload(0, rk0, rv0);
  sstore(0, rk0, rv0);
  if (1 < n_tiles) gload(1, rk1, rv1);
  __syncthreads();
  const int prow = pm_at_perm(ql);
  const float c2 = scale * 1.44269504f, lq2 = lq * 1.44269504f;       // base-2 units: exp(x) = exp2(x log2 e)
  auto tile = [&](int jt, int cur) __attribute__((always_inline)) {
    if (active && jt <= my_last) {
      pm_f32x16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        s[e] = 0.f;
        dp[e] = 0.f;
      }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag(sK[cur], prow, kk * 16, lane), fq[kk], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag(sV[cur], prow, kk * 16, lane), fdo[kk], dp, 0, 0, 0);
      }
      float ds[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) ds[e] = __builtin_amdgcn_exp2f(fmaf(s[e], c2, -lq2)) * (dp[e] - Dq);   // 1 / sqrt(dh): final store
      if (jt == my_last) {                        // the diagonal tile (uniform over the wave): causal mask
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int kidx = jt * 32 + 16 * (e >> 3) + 8 * g + (e & 7);
          if (kidx > q0 + ql) ds[e] = 0.f;
        }
      }
      const pm_bf16x8 b0 = pm_at_pack8(ds), b1 = pm_at_pack8(ds + 8);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag_tr(sK[cur], dt * 32, 0, lane), b0, acc[dt], 0, 0, 0);
        acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag_tr(sK[cur], dt * 32, 16, lane), b1, acc[dt], 0, 0, 0);
      }
    }
  };
  // steady part: the loads are unconditional, so the compiler counts outstanding loads exactly and the
  // wait before an LDS store covers only the older register set (a load under a condition would force a
  // wait for everything in flight, the fresh loads included)
  int jt = 0;
  for (; jt + 3 < n_tiles; jt += 2) {
    gload(jt + 2, rk0, rv0);
    tile(jt, 0);
    sstore(1, rk1, rv1);
    __syncthreads();
    gload(jt + 3, rk1, rv1);
    tile(jt + 1, 1);
    sstore(0, rk0, rv0);
    __syncthreads();
  }
  for (; jt < n_tiles; jt += 2) {           // the last one to three tiles
    if (jt + 2 < n_tiles) gload(jt + 2, rk0, rv0);
    tile(jt, 0);
    if (jt + 1 < n_tiles) sstore(1, rk1, rv1);
    __syncthreads();
    if (jt + 1 < n_tiles) {
      tile(jt + 1, 1);
      if (jt + 2 < n_tiles) sstore(0, rk0, rv0);
      __syncthreads();
    }
  }
  if (active) pm_at_store_t(dq + base + (int64_t)(q0 + ql) * d, acc, scale, lane);
}

// ---------------------------------------------------------------------------------------------
// backward, dK and dV: block = 4 waves x 32 keys; streams query tiles (Q, dO, and the row vectors
// log-sum-exp and D, the latter computed while the tile is loaded).
//   S = Q K^T, dP = dO V^T, dS = P (dP - D) / sqrt(dh), dV^T += dO^T P, dK^T += Q^T dS
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pm_attn_mfma_dkv_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                               const bf16_t* __restrict__ v, const bf16_t* __restrict__ o,
                                                               const bf16_t* __restrict__ dO, const float* __restrict__ lse,
                                                               bf16_t* __restrict__ dk, bf16_t* __restrict__ dv, int S, int H,
                                                               int BH, float scale) {
  __shared__ __attribute__((aligned(16))) bf16_t sQ[2][32 * PM_AT_ST];
  __shared__ __attribute__((aligned(16))) bf16_t sO[2][32 * PM_AT_ST];     // dO
  __shared__ __attribute__((aligned(16))) float sL[2][32];
  __shared__ __attribute__((aligned(16))) float sD[2][32];
  const int bh = blockIdx.x % BH, kb = blockIdx.x / BH;                    // long blocks (early keys) first
  const int b = bh / H, h = bh % H, d = H * 64;
  const int64_t base = (int64_t)b * S * d + (int64_t)h * 64;
  const int64_t lbase = ((int64_t)b * H + h) * S;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, kl = lane & 31, g = lane >> 5;
  const int k0 = kb * 128 + wave * 32;
  const bool active = k0 < S;
  const int my_first = k0 >> 5;
  const int first = kb * 4, n_tiles = S >> 5;

  pm_bf16x8 fk[4], fv[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    fk[kk] = active ? *reinterpret_cast<const pm_bf16x8*>(k + base + (int64_t)(k0 + kl) * d + kk * 16 + 8 * g) : pm_at_zero8();
    fv[kk] = active ? *reinterpret_cast<const pm_bf16x8*>(v + base + (int64_t)(k0 + kl) * d + kk * 16 + 8 * g) : pm_at_zero8();
  }
  pm_f32x16 ak[2], av[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      ak[dt][e] = 0.f;
      av[dt][e] = 0.f;
    }

  const int lrow = threadIdx.x >> 3, lcol = (threadIdx.x & 7) * 8;
  // two register sets (a query tile is loaded two iterations before its use); D of the tile's rows is
  // computed when the set moves to LDS
  struct Regs {
    uint4 q, dO, o;
    float L;
  };
  Regs r0, r1;
  r1.q = r1.dO = r1.o = make_uint4(0, 0, 0, 0);
  r0.L = r1.L = 0.f;
  auto gload = [&](int it, Regs& r) __attribute__((always_inline)) {
    const int64_t ro = base + (int64_t)(it * 32 + lrow) * d + lcol;
    r.q = *reinterpret_cast<const uint4*>(q + ro);
    r.dO = *reinterpret_cast<const uint4*>(dO + ro);
    r.o = *reinterpret_cast<const uint4*>(o + ro);
    r.L = lse[lbase + it * 32 + (threadIdx.x & 31)];       // every thread (no load under a condition)
  };
  auto sstore = [&](int buf, const Regs& r) __attribute__((always_inline)) {
    *reinterpret_cast<uint4*>(&sQ[buf][lrow * PM_AT_ST + lcol]) = r.q;
    *reinterpret_cast<uint4*>(&sO[buf][lrow * PM_AT_ST + lcol]) = r.dO;
    const uint32_t a[4] = {r.dO.x, r.dO.y, r.dO.z, r.dO.w}, c[4] = {r.o.x, r.o.y, r.o.z, r.o.w};
    float part = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      part = fmaf(__uint_as_float(a[e] << 16), __uint_as_float(c[e] << 16), part);
      part = fmaf(__uint_as_float(a[e] & 0xffff0000u), __uint_as_float(c[e] & 0xffff0000u), part);
    }
    part += __shfl_xor(part, 1, 64);
    part += __shfl_xor(part, 2, 64);
    part += __shfl_xor(part, 4, 64);
    if ((threadIdx.x & 7) == 0) sD[buf][lrow] = part;
    if (threadIdx.x < 32) sL[buf][threadIdx.x] = r.L * 1.44269504f;       // base-2 units
  };
  gload(first, r0);
  sstore(0, r0);
  if (first + 1 < n_tiles) gload(first + 1, r1);
  __syncthreads();
  const int prow = pm_at_perm(kl);
  const float c2 = scale * 1.44269504f;
  auto tile = [&](int it, int cur) __attribute__((always_inline)) {
    if (active && it >= my_first) {
      pm_f32x16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        s[e] = 0.f;
        dp[e] = 0.f;
      }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag(sQ[cur], prow, kk * 16, lane), fk[kk], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag(sO[cur], prow, kk * 16, lane), fv[kk], dp, 0, 0, 0);
      }
      float p[16], ds[16], lv[16], Dv[16];
#pragma unroll
      for (int c4 = 0; c4 < 4; ++c4) {
        // streamed (query) rows of this lane: 16 (e / 8) + 8 g + e % 8, i.e. two runs of 8 consecutive rows
        const int r = 16 * (c4 >> 1) + 8 * g + 4 * (c4 & 1);
        const float4 l4 = *reinterpret_cast<const float4*>(&sL[cur][r]);
        const float4 d4 = *reinterpret_cast<const float4*>(&sD[cur][r]);
        lv[4 * c4] = l4.x; lv[4 * c4 + 1] = l4.y; lv[4 * c4 + 2] = l4.z; lv[4 * c4 + 3] = l4.w;
        Dv[4 * c4] = d4.x; Dv[4 * c4 + 1] = d4.y; Dv[4 * c4 + 2] = d4.z; Dv[4 * c4 + 3] = d4.w;
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) p[e] = __builtin_amdgcn_exp2f(fmaf(s[e], c2, -lv[e]));
      if (it == my_first) {                       // the diagonal tile (uniform over the wave): causal mask
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int qidx = it * 32 + 16 * (e >> 3) + 8 * g + (e & 7);
          if (qidx < k0 + kl) p[e] = 0.f;
        }
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) ds[e] = p[e] * (dp[e] - Dv[e]);       // the factor 1 / sqrt(dh) goes into the final store
      const pm_bf16x8 p0 = pm_at_pack8(p), p1 = pm_at_pack8(p + 8), s0 = pm_at_pack8(ds), s1 = pm_at_pack8(ds + 8);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        av[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag_tr(sO[cur], dt * 32, 0, lane), p0, av[dt], 0, 0, 0);
        av[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag_tr(sO[cur], dt * 32, 16, lane), p1, av[dt], 0, 0, 0);
        ak[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag_tr(sQ[cur], dt * 32, 0, lane), s0, ak[dt], 0, 0, 0);
        ak[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_at_frag_tr(sQ[cur], dt * 32, 16, lane), s1, ak[dt], 0, 0, 0);
      }
    }
  };
  int it = first;
  for (; it + 3 < n_tiles; it += 2) {        // steady part: unconditional loads (see the forward kernel)
    gload(it + 2, r0);
    tile(it, 0);
    sstore(1, r1);
    __syncthreads();
    gload(it + 3, r1);
    tile(it + 1, 1);
    sstore(0, r0);
    __syncthreads();
  }
  for (; it < n_tiles; it += 2) {            // the last one to three tiles
    if (it + 2 < n_tiles) gload(it + 2, r0);
    tile(it, 0);
    if (it + 1 < n_tiles) sstore(1, r1);
    __syncthreads();
    if (it + 1 < n_tiles) {
      tile(it + 1, 1);
      if (it + 2 < n_tiles) sstore(0, r0);
      __syncthreads();
    }
  }
  if (active) {
    pm_at_store_t(dk + base + (int64_t)(k0 + kl) * d, ak, scale, lane);
    pm_at_store_t(dv + base + (int64_t)(k0 + kl) * d, av, 1.f, lane);
  }
}

