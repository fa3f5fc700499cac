// Weight-free and vector-weight kernels of the fine-grained Transformer stages: embedding,
// LayerNorm, causal attention core.  The matrix stages reuse the Linear GEMMs.
//
// Row t = b * S + s of every [tokens, width] matrix is token s of sequence b.  The residual stream
// and its gradient are fp32; GEMM operands are in the compute dtype T (bf16 or fp32).
//
// Two-weight backward (Sec. 2.1): a backward kernel reads a weight only where a gradient flows
// through it: LayerNorm's dx uses the backward gain (corrected buffer or ring slot, like the
// Linear units' dz . W); the gain / bias gradients use forward quantities only.
#pragma once
#include "pm_common.hpp"
#include "pm_update.hpp"
#include "pm_attn_api.hpp"

constexpr float PM_LN_EPS = 1e-5f;

// ---------------------------------------------------------------------------------------------
// GEMM epilogues of the residual blocks (used with the same GEMM kernels as the Linear epilogues)
// ---------------------------------------------------------------------------------------------
// out[i, j] = res[i, j] + acc + b[j], fp32: the residual stream after an attention / feed-forward block
template <typename T>
struct PmEpiFwdRes {
  static constexpr bool kColSumA = false;
  __device__ __forceinline__ bool wants_colsum() const { return false; }
  __device__ __forceinline__ void colsum(int, float) const {}
  PmWLoc<T> bias;
  const float* res; float* out; int ld;
  const T* b_;
  __device__ __forceinline__ void begin() { b_ = bias.get(); }
  __device__ __forceinline__ void operator()(int i, int j, float acc) const {
    const int64_t o = (int64_t)i * ld + j;
    out[o] = res[o] + acc + ldf(b_ + j);
  }
  struct Pre { PmRaw8<T> b; PmRaw8<float> r; };
  __device__ __forceinline__ Pre pre8(int i, int j) const {
    Pre p;
    p.b.load(b_ + j);
    p.r.load(res + (int64_t)i * ld + j);
    return p;
  }
  __device__ __forceinline__ void op8(int i, int j, const float* acc, const Pre& p) const {
    const int64_t o = (int64_t)i * ld + j;
    float v[8], bb[8], rr[8];
    p.b.widen(bb);
    p.r.widen(rr);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = rr[e] + acc[e] + bb[e];
    pm_st8(out + o, v);
  }
};
// out[i, j] (+)= acc, fp32: data gradients that enter a LayerNorm backward (summed over the
// consumers of the LayerNorm output)
struct PmEpiF32 {
  static constexpr bool kColSumA = false;
  __device__ __forceinline__ bool wants_colsum() const { return false; }
  __device__ __forceinline__ void colsum(int, float) const {}
  float* out; int ld; int accumulate;
  __device__ __forceinline__ void begin() {}
  __device__ __forceinline__ void operator()(int i, int j, float acc) const {
    const int64_t o = (int64_t)i * ld + j;
    out[o] = accumulate ? out[o] + acc : acc;
  }
  struct Pre { float o[8]; };
  __device__ __forceinline__ Pre pre8(int i, int j) const {
    Pre p;
    if (accumulate) pm_ld8(out + (int64_t)i * ld + j, p.o);
    return p;
  }
  __device__ __forceinline__ void op8(int i, int j, const float* acc, const Pre& p) const {
    const int64_t o = (int64_t)i * ld + j;
    float v[8];
    if (accumulate) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = p.o[e] + acc[e];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = acc[e];
    }
    pm_st8(out + o, v);
  }
};

// Inside a step of the 12-layer workload (kernel trace, same box): residual products 54.0 -> 51.8 us, fp32 data gradient
// with K = 4096 77.2 -> 75.0 us on the rectangular blocks; the bf16 data gradients (58.2 -> 59.1 us) and the feed-forward
// expansion (87.1 -> 88.3 us) lose what they gain stand-alone, the three projections in one launch stay the same.
template <typename T> struct pm_rect_tiles<PmEpiFwdRes<T>> : std::true_type {};
template <> struct pm_rect_tiles<PmEpiF32> : std::true_type {};

// zero a list of regions of a flat fp32 array: region r = [reg[2r], reg[2r] + reg[2r+1]); grid (x, regions)
__global__ __launch_bounds__(256) void pm_zero_regions_kernel(float* base, const int64_t* __restrict__ reg) {
  const int64_t off = reg[2 * blockIdx.y], n = reg[2 * blockIdx.y + 1];
  float4* p = reinterpret_cast<float4*>(base + off);          // regions are chunk-aligned and chunk-sized
  const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < (n >> 2); i += (int64_t)gridDim.x * blockDim.x) p[i] = z;
}

// First kernel of a Transformer microbatch: refreshes the step table at the start of a minibatch
// (L > 0) and clears the loss accumulator.  A launch of its own because the next kernel (the
// embedding lookup) already reads its ring slot from the table.
__global__ void pm_begin_tokens_kernel(PmStepHdr* hdr, const PmLayerStatic* ls, PmLayerStep* ld, int L, PmSchedDev sc,
                                       int par) {
  if (L > 0) pm_prologue_block(hdr, ls, ld, L, sc, par);
  if (threadIdx.x == 0) hdr->loss = 0.f;
}

// ---------------------------------------------------------------------------------------------
// embedding: x[t, :] = E[token[t], :] + pos[t mod S, :]
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void pm_embed_fwd_kernel(const int32_t* __restrict__ tokens, PmWLoc<T> E,
                                                           const float* __restrict__ pos, float* __restrict__ x,
                                                           int tokens_n, int S, int d, int vocab) {
  const T* e = E.get();
  const int64_t total = (int64_t)tokens_n * d;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int t = (int)(i / d), j = (int)(i % d);
    int tok = tokens[t];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);          // out-of-range ids are clamped
    x[i] = ldf(e + (int64_t)tok * d + j) + pos[(int64_t)(t % S) * d + j];
  }
}

// dE[token[t], :] += dx[t, :]   (fp32 atomics; the caller zeroes dE first unless accumulating)
__global__ __launch_bounds__(256) void pm_embed_bwd_kernel(const int32_t* __restrict__ tokens,
                                                           const float* __restrict__ dx, float* __restrict__ dE,
                                                           int tokens_n, int d, int vocab) {
  const int64_t total = (int64_t)tokens_n * d;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int t = (int)(i / d), j = (int)(i % d);
    int tok = tokens[t];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
    atomicAdd(dE + (int64_t)tok * d + j, dx[i]);
  }
}

// ---------------------------------------------------------------------------------------------
// LayerNorm forward: one wavefront per row, the row held in registers (lane l owns columns
// 256 c + 4 l .. + 3, d <= 256 NC, d a multiple of 4).  Stores mean and 1/sqrt(var + eps) for the
// backward.  gb: gain at offset 0, bias at offset boff of the unit's ring slot.
// ---------------------------------------------------------------------------------------------
template <typename T, int NC>
__global__ __launch_bounds__(256) void pm_ln_fwd_kernel(const float* __restrict__ x, PmWLoc<T> gb, int boff,
                                                        T* __restrict__ out, float* __restrict__ mean,
                                                        float* __restrict__ rstd, int rows, int d) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const int64_t ro = (int64_t)row * d;
  float4 xv[NC];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j = 256 * c + 4 * lane;
    xv[c] = j < d ? pm_ld4(x + ro + j) : make_float4(0.f, 0.f, 0.f, 0.f);
    s += xv[c].x + xv[c].y + xv[c].z + xv[c].w;
  }
  const float mu = pm_wave_sum(s) / (float)d;
  float v = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j = 256 * c + 4 * lane;
    if (j < d) {
      xv[c] = make_float4(xv[c].x - mu, xv[c].y - mu, xv[c].z - mu, xv[c].w - mu);
      v += xv[c].x * xv[c].x + xv[c].y * xv[c].y + xv[c].z * xv[c].z + xv[c].w * xv[c].w;
    }
  }
  const float rs = rsqrtf(pm_wave_sum(v) / (float)d + PM_LN_EPS);
  const T* g = gb.get();
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j = 256 * c + 4 * lane;
    if (j < d) {
      const float4 gg = pm_ld4(g + j), bb = pm_ld4(g + boff + j);
      pm_st4(out + ro + j, make_float4(xv[c].x * rs * gg.x + bb.x, xv[c].y * rs * gg.y + bb.y, xv[c].z * rs * gg.z + bb.z,
                                       xv[c].w * rs * gg.w + bb.w));
    }
  }
  if (lane == 0) {
    mean[row] = mu;
    rstd[row] = rs;
  }
}

// ---------------------------------------------------------------------------------------------
// LayerNorm backward.  dy fp32 [rows, d] is the gradient w.r.t. the LayerNorm output.
//   dx_out = dx_res + rstd * (dxh - mean(dxh) - xhat * mean(dxh * xhat)),  dxh = dy * gain_bkwd
//   dgain += sum_rows dy * xhat,  dbias += sum_rows dy      (fp32 atomics, one set per block)
// dx_res is the gradient already on the residual stream (same shape); dx_out may alias it.
// dx_out_t (optional) receives a copy in the compute dtype for the GEMMs that consume it.
// Block = 8 waves x 4 rows; lane l owns columns 256 c + 4 l .. + 3 (16-byte accesses), d <= 256 NC,
// d a multiple of 4.
// ---------------------------------------------------------------------------------------------
template <typename T, int NC>
__global__ __launch_bounds__(512) void pm_ln_bwd_kernel(const float* __restrict__ dy, const float* __restrict__ x,
                                                        const float* __restrict__ mean, const float* __restrict__ rstd,
                                                        PmWLoc<T> gain_bkwd, const float* dx_res, float* dx_out,
                                                        T* dx_out_t, float* __restrict__ dgain, float* __restrict__ dbias,
                                                        int rows, int d, const float* dy2) {
  __shared__ float4 red[8][2][64 * NC];                       // per wave: gain and bias partial sums
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const T* g = gain_bkwd.get();
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 gj[NC], ag[NC], ab[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j = 256 * c + 4 * lane;
    gj[c] = j < d ? pm_ld4(g + j) : zero4;
    ag[c] = zero4;
    ab[c] = zero4;
  }
  // all loads of the wave's four rows go out first (rows past the end re-read the last row and are
  // masked out below), so the wave pays the memory latency once instead of once per row
  float4 dyr[4][NC], xr[4][NC], rrr[4][NC];
  float mur[4], rsr[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int row = blockIdx.x * 32 + wave * 4 + r;
    const int rowc = row < rows ? row : rows - 1;
    const int64_t ro = (int64_t)rowc * d;
    mur[r] = mean[rowc];
    rsr[r] = rstd[rowc];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int j = 256 * c + 4 * lane;
      dyr[r][c] = j < d ? pm_ld4(dy + ro + j) : zero4;
      if (dy2 && j < d) {       // the gradient arrives as two addends (dy2 may be the buffer dx_out is written to below)
        const float4 e = pm_ld4(dy2 + ro + j);
        dyr[r][c].x += e.x; dyr[r][c].y += e.y; dyr[r][c].z += e.z; dyr[r][c].w += e.w;
      }
      xr[r][c] = j < d ? pm_ld4(x + ro + j) : zero4;
      // (requested here, not row by row below: a load issued behind the stores of the row before would wait for them)
      rrr[r][c] = (dx_res && j < d) ? pm_ld4(dx_res + ro + j) : zero4;
    }
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int row = blockIdx.x * 32 + wave * 4 + r;
    if (row >= rows) break;                                   // wave-uniform
    const float mu = mur[r], rs = rsr[r];
    const int64_t ro = (int64_t)row * d;
    float4 xh[NC], dxh[NC], rr[NC];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int j = 256 * c + 4 * lane;
      float4 dyv = dyr[r][c], xv = zero4;
      rr[c] = rrr[r][c];
      if (j < d) {
        xv = xr[r][c];
        xv = make_float4((xv.x - mu) * rs, (xv.y - mu) * rs, (xv.z - mu) * rs, (xv.w - mu) * rs);
      }
      xh[c] = xv;
      dxh[c] = make_float4(dyv.x * gj[c].x, dyv.y * gj[c].y, dyv.z * gj[c].z, dyv.w * gj[c].w);
      ag[c].x += dyv.x * xv.x; ag[c].y += dyv.y * xv.y; ag[c].z += dyv.z * xv.z; ag[c].w += dyv.w * xv.w;
      ab[c].x += dyv.x; ab[c].y += dyv.y; ab[c].z += dyv.z; ab[c].w += dyv.w;
      s1 += dxh[c].x + dxh[c].y + dxh[c].z + dxh[c].w;
      s2 += dxh[c].x * xv.x + dxh[c].y * xv.y + dxh[c].z * xv.z + dxh[c].w * xv.w;
    }
    s1 = pm_wave_sum(s1) / (float)d;
    s2 = pm_wave_sum(s2) / (float)d;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int j = 256 * c + 4 * lane;
      if (j < d) {
        float4 v;
        v.x = rr[c].x + rs * (dxh[c].x - s1 - xh[c].x * s2);
        v.y = rr[c].y + rs * (dxh[c].y - s1 - xh[c].y * s2);
        v.z = rr[c].z + rs * (dxh[c].z - s1 - xh[c].z * s2);
        v.w = rr[c].w + rs * (dxh[c].w - s1 - xh[c].w * s2);
        pm_st4(dx_out + ro + j, v);
        if (dx_out_t) pm_st4(dx_out_t + ro + j, v);
      }
    }
  }
  // block sum of the per-wave partials (plain LDS stores and loads: LDS float atomics were measured
  // several times slower), then one fp32 atomic per column and block
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    red[wave][0][64 * c + lane] = ag[c];
    red[wave][1][64 * c + lane] = ab[c];
  }
  __syncthreads();
  for (int j = threadIdx.x; j < d; j += 512) {
    float sg = 0.f, sb = 0.f;
    const int c = j >> 8, l4 = (j & 255) >> 2, e = j & 3;      // column j = 256 c + 4 lane + e
#pragma unroll
    for (int w = 0; w < 8; ++w) {
      const float* pg = reinterpret_cast<const float*>(&red[w][0][64 * c + l4]);
      const float* pb = reinterpret_cast<const float*>(&red[w][1][64 * c + l4]);
      sg += pg[e];
      sb += pb[e];
    }
    atomicAdd(dgain + j, sg);
    atomicAdd(dbias + j, sb);
  }
}

// copy fp32 -> compute dtype (the residual gradient entering a GEMM)
template <typename T>
__global__ __launch_bounds__(256) void pm_cast_kernel(const float* __restrict__ in, T* __restrict__ out, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    stf(out + i, in[i]);
}

// ---------------------------------------------------------------------------------------------
// Causal attention core, one block per (sequence, head), one thread per query row.
// q, k, v, o: [tokens, d_model] in T, head h in columns h*DH .. h*DH+DH-1.  lse: fp32 [B, H, S].
// K and V of the head sit in LDS as fp32 (S * DH * 8 bytes <= ~140 KB); all lanes read the same
// key row at a time (LDS broadcast), scores are never materialised (running max / sum).
// ---------------------------------------------------------------------------------------------
template <typename T, int DH>
__global__ void pm_attn_fwd_kernel(const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
                                   T* __restrict__ o, float* __restrict__ lse, int S, int H, float scale) {
  extern __shared__ float sm[];
  float* sK = sm;
  float* sV = sm + (size_t)S * DH;
  const int b = blockIdx.x / H, h = blockIdx.x % H;
  const int d = H * DH;
  const int64_t base = (int64_t)b * S * d + (int64_t)h * DH;
  for (int e = threadIdx.x; e < S * DH; e += blockDim.x) {
    const int r = e / DH, c = e % DH;
    sK[e] = ldf(k + base + (int64_t)r * d + c);
    sV[e] = ldf(v + base + (int64_t)r * d + c);
  }
  __syncthreads();
  const int i = threadIdx.x;
  if (i >= S) return;
  float qi[DH], acc[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) {
    qi[c] = ldf(q + base + (int64_t)i * d + c) * scale;
    acc[c] = 0.f;
  }
  float m = -3.0e38f, l = 0.f;
  for (int j = 0; j <= i; ++j) {
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < DH; ++c) s += qi[c] * sK[j * DH + c];
    const float mn = fmaxf(m, s);
    const float corr = __expf(m - mn), p = __expf(s - mn);
    l = l * corr + p;
#pragma unroll
    for (int c = 0; c < DH; ++c) acc[c] = acc[c] * corr + p * sV[j * DH + c];
    m = mn;
  }
  const float inv = 1.f / l;
#pragma unroll
  for (int c = 0; c < DH; ++c) stf(o + base + (int64_t)i * d + c, acc[c] * inv);
  lse[((int64_t)b * H + h) * S + i] = m + __logf(l);
}

// Backward of the attention core.  Pass 1 (thread = query row i): dq_i.  Pass 2 (thread = key
// row j): dk_j, dv_j.  Probabilities are recomputed from q, k and the stored log-sum-exp;
// D_i = do_i . o_i is the row term of the softmax Jacobian.
template <typename T, int DH>
__global__ void pm_attn_bwd_kernel(const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
                                   const T* __restrict__ o, const T* __restrict__ dO, const float* __restrict__ lse,
                                   T* __restrict__ dq, T* __restrict__ dk, T* __restrict__ dv, int S, int H, float scale) {
  extern __shared__ float sm[];
  float* sA = sm;                          // pass 1: K      pass 2: Q
  float* sB = sm + (size_t)S * DH;         // pass 1: V      pass 2: dO
  float* sL = sm + (size_t)2 * S * DH;     // log-sum-exp per row
  float* sD = sL + S;                      // D per row
  const int b = blockIdx.x / H, h = blockIdx.x % H;
  const int d = H * DH;
  const int64_t base = (int64_t)b * S * d + (int64_t)h * DH;
  const int i = threadIdx.x;
  for (int e = threadIdx.x; e < S * DH; e += blockDim.x) {
    const int r = e / DH, c = e % DH;
    sA[e] = ldf(k + base + (int64_t)r * d + c);
    sB[e] = ldf(v + base + (int64_t)r * d + c);
  }
  float qi[DH], doi[DH];
  float Di = 0.f, li = 0.f;
  if (i < S) {
#pragma unroll
    for (int c = 0; c < DH; ++c) {
      qi[c] = ldf(q + base + (int64_t)i * d + c);
      doi[c] = ldf(dO + base + (int64_t)i * d + c);
      Di += doi[c] * ldf(o + base + (int64_t)i * d + c);
    }
    li = lse[((int64_t)b * H + h) * S + i];
    sL[i] = li;
    sD[i] = Di;
  }
  __syncthreads();
  if (i < S) {
    float acc[DH];
#pragma unroll
    for (int c = 0; c < DH; ++c) acc[c] = 0.f;
    for (int j = 0; j <= i; ++j) {
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int c = 0; c < DH; ++c) {
        s += qi[c] * sA[j * DH + c];
        dp += doi[c] * sB[j * DH + c];
      }
      const float p = __expf(s * scale - li);
      const float ds = p * (dp - Di) * scale;
#pragma unroll
      for (int c = 0; c < DH; ++c) acc[c] += ds * sA[j * DH + c];
    }
#pragma unroll
    for (int c = 0; c < DH; ++c) stf(dq + base + (int64_t)i * d + c, acc[c]);
  }
  __syncthreads();
  // pass 2: this thread is key row j = threadIdx.x; Q and dO of the head go to LDS
  float kj[DH], vj[DH];
  if (i < S) {
#pragma unroll
    for (int c = 0; c < DH; ++c) {
      kj[c] = sA[i * DH + c];
      vj[c] = sB[i * DH + c];
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < S * DH; e += blockDim.x) {
    const int r = e / DH, c = e % DH;
    sA[e] = ldf(q + base + (int64_t)r * d + c);
    sB[e] = ldf(dO + base + (int64_t)r * d + c);
  }
  __syncthreads();
  if (i < S) {
    float ak[DH], av[DH];
#pragma unroll
    for (int c = 0; c < DH; ++c) {
      ak[c] = 0.f;
      av[c] = 0.f;
    }
    for (int r = i; r < S; ++r) {
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int c = 0; c < DH; ++c) {
        s += sA[r * DH + c] * kj[c];
        dp += sB[r * DH + c] * vj[c];
      }
      const float p = __expf(s * scale - sL[r]);
      const float ds = p * (dp - sD[r]) * scale;
#pragma unroll
      for (int c = 0; c < DH; ++c) {
        av[c] += p * sB[r * DH + c];
        ak[c] += ds * sA[r * DH + c];
      }
    }
#pragma unroll
    for (int c = 0; c < DH; ++c) {
      stf(dk + base + (int64_t)i * d + c, ak[c]);
      stf(dv + base + (int64_t)i * d + c, av[c]);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// host-side dispatch
// ---------------------------------------------------------------------------------------------
template <typename T>
inline bool pm_ln_fwd_launch(hipStream_t st, const float* x, PmWLoc<T> gb, int boff, T* out, float* mean, float* rstd,
                             int rows, int d) {
  if ((d & 3) || (boff & 3)) return false;
  const dim3 grid((rows + 3) / 4), blk(256);
#define PM_LNF(NC) hipLaunchKernelGGL((pm_ln_fwd_kernel<T, NC>), grid, blk, 0, st, x, gb, boff, out, mean, rstd, rows, d)
  if (d <= 256) PM_LNF(1);
  else if (d <= 512) PM_LNF(2);
  else if (d <= 768) PM_LNF(3);
  else if (d <= 1024) PM_LNF(4);
  else return false;
#undef PM_LNF
  return true;
}

template <typename T>
inline bool pm_ln_bwd_launch(hipStream_t st, const float* dy, const float* x, const float* mean, const float* rstd,
                             PmWLoc<T> gain_bkwd, const float* dx_res, float* dx_out, T* dx_out_t, float* dgain,
                             float* dbias, int rows, int d, const float* dy2 = nullptr) {
  if (d & 3) return false;
  const dim3 grid((rows + 31) / 32), blk(512);
#define PM_LNB(NC) hipLaunchKernelGGL((pm_ln_bwd_kernel<T, NC>), grid, blk, 0, st, dy, x, mean, rstd, gain_bkwd, dx_res, dx_out, dx_out_t, dgain, dbias, rows, d, dy2)
  if (d <= 256) PM_LNB(1);
  else if (d <= 512) PM_LNB(2);
  else if (d <= 768) PM_LNB(3);
  else if (d <= 1024) PM_LNB(4);
  else return false;
#undef PM_LNB
  return true;
}

// plain attention kernels: one thread per query / key row, K and V (Q and dO) of a head in LDS as fp32
inline bool pm_attn_plain_fits(int S, int dh) {
  // K, V (Q, dO) + two row vectors as fp32 in 64 KB of LDS
  return (int64_t)S * (dh + 1) * 8 <= 65536 && S <= 1024 && (dh == 4 || dh == 8 || dh == 16 || dh == 32 || dh == 64);
}

template <typename T>
inline bool pm_attn_fwd_launch(hipStream_t st, int B, int S, int H, int dh, const T* q, const T* k, const T* v, T* o,
                               float* lse) {
  if constexpr (sizeof(T) == 2) {
    if (pm_attn_mfma_fits(S, dh)) {
      pm_attn_mfma_fwd(st, B, S, H, q, k, v, o, lse);
      return true;
    }
  }
  if (!pm_attn_plain_fits(S, dh)) return false;
  const float scale = 1.f / sqrtf((float)dh);
  const dim3 grid(B * H), blk((S + 63) / 64 * 64);
  const size_t lds = (size_t)2 * S * dh * 4;
#define PM_AF(DH) hipLaunchKernelGGL((pm_attn_fwd_kernel<T, DH>), grid, blk, lds, st, q, k, v, o, lse, S, H, scale)
  switch (dh) {
    case 4: PM_AF(4); break;
    case 8: PM_AF(8); break;
    case 16: PM_AF(16); break;
    case 32: PM_AF(32); break;
    default: PM_AF(64); break;
  }
#undef PM_AF
  return true;
}

template <typename T>
inline bool pm_attn_bwd_launch(hipStream_t st, int B, int S, int H, int dh, const T* q, const T* k, const T* v, const T* o,
                               const T* dO, const float* lse, T* dq, T* dk, T* dv) {
  if constexpr (sizeof(T) == 2) {
    if (pm_attn_mfma_fits(S, dh)) {
      pm_attn_mfma_bwd(st, B, S, H, q, k, v, o, dO, lse, dq, dk, dv);
      return true;
    }
  }
  if (!pm_attn_plain_fits(S, dh)) return false;
  const float scale = 1.f / sqrtf((float)dh);
  const dim3 grid(B * H), blk((S + 63) / 64 * 64);
  const size_t lds = (size_t)2 * S * dh * 4 + (size_t)2 * S * 4;
#define PM_AB(DH) hipLaunchKernelGGL((pm_attn_bwd_kernel<T, DH>), grid, blk, lds, st, q, k, v, o, dO, lse, dq, dk, dv, S, H, scale)
  switch (dh) {
    case 4: PM_AB(4); break;
    case 8: PM_AB(8); break;
    case 16: PM_AB(16); break;
    case 32: PM_AB(32); break;
    default: PM_AB(64); break;
  }
#undef PM_AB
  return true;
}
