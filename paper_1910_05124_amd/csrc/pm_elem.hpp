// Input staging, loss kernels, bias gradient and the plain (non-MFMA) GEMM used for fp32 contexts.
#pragma once
#include <type_traits>

#include "pm_common.hpp"

// x (fp32 [M, n]) -> compute dtype [M, ld]; pad columns zeroed.  Also clears the loss accumulator
// of the microbatch (first kernel of every microbatch).
template <typename T>
__global__ __launch_bounds__(256) void pm_stage_input_kernel(const float* __restrict__ x, T* __restrict__ out,
                                                             int M, int n, int ld, PmStepHdr* hdr) {
  if (blockIdx.x == 0 && threadIdx.x == 0) hdr->loss = 0.f;
  const int64_t total = (int64_t)M * ld;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int m = (int)(i / ld), c = (int)(i % ld);
    stf(out + i, c < n ? x[(int64_t)m * n + c] : 0.f);
  }
}

// Softmax cross-entropy, mean over rows.  One wavefront per row; logits fp32 [M, ld], ld a multiple
// of 8.  Writes dz = (softmax - onehot)/M in the compute dtype (pad columns zero) and adds the row's
// loss / M to hdr->loss.  Two passes over the row: running (max, sum of exponentials) per lane,
// merged across the wave; then the gradient, eight columns per lane and access.
template <typename T>
__global__ __launch_bounds__(256) void pm_xent_kernel(const float* __restrict__ logits, const int32_t* __restrict__ y,
                                                      T* __restrict__ dz, int M, int C, int ld, PmStepHdr* hdr) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= M) return;
  const float* z = logits + (int64_t)row * ld;
  float mx = -3.0e38f, se = 0.f;
  const int C4 = C >> 2;
  for (int c = lane; c < C4; c += 64) {
    const float4 v = reinterpret_cast<const float4*>(z)[c];
    const float m4 = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
    if (m4 > mx) {
      se *= __expf(mx - m4);
      mx = m4;
    }
    se += __expf(v.x - mx) + __expf(v.y - mx) + __expf(v.z - mx) + __expf(v.w - mx);
  }
  for (int c = 4 * C4 + lane; c < C; c += 64) {
    const float v = z[c];
    if (v > mx) {
      se *= __expf(mx - v);
      mx = v;
    }
    se += __expf(v - mx);
  }
  const float mall = pm_wave_max(mx);
  se = pm_wave_sum(se * __expf(mx - mall));        // a lane that saw nothing has se = 0
  const int label = y[row];
  const bool label_ok = label >= 0 && label < C;      // an out-of-range label contributes nothing
  const float inv = 1.f / se, invM = 1.f / (float)M;
  for (int c = lane * 8; c < ld; c += 512) {
    float v[8], o[8];
    pm_ld8(z + c, v);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      o[e] = (c + e < C) ? (__expf(v[e] - mall) * inv - (c + e == label ? 1.f : 0.f)) * invM : 0.f;
    pm_st8(dz + (int64_t)row * ld + c, o);
  }
  if (lane == 0 && label_ok) atomicAdd(&hdr->loss, (logf(se) + mall - z[label]) * invM);
}

// The same for wide rows (thousands of classes): one block of 512 threads per row keeps the whole row
// in registers (up to NV float4 per thread), so the logits are read from memory once instead of once
// per pass; maximum, then sum of exponentials (block reductions through LDS), then the gradient.
template <typename T, int NV>
__global__ __launch_bounds__(512) void pm_xent_row_kernel(const float* __restrict__ logits, const int32_t* __restrict__ y,
                                                          T* __restrict__ dz, int M, int C, int ld, PmStepHdr* hdr) {
  __shared__ float red[2][8];
  const int row = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float* z = logits + (int64_t)row * ld;
  const int ld4 = ld >> 2;
  float4 v[NV];
  float mx = -3.0e38f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c4 = i * 512 + tid;
    v[i] = make_float4(-3.0e38f, -3.0e38f, -3.0e38f, -3.0e38f);
    if (c4 < ld4) {
      const float4 t = reinterpret_cast<const float4*>(z)[c4];
      const int c = 4 * c4;                      // pad columns (c >= C) take no part
      v[i].x = c < C ? t.x : -3.0e38f;
      v[i].y = c + 1 < C ? t.y : -3.0e38f;
      v[i].z = c + 2 < C ? t.z : -3.0e38f;
      v[i].w = c + 3 < C ? t.w : -3.0e38f;
    }
    mx = fmaxf(mx, fmaxf(fmaxf(v[i].x, v[i].y), fmaxf(v[i].z, v[i].w)));
  }
  mx = pm_wave_max(mx);
  if (lane == 0) red[0][wave] = mx;
  __syncthreads();
  float mall = red[0][0];
#pragma unroll
  for (int w = 1; w < 8; ++w) mall = fmaxf(mall, red[0][w]);
  float se = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    if (i * 512 < ld4) {                         // uniform over the block
      v[i].x = __expf(v[i].x - mall);            // masked entries: exp(-huge) = 0
      v[i].y = __expf(v[i].y - mall);
      v[i].z = __expf(v[i].z - mall);
      v[i].w = __expf(v[i].w - mall);
      se += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
  }
  se = pm_wave_sum(se);
  if (lane == 0) red[1][wave] = se;
  __syncthreads();
  se = 0.f;
#pragma unroll
  for (int w = 0; w < 8; ++w) se += red[1][w];
  const int label = y[row];
  const bool label_ok = label >= 0 && label < C;      // an out-of-range label contributes nothing
  const float inv = 1.f / se, invM = 1.f / (float)M, k = inv * invM;
  const int lab = label_ok ? label : -1;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c4 = i * 512 + tid;
    if (c4 < ld4) {
      const int c = 4 * c4;
      float4 o;
      o.x = v[i].x * k - (c == lab ? invM : 0.f);
      o.y = v[i].y * k - (c + 1 == lab ? invM : 0.f);
      o.z = v[i].z * k - (c + 2 == lab ? invM : 0.f);
      o.w = v[i].w * k - (c + 3 == lab ? invM : 0.f);
      pm_st4(dz + (int64_t)row * ld + c, o);
    }
  }
  if (tid == 0 && label_ok) atomicAdd(&hdr->loss, (logf(se) + mall - z[label]) * invM);
}

// softmax cross-entropy of M rows: row-resident kernel for wide rows, one wavefront per row otherwise
template <typename T>
inline void pm_xent_launch(hipStream_t st, const float* logits, const int32_t* y, T* dz, int M, int C, int ld,
                           PmStepHdr* hdr) {
  constexpr int NV = 16;
  if (C >= 2048 && (ld >> 2) <= NV * 512)
    hipLaunchKernelGGL((pm_xent_row_kernel<T, NV>), dim3(M), dim3(512), 0, st, logits, y, dz, M, C, ld, hdr);
  else
    hipLaunchKernelGGL((pm_xent_kernel<T>), dim3((M + 3) / 4), dim3(256), 0, st, logits, y, dz, M, C, ld, hdr);
}

// Mean squared error over all M*C outputs: dz = 2 (out - y) / (M C).
template <typename T>
__global__ __launch_bounds__(256) void pm_mse_kernel(const float* __restrict__ out, const float* __restrict__ y,
                                                     T* __restrict__ dz, int M, int C, int ld, PmStepHdr* hdr) {
  const int64_t total = (int64_t)M * ld;
  const float inv = 1.f / ((float)M * (float)C);
  float acc = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int m = (int)(i / ld), c = (int)(i % ld);
    float v = 0.f;
    if (c < C) {
      const float diff = out[i] - y[(int64_t)m * C + c];
      acc += diff * diff;
      v = 2.f * diff * inv;
    }
    stf(dz + i, v);
  }
  acc = pm_wave_sum(acc);
  if ((threadIdx.x & 63) == 0 && acc != 0.f) atomicAdd(&hdr->loss, acc * inv);
}

// Bias gradient db[n] = sum_m dz[m, n] into the fp32 gradient buffer (optionally accumulating).
// One wavefront per 64 columns would idle for narrow layers, so: block = 256 threads =
// 64 columns x 4 row groups, reduced through LDS.
template <typename T>
__global__ __launch_bounds__(256) void pm_bias_grad_kernel(const T* __restrict__ dz, float* __restrict__ db,
                                                           int M, int N, int ld, int accumulate) {
  const int col = blockIdx.x * 64 + (threadIdx.x & 63);
  const int rg = threadIdx.x >> 6;
  float acc = 0.f;
  if (col < N)
    for (int m = rg; m < M; m += 4) acc += ldf(dz + (int64_t)m * ld + col);
  __shared__ float part[4][64];
  part[rg][threadIdx.x & 63] = acc;
  __syncthreads();
  if (rg == 0 && col < N) {
    const float s = part[0][threadIdx.x] + part[1][threadIdx.x] + part[2][threadIdx.x] + part[3][threadIdx.x];
    db[col] = accumulate ? db[col] + s : s;
  }
}

// Bias gradient for many rows (token-rich microbatches): the rows are cut into chunks of 256 so
// that the whole chip reads dz once at full bandwidth; partial column sums meet in fp32 atomics
// (db must be zero, or hold the value to accumulate onto, when the kernel starts).
template <typename T>
__global__ __launch_bounds__(256) void pm_bias_grad_chunked_kernel(const T* __restrict__ dz, float* __restrict__ db,
                                                                   int M, int N, int ld) {
  const int col = blockIdx.x * 64 + (threadIdx.x & 63);
  const int rg = threadIdx.x >> 6;
  const int m0 = blockIdx.y * 256, m1 = m0 + 256 < M ? m0 + 256 : M;
  float acc = 0.f;
  if (col < N)
    for (int m = m0 + rg; m < m1; m += 4) acc += ldf(dz + (int64_t)m * ld + col);
  __shared__ float part[4][64];
  part[rg][threadIdx.x & 63] = acc;
  __syncthreads();
  if (rg == 0 && col < N)
    atomicAdd(db + col, part[0][threadIdx.x] + part[1][threadIdx.x] + part[2][threadIdx.x] + part[3][threadIdx.x]);
}

// dz <- dz * act'(z), element by element (n a multiple of 4): the activation derivative of a unit applied
// apart from the matrix product that produced dz, for the case where the two belong to different segments
// of a recomputing backward pass (the derivative must then wait for the rebuilt pre-activations).
template <typename T>
__global__ __launch_bounds__(256) void pm_act_bwd_apply_kernel(T* __restrict__ dz, const T* __restrict__ z, int act, int64_t n) {
  const int64_t n4 = n >> 2;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) {
    const float4 g = pm_ld4(dz + 4 * i), zz = pm_ld4(z + 4 * i);
    pm_st4(dz + 4 * i, make_float4(g.x * pm_act_bwd(zz.x, act), g.y * pm_act_bwd(zz.y, act), g.z * pm_act_bwd(zz.z, act),
                                   g.w * pm_act_bwd(zz.w, act)));
  }
}

__global__ __launch_bounds__(256) void pm_zero_f32_kernel(float* p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0.f;
}

// ---------------------------------------------------------------------------------------------
// Epilogues shared by the plain and the MFMA GEMMs.  acc is the fp32 contraction result for
// output element (i, j).
// ---------------------------------------------------------------------------------------------
// forward: z = acc + b[j]; stores z (compute dtype and/or fp32) and a = act(z)
template <typename T>
struct PmEpiFwd {
  static constexpr bool kColSumA = false;
  __device__ __forceinline__ bool wants_colsum() const { return false; }
  __device__ __forceinline__ void colsum(int, float) const {}
  PmWLoc<T> bias;   // the bias lives in the same ring slot as its weight matrix
  T* z; T* a; float* z32; int ld; int act;
  const T* b_;
  __device__ __forceinline__ void begin() { b_ = bias.get(); }
  __device__ __forceinline__ void operator()(int i, int j, float acc) const {
    const float zz = acc + ldf(b_ + j);
    const int64_t o = (int64_t)i * ld + j;
    if (z) stf(z + o, zz);
    if (z32) z32[o] = zz;
    if (a) stf(a + o, pm_act_fwd(zz, act));
  }
  // eight consecutive columns j .. j+7 (j a multiple of 8) of row i: 16-byte accesses.  pre8 requests what the
  // epilogue reads from memory; the caller issues it for several groups before it finishes the first one, so the
  // loads do not queue behind the stores of the group before (loads and stores complete in issue order).
  struct Pre { PmRaw8<T> b; };
  __device__ __forceinline__ Pre pre8(int, int j) const { Pre p; p.b.load(b_ + j); return p; }
  __device__ __forceinline__ void op8(int i, int j, const float* acc, const Pre& p) const {
    float zz[8], aa[8], bb[8];
    p.b.widen(bb);
#pragma unroll
    for (int e = 0; e < 8; ++e) zz[e] = acc[e] + bb[e];
    const int64_t o = (int64_t)i * ld + j;
    if (z) pm_st8(z + o, zz);
    if (z32) pm_st8(z32 + o, zz);
    if (a) {
      pm_act_fwd8(zz, aa, act);
      pm_st8(a + o, aa);
    }
  }
};
// backward data: dz_prev = acc * act'(z_prev)   (act == 0: dz_prev = acc, z_prev is not read)
template <typename T>
struct PmEpiBwdData {
  static constexpr bool kColSumA = false;
  __device__ __forceinline__ bool wants_colsum() const { return false; }
  __device__ __forceinline__ void colsum(int, float) const {}
  const T* zprev; T* dzprev; int ld; int act;
  __device__ __forceinline__ void begin() {}
  __device__ __forceinline__ void operator()(int i, int j, float acc) const {
    const int64_t o = (int64_t)i * ld + j;
    stf(dzprev + o, act ? acc * pm_act_bwd(ldf(zprev + o), act) : acc);
  }
  struct Pre { PmRaw8<T> zp; };
  __device__ __forceinline__ Pre pre8(int i, int j) const {
    Pre p;
    if (act) p.zp.load(zprev + (int64_t)i * ld + j);
    return p;
  }
  __device__ __forceinline__ void op8(int i, int j, const float* acc, const Pre& p) const {
    const int64_t o = (int64_t)i * ld + j;
    float out[8];
    if (act) {
      float zp[8];
      p.zp.widen(zp);
      pm_act_bwd8(acc, zp, out, act);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = acc[e];
    }
    pm_st8(dzprev + o, out);
  }
};
// backward weight: g[i, j] (+)= acc, fp32; db[i] (+)= column sum of the A operand (MFMA path only)
// (runs in table-driven launches: its accesses name the global address space, see pm_ldg16)
struct PmEpiBwdWeight {
  static constexpr bool kColSumA = true;
  float* g; int ld; int accumulate;
  float* db;   // bias gradient, or nullptr when a separate kernel produces it
  __device__ __forceinline__ bool wants_colsum() const { return db != nullptr; }
  __device__ __forceinline__ void colsum(int i, float s) const { db[i] = accumulate ? db[i] + s : s; }
  __device__ __forceinline__ void begin() {}
  __device__ __forceinline__ void operator()(int i, int j, float acc) const {
    const int64_t o = (int64_t)i * ld + j;
    g[o] = accumulate ? g[o] + acc : acc;
  }
  struct Pre { float o[8]; };
  __device__ __forceinline__ Pre pre8(int i, int j) const {
    Pre p;
    if (accumulate) pm_ld8_g(g + (int64_t)i * ld + j, p.o);
    return p;
  }
  __device__ __forceinline__ void op8(int i, int j, const float* acc, const Pre& p) const {
    const int64_t o = (int64_t)i * ld + j;
    float out[8];
    if (accumulate) {
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = p.o[e] + acc[e];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = acc[e];
    }
    pm_st8_g(g + o, out);
  }
};

// backward weight of a unit whose gradient is final after this product (one microbatch per step, no clipping):
// g[i, j] = acc as above, and then the block applies the update of its own tile of parameters - the Sec. 2.1
// recurrence with the T1 step size of Sec. 3.1, the delta accumulator and the corrected backward weights of
// Sec. 3.2, with the arithmetic of pm_fused_update_kernel - while other tiles of the launch still multiply.
// The update pass then leaves these parameters out.
struct PmEpiBwdWeightUpd {
  static constexpr bool kColSumA = true;
  static constexpr bool kTileUpdate = true;
  float* g; int ld;
  float* db;
  PmFuseUpd f;
  __device__ __forceinline__ bool wants_colsum() const { return db != nullptr; }
  __device__ __forceinline__ void colsum(int i, float s) const { db[i] = s; }
  __device__ __forceinline__ void begin() {}
  struct Pre {};
  __device__ __forceinline__ Pre pre8(int, int) const { return Pre(); }
  __device__ __forceinline__ void op8(int i, int j, const float* acc, const Pre&) const { pm_st8_g(g + (int64_t)i * ld + j, acc); }
  // single elements are never needed: the launch that uses this epilogue takes whole tiles only
  __device__ __forceinline__ void operator()(int, int, float) const {}

  // Parameters [i0, i0 + BI) x [j0, j0 + BJ) of the unit's matrix, by a block of NT threads that has stored their
  // gradients (and passed a barrier since).  A lane takes 8 consecutive parameters of U rows at a time and
  // requests all their state before it computes: with the accumulators dead there is room to keep 5 U 32-byte
  // loads per lane in flight, and what bounds this phase is memory latency times the bytes in flight.
  template <int BI, int BJ, int NT>
  __device__ __forceinline__ void update_tile(int i0, int j0) const {
    constexpr int LPR = BJ / 8, RPP = NT / LPR, U = 4;       // lanes per row, rows per pass of the block, rows per lane and pass
    static_assert(BI % (RPP * U) == 0, "tile rows");
    const PmLayerStep D = *f.step;
    const float lr = D.lr, corr = D.corr_next;
    const float gs = f.hdr->gscale[0], bc1 = f.hdr->bc1[0], bc2 = f.hdr->bc2[0];
    const bool ub_from_ring = (corr != 0.f) && (f.tau_b > 0);
    const int64_t wslot = (int64_t)D.write_slot * f.n_pad, ubslot = (int64_t)D.ub_slot * f.n_pad;
    const int r = (int)threadIdx.x / LPR, c8 = ((int)threadIdx.x % LPR) * 8;
    bool bad = false;
    for (int p = 0; p < BI; p += RPP * U) {
      float gr[U][8], w[U][8], v[U][8], d[U][8], s[U][8];
      int64_t o[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        o[u] = (int64_t)(i0 + p + u * RPP + r) * ld + j0 + c8;
        pm_ld8_g(g + o[u], gr[u]);
        pm_ld8_g(f.w + o[u], w[u]);
        pm_ld8_g(f.v + o[u], v[u]);
        pm_ld8_g(f.d + o[u], d[u]);
        if (f.opt == 1) pm_ld8_g(f.s + o[u], s[u]);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float wn[8], ubv[8];
        if (ub_from_ring) pm_ld8_g(f.ring + ubslot + o[u], ubv);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float ge = gr[u][e] * gs;
          float dw;
          if (f.opt == 0) {
            ge += f.wd * w[u][e];
            v[u][e] = f.beta1 * v[u][e] - lr * ge;
            dw = v[u][e];
          } else {
            v[u][e] = f.beta1 * v[u][e] + (1.f - f.beta1) * ge;
            s[u][e] = f.beta2 * s[u][e] + (1.f - f.beta2) * ge * ge;
            const float mh = v[u][e] * bc1;
            const float sh = s[u][e] * bc2;
            dw = -lr * (mh / (sqrtf(sh) + f.eps) + f.wd * w[u][e]);
          }
          wn[e] = w[u][e] + dw;
          d[u][e] = f.gamma * d[u][e] + (1.f - f.gamma) * dw;
          bad |= !(fabsf(wn[e]) <= 3.0e38f);
        }
        pm_st8_g(f.w + o[u], wn);
        pm_st8_g(f.v + o[u], v[u]);
        pm_st8_g(f.d + o[u], d[u]);
        if (f.opt == 1) pm_st8_g(f.s + o[u], s[u]);
        pm_st8_g(f.ring + wslot + o[u], wn);
        if (f.has_ub) {
#pragma unroll
          for (int e = 0; e < 8; ++e) ubv[e] = (ub_from_ring ? ubv[e] : wn[e]) - corr * d[u][e];
          pm_st8_g(f.ub + o[u], ubv);
        }
      }
    }
    if (bad) f.hdr->diverged = 1;
  }
};
// true for the epilogues whose products run faster on the rectangular 8-wave blocks inside a training step too (see
// PmBigTall / PmBigWide); specialised next to those epilogues
template <class E> struct pm_rect_tiles : std::false_type {};
// true for an epilogue with a tile-wide second phase (update_tile)
template <class E, class = void> struct pm_has_tile_update : std::false_type {};
template <class E> struct pm_has_tile_update<E, std::void_t<decltype(E::kTileUpdate)>> : std::true_type {};

// ---------------------------------------------------------------------------------------------
// Plain tiled GEMM  C[i, j] = sum_k A(i, k) * B(j, k)  with arbitrary strides; fp32 FMA.
// Used for fp32 contexts (tiny layers where launch latency dominates) and for any bf16 shape the
// MFMA kernel's alignment rules exclude.  16x16 outputs per block, K staged 16 at a time.
// ---------------------------------------------------------------------------------------------
template <typename TA, typename TB, class Epi>
__global__ __launch_bounds__(256) void pm_gemm_plain_kernel(int I, int J, int K,
                                                            const TA* __restrict__ A, int64_t sai, int64_t sak,
                                                            PmWLoc<TB> bloc, int64_t sbj, int64_t sbk,
                                                            Epi epi) {
  __shared__ float sA[16][17], sB[16][17];
  const TB* B = bloc.get();
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int i0 = blockIdx.y * 16, j0 = blockIdx.x * 16;
  float acc = 0.f;
  for (int k0 = 0; k0 < K; k0 += 16) {
    const int ia = i0 + ty, jb = j0 + ty, kk = k0 + tx;
    sA[ty][tx] = (ia < I && kk < K) ? ldf(A + ia * sai + kk * sak) : 0.f;
    sB[ty][tx] = (jb < J && kk < K) ? ldf(B + jb * sbj + kk * sbk) : 0.f;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) acc += sA[ty][k] * sB[tx][k];
    __syncthreads();
  }
  const int i = i0 + ty, j = j0 + tx;
  epi.begin();
  if (i < I && j < J) epi(i, j, acc);
}
