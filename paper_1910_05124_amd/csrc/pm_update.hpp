// Prologue (slot / step-size table), gradient norm and the fused PipeMare update pass.
#pragma once
#include "pm_common.hpp"

// ---------------------------------------------------------------------------------------------
// Prologue: one launch per optimizer step.  Reads the device step counter t, writes per unit the
// ring slots of the delayed reads (Sec. 2.1: versions t - tau_fwd,i and t - tau_bkwd,i, clamped
// to 0 during pipeline fill) and the rescheduled step size (Sec. 3.1, T1), then advances t.
// A single block so that the counter update is ordered after every table entry.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void pm_prologue_block(PmStepHdr* hdr, const PmLayerStatic* ls, PmLayerStep* ld, int L,
                                                  const PmSchedDev& sc, int par) {
  const long long t = hdr->t_next;
  const bool warm = t < sc.sync_warmup;            // synchronous warm-up (PipeMareW): no delays, no T1/T2
  const bool warm_next = t + 1 < sc.sync_warmup;
  const long long k = warm ? 0 : t - sc.sync_warmup;   // T1 counts from the switch
  double a_base;
  if (sc.kind == 0) {
    a_base = sc.base;
  } else if (sc.kind == 1) {
    a_base = sc.base * pow(sc.factor, (double)(t / sc.interval));
  } else {
    if (t < sc.interval) a_base = sc.init + (sc.base - sc.init) * ((double)t / (double)sc.interval);
    else a_base = t > 0 ? sc.base * sqrt((double)sc.interval / (double)t) : sc.base;
  }
  double p = 0.0;
  if (sc.K > 0 && !warm) {
    double f = (double)k / (double)sc.K;
    p = 1.0 - (f < 1.0 ? f : 1.0);
  }
  for (int l = threadIdx.x; l < L; l += blockDim.x) {
    const PmLayerStatic S = ls[l];
    PmLayerStep D;
    long long tf = warm ? 0 : S.tau_f, tb = warm ? 0 : S.tau_b;
    const long long tbn = warm_next ? 0 : S.tau_b;
    const long long tr = warm ? 0 : S.tau_r, trn = warm_next ? 0 : S.tau_r;
    if (sc.stoch && !warm) {
      // this step's delay of the unit's stage; both passes read that version (no discrepancy, no T2)
      tf = tb = pm_delay_from_u32(pm_counter_u32(sc.seed, t, S.stage, sc.P), sc.cdf + (size_t)(S.stage - 1) * sc.tau_max,
                                  sc.tau_max);
    }
    const long long vf = t - tf > 0 ? t - tf : 0;
    const long long vb = t - tb > 0 ? t - tb : 0;
    const long long vu = t + 1 - tbn > 0 ? t + 1 - tbn : 0;
    const long long vr = t - tr > 0 ? t - tr : 0;
    const long long vur = t + 1 - trn > 0 ? t + 1 - trn : 0;
    D.fwd_slot = (int32_t)(vf % S.R);
    D.bkwd_slot = (int32_t)(vb % S.R);
    D.write_slot = (int32_t)((t + 1) % S.R);
    D.ub_slot = (int32_t)(vu % S.R);
    double lr = a_base;
    if (sc.t1_enabled && p > 0.0) {
      const int tau = S.tau_f > 1 ? S.tau_f : 1;
      lr = a_base / pow((double)tau, p);
    }
    D.lr = (float)lr;
    D.corr_next = warm_next ? 0.f : S.corr;
    D.rec_slot = (int32_t)(vr % S.R);
    D.ur_slot = (int32_t)(vur % S.R);
    D.corr_r_next = warm_next ? 0.f : S.corr_r;
    D.rev = (int32_t)(t & 1);
    D.pad_[0] = D.pad_[1] = 0;
    ld[l] = D;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    hdr->t_used = t;
    hdr->t_next = t + 1;
    hdr->gnorm2[par] = 0.f;
    hdr->gscale[par] = (float)sc.gscale0;
    hdr->bc1[par] = (float)(1.0 / (1.0 - pow(sc.beta1, (double)(t + 1))));
    hdr->bc2[par] = (float)(1.0 / (1.0 - pow(sc.beta2, (double)(t + 1))));
  }
}

__global__ void pm_prologue_kernel(PmStepHdr* hdr, const PmLayerStatic* ls, PmLayerStep* ld, int L, PmSchedDev sc,
                                   int par) {
  pm_prologue_block(hdr, ls, ld, L, sc, par);
}

// First kernel of every microbatch: stages the fp32 input batch into the compute dtype (pad columns
// zero), clears the loss accumulator, and - in block 0, when L > 0, i.e. at the start of a
// minibatch - refreshes the step table (so the step costs one launch less).
template <typename T>
__global__ __launch_bounds__(256) void pm_begin_step_kernel(const float* __restrict__ x, T* __restrict__ out, int M,
                                                            int n, int ld_x, PmStepHdr* hdr, const PmLayerStatic* ls,
                                                            PmLayerStep* ld, int L, PmSchedDev sc, int par,
                                                            uint4* shared_fill, int64_t n_shared_fill) {
  if (blockIdx.x == 0) {
    if (L > 0) pm_prologue_block(hdr, ls, ld, L, sc, par);
    if (threadIdx.x == 0) hdr->loss = 0.f;
  }
  // the tensors that the chained forward / data-gradient launches of this microbatch pass from block to block
  // start as all-ones words ("not written yet", see pm_chain.hpp)
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_shared_fill; i += (int64_t)gridDim.x * blockDim.x)
    shared_fill[i] = make_uint4(~0u, ~0u, ~0u, ~0u);
  const int64_t total = (int64_t)M * ld_x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int m = (int)(i / ld_x), c = (int)(i % ld_x);
    stf(out + i, c < n ? x[(int64_t)m * n + c] : 0.f);
  }
}

// ---------------------------------------------------------------------------------------------
// Sum of squares over a flat fp32 array (global gradient norm for clipping, parameter norm for
// the divergence monitor): wavefront shuffles, one LDS stage, one atomic per block.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pm_sumsq_kernel(const float* __restrict__ x, int64_t n, float* out) {
  float acc = 0.f;
  const int64_t n4 = n >> 2;
  const float4* x4 = reinterpret_cast<const float4*>(x);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) {
    const float4 v = x4[i];
    acc += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  acc = pm_wave_sum(acc);
  __shared__ float part[4];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) atomicAdd(out, part[0] + part[1] + part[2] + part[3]);
}

// gscale <- (1/N) * min(1, clip / ||g/N||)
__global__ void pm_clip_scale_kernel(PmStepHdr* hdr, float clip, int par) {
  const float gn = sqrtf(hdr->gnorm2[par]) * hdr->gscale[par];
  if (gn > clip) hdr->gscale[par] *= clip / gn;
}

// ---------------------------------------------------------------------------------------------
// The fused update: ONE launch over the flat parameter space of all units.
//   g' = gscale * g (+ wd * w for SGD)
//   SGD momentum (App. B.3 form)  v <- beta v - lr_i g' ;  w <- w + v
//   AdamW                         m,s moments with bias correction; w <- w - lr_i (mhat/(sqrt(shat)+eps) + wd w)
//   delta <- gamma_i delta + (1 - gamma_i)(w_new - w)                 (Sec. 3.2, T2 accumulator)
//   ring[(t+1) mod R_i] <- round(w_new)                               (the version the forward reads later)
//   ub <- round(base - (tau_fwd,i - tau_bkwd,i) delta_new)            (Sec. 3.2, corrected backward weights
//        of the NEXT step; base = w_new when tau_bkwd = 0, else the stored version t+1-tau_bkwd)
//   ur <- round(base_r - (tau_fwd,i - tau_recomp,i) delta_new)        (App. on recompute, "T2 for Recompute":
//        corrected recompute weights of the NEXT step, only for units that keep such a buffer;
//        base_r = w_new when tau_recomp = 0, else the stored version t+1-tau_recomp)
// Each block owns PM_CHUNK (or half of it, see PmAcc) consecutive elements, all of one unit (units are
// padded to the chunk), so the per-unit scalars are wave-uniform.
// ---------------------------------------------------------------------------------------------
template <typename RT>
struct PmUpdArgs {
  const float* g;
  float* w;
  float* v;   // momentum, or Adam m
  float* s;   // Adam second moment
  float* d;   // delta
  RT* ring;
  RT* ub;
  RT* ur;     // corrected recompute weights (NULL when no unit keeps any)
  const int32_t* chunk_layer;
  const int32_t* blocks;   // NULL: block b of the grid takes block b of the flat space (or its mirror image); else the
                           // list of the blocks to visit (the rest was updated in the weight-gradient epilogues)
  const PmLayerStatic* ls;
  const PmLayerStep* ld;
  PmStepHdr* hdr;
  int par;    // which set of step scalars (step parity)
  float beta1, beta2, eps, wd;
};

// Element access pattern of one thread: G groups of 4 elements 1024 apart (a block of 256 threads covers
// 1024 G consecutive elements: a whole chunk, or half of one), so every load / store instruction of a
// wave covers one dense 1 KB (fp32) or 512 B (bf16) span.
// VAR 1: two groups, ordinary accesses (streams small enough to stay partly cached from step to step).
// VAR 2: ONE group, non-temporal loads and stores (streams of GBs).  Measured on an 8.7 GB pass of this
//        shape: one group per thread 5.80 TB/s, two 5.50, four 5.57; ordinary accesses 5.27-5.32.
template <int VAR> struct PmAcc;
template <bool NT, int G> struct PmAccSplit {
  static constexpr int GROUPS = G;
  static constexpr int PER_BLOCK = 1024 * G;
  static constexpr int N = 4 * G;       // elements per thread
  static __device__ __forceinline__ int64_t base(int tid) { return tid * 4; }
  typedef float __attribute__((ext_vector_type(4))) f4;
  typedef unsigned int __attribute__((ext_vector_type(2))) u2;
  static __device__ __forceinline__ float4 l4(const float4* p) {
    if (!NT) return *p;
    const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
  }
  static __device__ __forceinline__ void s4(float4* p, float4 v) {
    if (!NT) { *p = v; return; }
    f4 t; t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    __builtin_nontemporal_store(t, reinterpret_cast<f4*>(p));
  }
  static __device__ __forceinline__ uint2 l2(const uint2* p) {
    if (!NT) return *p;
    const u2 v = __builtin_nontemporal_load(reinterpret_cast<const u2*>(p));
    return make_uint2(v.x, v.y);
  }
  static __device__ __forceinline__ void s2(uint2* p, uint2 v) {
    if (!NT) { *p = v; return; }
    u2 t; t.x = v.x; t.y = v.y;
    __builtin_nontemporal_store(t, reinterpret_cast<u2*>(p));
  }
  static __device__ __forceinline__ void ld(const float* p, float* x) {
#pragma unroll
    for (int k = 0; k < G; ++k) {
      const float4 a = l4(reinterpret_cast<const float4*>(p + 1024 * k));
      x[4 * k + 0] = a.x; x[4 * k + 1] = a.y; x[4 * k + 2] = a.z; x[4 * k + 3] = a.w;
    }
  }
  static __device__ __forceinline__ void ld(const bf16_t* p, float* x) {
#pragma unroll
    for (int k = 0; k < G; ++k) {
      const uint2 a = l2(reinterpret_cast<const uint2*>(p + 1024 * k));
      x[4 * k + 0] = __uint_as_float(a.x << 16); x[4 * k + 1] = __uint_as_float(a.x & 0xffff0000u);
      x[4 * k + 2] = __uint_as_float(a.y << 16); x[4 * k + 3] = __uint_as_float(a.y & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void st(float* p, const float* x) {
#pragma unroll
    for (int k = 0; k < G; ++k)
      s4(reinterpret_cast<float4*>(p + 1024 * k), make_float4(x[4 * k], x[4 * k + 1], x[4 * k + 2], x[4 * k + 3]));
  }
  static __device__ __forceinline__ void st(bf16_t* p, const float* x) {
#pragma unroll
    for (int k = 0; k < G; ++k) {
      uint2 a;
      a.x = pm_pack_bf16(x[4 * k], x[4 * k + 1]);
      a.y = pm_pack_bf16(x[4 * k + 2], x[4 * k + 3]);
      s2(reinterpret_cast<uint2*>(p + 1024 * k), a);
    }
  }
};
template <> struct PmAcc<1> : PmAccSplit<false, 2> {};
template <> struct PmAcc<2> : PmAccSplit<true, 1> {};

template <typename RT, int OPT, int VAR>
__global__ __launch_bounds__(256) void pm_fused_update_kernel(PmUpdArgs<RT> a) {
  using X = PmAcc<VAR>;
  constexpr int NE = X::N;
  static_assert(PM_CHUNK % X::PER_BLOCK == 0, "a block covers a whole chunk or a whole fraction of one");
  // Blocks are walked in opposite directions on alternate steps: the pass streams more state than the
  // 256 MB last-level cache holds, so what survives there from the previous pass is its tail, and the
  // next pass starts with exactly that part instead of evicting it before reaching it.
  // (the direction comes from this step's table, which is not rewritten while the pass runs)
  const int64_t pos = a.ld[0].rev ? (int64_t)(gridDim.x - 1 - blockIdx.x) : (int64_t)blockIdx.x;
  const int64_t blk = a.blocks ? (int64_t)a.blocks[pos] : pos;
  const int64_t e = blk * X::PER_BLOCK + X::base(threadIdx.x);
  // the streams whose addresses need no table go out first; the table reads overlap their latency
  float g[NE], w[NE], v[NE], d[NE], s[NE], wn[NE], ubv[NE];
  X::ld(a.g + e, g);
  X::ld(a.w + e, w);
  X::ld(a.v + e, v);
  X::ld(a.d + e, d);
  if (OPT == 1) X::ld(a.s + e, s);
  const int l = a.chunk_layer[blk / (PM_CHUNK / X::PER_BLOCK)];
  const PmLayerStatic S = a.ls[l];
  const PmLayerStep D = a.ld[l];
  // S.corr != 0 says the backward reads the corrected buffer at all; D.corr_next is the coefficient
  // of the step that will read it (0 while that step is still in the synchronous warm-up)
  const float lr = D.lr, gam = S.gamma, corr = D.corr_next;
  const bool has_ub = S.corr != 0.f;
  const float gs = a.hdr->gscale[a.par];
  const int64_t rel = e - S.off;
  const bool ub_from_ring = (corr != 0.f) && (S.tau_b > 0);
  if (ub_from_ring) X::ld(a.ring + S.ring_off + (int64_t)D.ub_slot * S.n_pad + rel, ubv);

  bool bad = false;
#pragma unroll
  for (int j = 0; j < NE; ++j) {
    float gj = g[j] * gs;
    float dw;   // w_{t+1} - w_t, kept as computed (not re-derived by subtraction) so delta keeps its low bits
    if (OPT == 0) {
      gj += a.wd * w[j];
      v[j] = a.beta1 * v[j] - lr * gj;
      dw = v[j];
    } else {
      v[j] = a.beta1 * v[j] + (1.f - a.beta1) * gj;
      s[j] = a.beta2 * s[j] + (1.f - a.beta2) * gj * gj;
      const float mh = v[j] * a.hdr->bc1[a.par];
      const float sh = s[j] * a.hdr->bc2[a.par];
      dw = -lr * (mh / (sqrtf(sh) + a.eps) + a.wd * w[j]);
    }
    wn[j] = w[j] + dw;
    d[j] = gam * d[j] + (1.f - gam) * dw;
    bad |= !(fabsf(wn[j]) <= 3.0e38f);
  }
  X::st(a.w + e, wn);
  X::st(a.v + e, v);
  X::st(a.d + e, d);
  if (OPT == 1) X::st(a.s + e, s);
  X::st(a.ring + S.ring_off + (int64_t)D.write_slot * S.n_pad + rel, wn);
  if (has_ub) {
#pragma unroll
    for (int j = 0; j < NE; ++j) ubv[j] = (ub_from_ring ? ubv[j] : wn[j]) - corr * d[j];
    X::st(a.ub + e, ubv);
  }
  if (S.corr_r != 0.f) {        // block-uniform; the ring slot read here is never the one written above (tau_recomp >= 1)
    const float cr = D.corr_r_next;
    const bool ur_from_ring = (cr != 0.f) && (S.tau_r > 0);
    if (ur_from_ring) X::ld(a.ring + S.ring_off + (int64_t)D.ur_slot * S.n_pad + rel, ubv);
#pragma unroll
    for (int j = 0; j < NE; ++j) ubv[j] = (ur_from_ring ? ubv[j] : wn[j]) - cr * d[j];
    X::st(a.ur + e, ubv);
  }
  if (bad) a.hdr->diverged = 1;
}

// Fill every ring slot and the corrected-weight buffer of all units with the initial weights.
template <typename RT>
__global__ __launch_bounds__(256) void pm_init_ring_kernel(const float* __restrict__ w, RT* ring, RT* ub, RT* ur,
                                                           const int32_t* chunk_layer,
                                                           const PmLayerStatic* ls) {
  const int c = blockIdx.x;
  const PmLayerStatic S = ls[chunk_layer[c]];
  const int64_t e = (int64_t)c * PM_CHUNK + threadIdx.x * 8;
  float x[8];
  pm_ld8(w + e, x);
  pm_st8(ub + e, x);
  if (ur) pm_st8(ur + e, x);
  for (int r = 0; r < S.R; ++r) pm_st8(ring + S.ring_off + (int64_t)r * S.n_pad + (e - S.off), x);
}
