// Shared device-side types of the PipeMare step library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned short bf16_t;   // raw bfloat16 bits

constexpr int PM_CHUNK = 2048;   // elements of the flat parameter space handled by one update block
constexpr int PM_ALIGN = 256;    // byte alignment of every arena region

// Static per-unit description, written once by pm_create.
struct PmLayerStatic {
  int64_t off;       // element offset of the unit in the flat fp32 arrays (multiple of PM_CHUNK)
  int64_t n_pad;     // padded element count (multiple of PM_CHUNK) = ring slot stride
  int64_t ring_off;  // element offset of slot 0 of this unit in the ring
  int32_t R;         // ring slots = tau_fwd + 1
  int32_t tau_f;
  int32_t tau_b;
  int32_t stage;
  float gamma;       // decay of the delta accumulator (T2)
  float corr;        // tau_fwd - tau_bkwd if the correction is active, else 0
  int32_t tau_r;     // recomputation delay (App. on recompute); equals tau_b when nothing is recomputed
  float corr_r;      // tau_fwd - tau_recomp if the unit keeps corrected recompute weights of its own, else 0
};

// Per-step values for a unit, rewritten by the prologue kernel from the device step counter.
struct PmLayerStep {
  int32_t fwd_slot;    // (max(t - tau_fwd, 0)) mod R
  int32_t bkwd_slot;   // (max(t - tau_bkwd, 0)) mod R
  int32_t write_slot;  // (t + 1) mod R
  int32_t ub_slot;     // (max(t + 1 - tau_bkwd, 0)) mod R : base of the next corrected weights
  float lr;            // alpha_{t,i}
  float corr_next;     // T2 coefficient of the NEXT step's corrected weights (0 during synchronous warm-up)
  int32_t rec_slot;    // (max(t - tau_recomp, 0)) mod R : version the recomputation reads when it needs no correction
  int32_t ur_slot;     // (max(t + 1 - tau_recomp, 0)) mod R : base of the next corrected recompute weights
  float corr_r_next;   // coefficient of the NEXT step's corrected recompute weights (0 during synchronous warm-up)
  int32_t rev;         // t mod 2: direction in which this step's update pass walks the parameter chunks
  int32_t pad_[2];
};

// The step table and the per-step scalars exist twice (index = step parity): the update of step t,
// which may run on the library's second stream, reads set t&1 while the first kernel of step t+1
// already writes set (t+1)&1.
struct PmStepHdr {
  long long t_next;    // optimizer steps completed = index of the next step
  long long t_used;    // index of the step the tables were last computed for
  float loss;          // accumulated by the loss kernel
  int32_t diverged;    // set when a non-finite weight is written
  float pnorm2;        // scratch for pm_stats
  int32_t chain_err;   // set (sticky) when a block of a chained launch gave up waiting for its producers
  float gnorm2[2];     // sum of squares of the accumulated gradients (clipping only)
  float gscale[2];     // factor applied to the gradient buffer inside the update
  float bc1[2], bc2[2];  // Adam bias corrections 1/(1-beta^(t+1))
};

// What the weight-gradient product of a unit needs to apply that unit's update (Sec. 2.1 recurrence with the T1
// step size of Sec. 3.1, the delta accumulator and the corrected backward weights of Sec. 3.2) in the epilogue of
// its own tiles.  Pointers address the unit's weight matrix (element 0 = row 0, column 0).
struct PmFuseUpd {
  float* w;                   // master weights
  float* v;                   // momentum, or Adam's first moment
  float* s;                   // Adam's second moment
  float* d;                   // delta
  bf16_t* ring;               // slot 0 of the unit's ring
  bf16_t* ub;                 // corrected backward weights
  const PmLayerStep* step;    // the unit's entry of the step table
  PmStepHdr* hdr;
  int64_t n_pad;              // ring slot stride
  float gamma, beta1, beta2, eps, wd;
  int32_t opt;                // 0: SGD with momentum, 1: AdamW
  int32_t has_ub, tau_b;
};

struct PmSchedDev {
  int32_t kind;
  double base, init, factor;
  long long interval, K;
  int32_t t1_enabled;
  double beta1, beta2;
  double gscale0;      // 1 / N (mean over microbatches)
  long long sync_warmup;  // E_w: steps t < E_w run with all delays 0 and the base step size
  // Hogwild-style stochastic delays (App. "Hogwild! asynchrony"): every step draws a delay per stage
  int32_t stoch;            // 1: on
  int32_t tau_max;          // delays lie in 0 .. tau_max; every ring has tau_max + 1 slots
  int32_t P;                // stages
  unsigned long long seed;
  const uint32_t* cdf;      // device: per stage tau_max thresholds T[k] = floor(2^32 P(delay <= k))
};

// 32 random bits for (step t, stage i of P), i 1-based: output number t * P + i of the SplitMix64
// generator (Steele, Lea, Flood 2014) started at `seed`, upper half.  A pure function, the same on
// host and device.
__host__ __device__ inline uint32_t pm_counter_u32(unsigned long long seed, long long t, int i, int P) {
  unsigned long long z = seed + (unsigned long long)(t * P + i) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  return (uint32_t)(z >> 32);
}
// delay = number of thresholds the draw exceeds (the table is non-decreasing)
__host__ __device__ inline int pm_delay_from_u32(uint32_t r, const uint32_t* T, int tau_max) {
  int d = 0;
  for (int k = 0; k < tau_max; ++k) d += r > T[k];
  return d;
}

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round-to-nearest-even, NaN kept quiet: the gfx950 conversion instruction (v_cvt_pk_bf16_f32, two
// values per instruction, no branches), reached through the compiler's own float -> bfloat conversion
typedef float pm_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 pm_bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// (lo, hi) -> two bf16 in one 32-bit word, lo in the low half
__device__ __forceinline__ uint32_t pm_pack_bf16(float lo, float hi) {
  const pm_f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, pm_bf16x2));
}

__device__ __forceinline__ float ldf(const float* p) { return *p; }
__device__ __forceinline__ float ldf(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void stf(float* p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// eight consecutive elements, 16-byte aligned: two float4 / one uint4
__device__ __forceinline__ void pm_ld8(const float* p, float* x) {
  const float4 a = reinterpret_cast<const float4*>(p)[0];
  const float4 b = reinterpret_cast<const float4*>(p)[1];
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
__device__ __forceinline__ void pm_ld8(const bf16_t* p, float* x) {
  const uint4 a = *reinterpret_cast<const uint4*>(p);
  x[0] = __uint_as_float(a.x << 16); x[1] = __uint_as_float(a.x & 0xffff0000u);
  x[2] = __uint_as_float(a.y << 16); x[3] = __uint_as_float(a.y & 0xffff0000u);
  x[4] = __uint_as_float(a.z << 16); x[5] = __uint_as_float(a.z & 0xffff0000u);
  x[6] = __uint_as_float(a.w << 16); x[7] = __uint_as_float(a.w & 0xffff0000u);
}
__device__ __forceinline__ void pm_st8(float* p, const float* x) {
  reinterpret_cast<float4*>(p)[0] = make_float4(x[0], x[1], x[2], x[3]);
  reinterpret_cast<float4*>(p)[1] = make_float4(x[4], x[5], x[6], x[7]);
}
__device__ __forceinline__ void pm_st8(bf16_t* p, const float* x) {
  uint4 o;
  o.x = pm_pack_bf16(x[0], x[1]);
  o.y = pm_pack_bf16(x[2], x[3]);
  o.z = pm_pack_bf16(x[4], x[5]);
  o.w = pm_pack_bf16(x[6], x[7]);
  *reinterpret_cast<uint4*>(p) = o;
}
// Eight consecutive elements as they come from memory: requesting and widening are separate steps, so that several
// requests can be in flight before the first one is waited for (widening bf16 right behind its load would wait).
template <typename T> struct PmRaw8;
template <> struct PmRaw8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p) { a = reinterpret_cast<const float4*>(p)[0]; b = reinterpret_cast<const float4*>(p)[1]; }
  __device__ __forceinline__ void widen(float* x) const { x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w; }
};
template <> struct PmRaw8<bf16_t> {
  uint4 a;
  __device__ __forceinline__ void load(const bf16_t* p) { a = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void widen(float* x) const {
    x[0] = __uint_as_float(a.x << 16); x[1] = __uint_as_float(a.x & 0xffff0000u);
    x[2] = __uint_as_float(a.y << 16); x[3] = __uint_as_float(a.y & 0xffff0000u);
    x[4] = __uint_as_float(a.z << 16); x[5] = __uint_as_float(a.z & 0xffff0000u);
    x[6] = __uint_as_float(a.w << 16); x[7] = __uint_as_float(a.w & 0xffff0000u);
  }
};

// Eight elements / 16 bytes of operands through pointers known to address device memory.  A pointer read from a
// table in device memory is generic to the compiler, which then emits flat accesses: slower to issue, and counted
// with the LDS operations, so that no wait of a software pipeline can be a counted one.
typedef float __attribute__((ext_vector_type(4))) pm_vf4;
typedef unsigned int __attribute__((ext_vector_type(4))) pm_vu4;
#define PM_GLOBAL __attribute__((address_space(1)))
// 16 bytes of bf16 operands
__device__ __forceinline__ uint4 pm_ldg16(const bf16_t* p) {
  return __builtin_bit_cast(uint4, *(const pm_vu4 PM_GLOBAL*)p);
}
__device__ __forceinline__ void pm_ld8_g(const float* p, float* x) {
  const pm_vf4 PM_GLOBAL* q = (const pm_vf4 PM_GLOBAL*)p;
  const pm_vf4 a = q[0], b = q[1];
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
__device__ __forceinline__ void pm_ld8_g(const bf16_t* p, float* x) {
  const pm_vu4 a = *(const pm_vu4 PM_GLOBAL*)p;
  x[0] = __uint_as_float(a.x << 16); x[1] = __uint_as_float(a.x & 0xffff0000u);
  x[2] = __uint_as_float(a.y << 16); x[3] = __uint_as_float(a.y & 0xffff0000u);
  x[4] = __uint_as_float(a.z << 16); x[5] = __uint_as_float(a.z & 0xffff0000u);
  x[6] = __uint_as_float(a.w << 16); x[7] = __uint_as_float(a.w & 0xffff0000u);
}
__device__ __forceinline__ void pm_st8_g(float* p, const float* x) {
  pm_vf4 PM_GLOBAL* q = (pm_vf4 PM_GLOBAL*)p;
  pm_vf4 a, b;
  a.x = x[0]; a.y = x[1]; a.z = x[2]; a.w = x[3]; b.x = x[4]; b.y = x[5]; b.z = x[6]; b.w = x[7];
  q[0] = a;
  q[1] = b;
}
__device__ __forceinline__ void pm_st8_g(bf16_t* p, const float* x) {
  pm_vu4 o;
  o.x = pm_pack_bf16(x[0], x[1]);
  o.y = pm_pack_bf16(x[2], x[3]);
  o.z = pm_pack_bf16(x[4], x[5]);
  o.w = pm_pack_bf16(x[6], x[7]);
  *(pm_vu4 PM_GLOBAL*)p = o;
}

// four consecutive elements: one float4 / one uint2
__device__ __forceinline__ float4 pm_ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 pm_ld4(const bf16_t* p) {
  const uint2 a = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(a.x << 16), __uint_as_float(a.x & 0xffff0000u), __uint_as_float(a.y << 16),
                     __uint_as_float(a.y & 0xffff0000u));
}
__device__ __forceinline__ void pm_st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void pm_st4(bf16_t* p, float4 v) {
  uint2 o;
  o.x = pm_pack_bf16(v.x, v.y);
  o.y = pm_pack_bf16(v.z, v.w);
  *reinterpret_cast<uint2*>(p) = o;
}

// Where a weight matrix lives this step: base + slot * stride (slot read from the device step
// table so that a captured graph stays valid from step to step); slot == nullptr -> base.
template <typename T>
struct PmWLoc {
  const T* base;
  const int32_t* slot;
  int64_t stride;
  __device__ __forceinline__ const T* get() const { return slot ? base + (int64_t)(*slot) * stride : base; }
};

// erf by the classical 5-term rational/exponential approximation (Abramowitz & Stegun 7.1.26,
// |error| <= 1.5e-7): about a third of the instructions of the library erff, which matters in
// GEMM epilogues that evaluate it once per output element.  Returns erf(x) and exp(-x^2).
__device__ __forceinline__ float pm_erf(float x, float* exp_mx2) {
  const float ax = fabsf(x);
  const float t = __frcp_rn(fmaf(0.3275911f, ax, 1.f));
  const float e = __expf(-ax * ax);
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float r = fmaf(-p * t, e, 1.f);
  *exp_mx2 = e;
  return copysignf(r, x);
}
__device__ __forceinline__ float pm_act_fwd(float z, int act) {
  if (act == 1) return z > 0.f ? z : 0.f;
  if (act == 2) {
    float e;
    return 0.5f * z * (1.f + pm_erf(z * 0.70710678118654752f, &e));
  }
  return z;
}
__device__ __forceinline__ float pm_act_bwd(float z, int act) {
  if (act == 1) return z > 0.f ? 1.f : 0.f;
  if (act == 2) {
    float e;   // exp(-z^2/2), shared between the two terms
    const float cdf = 0.5f * (1.f + pm_erf(z * 0.70710678118654752f, &e));
    return cdf + z * e * 0.39894228040143268f;
  }
  return 1.f;
}

// eight values at once with the (wave-uniform) choice of the activation taken once, not per element
__device__ __forceinline__ void pm_act_fwd8(const float* z, float* a, int act) {
  if (act == 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = z[e] > 0.f ? z[e] : 0.f;
  } else if (act == 2) {
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = pm_act_fwd(z[e], 2);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = z[e];
  }
}
// out[e] = acc[e] * act'(z[e])
__device__ __forceinline__ void pm_act_bwd8(const float* acc, const float* z, float* out, int act) {
  if (act == 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = z[e] > 0.f ? acc[e] : 0.f;
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = acc[e] * pm_act_bwd(z[e], act);
  }
}

__device__ __forceinline__ float pm_wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float pm_wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
