// 3x3 convolution stages (zero padding 1, stride 1 or 2) with a folded per-channel affine, ReLU and
// parameter-free residual shortcuts, for the ResNet-shaped stages of the training step.  gfx950.
//
// Activations are NHWC in the compute dtype T; pixel index p = (b * H + y) * W + x.  A convolution
// unit's parameters lie in one ring slot: W [C_out][tap = 3 dy + dx][C_in], then scale [C_out],
// shift [C_out].  forward:  z = conv(x, W_fwd);  a = scale_fwd * z + shift_fwd (+ shortcut);  y = relu(a).
// backward (two weight sets, Sec. 2.1): da = dy * [y > 0];  d scale = sum da * z;  d shift = sum da;
// dz = da * scale_bkwd;  dW = correlation of dz with the stored input;  d input = transposed convolution
// of dz with W_bkwd (+ da of the block's second convolution through the shortcut).
//
// The convolutions are implicit GEMMs on v_mfma_f32_32x32x16_bf16 (bf16, channel counts multiples
// of 16): no patch matrix is ever written.  Every product is computed transposed, channels on the
// MFMA rows and pixels on the MFMA columns, so a lane owns one pixel and 4 consecutive channels per
// accumulator group: the gathered operand (8 consecutive channels of one input pixel of one tap) is
// a single 16-byte global load, and results leave as 8-byte pieces of NHWC rows.
//   forward   out^T [co][pixel]    = sum_{tap, ci} W[co][tap][ci] x[pixel + tap][ci]
//   data      dx^T  [ci][in pixel] = sum_{tap, co} W[co][tap][ci] dz[pixel - tap][co]   (W^T via LDS transpose loads)
//   weight    dW    [co][tap, ci]  = sum_{pixel}   dz[pixel][co] x[pixel + tap][ci]     (both operands via LDS transpose loads)
// These layers are bound by launch latency and HBM traffic, not by MFMA rate (channel counts of
// 16 .. 64 give 70 - 300 flop per byte of activation traffic), so the kernels favour simplicity:
// no block-level barriers in the hot loops.  fp32 contexts and odd channel counts (the 3-channel
// input convolution) use the plain kernels below.
#pragma once
#include "pm_common.hpp"
#include "pm_attn_mfma.hpp"

struct PmConvGeom {
  int B, H, W, Cin, Cout, stride, Ho, Wo;   // input H x W, output Ho x Wo
};

// Shortcut added to a block's second convolution: the block input (Hs x Ws x Cs), subsampled by
// `stride` with the new channels zero.  src == nullptr: none.
template <typename T>
struct PmShortcut {
  const T* src;
  int Hs, Ws, Cs, stride;
  __device__ __forceinline__ float at(int b, int oy, int ox, int c) const {
    if (!src || c >= Cs) return 0.f;
    return ldf(src + (((int64_t)b * Hs + oy * stride) * Ws + ox * stride) * Cs + c);
  }
};

// Gradient that reaches a block's input through its shortcut: da of the block's second convolution
// (Ho x Wo x Co) placed on every stride-th input pixel, first Cin channels.
template <typename T>
struct PmShortcutBwd {
  const T* da;
  int Ho, Wo, Co, stride;
  __device__ __forceinline__ float at(int b, int iy, int ix, int c) const {
    if (!da) return 0.f;
    if (stride == 2 && ((iy | ix) & 1)) return 0.f;
    return ldf(da + (((int64_t)b * Ho + iy / stride) * Wo + ix / stride) * Co + c);
  }
};

// ---------------------------------------------------------------------------------------------
// plain kernels (any T, any channel counts)
// ---------------------------------------------------------------------------------------------
// NCHW fp32 image batch -> NHWC compute dtype
template <typename T>
__global__ __launch_bounds__(256) void pm_image_stage_kernel(const float* __restrict__ x, T* __restrict__ out, int B, int C,
                                                             int H, int W) {
  const int64_t total = (int64_t)B * H * W * C;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(i % C);
    const int64_t p = i / C;
    const int xw = (int)(p % W), yh = (int)((p / W) % H), b = (int)(p / ((int64_t)W * H));
    stf(out + i, x[(((int64_t)b * C + c) * H + yh) * W + xw]);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void pm_conv_fwd_plain_kernel(PmConvGeom g, const T* __restrict__ x, PmWLoc<T> wloc,
                                                                PmShortcut<T> sc, T* __restrict__ z, T* __restrict__ y) {
  const T* Wt = wloc.get();
  const T* scale = Wt + (int64_t)g.Cout * 9 * g.Cin;
  const T* shift = scale + g.Cout;
  const int64_t total = (int64_t)g.B * g.Ho * g.Wo * g.Cout;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int co = (int)(i % g.Cout);
    const int64_t p = i / g.Cout;
    const int ox = (int)(p % g.Wo), oy = (int)((p / g.Wo) % g.Ho), b = (int)(p / ((int64_t)g.Wo * g.Ho));
    float acc = 0.f;
    for (int dy = 0; dy < 3; ++dy) {
      const int iy = oy * g.stride + dy - 1;
      if (iy < 0 || iy >= g.H) continue;
      for (int dx = 0; dx < 3; ++dx) {
        const int ix = ox * g.stride + dx - 1;
        if (ix < 0 || ix >= g.W) continue;
        const T* xr = x + (((int64_t)b * g.H + iy) * g.W + ix) * g.Cin;
        const T* wr = Wt + ((int64_t)co * 9 + dy * 3 + dx) * g.Cin;
        for (int ci = 0; ci < g.Cin; ++ci) acc += ldf(xr + ci) * ldf(wr + ci);
      }
    }
    const float a = ldf(scale + co) * acc + ldf(shift + co) + sc.at(b, oy, ox, co);
    stf(z + i, acc);
    stf(y + i, a > 0.f ? a : 0.f);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void pm_conv_dgrad_plain_kernel(PmConvGeom g, const T* __restrict__ dz, PmWLoc<T> wloc,
                                                                  PmShortcutBwd<T> sb, T* __restrict__ dx) {
  const T* Wt = wloc.get();
  const int64_t total = (int64_t)g.B * g.H * g.W * g.Cin;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int ci = (int)(i % g.Cin);
    const int64_t p = i / g.Cin;
    const int ix = (int)(p % g.W), iy = (int)((p / g.W) % g.H), b = (int)(p / ((int64_t)g.W * g.H));
    float acc = 0.f;
    for (int dy = 0; dy < 3; ++dy) {
      const int ny = iy + 1 - dy;
      if (ny < 0 || ny % g.stride) continue;
      const int oy = ny / g.stride;
      if (oy >= g.Ho) continue;
      for (int dxx = 0; dxx < 3; ++dxx) {
        const int nx = ix + 1 - dxx;
        if (nx < 0 || nx % g.stride) continue;
        const int ox = nx / g.stride;
        if (ox >= g.Wo) continue;
        const T* dr = dz + (((int64_t)b * g.Ho + oy) * g.Wo + ox) * g.Cout;
        const T* wr = Wt + (int64_t)(dy * 3 + dxx) * g.Cin + ci;
        for (int co = 0; co < g.Cout; ++co) acc += ldf(dr + co) * ldf(wr + (int64_t)co * 9 * g.Cin);
      }
    }
    stf(dx + i, acc + sb.at(b, iy, ix, ci));
  }
}

// one block per weight element (co, tap, ci): sum over all output pixels
template <typename T>
__global__ __launch_bounds__(256) void pm_conv_wgrad_plain_kernel(PmConvGeom g, const T* __restrict__ dz,
                                                                  const T* __restrict__ x, float* __restrict__ dW,
                                                                  int accumulate) {
  const int e = blockIdx.x;
  const int ci = e % g.Cin, tap = (e / g.Cin) % 9, co = e / (9 * g.Cin);
  const int dy = tap / 3, dxx = tap % 3;
  const int64_t npix = (int64_t)g.B * g.Ho * g.Wo;
  float acc = 0.f;
  for (int64_t p = threadIdx.x; p < npix; p += blockDim.x) {
    const int ox = (int)(p % g.Wo), oy = (int)((p / g.Wo) % g.Ho), b = (int)(p / ((int64_t)g.Wo * g.Ho));
    const int iy = oy * g.stride + dy - 1, ix = ox * g.stride + dxx - 1;
    if (iy < 0 || iy >= g.H || ix < 0 || ix >= g.W) continue;
    acc += ldf(dz + p * g.Cout + co) * ldf(x + (((int64_t)b * g.H + iy) * g.W + ix) * g.Cin + ci);
  }
  acc = pm_wave_sum(acc);
  __shared__ float part[4];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    const float s = part[0] + part[1] + part[2] + part[3];
    dW[e] = accumulate ? dW[e] + s : s;
  }
}

// da = dy * [y > 0];  dz = da * scale_bkwd;  dscale += sum da * z;  dshift += sum da   (fp32 atomics;
// the caller zeroes dscale / dshift at the start of a minibatch).  Thread t of a block always sees
// channel (t * 8 .. t * 8 + 7) mod C because a block's span is a multiple of C elements.
template <typename T>
__global__ __launch_bounds__(256) void pm_conv_affine_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ y,
                                                                 const T* __restrict__ z, PmWLoc<T> scale_bkwd,
                                                                 T* __restrict__ da, T* __restrict__ dz,
                                                                 float* __restrict__ dscale, float* __restrict__ dshift,
                                                                 int64_t total, int C) {
  __shared__ float red[2][256];
  for (int j = threadIdx.x; j < 2 * 256; j += 256) (&red[0][0])[j] = 0.f;
  __syncthreads();
  const T* sbk = scale_bkwd.get();
  const int c0 = (threadIdx.x * 8) % C;            // C is a multiple of 8 and divides 2048
  float s8[8], as[8], at[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    s8[e] = ldf(sbk + c0 + e);
    as[e] = 0.f;
    at[e] = 0.f;
  }
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8; i < total; i += (int64_t)gridDim.x * 2048) {
    float a[8], b[8], c[8], o1[8], o2[8];
    pm_ld8(dy + i, a);
    pm_ld8(y + i, b);
    pm_ld8(z + i, c);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float d = b[e] > 0.f ? a[e] : 0.f;
      o1[e] = d;
      o2[e] = d * s8[e];
      as[e] += d * c[e];
      at[e] += d;
    }
    pm_st8(da + i, o1);
    pm_st8(dz + i, o2);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    atomicAdd(&red[0][c0 + e], as[e]);
    atomicAdd(&red[1][c0 + e], at[e]);
  }
  __syncthreads();
  for (int j = threadIdx.x; j < C; j += 256) {
    atomicAdd(dscale + j, red[0][j]);
    atomicAdd(dshift + j, red[1][j]);
  }
}

// global average pool: out[b][c] = mean over the HW pixels
template <typename T>
__global__ __launch_bounds__(256) void pm_pool_fwd_kernel(const T* __restrict__ y, T* __restrict__ out, int B, int HW, int C) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * C) return;
  const int b = i / C, c = i % C;
  float acc = 0.f;
  for (int p = 0; p < HW; ++p) acc += ldf(y + ((int64_t)b * HW + p) * C + c);
  stf(out + i, acc / (float)HW);
}
template <typename T>
__global__ __launch_bounds__(256) void pm_pool_bwd_kernel(const T* __restrict__ dpool, T* __restrict__ dy, int B, int HW, int C) {
  const int64_t total = (int64_t)B * HW * C;
  const float inv = 1.f / (float)HW;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(i % C), b = (int)(i / ((int64_t)HW * C));
    stf(dy + i, ldf(dpool + (int64_t)b * C + c) * inv);
  }
}

// ---------------------------------------------------------------------------------------------
// implicit-GEMM kernels (bf16, Cin and Cout multiples of 16, at most 64)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ pm_bf16x8 pm_cv_ld8(const bf16_t* p) { return *reinterpret_cast<const pm_bf16x8*>(p); }

// forward.  One wave = 32 output pixels x all output channels; 4 waves per block, no LDS.
template <int NCT>   // output-channel tiles of 32 (Cout <= 32 NCT)
__global__ __launch_bounds__(256) void pm_conv_fwd_mfma_kernel(PmConvGeom g, const bf16_t* __restrict__ x,
                                                               PmWLoc<bf16_t> wloc, PmShortcut<bf16_t> sc,
                                                               bf16_t* __restrict__ z, bf16_t* __restrict__ y) {
  const bf16_t* Wt = wloc.get();
  const bf16_t* scale = Wt + (int64_t)g.Cout * 9 * g.Cin;
  const bf16_t* shift = scale + g.Cout;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, pl = lane & 31, kg = lane >> 5;
  const int64_t npix = (int64_t)g.B * g.Ho * g.Wo;
  const int64_t p = ((int64_t)blockIdx.x * 4 + wave) * 32 + pl;
  const bool pv = p < npix;
  const int ox = (int)(p % g.Wo), oy = (int)((p / g.Wo) % g.Ho), b = (int)(p / ((int64_t)g.Wo * g.Ho));
  pm_f32x16 acc[NCT];
#pragma unroll
  for (int t = 0; t < NCT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  const int K9 = 9 * g.Cin;
  for (int tap = 0; tap < 9; ++tap) {
    const int iy = oy * g.stride + tap / 3 - 1, ix = ox * g.stride + tap % 3 - 1;
    const bool ok = pv && iy >= 0 && iy < g.H && ix >= 0 && ix < g.W;
    const bf16_t* xr = x + (((int64_t)b * g.H + iy) * g.W + ix) * g.Cin + 8 * kg;
    for (int kc = 0; kc < g.Cin; kc += 16) {
      const pm_bf16x8 fb = ok ? pm_cv_ld8(xr + kc) : pm_at_zero8();
#pragma unroll
      for (int t = 0; t < NCT; ++t) {
        const int co = t * 32 + pl;
        const pm_bf16x8 fa = co < g.Cout ? pm_cv_ld8(Wt + (int64_t)co * K9 + tap * g.Cin + kc + 8 * kg) : pm_at_zero8();
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[t], 0, 0, 0);
      }
    }
  }
  if (!pv) return;
#pragma unroll
  for (int t = 0; t < NCT; ++t)
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int co = t * 32 + 8 * a + 4 * kg;
      if (co >= g.Cout) continue;
      float zz[4], yy[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        zz[j] = acc[t][4 * a + j];
        const float av = ldf(scale + co + j) * zz[j] + ldf(shift + co + j) + sc.at(b, oy, ox, co + j);
        yy[j] = av > 0.f ? av : 0.f;
      }
      pm_st4(z + p * g.Cout + co, make_float4(zz[0], zz[1], zz[2], zz[3]));
      pm_st4(y + p * g.Cout + co, make_float4(yy[0], yy[1], yy[2], yy[3]));
    }
}

// data gradient.  One wave = 32 input pixels x all input channels.  The whole kernel tensor of the
// backward weights sits in LDS as it lies in memory ([co][tap * Cin + ci], padded rows); its
// transposed fragments (row = ci, contraction = co) come from LDS transpose loads.
template <int NCO, int NCT>   // channel tiles of 32: Cout <= 32 NCO, Cin <= 32 NCT
__global__ __launch_bounds__(256) void pm_conv_dgrad_mfma_kernel(PmConvGeom g, const bf16_t* __restrict__ dz,
                                                                 PmWLoc<bf16_t> wloc, PmShortcutBwd<bf16_t> sb,
                                                                 bf16_t* __restrict__ dx) {
  __shared__ __attribute__((aligned(16))) bf16_t sW[(32 * NCO + 16) * (9 * 32 * NCT + 8)];
  const int K9 = 9 * g.Cin, WS = K9 + 8;                 // LDS row stride: 16-byte aligned rows
  {
    const bf16_t* Wt = wloc.get();
    const int chunks = g.Cout * (K9 / 8);
    for (int c = threadIdx.x; c < chunks; c += 256) {
      const int r = c / (K9 / 8), col = (c % (K9 / 8)) * 8;
      *reinterpret_cast<uint4*>(sW + r * WS + col) = *reinterpret_cast<const uint4*>(Wt + (int64_t)r * K9 + col);
    }
    // fragment reads of a channel tile wider than Cin run past a row's end into the next row (those
    // MFMA rows are discarded); the 16 tail rows keep such reads of the last row inside the array
    for (int c = threadIdx.x; c < 16 * WS / 8; c += 256) *reinterpret_cast<uint4*>(sW + g.Cout * WS + c * 8) = make_uint4(0, 0, 0, 0);
  }
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, pl = lane & 31, kg = lane >> 5;
  const int64_t npix = (int64_t)g.B * g.H * g.W;
  const int64_t p = ((int64_t)blockIdx.x * 4 + wave) * 32 + pl;
  const bool pv = p < npix;
  const int ix = (int)(p % g.W), iy = (int)((p / g.W) % g.H), b = (int)(p / ((int64_t)g.W * g.H));
  pm_f32x16 acc[NCT];
#pragma unroll
  for (int t = 0; t < NCT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  const int ql = lane >> 4, q = lane & 15;               // transpose-load lane mapping (see pm_at_frag_tr)
  for (int tap = 0; tap < 9; ++tap) {
    const int ny = iy + 1 - tap / 3, nx = ix + 1 - tap % 3;
    bool ok = pv && ny >= 0 && nx >= 0 && (ny % g.stride) == 0 && (nx % g.stride) == 0;
    const int oy = ny / g.stride, ox = nx / g.stride;
    ok = ok && oy < g.Ho && ox < g.Wo;
    const bf16_t* dr = dz + (((int64_t)b * g.Ho + oy) * g.Wo + ox) * g.Cout + 8 * kg;
    for (int kc = 0; kc < g.Cout; kc += 16) {
      const pm_bf16x8 fb = ok ? pm_cv_ld8(dr + kc) : pm_at_zero8();
#pragma unroll
      for (int t = 0; t < NCT; ++t) {
        // A = W^T: MFMA row = ci = t * 32 + lane % 32 (LDS column tap * Cin + ci), contraction = co rows kc ..
        const bf16_t* pp = sW + (kc + 8 * (ql >> 1) + (q >> 2)) * WS + tap * g.Cin + t * 32 + 16 * (ql & 1) + 4 * (q & 3);
        typedef pm_v4s __attribute__((address_space(3))) * lds_v4s;
        union { pm_bf16x8 v; pm_v4s h[2]; } u;
        u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(pp));
        u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(pp + 4 * WS));
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u.v, fb, acc[t], 0, 0, 0);
      }
    }
  }
  if (!pv) return;
#pragma unroll
  for (int t = 0; t < NCT; ++t)
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int ci = t * 32 + 8 * a + 4 * kg;
      if (ci >= g.Cin) continue;
      float v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = acc[t][4 * a + j] + sb.at(b, iy, ix, ci + j);
      pm_st4(dx + p * g.Cin + ci, make_float4(v[0], v[1], v[2], v[3]));
    }
}

// weight gradient.  Each wave owns a run of output pixels, 32 at a time: it parks the dz rows and
// the (tap-shifted) input rows of the 32 pixels in a private LDS region and reads both transposed
// (contraction = pixels).  One tap at a time; partial sums leave through fp32 atomics (the caller
// zeroes the gradient at the start of a minibatch).  No block-level barrier after the set-up.
template <int NTO, int NTI>   // channel tiles of 32 of Cout and Cin
__global__ __launch_bounds__(256) void pm_conv_wgrad_mfma_kernel(PmConvGeom g, const bf16_t* __restrict__ dz,
                                                                 const bf16_t* __restrict__ x, float* __restrict__ dW,
                                                                 int chunks_per_wave) {
  constexpr int SA = NTO * 32 + 8, SB = NTI * 32 + 8;     // LDS row strides (elements)
  __shared__ __attribute__((aligned(16))) bf16_t sA[4][32 * SA];
  __shared__ __attribute__((aligned(16))) bf16_t sB[4][32 * SB];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  bf16_t* wa = sA[wave];
  bf16_t* wb = sB[wave];
  for (int c = lane; c < 32 * SA / 8; c += 64) *reinterpret_cast<uint4*>(wa + c * 8) = make_uint4(0, 0, 0, 0);
  for (int c = lane; c < 32 * SB / 8; c += 64) *reinterpret_cast<uint4*>(wb + c * 8) = make_uint4(0, 0, 0, 0);
  __builtin_amdgcn_wave_barrier();
  const int64_t npix = (int64_t)g.B * g.Ho * g.Wo;
  const int64_t p_begin = ((int64_t)blockIdx.x * 4 + wave) * chunks_per_wave * 32;
  const int pa = g.Cout / 8, pb = g.Cin / 8;               // 16-byte pieces per row
  for (int tap = 0; tap < 9; ++tap) {
    pm_f32x16 acc[NTO][NTI];
#pragma unroll
    for (int a = 0; a < NTO; ++a)
#pragma unroll
      for (int bb = 0; bb < NTI; ++bb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[a][bb][e] = 0.f;
    for (int ch = 0; ch < chunks_per_wave; ++ch) {
      const int64_t p0 = p_begin + (int64_t)ch * 32;
      if (p0 >= npix) break;                                // wave-uniform
      for (int c = lane; c < 32 * pa; c += 64) {
        const int r = c / pa, col = (c % pa) * 8;
        const int64_t p = p0 + r;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (p < npix) v = *reinterpret_cast<const uint4*>(dz + p * g.Cout + col);
        *reinterpret_cast<uint4*>(wa + r * SA + col) = v;
      }
      for (int c = lane; c < 32 * pb; c += 64) {
        const int r = c / pb, col = (c % pb) * 8;
        const int64_t p = p0 + r;
        const int ox = (int)(p % g.Wo), oy = (int)((p / g.Wo) % g.Ho), b = (int)(p / ((int64_t)g.Wo * g.Ho));
        const int iy = oy * g.stride + tap / 3 - 1, ix = ox * g.stride + tap % 3 - 1;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (p < npix && iy >= 0 && iy < g.H && ix >= 0 && ix < g.W)
          v = *reinterpret_cast<const uint4*>(x + (((int64_t)b * g.H + iy) * g.W + ix) * g.Cin + col);
        *reinterpret_cast<uint4*>(wb + r * SB + col) = v;
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        pm_bf16x8 fa[NTO], fb[NTI];
        const int ql = lane >> 4, q = lane & 15;
        typedef pm_v4s __attribute__((address_space(3))) * lds_v4s;
#pragma unroll
        for (int a = 0; a < NTO; ++a) {
          const bf16_t* pp = wa + (ks * 16 + 8 * (ql >> 1) + (q >> 2)) * SA + a * 32 + 16 * (ql & 1) + 4 * (q & 3);
          union { pm_bf16x8 v; pm_v4s h[2]; } u;
          u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(pp));
          u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(pp + 4 * SA));
          fa[a] = u.v;
        }
#pragma unroll
        for (int bb = 0; bb < NTI; ++bb) {
          const bf16_t* pp = wb + (ks * 16 + 8 * (ql >> 1) + (q >> 2)) * SB + bb * 32 + 16 * (ql & 1) + 4 * (q & 3);
          union { pm_bf16x8 v; pm_v4s h[2]; } u;
          u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(pp));
          u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(pp + 4 * SB));
          fb[bb] = u.v;
        }
#pragma unroll
        for (int a = 0; a < NTO; ++a)
#pragma unroll
          for (int bb = 0; bb < NTI; ++bb)
            acc[a][bb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[bb], acc[a][bb], 0, 0, 0);
      }
      __builtin_amdgcn_wave_barrier();
    }
    // accumulator value v of lane l: row co = 32 a + 8 (v / 4) + 4 (l / 32) + v % 4, column ci = 32 bb + l % 32
    const int kg = lane >> 5, cl = lane & 31;
#pragma unroll
    for (int a = 0; a < NTO; ++a)
#pragma unroll
      for (int bb = 0; bb < NTI; ++bb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int co = a * 32 + 8 * (v >> 2) + 4 * kg + (v & 3), ci = bb * 32 + cl;
          if (co < g.Cout && ci < g.Cin) atomicAdd(dW + ((int64_t)co * 9 + tap) * g.Cin + ci, acc[a][bb][v]);
        }
  }
}

// ---------------------------------------------------------------------------------------------
// host-side dispatch
// ---------------------------------------------------------------------------------------------
inline bool pm_conv_mfma_fits(int Cin, int Cout) { return (Cin % 16) == 0 && (Cout % 16) == 0 && Cin <= 64 && Cout <= 64; }

template <typename T>
inline void pm_conv_fwd_launch(hipStream_t st, const PmConvGeom& g, const T* x, PmWLoc<T> w, PmShortcut<T> sc, T* z, T* y) {
  const int64_t npix = (int64_t)g.B * g.Ho * g.Wo;
  if constexpr (sizeof(T) == 2) {
    if (pm_conv_mfma_fits(g.Cin, g.Cout)) {
      const dim3 grid((unsigned)((npix + 127) / 128)), blk(256);
      if (g.Cout <= 32) hipLaunchKernelGGL((pm_conv_fwd_mfma_kernel<1>), grid, blk, 0, st, g, x, w, sc, z, y);
      else hipLaunchKernelGGL((pm_conv_fwd_mfma_kernel<2>), grid, blk, 0, st, g, x, w, sc, z, y);
      return;
    }
  }
  const int64_t total = npix * g.Cout;
  hipLaunchKernelGGL((pm_conv_fwd_plain_kernel<T>), dim3((unsigned)std::min<int64_t>(65535, (total + 255) / 256)), dim3(256), 0,
                     st, g, x, w, sc, z, y);
}

template <typename T>
inline void pm_conv_dgrad_launch(hipStream_t st, const PmConvGeom& g, const T* dz, PmWLoc<T> w, PmShortcutBwd<T> sb, T* dx) {
  const int64_t npix = (int64_t)g.B * g.H * g.W;
  if constexpr (sizeof(T) == 2) {
    if (pm_conv_mfma_fits(g.Cin, g.Cout)) {
      const dim3 grid((unsigned)((npix + 127) / 128)), blk(256);
#define PM_CD(A, B) hipLaunchKernelGGL((pm_conv_dgrad_mfma_kernel<A, B>), grid, blk, 0, st, g, dz, w, sb, dx)
      if (g.Cout <= 32 && g.Cin <= 32) PM_CD(1, 1);
      else if (g.Cout <= 32) PM_CD(1, 2);
      else if (g.Cin <= 32) PM_CD(2, 1);
      else PM_CD(2, 2);
#undef PM_CD
      return;
    }
  }
  const int64_t total = npix * g.Cin;
  hipLaunchKernelGGL((pm_conv_dgrad_plain_kernel<T>), dim3((unsigned)std::min<int64_t>(65535, (total + 255) / 256)), dim3(256),
                     0, st, g, dz, w, sb, dx);
}

// dW (fp32 [Cout][9][Cin]).  The MFMA path ADDS to dW (atomics): the caller clears it first unless
// accumulating.  The plain path overwrites or accumulates per `accumulate`.
template <typename T>
inline void pm_conv_wgrad_launch(hipStream_t st, const PmConvGeom& g, const T* dz, const T* x, float* dW, int accumulate) {
  if constexpr (sizeof(T) == 2) {
    if (pm_conv_mfma_fits(g.Cin, g.Cout)) {
      const int64_t npix = (int64_t)g.B * g.Ho * g.Wo;
      const int64_t chunks = (npix + 31) / 32;
      // about 256 blocks of 4 waves; fewer, longer runs for the small late maps (fewer atomics)
      int cpw = (int)((chunks + 1023) / 1024);
      if (cpw < 4) cpw = 4;
      const unsigned blocks = (unsigned)((chunks + (int64_t)cpw * 4 - 1) / ((int64_t)cpw * 4));
      const dim3 grid(blocks), blk(256);
#define PM_CW(A, B) hipLaunchKernelGGL((pm_conv_wgrad_mfma_kernel<A, B>), grid, blk, 0, st, g, dz, x, dW, cpw)
      if (g.Cout <= 32 && g.Cin <= 32) PM_CW(1, 1);
      else if (g.Cout <= 32) PM_CW(1, 2);
      else if (g.Cin <= 32) PM_CW(2, 1);
      else PM_CW(2, 2);
#undef PM_CW
      return;
    }
  }
  hipLaunchKernelGGL((pm_conv_wgrad_plain_kernel<T>), dim3((unsigned)(g.Cout * 9 * g.Cin)), dim3(256), 0, st, g, dz, x, dW,
                     accumulate);
}

template <typename T>
inline bool pm_conv_affine_bwd_launch(hipStream_t st, const T* dy, const T* y, const T* z, PmWLoc<T> scale_bkwd, T* da, T* dz,
                                      float* dscale, float* dshift, int64_t total, int C) {
  if ((C & 7) || (2048 % C) || C > 256) return false;
  const unsigned blocks = (unsigned)std::max<int64_t>(1, std::min<int64_t>(512, (total + 2047) / 2048));
  hipLaunchKernelGGL((pm_conv_affine_bwd_kernel<T>), dim3(blocks), dim3(256), 0, st, dy, y, z, scale_bkwd, da, dz, dscale,
                     dshift, total, C);
  return true;
}
