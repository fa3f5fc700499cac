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
#include "pm_mfma_types.hpp"

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

// Forward of the image layer (3 input channels, 16 output channels): one thread per output pixel
// computes all 16 channels from the 27 inputs of its window, with the kernel tensor, scale and shift
// held in LDS as fp32 (every lane reads the same entry: a broadcast); outputs go out as 16-byte pieces.
// The one-thread-per-output-element kernel above spends 61 us on the 128 x 32 x 32 images of the
// ResNet workload (2-byte loads, a 27-element stride between the lanes' weights), this one a few.
template <typename T>
__global__ __launch_bounds__(256) void pm_conv_fwd_thin_kernel(PmConvGeom g, const T* __restrict__ x, PmWLoc<T> wloc,
                                                               PmShortcut<T> sc, T* __restrict__ z, T* __restrict__ y) {
  constexpr int CO = 16, CI = 3, NW = CO * 9 * CI;
  __shared__ float sw[NW + 2 * CO];                   // W [CO][9][CI], then scale [CO], shift [CO] (as in memory)
  const T* Wt = wloc.get();
  for (int i = threadIdx.x; i < NW + 2 * CO; i += blockDim.x) sw[i] = ldf(Wt + i);
  __syncthreads();
  const int64_t npix = (int64_t)g.B * g.Ho * g.Wo;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < npix; p += (int64_t)gridDim.x * blockDim.x) {
    const int ox = (int)(p % g.Wo), oy = (int)((p / g.Wo) % g.Ho), b = (int)(p / ((int64_t)g.Wo * g.Ho));
    float acc[CO];
#pragma unroll
    for (int co = 0; co < CO; ++co) acc[co] = 0.f;
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
      const int iy = oy * g.stride + dy - 1;
      if (iy < 0 || iy >= g.H) continue;
#pragma unroll
      for (int dx = 0; dx < 3; ++dx) {
        const int ix = ox * g.stride + dx - 1;
        if (ix < 0 || ix >= g.W) continue;
        const T* xr = x + (((int64_t)b * g.H + iy) * g.W + ix) * CI;
        const float x0 = ldf(xr), x1 = ldf(xr + 1), x2 = ldf(xr + 2);
        const float* w = sw + (dy * 3 + dx) * CI;
#pragma unroll
        for (int co = 0; co < CO; ++co) {             // same order of additions as the plain kernel
          acc[co] = fmaf(x0, w[co * 9 * CI], acc[co]);
          acc[co] = fmaf(x1, w[co * 9 * CI + 1], acc[co]);
          acc[co] = fmaf(x2, w[co * 9 * CI + 2], acc[co]);
        }
      }
    }
    float a[CO];
#pragma unroll
    for (int co = 0; co < CO; ++co) {
      const float v = sw[NW + co] * acc[co] + sw[NW + CO + co] + sc.at(b, oy, ox, co);
      a[co] = v > 0.f ? v : 0.f;
    }
    pm_st8(z + p * CO, acc);
    pm_st8(z + p * CO + 8, acc + 8);
    pm_st8(y + p * CO, a);
    pm_st8(y + p * CO + 8, a + 8);
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

// weight gradient of a convolution with very few input channels (the 3-channel input layer), any T.
// grid (pixel groups, 9 taps); a thread walks pixels of its group and keeps the CO x CI outer-product
// sums of its pixels in registers; wave shuffles, then LDS across the four waves; the block writes
// its partial of the tap to scratch [group][co][tap][ci] for pm_conv_wgrad_reduce_kernel.
template <typename T, int CO, int CI>
__global__ __launch_bounds__(256) void pm_conv_wgrad_thin_kernel(PmConvGeom g, const T* __restrict__ dz,
                                                                 const T* __restrict__ x, float* __restrict__ part) {
  const int tap = blockIdx.y, dy = tap / 3 - 1, dx = tap % 3 - 1;
  const int npix = g.B * g.Ho * g.Wo;
  float acc[CO][CI];
#pragma unroll
  for (int a = 0; a < CO; ++a)
#pragma unroll
    for (int b = 0; b < CI; ++b) acc[a][b] = 0.f;
  for (int p = blockIdx.x * 256 + threadIdx.x; p < npix; p += gridDim.x * 256) {
    const unsigned up = (unsigned)p, wo = (unsigned)g.Wo, ho = (unsigned)g.Ho;
    const int ox = (int)(up % wo), oy = (int)((up / wo) % ho), bb = (int)(up / (wo * ho));
    const int iy = oy * g.stride + dy, ix = ox * g.stride + dx;
    if (iy < 0 || iy >= g.H || ix < 0 || ix >= g.W) continue;
    float xv[CI], dv[CO];
    const T* xr = x + ((int64_t)(bb * g.H + iy) * g.W + ix) * CI;
#pragma unroll
    for (int b = 0; b < CI; ++b) xv[b] = ldf(xr + b);
#pragma unroll
    for (int a = 0; a < CO; a += 8) pm_ld8(dz + (int64_t)p * CO + a, dv + a);
#pragma unroll
    for (int a = 0; a < CO; ++a)
#pragma unroll
      for (int b = 0; b < CI; ++b) acc[a][b] += dv[a] * xv[b];
  }
  __shared__ float red[4][CO * CI];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int a = 0; a < CO; ++a)
#pragma unroll
    for (int b = 0; b < CI; ++b) {
      const float s = pm_wave_sum(acc[a][b]);
      if (lane == 0) red[wave][a * CI + b] = s;
    }
  __syncthreads();
  if (threadIdx.x < CO * CI) {
    const int a = threadIdx.x / CI, b = threadIdx.x % CI;
    part[(int64_t)blockIdx.x * (CO * 9 * CI) + ((int64_t)a * 9 + tap) * CI + b] =
        red[0][threadIdx.x] + red[1][threadIdx.x] + red[2][threadIdx.x] + red[3][threadIdx.x];
  }
}
constexpr int PM_CONV_THIN_GROUPS = 64;

// da = dy * [y > 0];  dz = da * scale_bkwd;  dscale += sum da * z;  dshift += sum da.  The caller zeroes
// dscale / dshift at the start of a minibatch.  With `part` the block writes its sums to
// part[block][0 = scale | 1 = shift][C] and the weight-gradient reduce kernel that follows adds them up
// (hundreds of blocks adding into the same few dozen addresses with fp32 atomics serialise: that tail
// cost more than the streaming part of the kernel); without it, fp32 atomics.  Thread t of a block always
// sees channel (t * 8 .. t * 8 + 7) mod C because a block's span is a multiple of C elements.
template <typename T>
__global__ __launch_bounds__(256) void pm_conv_affine_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ y,
                                                                 const T* __restrict__ z, PmWLoc<T> scale_bkwd,
                                                                 T* __restrict__ da, T* __restrict__ dz,
                                                                 float* __restrict__ dscale, float* __restrict__ dshift,
                                                                 float* __restrict__ part, int64_t total, int C) {
  __shared__ float red[4][2][256];
  const T* sbk = scale_bkwd.get();
  const int c0 = (threadIdx.x * 8) % C;            // C is a power of two, 8 <= C <= 256
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
  // lanes l and l + C / 8 (mod 64) own the same channels: butterfly over the lane bits above C / 8, then
  // the four waves meet in LDS (plain stores: LDS float atomics are slow), one fp32 atomic per channel and block
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, per = C >> 3;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    for (int o = 32; o >= per && o > 0; o >>= 1) {
      as[e] += __shfl_xor(as[e], o, 64);
      at[e] += __shfl_xor(at[e], o, 64);
    }
  }
  if (lane < per || per > 64) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      red[wave][0][c0 + e] = as[e];
      red[wave][1][c0 + e] = at[e];
    }
  }
  __syncthreads();
  for (int j = threadIdx.x; j < C; j += 256) {
    const float vs = red[0][0][j] + red[1][0][j] + red[2][0][j] + red[3][0][j];
    const float vt = red[0][1][j] + red[1][1][j] + red[2][1][j] + red[3][1][j];
    if (part) {
      part[((int64_t)blockIdx.x * 2 + 0) * C + j] = vs;
      part[((int64_t)blockIdx.x * 2 + 1) * C + j] = vt;
    } else {
      atomicAdd(dscale + j, vs);
      atomicAdd(dshift + j, vt);
    }
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
// The same with one block per image when the channel count divides 256: the block's 256 / C groups of
// threads each sum a share of the pixels (independent loads, consecutive lanes on consecutive channels),
// then the shares are added through LDS - instead of one thread walking all pixels of a channel with
// dependent 2-byte loads (20 us for 64 pixels).
template <typename T>
__global__ __launch_bounds__(256) void pm_pool_fwd_block_kernel(const T* __restrict__ y, T* __restrict__ out, int HW, int C) {
  __shared__ float part[256];
  const int b = blockIdx.x, c = threadIdx.x % C, grp = threadIdx.x / C, ngrp = 256 / C;
  float acc = 0.f;
  for (int p = grp; p < HW; p += ngrp) acc += ldf(y + ((int64_t)b * HW + p) * C + c);
  part[threadIdx.x] = acc;
  __syncthreads();
  if (grp == 0) {
    for (int q = 1; q < ngrp; ++q) acc += part[q * C + c];
    stf(out + (int64_t)b * C + c, acc / (float)HW);
  }
}
template <typename T>
inline void pm_pool_fwd_launch(hipStream_t st, const T* y, T* out, int B, int HW, int C) {
  if (C <= 256 && 256 % C == 0)
    hipLaunchKernelGGL((pm_pool_fwd_block_kernel<T>), dim3(B), dim3(256), 0, st, y, out, HW, C);
  else
    hipLaunchKernelGGL((pm_pool_fwd_kernel<T>), dim3((B * C + 255) / 256), dim3(256), 0, st, y, out, B, HW, C);
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

struct PmReduceJob {
  const float* part;
  int nparts;
  int64_t n;
  float* out;
  int accumulate;
};
// work of block `bid` (256 threads) of a reduce over two jobs; blocks0 = blocks of the first job
__device__ __forceinline__ void pm_conv_reduce_block(const PmReduceJob& j0, const PmReduceJob& j1, int blocks0, int bid) {
  const bool second = bid >= blocks0;
  const PmReduceJob jb = second ? j1 : j0;
  const int el = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int64_t e = (int64_t)(second ? bid - blocks0 : bid) * 16 + el;
  float acc = 0.f;
  if (e < jb.n) {
    int p = sl;
#pragma unroll 1
    for (; p + 48 < jb.nparts; p += 64) {
      const float a0 = jb.part[(int64_t)p * jb.n + e], a1 = jb.part[(int64_t)(p + 16) * jb.n + e];
      const float a2 = jb.part[(int64_t)(p + 32) * jb.n + e], a3 = jb.part[(int64_t)(p + 48) * jb.n + e];
      acc += (a0 + a1) + (a2 + a3);
    }
    for (; p < jb.nparts; p += 16) acc += jb.part[(int64_t)p * jb.n + e];
  }
  __shared__ float s[16][16];
  s[sl][el] = acc;
  __syncthreads();
  if (sl == 0 && e < jb.n) {
    float v = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) v += s[q][el];
    jb.out[e] = jb.accumulate ? jb.out[e] + v : v;
  }
}
__global__ __launch_bounds__(256) void pm_conv_wgrad_reduce_kernel(PmReduceJob j0, PmReduceJob j1, int blocks0) {
  pm_conv_reduce_block(j0, j1, blocks0, blockIdx.x);
}
// a reduce that has not been launched yet: it can ride as extra blocks on the next independent launch
struct PmReducePending {
  PmReduceJob j0, j1;
  bool valid;
  int blocks0() const { return (int)((j0.n + 15) / 16); }
  int blocks() const { return blocks0() + (j1.part ? (int)((j1.n + 15) / 16) : 0); }
};

// ---------------------------------------------------------------------------------------------
// implicit-GEMM kernels (bf16, Cin and Cout multiples of 16, at most 64)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ pm_bf16x8 pm_cv_ld8(const bf16_t* p) { return *reinterpret_cast<const pm_bf16x8*>(p); }

// forward.  One wave = 32 output pixels x all output channels; blockDim.x / 64 waves per block (4 on large
// maps, 1 on small ones so that the few pixel groups still spread over the chip), no LDS.
template <int NCT>   // output-channel tiles of 32 (Cout <= 32 NCT)
__global__ __launch_bounds__(256) void pm_conv_fwd_mfma_kernel(PmConvGeom g, const bf16_t* __restrict__ x,
                                                               PmWLoc<bf16_t> wloc, PmShortcut<bf16_t> sc,
                                                               bf16_t* __restrict__ z, bf16_t* __restrict__ y) {
  const bf16_t* Wt = wloc.get();
  const bf16_t* scale = Wt + (int64_t)g.Cout * 9 * g.Cin;
  const bf16_t* shift = scale + g.Cout;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, pl = lane & 31, kg = lane >> 5;
  const int64_t npix = (int64_t)g.B * g.Ho * g.Wo;
  const int64_t p = ((int64_t)blockIdx.x * (blockDim.x >> 6) + wave) * 32 + pl;
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
                                                                 bf16_t* __restrict__ dx, PmReduceJob r0, PmReduceJob r1,
                                                                 int rblocks0, int dgrad_blocks) {
  __shared__ __attribute__((aligned(16))) bf16_t sW[(32 * NCO + 16) * (9 * 32 * NCT + 8)];
  // blocks past the data gradient's own carry the pending reduce of the same layer's weight gradient
  // (independent work: one launch less per layer on maps where a launch costs as much as the kernel)
  if ((int)blockIdx.x >= dgrad_blocks) {
    pm_conv_reduce_block(r0, r1, rblocks0, (int)blockIdx.x - dgrad_blocks);
    return;
  }
  const int K9 = 9 * g.Cin, WS = K9 + 8;                 // LDS row stride: 16-byte aligned rows
  {
    const bf16_t* Wt = wloc.get();
    const int chunks = g.Cout * (K9 / 8);
    for (int c = threadIdx.x; c < chunks; c += blockDim.x) {
      const int r = c / (K9 / 8), col = (c % (K9 / 8)) * 8;
      *reinterpret_cast<uint4*>(sW + r * WS + col) = *reinterpret_cast<const uint4*>(Wt + (int64_t)r * K9 + col);
    }
    // fragment reads of a channel tile wider than Cin run past a row's end into the next row (those
    // MFMA rows are discarded); the 16 tail rows keep such reads of the last row inside the array
    for (int c = threadIdx.x; c < 16 * WS / 8; c += blockDim.x) *reinterpret_cast<uint4*>(sW + g.Cout * WS + c * 8) = make_uint4(0, 0, 0, 0);
  }
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, pl = lane & 31, kg = lane >> 5;
  const int64_t npix = (int64_t)g.B * g.H * g.W;
  const int64_t p = ((int64_t)blockIdx.x * (blockDim.x >> 6) + wave) * 32 + pl;
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

// weight gradient.  Each wave owns a run of output pixels, 32 at a time ("chunk"): it parks the dz
// rows and the (tap-shifted) input rows of the 32 pixels in a private LDS region and reads both
// transposed (contraction = pixels).  Work items are (tap, chunk) pairs, tap outermost so that one
// accumulator set serves a tap; the global loads of the next item are in flight in a second register
// set while the current item is stored to LDS and multiplied (a wave has no other wave to hide its
// load latency behind here).  At the end of a tap the four waves of the block park their accumulators
// in LDS, the block sums them and writes ITS partial dW of that tap to a scratch area;
// pm_conv_wgrad_reduce_kernel sums the blocks' partials.  (Measured alternatives: fp32 atomics of
// every wave straight into dW, or LDS float atomics for the block sum, each cost several times the
// rest of the kernel.)
// TPB taps per block (9: all of them; 3: blockIdx.y picks the tap row dy = blockIdx.y - 1, for small
// maps whose pixel chunks alone would leave most of the chip idle; the rows write disjoint entries of
// the block's partial, so nothing else changes).
template <int NTO, int NTI, int NCH, int TPB = 9>   // channel tiles of 32 of Cout and Cin; chunks of 32 pixels per wave
__global__ __launch_bounds__(256) void pm_conv_wgrad_mfma_kernel(PmConvGeom g, const bf16_t* __restrict__ dz,
                                                                 const bf16_t* __restrict__ x, float* __restrict__ part) {
  const int tap0 = TPB == 9 ? 0 : (int)blockIdx.y * 3;
  constexpr int SA = NTO * 32 + 8, SB = NTI * 32 + 8;     // LDS row strides (elements)
  constexpr int PA = NTO * 2, PB = NTI * 2;               // 16-byte pieces per lane of a 32-pixel tile
  constexpr int RW = NTI * 32;                            // row width of the block's reduction tile
  __shared__ __attribute__((aligned(16))) bf16_t sA[4][32 * SA];
  __shared__ __attribute__((aligned(16))) bf16_t sB[4][32 * SB];
  __shared__ float red[4][NTO * 32 * RW];                 // one accumulator image per wave
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  bf16_t* wa = sA[wave];
  bf16_t* wb = sB[wave];
  for (int c = lane; c < 32 * SA / 8; c += 64) *reinterpret_cast<uint4*>(wa + c * 8) = make_uint4(0, 0, 0, 0);
  for (int c = lane; c < 32 * SB / 8; c += 64) *reinterpret_cast<uint4*>(wb + c * 8) = make_uint4(0, 0, 0, 0);
  __syncthreads();
  const int npix = g.B * g.Ho * g.Wo;                      // fits 32 bits (checked by the dispatcher)
  const int p_begin = (blockIdx.x * 4 + wave) * NCH * 32;
  const int pa = g.Cout / 8, pb = g.Cin / 8;               // 16-byte pieces per row
  const int64_t nW = (int64_t)g.Cout * 9 * g.Cin;
  float* my_part = part + (int64_t)blockIdx.x * nW;

  // Per chunk and piece, once: where this lane's piece comes from.  Loads are unconditional (clamped
  // to a valid address) and zeroed by a select afterwards, so they issue back to back and the waits
  // before the LDS stores count only the older register set.
  int a_off[NCH][PA];        // element offset into dz, or -1 (piece not used / pixel past the end)
  int b_ctr[NCH][PB];        // input pixel index of the centre tap, or -1
  int b_yx[NCH][PB];         // (iy << 16 | ix) of the centre tap
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
#pragma unroll
    for (int j = 0; j < PA; ++j) {
      const int c = lane + 64 * j, p = p_begin + ch * 32 + c / pa;
      a_off[ch][j] = (c < 32 * pa && p < npix) ? p * g.Cout + (c % pa) * 8 : -1;
    }
#pragma unroll
    for (int j = 0; j < PB; ++j) {
      const int c = lane + 64 * j, p = p_begin + ch * 32 + c / pb;
      if (c < 32 * pb && p < npix) {
        const unsigned up = (unsigned)p, wo = (unsigned)g.Wo, ho = (unsigned)g.Ho;
        const int ox = (int)(up % wo), oy = (int)((up / wo) % ho), bb = (int)(up / (wo * ho));
        const int iy = oy * g.stride, ix = ox * g.stride;
        b_ctr[ch][j] = (bb * g.H + iy) * g.W + ix;
        b_yx[ch][j] = (iy << 16) | ix;
      } else {
        b_ctr[ch][j] = -1;
        b_yx[ch][j] = 0;
      }
    }
  }
  int cbv[PB];                                             // column of this lane's j-th input piece
#pragma unroll
  for (int j = 0; j < PB; ++j) cbv[j] = ((lane + 64 * j) % pb) * 8;

  auto load_regs = [&](int tl, int ch, uint4* ra, uint4* rb) __attribute__((always_inline)) {
    const int dy = (tap0 + tl) / 3 - 1, dx = tl % 3 - 1;       // tap0 is a multiple of 3
#pragma unroll
    for (int j = 0; j < PA; ++j) {
      const int o = a_off[ch][j];
      ra[j] = *reinterpret_cast<const uint4*>(dz + (o < 0 ? 0 : o));
    }
#pragma unroll
    for (int j = 0; j < PB; ++j) {
      const int ctr = b_ctr[ch][j];
      const int iy = (b_yx[ch][j] >> 16) + dy, ix = (b_yx[ch][j] & 0xffff) + dx;
      const bool ok = ctr >= 0 && iy >= 0 && iy < g.H && ix >= 0 && ix < g.W;
      rb[j] = *reinterpret_cast<const uint4*>(x + (ok ? (int64_t)(ctr + dy * g.W + dx) * g.Cin + cbv[j] : 0));
    }
  };
  // zero what must not contribute (after the data has arrived, right before it is parked)
  auto store_regs = [&](int tl, int ch, const uint4* ra, const uint4* rb) __attribute__((always_inline)) {
    const int dy = (tap0 + tl) / 3 - 1, dx = tl % 3 - 1;
    // (component-wise selects: a select between whole uint4 objects would go through memory)
#pragma unroll
    for (int j = 0; j < PA; ++j) {
      const int c = lane + 64 * j;
      const unsigned m = a_off[ch][j] < 0 ? 0u : 0xffffffffu;
      if (c < 32 * pa)
        *reinterpret_cast<uint4*>(wa + (c / pa) * SA + (c % pa) * 8) = make_uint4(ra[j].x & m, ra[j].y & m, ra[j].z & m, ra[j].w & m);
    }
#pragma unroll
    for (int j = 0; j < PB; ++j) {
      const int c = lane + 64 * j;
      const int iy = (b_yx[ch][j] >> 16) + dy, ix = (b_yx[ch][j] & 0xffff) + dx;
      const bool ok = b_ctr[ch][j] >= 0 && iy >= 0 && iy < g.H && ix >= 0 && ix < g.W;
      const unsigned m = ok ? 0xffffffffu : 0u;
      if (c < 32 * pb) *reinterpret_cast<uint4*>(wb + (c / pb) * SB + cbv[j]) = make_uint4(rb[j].x & m, rb[j].y & m, rb[j].z & m, rb[j].w & m);
    }
  };
  pm_f32x16 acc[NTO][NTI];
  auto mma = [&]() __attribute__((always_inline)) {
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
  };
  uint4 ra[2][PA], rb[2][PB];
  load_regs(0, 0, ra[0], rb[0]);
#pragma unroll
  for (int tap = 0; tap < TPB; ++tap) {     // fully unrolled: every register-set and table index is static
#pragma unroll
    for (int a = 0; a < NTO; ++a)
#pragma unroll
      for (int bb = 0; bb < NTI; ++bb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[a][bb][e] = 0.f;
    // items (tap, 0 .. NCH - 1); item (tap, ch) sits in register set ch & 1 (NCH is even or 1, and the
    // first item of the next tap is requested during the last item of this one into set 0)
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const int cur = NCH == 1 ? (tap & 1) : (ch & 1);
      store_regs(tap, ch, ra[cur], rb[cur]);
      if (ch + 1 < NCH) load_regs(tap, ch + 1, ra[cur ^ 1], rb[cur ^ 1]);
      else if (tap + 1 < TPB) load_regs(tap + 1, 0, ra[cur ^ 1], rb[cur ^ 1]);
      __builtin_amdgcn_wave_barrier();
      mma();
      __builtin_amdgcn_wave_barrier();
    }
    // block reduction of the tap: accumulator value v of lane l is row co = 32 a + 8 (v / 4) + 4 (l / 32) + v % 4,
    // column ci = 32 bb + l % 32
    {
      const int kg = lane >> 5, cl = lane & 31;
#pragma unroll
      for (int a = 0; a < NTO; ++a)
#pragma unroll
        for (int bb = 0; bb < NTI; ++bb)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            red[wave][(a * 32 + 8 * (v >> 2) + 4 * kg + (v & 3)) * RW + bb * 32 + cl] = acc[a][bb][v];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < g.Cout * g.Cin; e += 256) {
      const int co = e / g.Cin, ci = e - co * g.Cin, o = co * RW + ci;
      my_part[((int64_t)co * 9 + tap0 + tap) * g.Cin + ci] = red[0][o] + red[1][o] + red[2][o] + red[3][o];
    }
    __syncthreads();
  }
}

// out[e] (+)= sum over nparts partial vectors of n elements each (part[p][e]).  Block = 16 elements x 16
// slices of the partial range: many short chains of independent loads instead of a few long ones (the
// arrays are small; what matters is the latency of the longest chain).  A launch carries up to two
// jobs: the blocks after the first job's work on the second one (used for the per-channel sums of the
// affine backward, whose out is always added to).
inline void pm_conv_reduce_launch(hipStream_t st, const PmReduceJob& j0, const PmReduceJob& j1) {
  const int b0 = (int)((j0.n + 15) / 16), b1 = j1.part ? (int)((j1.n + 15) / 16) : 0;
  hipLaunchKernelGGL(pm_conv_wgrad_reduce_kernel, dim3((unsigned)(b0 + b1)), dim3(256), 0, st, j0, j1, b0);
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
      const int wpb = npix >= 256 * 128 ? 4 : 1;          // waves (of 32 pixels) per block
      const dim3 grid((unsigned)((npix + 32 * wpb - 1) / (32 * wpb))), blk(64 * wpb);
      if (g.Cout <= 32) hipLaunchKernelGGL((pm_conv_fwd_mfma_kernel<1>), grid, blk, 0, st, g, x, w, sc, z, y);
      else hipLaunchKernelGGL((pm_conv_fwd_mfma_kernel<2>), grid, blk, 0, st, g, x, w, sc, z, y);
      return;
    }
  }
  if (g.Cin == 3 && g.Cout == 16) {                     // the image layer
    hipLaunchKernelGGL((pm_conv_fwd_thin_kernel<T>), dim3((unsigned)std::min<int64_t>(65535, (npix + 255) / 256)), dim3(256),
                       0, st, g, x, w, sc, z, y);
    return;
  }
  const int64_t total = npix * g.Cout;
  hipLaunchKernelGGL((pm_conv_fwd_plain_kernel<T>), dim3((unsigned)std::min<int64_t>(65535, (total + 255) / 256)), dim3(256), 0,
                     st, g, x, w, sc, z, y);
}

template <typename T>
inline void pm_conv_dgrad_launch(hipStream_t st, const PmConvGeom& g, const T* dz, PmWLoc<T> w, PmShortcutBwd<T> sb, T* dx,
                                 const PmReducePending* pend = nullptr) {
  const int64_t npix = (int64_t)g.B * g.H * g.W;
  const bool carry = pend && pend->valid;
  if constexpr (sizeof(T) == 2) {
    if (pm_conv_mfma_fits(g.Cin, g.Cout)) {
      // (fewer waves per block on small maps were measured slower here: every block first loads the kernel tensor)
      const int nb = (int)((npix + 127) / 128);
      const PmReduceJob none{nullptr, 0, 0, nullptr, 1};
      const PmReduceJob r0 = carry ? pend->j0 : none, r1 = carry ? pend->j1 : none;
      const int rb0 = carry ? pend->blocks0() : 0;
      const dim3 grid((unsigned)(nb + (carry ? pend->blocks() : 0))), blk(256);
#define PM_CD(A, B) hipLaunchKernelGGL((pm_conv_dgrad_mfma_kernel<A, B>), grid, blk, 0, st, g, dz, w, sb, dx, r0, r1, rb0, nb)
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
  if (carry) pm_conv_reduce_launch(st, pend->j0, pend->j1);
}

// blocks and chunks per wave (4 on large maps, 1 on small ones) of the MFMA weight-gradient kernel
inline void pm_conv_wgrad_plan(const PmConvGeom& g, int* blocks, int* cpw) {
  const int64_t npix = (int64_t)g.B * g.Ho * g.Wo;
  const int64_t chunks = (npix + 31) / 32;
  const int c = chunks >= 2048 ? 4 : 1;
  *cpw = c;
  *blocks = (int)((chunks + (int64_t)c * 4 - 1) / ((int64_t)c * 4));
}
// fp32 scratch elements the MFMA path needs (0: the plain path is used)
inline bool pm_conv_thin_fits(const PmConvGeom& g) {
  return g.Cin == 3 && g.Cout == 16 && (int64_t)g.B * g.H * g.W * 16 < ((int64_t)1 << 31);
}
template <typename T>
inline size_t pm_conv_wgrad_scratch_elems(const PmConvGeom& g) {
  if (pm_conv_thin_fits(g)) return (size_t)PM_CONV_THIN_GROUPS * g.Cout * 9 * g.Cin;
  if (sizeof(T) != 2 || !pm_conv_mfma_fits(g.Cin, g.Cout)) return 0;
  if ((int64_t)g.B * g.H * g.W * std::max(g.Cin, g.Cout) >= (int64_t)1 << 31) return 0;   // 32-bit indexing inside
  int blocks, cpw;
  pm_conv_wgrad_plan(g, &blocks, &cpw);
  return (size_t)blocks * g.Cout * 9 * g.Cin;
}

// dW (fp32 [Cout][9][Cin]) = (accumulate ? dW : 0) + correlation of dz with x.  `scratch` must hold
// pm_conv_wgrad_scratch_elems floats (unused by the plain path).
// true if the weight gradient of this geometry ends in a reduce launch (which can carry a second job)
template <typename T>
inline bool pm_conv_wgrad_has_reduce(const PmConvGeom& g) {
  return pm_conv_thin_fits(g) || pm_conv_wgrad_scratch_elems<T>(g) > 0;
}

template <typename T>
inline void pm_conv_wgrad_launch(hipStream_t st, const PmConvGeom& g, const T* dz, const T* x, float* dW, int accumulate,
                                 float* scratch, PmReduceJob extra = PmReduceJob{nullptr, 0, 0, nullptr, 1},
                                 PmReducePending* pend = nullptr) {
  // the reduce that ends the MFMA and thin paths is launched here, or handed back in *pend for the caller
  // to attach to its next launch
  auto finish = [&](const PmReduceJob& j0) {
    if (pend) *pend = PmReducePending{j0, extra, true};
    else pm_conv_reduce_launch(st, j0, extra);
  };
  if (pend) pend->valid = false;
  if constexpr (sizeof(T) == 2) {
    if (!pm_conv_thin_fits(g) && pm_conv_wgrad_scratch_elems<T>(g) > 0) {
      int blocks, cpw;
      pm_conv_wgrad_plan(g, &blocks, &cpw);
      const bool split = blocks < 128;                 // too few pixel chunks to fill the chip: one tap row per block
      const dim3 grid(blocks, split ? 3 : 1), blk(256);
#define PM_CW(A, B) do { if (cpw == 4) hipLaunchKernelGGL((pm_conv_wgrad_mfma_kernel<A, B, 4>), grid, blk, 0, st, g, dz, x, scratch); \
                         else if (split) hipLaunchKernelGGL((pm_conv_wgrad_mfma_kernel<A, B, 1, 3>), grid, blk, 0, st, g, dz, x, scratch); \
                         else hipLaunchKernelGGL((pm_conv_wgrad_mfma_kernel<A, B, 1>), grid, blk, 0, st, g, dz, x, scratch); } while (0)
      if (g.Cout <= 32 && g.Cin <= 32) PM_CW(1, 1);
      else if (g.Cout <= 32) PM_CW(1, 2);
      else if (g.Cin <= 32) PM_CW(2, 1);
      else PM_CW(2, 2);
#undef PM_CW
      const int64_t nW = (int64_t)g.Cout * 9 * g.Cin;
      finish(PmReduceJob{scratch, blocks, nW, dW, accumulate});
      return;
    }
  }
  if (pm_conv_thin_fits(g)) {
    const int64_t nW = (int64_t)g.Cout * 9 * g.Cin;
    hipLaunchKernelGGL((pm_conv_wgrad_thin_kernel<T, 16, 3>), dim3(PM_CONV_THIN_GROUPS, 9), dim3(256), 0, st, g, dz, x, scratch);
    finish(PmReduceJob{scratch, PM_CONV_THIN_GROUPS, nW, dW, accumulate});
    return;
  }
  hipLaunchKernelGGL((pm_conv_wgrad_plain_kernel<T>), dim3((unsigned)(g.Cout * 9 * g.Cin)), dim3(256), 0, st, g, dz, x, dW,
                     accumulate);
}

constexpr int PM_CONV_AFFINE_MAX_BLOCKS = 1024;
// part: NULL (fp32 atomics into dscale / dshift), or room for PM_CONV_AFFINE_MAX_BLOCKS * 2 * C floats; then
// *job receives the reduction the caller must hand to the next reduce launch (out = dscale, n = 2 C:
// dshift follows dscale in memory).
template <typename T>
inline bool pm_conv_affine_bwd_launch(hipStream_t st, const T* dy, const T* y, const T* z, PmWLoc<T> scale_bkwd, T* da, T* dz,
                                      float* dscale, float* dshift, int64_t total, int C, float* part = nullptr,
                                      PmReduceJob* job = nullptr) {
  if (C < 8 || C > 256 || (C & (C - 1))) return false;        // a power of two in 8 .. 256
  if (part && dshift != dscale + C) return false;
  const unsigned blocks = (unsigned)std::max<int64_t>(1, std::min<int64_t>(part ? PM_CONV_AFFINE_MAX_BLOCKS : 512, (total + 2047) / 2048));
  hipLaunchKernelGGL((pm_conv_affine_bwd_kernel<T>), dim3(blocks), dim3(256), 0, st, dy, y, z, scale_bkwd, da, dz, dscale,
                     dshift, part, total, C);
  if (part && job) *job = PmReduceJob{part, (int)blocks, (int64_t)2 * C, dscale, 1};
  return true;
}
