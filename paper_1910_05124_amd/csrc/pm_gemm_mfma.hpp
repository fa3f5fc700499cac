// bf16 MFMA GEMM for the stage forward / backward-data / backward-weight products (gfx950).
//
//   C[i, j] = sum_k A(i, k) * B(j, k),   fp32 accumulation on v_mfma_f32_32x32x16_bf16.
//
// Each operand is either "KC" (contraction index contiguous in memory: X[r * ld + k]) or "RC"
// (row index contiguous: X[k * ld + r]).  The three products of a Linear unit map to
//   forward          Z = A W^T      A: KC (activations)   B: KC (W[n_out, n_in])
//   backward data    dA = dZ W      A: KC (dZ)            B: RC (W read along n_in)
//   backward weight  dW = dZ^T A    A: RC (dZ)            B: RC (activations)
// Global -> LDS is always a straight 16-byte copy of the tile as it lies in memory; an RC tile
// is transposed on the LDS -> register side (eight 2-byte reads along k, consecutive lanes on
// consecutive addresses, so no bank conflicts), a KC tile is read with one 16-byte load per
// fragment.  LDS rows are padded by 8 elements so the 16-byte fragment reads of 16 lanes cover
// all banks once.
//
// Block = WI x WJ x WK wavefronts.  WI x WJ waves tile the BI x BJ output block in 32x32 MFMA
// tiles; WK > 1 additionally splits every K slab across waves (for skinny problems such as
// 128 x 1024 x 1024 where output tiles alone cannot fill 256 CUs) and the partial accumulators
// are summed through LDS before the epilogue.  The slab depth BK is a template parameter: the
// skinny shapes are bound by memory latency, not MFMA rate, so they use deep slabs (many
// 16-byte loads in flight per thread, few serialised round trips).
//
// A launch covers either one problem (passed by value) or a table of problems in device memory
// indexed by blockIdx.z (all weight-gradient products of a step go out as one launch).  The
// weight-gradient epilogue can also emit the bias gradient: column sums of the (RC) A tile,
// accumulated by the blocks of the first column of tiles while the tile sits in LDS.
//
// Requirements (checked by the dispatcher, which otherwise declines): leading dimensions and
// base pointers multiples of 8 elements; memory readable up to the next multiple of 8 along the
// contiguous index, holding zeros beyond the logical extent.
#pragma once
#include <type_traits>

#include "pm_common.hpp"
#include "pm_elem.hpp"
#include "pm_mfma_types.hpp"


template <int ROWS, bool KC, int BK>
struct PmTileShape {                       // how a (ROWS x BK) operand tile lies in LDS
  static constexpr int lds_rows = KC ? ROWS : BK;
  static constexpr int lds_cols = KC ? BK : ROWS;
  static constexpr int stride = lds_cols + 8;
  static constexpr int elems = lds_rows * stride;
  static constexpr int chunks = lds_rows * lds_cols / 8;    // 16-byte pieces
};

template <int ROWS, bool KC, int BK, int NT>
struct PmTileLoader {
  using S = PmTileShape<ROWS, KC, BK>;
  static constexpr int PER = (S::chunks + NT - 1) / NT;
  uint4 r[PER];
  // r0: first row of the tile, k0: first contraction index; R / K logical extents
  __device__ __forceinline__ void load(const bf16_t* __restrict__ X, int64_t ld, int r0, int k0, int R, int K) {
    const int R8 = (R + 7) & ~7, K8 = (K + 7) & ~7;
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      const int c = p * NT + threadIdx.x;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (S::chunks % NT == 0 || c < S::chunks) {
        const int lr = c / (S::lds_cols / 8), lc = (c % (S::lds_cols / 8)) * 8;
        if (KC) {
          const int row = r0 + lr, k = k0 + lc;
          if (row < R && k < K8) v = *reinterpret_cast<const uint4*>(X + (int64_t)row * ld + k);
        } else {
          const int k = k0 + lr, row = r0 + lc;
          if (k < K && row < R8) v = *reinterpret_cast<const uint4*>(X + (int64_t)k * ld + row);
        }
      }
      r[p] = v;
    }
  }
  __device__ __forceinline__ void store(bf16_t* s) const {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      const int c = p * NT + threadIdx.x;
      if (S::chunks % NT == 0 || c < S::chunks) {
        const int lr = c / (S::lds_cols / 8), lc = (c % (S::lds_cols / 8)) * 8;
        *reinterpret_cast<uint4*>(s + lr * S::stride + lc) = r[p];
      }
    }
  }
};


// MFMA operand fragment of the 32-row tile starting at tile row r32 for contraction indices
// kb .. kb+15 (kb a multiple of 16): lane l holds row r32 + l%32, k = kb + 8*(l/32) .. +7.
// KC tile: one 16-byte read.  RC tile ([k][row] in LDS): the gfx950 LDS transpose load - in each
// group of 16 lanes, lane q supplies the address of 4 consecutive elements (one k-row, 4 operand
// rows) and receives, for the operand row given by its index in the group, the elements of 4
// consecutive k-rows; lane q of group g addresses k-row kb + 8*(g/2) + q/4, operand rows
// r32 + 16*(g%2) + 4*(q%4) .. +3 (two such loads, k-rows +0 and +4, make the fragment).
template <int ROWS, bool KC, int BK>
__device__ __forceinline__ pm_bf16x8 pm_read_frag(const bf16_t* s, int r32, int kb, int lane) {
  using S = PmTileShape<ROWS, KC, BK>;
  if (KC) {
    return *reinterpret_cast<const pm_bf16x8*>(s + (r32 + (lane & 31)) * S::stride + kb + (lane >> 5) * 8);
  } else {
    static_assert((S::stride & 3) == 0, "transpose loads need 8-byte aligned k-rows");
    const int g = lane >> 4, q = lane & 15;
    const bf16_t* p = s + (kb + 8 * (g >> 1) + (q >> 2)) * S::stride + r32 + 16 * (g & 1) + 4 * (q & 3);
    typedef pm_v4s __attribute__((address_space(3))) * lds_v4s;
    union { pm_bf16x8 v; pm_v4s h[2]; } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 4 * S::stride));
    return u.v;
  }
}

template <class Epi>
struct PmGemmProb {
  int I, J, K;
  const bf16_t* A;
  int64_t lda;
  PmWLoc<bf16_t> B;
  int64_t ldb;
  Epi epi;
};

template <int BI_, int BJ_, int WI_, int WJ_, int WK_, int BK_>
struct PmGemmCfg {
  static constexpr int BI = BI_, BJ = BJ_, WI = WI_, WJ = WJ_, WK = WK_, BK = BK_;
  static constexpr int NT = WI * WJ * WK * 64;
};

template <class Cfg, bool AKC, bool BKC>
struct PmGemmLds {
  using SA = PmTileShape<Cfg::BI, AKC, Cfg::BK>;
  using SB = PmTileShape<Cfg::BJ, BKC, Cfg::BK>;
  static constexpr int ab = (SA::elems + SB::elems) * 2;
  static constexpr int red = Cfg::WK > 1 ? Cfg::WK * Cfg::BI * Cfg::BJ * 4 : 0;
  static constexpr int bytes = ab > red ? ab : red;
};

template <class Cfg, bool AKC, bool BKC, class Epi>
__device__ __forceinline__ void pm_gemm_body(const PmGemmProb<Epi>& pr, Epi epi, int bx, int by, unsigned char* smem) {
  constexpr int BI = Cfg::BI, BJ = Cfg::BJ, WI = Cfg::WI, WJ = Cfg::WJ, WK = Cfg::WK, BK = Cfg::BK, NT = Cfg::NT;
  constexpr int TI = BI / WI / 32, TJ = BJ / WJ / 32;     // 32x32 MFMA tiles per wave
  constexpr int KS = BK / 16 / WK;                        // k-steps of 16 per wave per slab
  static_assert(BI % (WI * 32) == 0 && BJ % (WJ * 32) == 0 && (BK / 16) % WK == 0, "tile shape");
  using SA = PmTileShape<BI, AKC, BK>;
  const int I = pr.I, J = pr.J, K = pr.K;
  const int i0 = by * BI, j0 = bx * BJ;
  if (i0 >= I || j0 >= J) return;                         // grouped launch: grid sized for the largest problem
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem);
  bf16_t* sB = sA + SA::elems;
  const bf16_t* __restrict__ A = pr.A;
  const bf16_t* __restrict__ B = pr.B.get();
  const int64_t lda = pr.lda, ldb = pr.ldb;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wk = wave % WK, wj = (wave / WK) % WJ, wi = wave / (WK * WJ);
  const int lr = lane & 31, kg = lane >> 5;

  pm_f32x16 acc[TI][TJ];
#pragma unroll
  for (int a = 0; a < TI; ++a)
#pragma unroll
    for (int b = 0; b < TJ; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
  float colsum = 0.f;                                     // bias gradient (weight-gradient epilogue only)
  const bool do_colsum = Epi::kColSumA && !AKC && bx == 0 && epi.wants_colsum();

  PmTileLoader<BI, AKC, BK, NT> la;
  PmTileLoader<BJ, BKC, BK, NT> lb;
  const int nk = (K + BK - 1) / BK;
  la.load(A, lda, i0, 0, I, K);
  lb.load(B, ldb, j0, 0, J, K);
  for (int kt = 0; kt < nk; ++kt) {
    la.store(sA);
    lb.store(sB);
    __syncthreads();
    if (kt + 1 < nk) {
      la.load(A, lda, i0, (kt + 1) * BK, I, K);
      lb.load(B, ldb, j0, (kt + 1) * BK, J, K);
    }
    if (Epi::kColSumA && !AKC) {
      if (do_colsum && threadIdx.x < BI) {
#pragma unroll 8
        for (int k = 0; k < BK; ++k) colsum += bf16_to_f32(sA[k * SA::stride + threadIdx.x]);
      }
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int kb = (wk * KS + ks) * 16;
      pm_bf16x8 fa[TI], fb[TJ];
#pragma unroll
      for (int a = 0; a < TI; ++a) fa[a] = pm_read_frag<BI, AKC, BK>(sA, (wi * TI + a) * 32, kb, lane);
#pragma unroll
      for (int b = 0; b < TJ; ++b) fb[b] = pm_read_frag<BJ, BKC, BK>(sB, (wj * TJ + b) * 32, kb, lane);
#pragma unroll
      for (int a = 0; a < TI; ++a)
#pragma unroll
        for (int b = 0; b < TJ; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
    __syncthreads();
  }

  epi.begin();
  if (Epi::kColSumA && !AKC) {
    if (do_colsum && threadIdx.x < BI && i0 + (int)threadIdx.x < I) epi.colsum(i0 + threadIdx.x, colsum);
  }
  if (WK == 1) {
    // accumulator layout of the 32x32 tile: value v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32
#pragma unroll
    for (int a = 0; a < TI; ++a)
#pragma unroll
      for (int b = 0; b < TJ; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = i0 + (wi * TI + a) * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
          const int j = j0 + (wj * TJ + b) * 32 + lr;
          if (i < I && j < J) epi(i, j, acc[a][b][v]);
        }
  } else {
    // sum the WK partial tiles through LDS; afterwards thread -> element mapping is row-major over
    // the block so the epilogue's stores are contiguous along j
    float* red = reinterpret_cast<float*>(smem);
#pragma unroll
    for (int a = 0; a < TI; ++a)
#pragma unroll
      for (int b = 0; b < TJ; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int li = (wi * TI + a) * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
          const int lj = (wj * TJ + b) * 32 + lr;
          red[(wk * BI + li) * BJ + lj] = acc[a][b][v];
        }
    __syncthreads();
    for (int e = threadIdx.x; e < BI * BJ; e += NT) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < WK; ++w) sum += red[w * BI * BJ + e];
      const int i = i0 + e / BJ, j = j0 + e % BJ;
      if (i < I && j < J) epi(i, j, sum);
    }
  }
}

// Weights of the NEXT product of a chain of small products, to be pulled towards the compute units while
// this one runs.  A 128 x 1024 x 1024 product keeps only half the chip busy and is bound by the latency
// of its weight matrix, which was last touched many steps ago (a ring slot) and, in the data gradient,
// is read in 64-byte pieces one row apart.  Extra blocks of the launch (grid rows beyond the real tile
// rows) read the next matrix in dense pieces; block x of any launch runs on XCD x % 8 and the tile
// order below gives XCD k the k-th eighth of the column tiles, so each XCD's extra blocks read exactly
// the part its own L2 will be asked for.
struct PmPrefetch {
  const unsigned char* base;   // nullptr: nothing to prefetch
  const int32_t* slot;         // ring slot index in the device step table, or nullptr
  int64_t stride_bytes;        // bytes between ring slots
  int rows;                    // matrix rows
  int row_bytes;               // useful bytes per row (a multiple of 16)
  int64_t ld_bytes;            // bytes between rows
  int by_rows;                 // 1: an XCD's share is a range of rows (the consumer's column tiles are rows of the
                               // matrix: forward); 0: a range of bytes of every row (data gradient)
  int share;                   // rows (by_rows) or bytes of a row (else) per XCD
};

__device__ __forceinline__ void pm_prefetch_block(const PmPrefetch& pf, int bx, int py, int gx, int npy) {
  const unsigned char* base = pf.base + (pf.slot ? (int64_t)(*pf.slot) * pf.stride_bytes : 0);
  const int xcd = bx & 7, q = (bx >> 3) + (gx >> 3) * py, nq = (gx >> 3) * npy;
  int r0 = 0, nr = pf.rows, c0 = 0, nb = pf.row_bytes;
  if (pf.by_rows) {
    r0 = xcd * pf.share;
    nr = pf.rows - r0 < pf.share ? pf.rows - r0 : pf.share;
  } else {
    c0 = xcd * pf.share;
    nb = pf.row_bytes - c0 < pf.share ? pf.row_bytes - c0 : pf.share;
  }
  if (nr <= 0 || nb <= 0) return;
  const int per_row = (nb + 63) >> 6;                     // one 4-byte read per 64 bytes brings the line in
  const int total = nr * per_row;
  uint32_t acc = 0;
  const int nt = (int)blockDim.x;
  for (int c = q * nt + (int)threadIdx.x; c < total; c += nq * nt) {
    const int r = c / per_row, piece = c - r * per_row;
    acc |= *reinterpret_cast<const uint32_t*>(base + (int64_t)(r0 + r) * pf.ld_bytes + c0 + piece * 64);
  }
  asm volatile("" ::"v"(acc));                            // the reads have no other use: keep them
}

// one problem, passed by value.  Grid (column tiles, row tiles + extra rows of prefetching blocks).
template <class Cfg, bool AKC, bool BKC, class Epi>
__global__ __launch_bounds__(Cfg::NT) void pm_gemm_mfma_kernel(PmGemmProb<Epi> pr, PmPrefetch pf, int tiles_i) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[PmGemmLds<Cfg, AKC, BKC>::bytes];
  if ((int)blockIdx.y >= tiles_i) {
    pm_prefetch_block(pf, blockIdx.x, blockIdx.y - tiles_i, gridDim.x, gridDim.y - tiles_i);
    return;
  }
  // XCD k (blocks with x % 8 == k) takes the k-th eighth of the column tiles: its L2 then holds one
  // contiguous part of the B operand
  int bx = blockIdx.x;
  if ((gridDim.x & 7) == 0) bx = (bx & 7) * (gridDim.x >> 3) + (bx >> 3);
  pm_gemm_body<Cfg, AKC, BKC, Epi>(pr, pr.epi, bx, blockIdx.y, smem);
}

// a table of problems in device memory, one per blockIdx.z
template <class Cfg, bool AKC, bool BKC, class Epi>
__global__ __launch_bounds__(Cfg::NT) void pm_gemm_mfma_grouped_kernel(const PmGemmProb<Epi>* __restrict__ probs) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[PmGemmLds<Cfg, AKC, BKC>::bytes];
  const PmGemmProb<Epi> pr = probs[blockIdx.z];   // by value: the fields become wave-uniform registers
  pm_gemm_body<Cfg, AKC, BKC, Epi>(pr, pr.epi, blockIdx.x, blockIdx.y, smem);
}

template <class Cfg, bool AKC, bool BKC, class Epi>
inline void pm_mfma_launch(hipStream_t st, const PmGemmProb<Epi>& pr, const PmPrefetch* pf = nullptr) {
  dim3 grid((pr.J + Cfg::BJ - 1) / Cfg::BJ, (pr.I + Cfg::BI - 1) / Cfg::BI);
  const int tiles_i = (int)grid.y;
  PmPrefetch none{nullptr, nullptr, 0, 0, 0, 0, 0, 0};
  // prefetching blocks only where the product leaves compute units idle, as many as are idle
  if (pf && pf->base && (grid.x & 7) == 0 && grid.x * grid.y < 256) grid.y += (256 - grid.x * grid.y) / grid.x;
  else pf = &none;
  hipLaunchKernelGGL((pm_gemm_mfma_kernel<Cfg, AKC, BKC, Epi>), grid, dim3(Cfg::NT), 0, st, pr, *pf, tiles_i);
}

using PmCfgBig = PmGemmCfg<128, 128, 2, 2, 1, 64>;      // MFMA-bound shapes
using PmCfgMid = PmGemmCfg<64, 64, 2, 2, 1, 64>;
using PmCfgShortK = PmGemmCfg<64, 64, 2, 2, 1, 128>;    // K <= 128 (weight gradient of a small microbatch): one slab
// few output tiles, long K: bound by latency, so the slab is as deep as LDS allows (all loads of up to
// 1024 k in flight at once, 132 KB LDS, one block per CU) and the contraction is split over as many waves
// as a block can have: 16 waves x 64 deep instead of 4 waves x 256 deep took the 128 x 1024 x 1024 products
// of the MLP chain from 7.1 to 5.4 us (four waves per SIMD cover each other's load, LDS and MFMA latencies,
// and each wave's dependent MFMA chain is a quarter as long)
using PmCfgSkinny256 = PmGemmCfg<32, 32, 1, 1, 8, 256>;
using PmCfgSkinny512 = PmGemmCfg<32, 32, 1, 1, 16, 512>;
using PmCfgSkinny1K = PmGemmCfg<32, 32, 1, 1, 16, 1024>;

template <bool AKC, bool BKC, class Epi>
inline bool pm_big_try(hipStream_t st, const PmGemmProb<Epi>& pr);
template <bool AKC, bool BKC, class Epi>
inline bool pm_mid_try(hipStream_t st, const PmGemmProb<Epi>& pr);

template <bool AKC, bool BKC, class Epi>
inline void pm_mfma_pick(hipStream_t st, const PmGemmProb<Epi>& pr, const PmPrefetch* pf = nullptr) {
  if (pm_big_try<AKC, BKC>(st, pr)) return;
  const long tiles128 = (long)((pr.I + 127) / 128) * ((pr.J + 127) / 128);
  const long tiles64 = (long)((pr.I + 63) / 64) * ((pr.J + 63) / 64);
  if (pm_mid_try<AKC, BKC>(st, pr)) return;
  if (tiles128 >= 512) pm_mfma_launch<PmCfgBig, AKC, BKC>(st, pr);
  else if (pr.K <= 128) pm_mfma_launch<PmCfgShortK, AKC, BKC>(st, pr, pf);
  else if (tiles64 >= 192 || pr.K <= 256) pm_mfma_launch<PmCfgMid, AKC, BKC>(st, pr, pf);
  else if (pr.K >= 768) pm_mfma_launch<PmCfgSkinny1K, AKC, BKC>(st, pr, pf);
  else if (pr.K >= 384) pm_mfma_launch<PmCfgSkinny512, AKC, BKC>(st, pr, pf);
  else pm_mfma_launch<PmCfgSkinny256, AKC, BKC>(st, pr, pf);
}

// Alignment rules of the MFMA path for one problem given element strides (exactly one of
// (sxr, sxk) must be 1 per operand).
inline bool pm_mfma_fits(int I, int J, int K, const void* A, int64_t sai, int64_t sak, const void* Bbase, int64_t Bstride,
                         int64_t sbj, int64_t sbk) {
  const bool akc = sak == 1, bkc = sbk == 1;
  if (!akc && sai != 1) return false;
  if (!bkc && sbj != 1) return false;
  const int64_t lda = akc ? sai : sak, ldb = bkc ? sbj : sbk;
  if ((lda & 7) || (ldb & 7) || (Bstride & 7)) return false;
  if (((uintptr_t)A & 15) || ((uintptr_t)Bbase & 15)) return false;
  // the contiguous index is read in whole groups of 8: the row must be that long
  if (lda < ((akc ? K : I) + 7) / 8 * 8) return false;
  if (ldb < ((bkc ? K : J) + 7) / 8 * 8) return false;
  return true;
}

// Whether pm_mfma_gemm_try takes a single product: the alignment rules, and a contraction longer than
// one MFMA depth (K <= 16, e.g. the data gradient through a 10-class head, goes to the plain kernel,
// whose single 16-deep step has less latency than staging 64 x 128 tiles of mostly padding).
inline bool pm_mfma_takes(int I, int J, int K, const void* A, int64_t sai, int64_t sak, const void* Bbase, int64_t Bstride,
                          int64_t sbj, int64_t sbk) {
  return K > 16 && pm_mfma_fits(I, J, K, A, sai, sak, Bbase, Bstride, sbj, sbk);
}

// Try to run the product on MFMA.  Returns false (nothing launched) when the alignment rules do
// not fit, in which case the caller uses the plain kernel.
template <class Epi>
inline bool pm_mfma_gemm_try(hipStream_t st, int I, int J, int K, const bf16_t* A, int64_t sai, int64_t sak,
                             PmWLoc<bf16_t> B, int64_t sbj, int64_t sbk, const Epi& epi, const PmPrefetch* pf = nullptr) {
  if (!pm_mfma_takes(I, J, K, A, sai, sak, B.base, B.stride, sbj, sbk)) return false;
  const bool akc = sak == 1, bkc = sbk == 1;
  PmGemmProb<Epi> pr{I, J, K, A, akc ? sai : sak, B, bkc ? sbj : sbk, epi};
  if (akc && bkc) pm_mfma_pick<true, true>(st, pr, pf);
  else if (akc && !bkc) pm_mfma_pick<true, false>(st, pr, pf);
  else if (!akc && bkc) pm_mfma_pick<false, true>(st, pr, pf);
  else pm_mfma_pick<false, false>(st, pr, pf);
  return true;
}

// ---------------------------------------------------------------------------------------------
// Large problems (MFMA bound): big block tiles, double-buffered LDS (one barrier per 64-deep slab,
// the next slab's global loads in flight during the MFMAs), RC operands read with the gfx950 LDS
// transpose load (ds_read_b64_tr_b16: two instructions per fragment instead of eight 2-byte
// reads), XCD-aware block -> tile mapping so that tiles sharing operand panels share an L2.
// ---------------------------------------------------------------------------------------------
template <int ROWS, bool KC>
struct PmBigTile {                         // (ROWS x 64) operand slab in LDS
  static constexpr int BK = 64;
  static constexpr int lds_rows = KC ? ROWS : BK;
  static constexpr int lds_cols = KC ? BK : ROWS;
  // KC: 16-byte fragment reads of 16 lanes cover all banks once with an 8-element pad.
  // RC: transpose reads touch 4 consecutive k-rows x 64 bytes; a row stride of 16 words mod 64 keeps them apart.
  static constexpr int stride = KC ? BK + 8 : ROWS + 32;
  static constexpr int elems = lds_rows * stride;
  static constexpr int chunks = lds_rows * lds_cols / 8;
};

template <int ROWS, bool KC, int NT>
struct PmBigLoader {
  using S = PmBigTile<ROWS, KC>;
  static_assert(S::chunks % NT == 0, "tile must split evenly over the block");
  static constexpr int PER = S::chunks / NT;
  uint4 r[PER];
  // CHECK false: the tile lies fully inside the operand (no predicates: the loads of a slab issue
  // back to back and the compiler can count them exactly when it waits for an older slab)
  template <bool CHECK>
  __device__ __forceinline__ void load(const bf16_t* __restrict__ X, int64_t ld, int r0, int k0, int R, int K) {
    const int R8 = (R + 7) & ~7, K8 = (K + 7) & ~7;
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      const int c = p * NT + threadIdx.x;
      const int lr = c / (S::lds_cols / 8), lc = (c % (S::lds_cols / 8)) * 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (KC) {
        const int row = r0 + lr, k = k0 + lc;
        // (the explicit global load only where the load is unconditional: under a predicate it came out with a wait
        // behind every second load)
        if (!CHECK) v = pm_ldg16(X + (int64_t)row * ld + k);
        else if (row < R && k < K8) v = *reinterpret_cast<const uint4*>(X + (int64_t)row * ld + k);
      } else {
        const int k = k0 + lr, row = r0 + lc;
        if (!CHECK) v = pm_ldg16(X + (int64_t)k * ld + row);
        else if (k < K && row < R8) v = *reinterpret_cast<const uint4*>(X + (int64_t)k * ld + row);
      }
      r[p] = v;
    }
  }
  __device__ __forceinline__ void store(bf16_t* s) const {
#pragma unroll
    for (int p = 0; p < PER; ++p) store_part(s, p);
  }
  __device__ __forceinline__ void store_part(bf16_t* s, int p) const {
    const int c = p * NT + threadIdx.x;
    const int lr = c / (S::lds_cols / 8), lc = (c % (S::lds_cols / 8)) * 8;
    *reinterpret_cast<uint4*>(s + lr * S::stride + lc) = r[p];
  }
};

// fragment of the 32-row tile starting at tile row r32, contraction indices kb .. kb+15
template <int ROWS, bool KC>
__device__ __forceinline__ pm_bf16x8 pm_big_frag(const bf16_t* s, int r32, int kb, int lane) {
  using S = PmBigTile<ROWS, KC>;
  if (KC) {
    return *reinterpret_cast<const pm_bf16x8*>(s + (r32 + (lane & 31)) * S::stride + kb + (lane >> 5) * 8);
  } else {
    // Transpose load: in each group of 16 lanes, lane q supplies the address of 4 consecutive
    // elements (one k-row, 4 rows of the operand) and receives, for operand row (its index in the
    // group), the elements of 4 consecutive k-rows.  Lane q of group g addresses
    // k-row kb + 8*(g/2) + q/4, operand rows r32 + 16*(g%2) + 4*(q%4) .. +3.
    const int g = lane >> 4, q = lane & 15;
    const bf16_t* p = s + (kb + 8 * (g >> 1) + (q >> 2)) * S::stride + r32 + 16 * (g & 1) + 4 * (q & 3);
    typedef pm_v4s __attribute__((address_space(3))) * lds_v4s;
    const pm_v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
    const pm_v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 4 * S::stride));
    union { pm_bf16x8 v; pm_v4s h[2]; } u;
    u.h[0] = lo;
    u.h[1] = hi;
    return u.v;
  }
}

template <int BI_, int BJ_, int WI_, int WJ_>
struct PmBigCfg {
  static constexpr int BI = BI_, BJ = BJ_, WI = WI_, WJ = WJ_, NT = WI_ * WJ_ * 64;
  // waves per SIMD the register budget is sized for: the 128 x 128 wave tile holds 256 accumulator
  // registers and needs the whole 512-entry file (its LDS footprint allows one block per CU anyway)
  static constexpr int WPE = (BI_ / WI_) * (BJ_ / WJ_) >= 128 * 128 ? 1 : (BI_ / WI_) * (BJ_ / WJ_) <= 32 * 32 ? 4 : 2;
};

template <class Cfg, bool AKC, bool BKC>
struct PmBigLds {
  static constexpr int elems = 2 * (PmBigTile<Cfg::BI, AKC>::elems + PmBigTile<Cfg::BJ, BKC>::elems);
};

// id: index of this block among the tiles_i * tiles_j blocks of the problem.
// CHECK false: I, J multiples of the block tile and K a multiple of 64 (no bounds tests anywhere).
//
// Software pipeline over the 64-deep slabs of the contraction: two LDS stages and two register sets.
// While the MFMAs of slab kt run on LDS stage kt & 1, the global loads of slab kt + 2 are issued into
// the register set that slab kt came from, and slab kt + 1 (loaded one iteration earlier) moves from
// the other register set into the other LDS stage, a part behind each k-step.  A load therefore has
// more than a slab of MFMA time to arrive before it is waited for; one barrier per slab.
//
// Seg: PmNoSeg, or PmKSeg3 = the contraction runs over three operand pairs of Kseg indices each
// (out = A0 B0 + A1 B1 + A2 B2 as ONE product with K = 3 Kseg: the slab loader switches base pointers
// at the segment boundaries, which fall on slab boundaries since Kseg is a multiple of 64).
struct PmNoSeg {
  static constexpr bool on = false;
};
struct PmKSeg3 {                     // pair 0 is the problem's own A and B
  static constexpr bool on = true;
  const bf16_t* A1;
  const bf16_t* A2;
  PmWLoc<bf16_t> B1, B2;
  int Kseg;
};
template <class Cfg, bool AKC, bool BKC, bool CHECK, class Epi, class Seg = PmNoSeg>
__device__ __forceinline__ void pm_gemm_big_body(const PmGemmProb<Epi>& pr, int id, int tiles_i, int tiles_j, bf16_t* smem,
                                                 bool xcd_remap = true, const Seg& sg = Seg()) {
  constexpr int BI = Cfg::BI, BJ = Cfg::BJ, WI = Cfg::WI, WJ = Cfg::WJ, NT = Cfg::NT, BK = 64;
  constexpr int TI = BI / WI / 32, TJ = BJ / WJ / 32;
  using SA = PmBigTile<BI, AKC>;
  using SB = PmBigTile<BJ, BKC>;
  constexpr int STAGE = SA::elems + SB::elems;      // stage s: A at s*STAGE, B at s*STAGE + SA::elems

  // XCD-aware mapping: consecutive block ids land on consecutive XCDs (8 of them), so give each
  // XCD a contiguous range of tiles, and inside it walk the tiles in column panels of 8 row tiles.
  const int nblk = tiles_i * tiles_j;
  if (xcd_remap && (nblk & 7) == 0) id = (id & 7) * (nblk >> 3) + (id >> 3);
  constexpr int GROUP = 8;
  const int panel = id / (GROUP * tiles_j);
  const int first_i = panel * GROUP;
  const int rows_in_panel = (tiles_i - first_i) < GROUP ? (tiles_i - first_i) : GROUP;
  const int by = first_i + (id % (GROUP * tiles_j)) % rows_in_panel;
  const int bx = (id % (GROUP * tiles_j)) / rows_in_panel;

  const int I = pr.I, J = pr.J, K = pr.K;
  const int i0 = by * BI, j0 = bx * BJ;
  const bf16_t* __restrict__ A = pr.A;
  const bf16_t* __restrict__ B = pr.B.get();
  const int64_t lda = pr.lda, ldb = pr.ldb;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wj = wave % WJ, wi = wave / WJ;
  const int lr = lane & 31, kg = lane >> 5;

  pm_f32x16 acc[TI][TJ];
#pragma unroll
  for (int a = 0; a < TI; ++a)
#pragma unroll
    for (int b = 0; b < TJ; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
  Epi epi = pr.epi;
  float colsum = 0.f;
  const bool do_colsum = Epi::kColSumA && !AKC && bx == 0 && epi.wants_colsum();

  using LA = PmBigLoader<BI, AKC, NT>;
  using LB = PmBigLoader<BJ, BKC, NT>;
  constexpr int QA = (LA::PER + 3) / 4, QB = (LB::PER + 3) / 4;
  LA la0, la1;
  LB lb0, lb1;
  const int nk = (K + BK - 1) / BK;
  // segment p > 0 is addressed with the running contraction index through a base pointer moved back by
  // p * Kseg contraction steps, so the loader's address arithmetic is the same as for a single pair
  const bf16_t* As1 = A;
  const bf16_t* As2 = A;
  const bf16_t* Bs1 = B;
  const bf16_t* Bs2 = B;
  int Kseg = K;
  if constexpr (Seg::on) {
    Kseg = sg.Kseg;
    const int64_t ka = AKC ? 1 : lda, kb = BKC ? 1 : ldb;
    As1 = sg.A1 - (int64_t)Kseg * ka;
    As2 = sg.A2 - 2 * (int64_t)Kseg * ka;
    Bs1 = sg.B1.get() - (int64_t)Kseg * kb;
    Bs2 = sg.B2.get() - 2 * (int64_t)Kseg * kb;
  }
  // global loads of slab kt into a register set.  (The selects work on copies of the pointers: a
  // conditional between the captured variables themselves is a conditional between their addresses,
  // which keeps every captured variable in memory.)
  auto load_slab = [&](LA& sa, LB& sb, int kt_) __attribute__((always_inline)) {
    const int k_ = kt_ * BK;
    const bf16_t* Xa_ = A;
    const bf16_t* Xb_ = B;
    if constexpr (Seg::on) {
      const bf16_t *a1_ = As1, *a2_ = As2, *b1_ = Bs1, *b2_ = Bs2;
      const int ks_ = Kseg;
      if (k_ >= ks_) Xa_ = a1_, Xb_ = b1_;
      if (k_ >= 2 * ks_) Xa_ = a2_, Xb_ = b2_;
    }
    sa.template load<CHECK>(Xa_, lda, i0, k_, I, K);
    sb.template load<CHECK>(Xb_, ldb, j0, k_, J, K);
  };
  load_slab(la0, lb0, 0);
  la0.store(smem);
  lb0.store(smem + SA::elems);
  if (nk > 1) load_slab(la1, lb1, 1);
  __syncthreads();

  // one slab: fa / fb = register set that is free (refilled with slab kt + 2), na / nb = register set
  // holding slab kt + 1 (moved to the other LDS stage).  steady (compile-time): slabs kt + 1 and
  // kt + 2 exist, so the loads and stores are unconditional and the compiler's wait counts before
  // the LDS stores cover exactly the older register set.
  auto slab = [&](auto steady, int kt, LA& fa_set, LB& fb_set, const LA& na_set, const LB& nb_set)
                  __attribute__((always_inline)) {
    constexpr bool STEADY = decltype(steady)::value;
    const int cur = kt & 1;
    const bf16_t* cA = smem + cur * STAGE;
    const bf16_t* cB = cA + SA::elems;
    if (STEADY || kt + 2 < nk) {
      load_slab(fa_set, fb_set, kt + 2);
      // keep the loads here, ahead of the slab's MFMAs (the instruction scheduler otherwise sinks
      // them to the end of the slab to shorten register live ranges, which costs the latency cover)
      __builtin_amdgcn_sched_barrier(0);
    }
    if (Epi::kColSumA && !AKC) {
      if (do_colsum && threadIdx.x < BI) {
#pragma unroll 8
        for (int k = 0; k < BK; ++k) colsum += bf16_to_f32(cA[k * SA::stride + threadIdx.x]);
      }
    }
    // fragments are double-buffered in registers: the LDS reads of k-step ks+1 are in flight
    // while the MFMAs of k-step ks issue
    pm_bf16x8 fa[2][TI], fb[2][TJ];
#pragma unroll
    for (int a = 0; a < TI; ++a) fa[0][a] = pm_big_frag<BI, AKC>(cA, (wi * TI + a) * 32, 0, lane);
#pragma unroll
    for (int b = 0; b < TJ; ++b) fb[0][b] = pm_big_frag<BJ, BKC>(cB, (wj * TJ + b) * 32, 0, lane);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      if (ks + 1 < BK / 16) {
#pragma unroll
        for (int a = 0; a < TI; ++a) fa[n][a] = pm_big_frag<BI, AKC>(cA, (wi * TI + a) * 32, (ks + 1) * 16, lane);
#pragma unroll
        for (int b = 0; b < TJ; ++b) fb[n][b] = pm_big_frag<BJ, BKC>(cB, (wj * TJ + b) * 32, (ks + 1) * 16, lane);
      }
#pragma unroll
      for (int a = 0; a < TI; ++a)
#pragma unroll
        for (int b = 0; b < TJ; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c][a], fb[c][b], acc[a][b], 0, 0, 0);
      if (STEADY || kt + 1 < nk) {
        if (ks * QA < LA::PER) {
#pragma unroll
          for (int q = 0; q < QA; ++q)
            if (ks * QA + q < LA::PER) na_set.store_part(smem + (cur ^ 1) * STAGE, ks * QA + q);
        }
        if (ks * QB < LB::PER) {
#pragma unroll
          for (int q = 0; q < QB; ++q)
            if (ks * QB + q < LB::PER) nb_set.store_part(smem + (cur ^ 1) * STAGE + SA::elems, ks * QB + q);
        }
      }
    }
    __syncthreads();
  };
  int kt = 0;
  for (; kt + 3 < nk; kt += 2) {          // both slabs of the pair have successors kt + 2 and kt + 3
    slab(std::true_type{}, kt, la0, lb0, la1, lb1);
    slab(std::true_type{}, kt + 1, la1, lb1, la0, lb0);
  }
  for (; kt < nk; kt += 2) {              // the last one to three slabs
    slab(std::false_type{}, kt, la0, lb0, la1, lb1);
    if (kt + 1 < nk) slab(std::false_type{}, kt + 1, la1, lb1, la0, lb0);
  }

  epi.begin();
  if (Epi::kColSumA && !AKC) {
    if (do_colsum && threadIdx.x < BI && (!CHECK || i0 + (int)threadIdx.x < I)) epi.colsum(i0 + threadIdx.x, colsum);
  }
  // Epilogue through LDS (the operand stages are dead after the last barrier): each wave parks one
  // 32-row stripe of its fp32 tile at a time, row-major in a private region, then every lane takes 8
  // consecutive columns of a row, so global accesses are 16-byte pieces of full row segments instead
  // of 2-byte scatters.  (A wave's LDS accesses complete in program order: no barrier is needed
  // between parking and reading back inside one wave.)
  constexpr int WT_I = TI * 32, WT_J = TJ * 32, ES = WT_J + 4;          // wave tile and its padded row stride
  static_assert((size_t)PmBigLds<Cfg, AKC, BKC>::elems * 2 >= (size_t)WI * WJ * 32 * ES * 4, "epilogue staging does not fit the operand stages");
  // all stripes of the wave tile at once when the stages are large enough (one write -> read round trip
  // through LDS per tile instead of one per stripe), else stripe by stripe
  constexpr bool ALL = (size_t)PmBigLds<Cfg, AKC, BKC>::elems * 2 >= (size_t)WI * WJ * WT_I * ES * 4;
  constexpr int SR = ALL ? WT_I : 32;                                   // rows staged per pass
  float* es = reinterpret_cast<float*>(smem) + (size_t)wave * SR * ES;
  const int wi0 = i0 + wi * WT_I, wj0 = j0 + wj * WT_J;
#pragma unroll
  for (int a0 = 0; a0 < TI; a0 += SR / 32) {
#pragma unroll
    for (int a = a0; a < a0 + SR / 32; ++a)
#pragma unroll
      for (int b = 0; b < TJ; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          es[((a - a0) * 32 + 8 * (v >> 2) + 4 * kg + (v & 3)) * ES + b * 32 + lr] = acc[a][b][v];
    // groups of up to four 8-column pieces per lane: what the epilogue reads from memory is requested for the
    // whole group first (a load issued behind a store waits for that store to complete)
    constexpr int ITERS = SR * (WT_J / 8) / 64, GRP = ITERS < 4 ? ITERS : 4;
    static_assert(SR * (WT_J / 8) % 64 == 0 && ITERS % GRP == 0, "staged pass must split evenly over the lanes");
#pragma unroll
    for (int it0 = 0; it0 < ITERS; it0 += GRP) {
      typename Epi::Pre pre[GRP];
      int ii[GRP], jj[GRP];
      bool full[GRP];
#pragma unroll
      for (int u = 0; u < GRP; ++u) {
        const int c = lane + 64 * (it0 + u);
        const int r = c / (WT_J / 8), c8 = (c % (WT_J / 8)) * 8;
        ii[u] = wi0 + a0 * 32 + r;
        jj[u] = wj0 + c8;
        full[u] = !CHECK || (ii[u] < I && jj[u] + 8 <= J);
        if (full[u]) pre[u] = epi.pre8(ii[u], jj[u]);
      }
#pragma unroll
      for (int u = 0; u < GRP; ++u) {
        const int c = lane + 64 * (it0 + u);
        const int r = c / (WT_J / 8), c8 = (c % (WT_J / 8)) * 8;
        const int i = ii[u], j = jj[u];
        if (CHECK && (i >= I || j >= J)) continue;
        float vals[8];
        const float4 v0 = *reinterpret_cast<const float4*>(es + r * ES + c8);
        const float4 v1 = *reinterpret_cast<const float4*>(es + r * ES + c8 + 4);
        vals[0] = v0.x; vals[1] = v0.y; vals[2] = v0.z; vals[3] = v0.w;
        vals[4] = v1.x; vals[5] = v1.y; vals[6] = v1.z; vals[7] = v1.w;
        if (full[u]) {
          epi.op8(i, j, vals, pre[u]);
        } else {
          for (int e = 0; e < 8 && j + e < J; ++e) epi(i, j + e, vals[e]);
        }
      }
    }
  }
  if constexpr (pm_has_tile_update<Epi>::value) {
    static_assert(!CHECK, "whole tiles only");
    __syncthreads();      // the block's stores of the tile are visible to all its waves
    epi.template update_tile<BI, BJ, NT>(i0, j0);
  }
}

template <class Cfg, bool AKC, bool BKC, bool CHECK, class Epi>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(Cfg::WPE, Cfg::WPE))) void pm_gemm_big_kernel(PmGemmProb<Epi> pr, int tiles_i, int tiles_j) {
  __shared__ __attribute__((aligned(16))) bf16_t smem[PmBigLds<Cfg, AKC, BKC>::elems];
  pm_gemm_big_body<Cfg, AKC, BKC, CHECK, Epi>(pr, blockIdx.x, tiles_i, tiles_j, smem);
}

// Three products of equal shape in one launch (the query / key / value projections share their
// input): block b works on problem b / (tiles_i * tiles_j).  One launch instead of three keeps the
// chip filled across the problems' first and last waves of tiles.
template <class Cfg, bool AKC, bool BKC, bool CHECK, class Epi>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(Cfg::WPE, Cfg::WPE))) void pm_gemm_big_multi3_kernel(PmGemmProb<Epi> p0, PmGemmProb<Epi> p1, PmGemmProb<Epi> p2, int tiles_i, int tiles_j) {
  __shared__ __attribute__((aligned(16))) bf16_t smem[PmBigLds<Cfg, AKC, BKC>::elems];
  const int nt = tiles_i * tiles_j;
  const int p = blockIdx.x / nt, id = blockIdx.x - p * nt;      // uniform over the block
  pm_gemm_big_body<Cfg, AKC, BKC, CHECK, Epi>(p == 0 ? p0 : p == 1 ? p1 : p2, id, tiles_i, tiles_j, smem);
}

// One product with a very long contraction and too few output tiles to fill the chip, cut into two halves of
// the contraction that run side by side: block b works on half b / (tiles_i * tiles_j); each half writes its
// own fp32 output and the consumer adds the two.  (256 x 256 tiles: the only block shape whose main loop gets
// past 1.1 PFLOP/s needs K >= 8192 to amortise its start and end.)
template <class Cfg, bool AKC, bool BKC, class Epi>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(Cfg::WPE, Cfg::WPE))) void pm_gemm_big_khalves_kernel(PmGemmProb<Epi> p0, PmGemmProb<Epi> p1, int tiles_i, int tiles_j) {
  __shared__ __attribute__((aligned(16))) bf16_t smem[PmBigLds<Cfg, AKC, BKC>::elems];
  const int nt = tiles_i * tiles_j;
  const int p = blockIdx.x / nt, id = blockIdx.x - p * nt;      // uniform over the block
  pm_gemm_big_body<Cfg, AKC, BKC, false, Epi>(p == 0 ? p0 : p1, id, tiles_i, tiles_j, smem);
}

// One product whose contraction runs over three operand pairs (PmKSeg3); pr.K = 3 * Kseg, pr.A / pr.B = pair 0.
template <class Cfg, bool AKC, bool BKC, bool CHECK, class Epi>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(Cfg::WPE, Cfg::WPE))) void pm_gemm_big_kseg3_kernel(PmGemmProb<Epi> pr, PmKSeg3 sg, int tiles_i, int tiles_j) {
  __shared__ __attribute__((aligned(16))) bf16_t smem[PmBigLds<Cfg, AKC, BKC>::elems];
  pm_gemm_big_body<Cfg, AKC, BKC, CHECK, Epi, PmKSeg3>(pr, blockIdx.x, tiles_i, tiles_j, smem, true, sg);
}

// Many problems in one launch, scheduled per XCD.  Consecutive block ids land on consecutive XCDs
// (8 of them, each with its own L2), so block b works for XCD b % 8 at position b / 8 of that XCD's
// own work list: a list of segments (problem, first tile, tile count) built by the host so that the
// tiles that run concurrently on one XCD come from one problem (or one row range of a huge one) and
// share their operand panels through that XCD's L2.  All weight-gradient products of a token-rich
// step go out together this way: single problems of 64 tiles cannot fill 256 compute units, and with
// the contraction over thousands of tokens every re-read of an operand panel from memory is what
// bounds the kernel.  No split of the contraction, no atomics.
struct PmXcdSeg {
  int32_t prob;        // problem index
  int32_t tile0;       // first tile of the problem handled by this segment (panel order, see the body)
  int32_t start;       // position of the segment's first tile in the XCD's list
  int32_t pad_;
};
// segs: 8 lists of `max_segs` entries each (unused entries have start = INT_MAX); nseg[x] entries are valid
template <class Cfg, bool AKC, bool BKC, bool CHECK, class Epi>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(Cfg::WPE, Cfg::WPE))) void pm_gemm_big_grouped_kernel(const PmGemmProb<Epi>* __restrict__ probs, const PmXcdSeg* __restrict__ segs, const int32_t* __restrict__ xcd_tiles, int max_segs) {
  __shared__ __attribute__((aligned(16))) bf16_t smem[PmBigLds<Cfg, AKC, BKC>::elems];
  const int x = blockIdx.x & 7, pos = blockIdx.x >> 3;
  if (pos >= xcd_tiles[x]) return;
  const PmXcdSeg* list = segs + (size_t)x * max_segs;
  int lo = 0, hi = max_segs - 1;                 // last segment with start <= pos
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (list[mid].start <= pos) lo = mid; else hi = mid - 1;
  }
  const PmXcdSeg sg = list[lo];
  const PmGemmProb<Epi> pr = probs[sg.prob];
  const int ti = (pr.I + Cfg::BI - 1) / Cfg::BI, tj = (pr.J + Cfg::BJ - 1) / Cfg::BJ;
  pm_gemm_big_body<Cfg, AKC, BKC, CHECK, Epi>(pr, sg.tile0 + (pos - sg.start), ti, tj, smem, false);
}

// 128 x 128 block, 4 waves x (64 x 64): 80 KB of LDS, so two blocks share a CU and cover each
// other's barriers.  Measured on 8192-row problems (K, N in {1024, 4096}) this beat 256 x 256
// (8 waves x 128 x 64) and 256 x 128 (4 waves x 128 x 64) blocks in 7 of 9 shape / layout cases.
using PmBig128 = PmBigCfg<128, 128, 2, 2>;
// 256 x 256 block, 8 waves x (128 x 64): one block per CU, two waves per SIMD (128 accumulator registers
// each).  Per MFMA it reads 3/4 of the LDS bytes of the 64 x 64 wave tile and writes half.  Measured on
// the 8192-deep weight gradients against 4 waves x (128 x 128) (one wave per SIMD, still less LDS
// traffic): 2.7 vs 3.5 ms - the second wave per SIMD, which covers the other's LDS and barrier waits,
// matters more than the traffic.
using PmBig256 = PmBigCfg<256, 256, 2, 4>;
// 64 x 64 block, 4 waves x (32 x 32): 37 KB of LDS, four blocks per CU.  For token counts in the low
// thousands with narrow layers (4096 x 512 x 512 ...): enough tiles to fill the chip, and the same
// software pipeline hides the memory latency that a load - store - compute loop pays once per slab.
using PmBig64 = PmBigCfg<64, 64, 2, 2>;

// 256 x 128 and 128 x 256 blocks, 8 waves x (64 x 64), one block per compute unit: the operand tile with 256 rows is
// written to LDS once for two of the other's (a quarter less LDS write traffic and global load issue than two
// 128 x 128 blocks), with the same eight waves per compute unit.  Measured stand-alone on the token-rich products of
// the 12-layer workload (8192 rows; one block per compute unit or a few rounds, operands warm) against 128 x 128:
// K = 4096 forward 78 -> 73 us, feed-forward expansion 88 -> 81 us (256 x 128); data gradients 23 -> 21 us (K = 1024),
// 79 -> 74 us (K = 4096), 92 -> 87 us (4096 columns; 128 x 256); the vocabulary projection (hundreds of rounds, fp32
// output) is slower on them.  Inside a step only some of these gains remain (pm_rect_tiles says which epilogues
// take the rectangular blocks).
using PmBigTall = PmBigCfg<256, 128, 4, 2>;
using PmBigWide = PmBigCfg<128, 256, 2, 4>;
// a problem for these blocks: whole tiles, at least one per compute unit and at most a few rounds, K >= 1024
template <class Cfg>
inline bool pm_big_rect_suits(int I, int J, int K);

// true if no tile of the problem needs a bounds test
template <class Cfg>
inline bool pm_big_aligned(int I, int J, int K) { return I % Cfg::BI == 0 && J % Cfg::BJ == 0 && K % 64 == 0; }

template <class Cfg>
inline bool pm_big_rect_suits(int I, int J, int K) {
  if (!pm_big_aligned<Cfg>(I, J, K) || K < 1024) return false;
  const long t = (long)(I / Cfg::BI) * (J / Cfg::BJ);
  return t >= 256 && t <= 2048;
}

template <class Cfg, bool AKC, bool BKC, class Epi>
inline void pm_big_launch(hipStream_t st, const PmGemmProb<Epi>& pr) {
  const int ti = (pr.I + Cfg::BI - 1) / Cfg::BI, tj = (pr.J + Cfg::BJ - 1) / Cfg::BJ;
  if (pm_big_aligned<Cfg>(pr.I, pr.J, pr.K))
    hipLaunchKernelGGL((pm_gemm_big_kernel<Cfg, AKC, BKC, false, Epi>), dim3(ti * tj), dim3(Cfg::NT), 0, st, pr, ti, tj);
  else
    hipLaunchKernelGGL((pm_gemm_big_kernel<Cfg, AKC, BKC, true, Epi>), dim3(ti * tj), dim3(Cfg::NT), 0, st, pr, ti, tj);
}

// mid-size problems on the pipelined kernel with 64 x 64 blocks
template <bool AKC, bool BKC, class Epi>
inline bool pm_mid_try(hipStream_t st, const PmGemmProb<Epi>& pr) {
  const long tiles64 = (long)((pr.I + 63) / 64) * ((pr.J + 63) / 64);
  if (tiles64 < 256 || pr.K < 256) return false;
  pm_big_launch<PmBig64, AKC, BKC>(st, pr);
  return true;
}

// true if the problem was large enough for (and was launched on) the big-tile kernel
template <bool AKC, bool BKC, class Epi>
inline bool pm_big_try(hipStream_t st, const PmGemmProb<Epi>& pr) {
  const long tiles = (long)((pr.I + 127) / 128) * ((pr.J + 127) / 128);
  if (pr.K < 256) return false;
  // enough tiles to fill the chip, or fewer tiles with a long contraction (the weight gradient of a
  // token-rich microbatch: the deep software pipeline matters more than idle CUs; splitting K
  // over blocks with fp32 atomics was measured slower than leaving 3/4 of the CUs idle)
  if (tiles < 200) {
    // too few 128 x 128 tiles to fill the chip: 64 x 64 blocks if those do (measured 1.3 - 1.6 x faster
    // on 4096 x 512 x 2048 and on the 1024 x 1024 weight gradient over 8192 tokens), else only for long K
    const long tiles64 = (long)((pr.I + 63) / 64) * ((pr.J + 63) / 64);
    if (tiles64 >= 256) return false;
    if (!(tiles >= 32 && pr.K >= 2048)) return false;
  }
  // long contraction and enough 256 x 256 tiles for every compute unit: the larger tile (measured on
  // 32000 x 1024 x 8192: 735 vs 937 us); with K <= 4096 the 128 x 128 tile is as fast or faster
  if (pr.K >= 8192 && (long)((pr.I + 255) / 256) * ((pr.J + 255) / 256) >= 256 && pm_big_aligned<PmBig256>(pr.I, pr.J, pr.K)) {
    pm_big_launch<PmBig256, AKC, BKC>(st, pr);
    return true;
  }
  // activations times weights with whole rectangular tiles: the tall block where the weights are read along the
  // contraction (forward), the wide one where they are read across it (data gradient)
  if constexpr (AKC && pm_rect_tiles<Epi>::value) {
    using Rect = std::conditional_t<BKC, PmBigTall, PmBigWide>;
    if (pm_big_rect_suits<Rect>(pr.I, pr.J, pr.K)) {
      const int ti = pr.I / Rect::BI, tj = pr.J / Rect::BJ;
      hipLaunchKernelGGL((pm_gemm_big_kernel<Rect, AKC, BKC, false, Epi>), dim3(ti * tj), dim3(Rect::NT), 0, st, pr, ti, tj);
      return true;
    }
  }
  pm_big_launch<PmBig128, AKC, BKC>(st, pr);
  return true;
}


// Which pipelined block tile a problem with `tiles128` / `tiles64` block tiles in total gets: 0 none, 128, 64.
inline int pm_big_choice(long tiles128, long tiles64, int K) {
  if (K < 256) return 0;
  if (tiles128 >= 200) return 128;
  if (tiles64 >= 256) return 64;
  return 0;
}

// Three products of equal shape and layout (A row-major over the contraction, B likewise) in one launch.
// False (nothing launched) if the shapes do not suit the pipelined kernels.
template <class Epi>
inline bool pm_gemm_multi3_try(hipStream_t st, const PmGemmProb<Epi> (&pr)[3]) {
  const int I = pr[0].I, J = pr[0].J, K = pr[0].K;
  for (int p = 0; p < 3; ++p) {
    if (pr[p].I != I || pr[p].J != J || pr[p].K != K) return false;
    if (!pm_mfma_fits(I, J, K, pr[p].A, pr[p].lda, 1, pr[p].B.base, pr[p].B.stride, pr[p].ldb, 1)) return false;
  }
  const long t128 = (long)((I + 127) / 128) * ((J + 127) / 128), t64 = (long)((I + 63) / 64) * ((J + 63) / 64);
  const int pick = pm_big_choice(3 * t128, 3 * t64, K);
  auto go = [&](auto cfg) {
    using Cfg = decltype(cfg);
    const int ti = (I + Cfg::BI - 1) / Cfg::BI, tj = (J + Cfg::BJ - 1) / Cfg::BJ;
    if (pm_big_aligned<Cfg>(I, J, K))
      hipLaunchKernelGGL((pm_gemm_big_multi3_kernel<Cfg, true, true, false, Epi>), dim3(3 * ti * tj), dim3(Cfg::NT), 0, st,
                         pr[0], pr[1], pr[2], ti, tj);
    else
      hipLaunchKernelGGL((pm_gemm_big_multi3_kernel<Cfg, true, true, true, Epi>), dim3(3 * ti * tj), dim3(Cfg::NT), 0, st,
                         pr[0], pr[1], pr[2], ti, tj);
  };
  if (pick == 128) go(PmBig128());
  else if (pick == 64) go(PmBig64());
  else return false;
  return true;
}

// out = sum over p of A_p B_p with A_p (I x Kseg, row-major) and B_p (Kseg x J, row-major) as one product.
template <class Epi>
inline bool pm_gemm_kseg3_try(hipStream_t st, int I, int J, int Kseg, const bf16_t* const (&A)[3], int64_t lda,
                              const PmWLoc<bf16_t> (&B)[3], int64_t ldb, const Epi& epi) {
  if (Kseg % 64) return false;
  for (int p = 0; p < 3; ++p)
    if (!pm_mfma_fits(I, J, Kseg, A[p], lda, 1, B[p].base, B[p].stride, 1, ldb)) return false;
  const long t128 = (long)((I + 127) / 128) * ((J + 127) / 128), t64 = (long)((I + 63) / 64) * ((J + 63) / 64);
  const int pick = pm_big_choice(t128, t64, 3 * Kseg);
  PmGemmProb<Epi> pr{I, J, 3 * Kseg, A[0], lda, B[0], ldb, epi};
  PmKSeg3 sg{A[1], A[2], B[1], B[2], Kseg};
  if (pm_big_rect_suits<PmBigTall>(I, J, Kseg)) {      // (measured 56.6 us tall, 58.0 wide, 60.5 on 128 x 128)
    const int ti = I / 256, tj = J / 128;
    hipLaunchKernelGGL((pm_gemm_big_kseg3_kernel<PmBigTall, true, false, false, Epi>), dim3(ti * tj), dim3(PmBigTall::NT), 0, st, pr,
                       sg, ti, tj);
    return true;
  }
  auto go = [&](auto cfg) {
    using Cfg = decltype(cfg);
    const int ti = (I + Cfg::BI - 1) / Cfg::BI, tj = (J + Cfg::BJ - 1) / Cfg::BJ;
    if (pm_big_aligned<Cfg>(I, J, Kseg))
      hipLaunchKernelGGL((pm_gemm_big_kseg3_kernel<Cfg, true, false, false, Epi>), dim3(ti * tj), dim3(Cfg::NT), 0, st, pr,
                         sg, ti, tj);
    else
      hipLaunchKernelGGL((pm_gemm_big_kseg3_kernel<Cfg, true, false, true, Epi>), dim3(ti * tj), dim3(Cfg::NT), 0, st, pr,
                         sg, ti, tj);
  };
  if (pick == 128) go(PmBig128());
  else if (pick == 64) go(PmBig64());
  else return false;
  return true;
}
