// The forward chain and the data-gradient chain of an MLP with few rows per microbatch, each as ONE
// persistent launch (bf16, gfx950).
//
// With 128 rows a stage product (128 x 1024 x 1024) takes about a microsecond of work, a dependent
// kernel launch 4.4 us, and a step has two such products per stage in sequence (the per-stage forward
// and backward of Sec. 2.1).  Here one grid of co-resident blocks walks the whole chain.  A block owns
// 32 x 32 output tiles; it stages the 32 input rows of a tile in LDS (panels of up to 1024 columns), its
// 16 waves split the contraction in slices of 64 and sum their partial tiles through LDS.  The tile of
// unit l needs row tile rt of unit l-1's output, which other blocks of the same launch are still writing.
// There is no grid-wide barrier, no flag and no cache maintenance - the data itself says when it is there:
//   * before the launch (in the kernel that stages the batch) every tensor that travels between blocks
//     inside the launch (activations a, gradients dz) is filled with all-ones 8-byte words.  Such a word
//     is four bf16 NaNs with a full payload; a producer that would store exactly that word stores another
//     NaN instead, so a finished tensor holds none;
//   * a producer writes its tile as 8-byte agent-scope stores (written through to the memory side, where
//     all eight XCDs see them; a word appears whole or not at all);
//   * a consumer reads with 8-byte agent-scope loads (which do not trust an XCD-local cached copy),
//     consecutive threads taking consecutive words so that every request covers whole cache lines: each
//     thread first polls ONE word of its share until it is there (little traffic while nothing has arrived
//     yet), then loads the rest and asks again for every word that still reads all ones.
//   One memory-side hop (0.6 us between two compute units, measured) separates two units: store lands, next
//   poll sees it.  A counter per row tile instead needs the stores' acknowledgement, the increment, the poll
//   and then the loads.
//   * the weights (never written inside the launch) are read with ordinary loads; the first slice of a
//     tile's weights and its bias (forward) or stored pre-activation (backward) are requested one tile
//     AHEAD, right after the current tile's inputs have arrived, so their memory latency - a ring slot last
//     written tau steps ago - is spent while the tile is computed and the next one waited for; the unit
//     tables are resolved (ring slot -> address) once, into LDS, when the launch starts.
// Every wait is bounded: after PM_CHAIN_SPINS polls a thread sets hdr->chain_err (sticky, reported by the
// next synchronising call as PM_EHIP) and carries on with what it has, and once the flag is up nobody waits
// any more, so the launch always ends.  The host launches at most one block per compute unit, all of them
// resident (nothing else runs on the stream's device meanwhile: the launch is stream-ordered after its
// producers).
//
// Shapes (checked on the host; anything else keeps the launch-per-product path): rows M a multiple of 32,
// at most 128; a unit's n_in a multiple of 64, n_out a multiple of 32; dense rows (leading dimension =
// width).
#pragma once
#include "pm_common.hpp"
#include "pm_mfma_types.hpp"

constexpr unsigned PM_CHAIN_SPINS = 1u << 17;   // polls of one wait before giving up (a fraction of a second)
constexpr int PM_CHAIN_NT = 1024;               // 16 waves per block
constexpr int PM_CHAIN_MAX_ROW_TILES = 4;       // M <= 128 (bounds the tiles per unit, nothing is sized by it)
constexpr int PM_CHAIN_MAX_UNITS = 96;          // units of one chained launch (their resolved tables sit in LDS)
constexpr int PM_CHAIN_KP = 1024;               // columns of the input panel staged in LDS
constexpr int PM_CHAIN_LDA = PM_CHAIN_KP + 8;   // its row stride in elements (16-byte aligned rows, staggered banks)
constexpr int PM_CHAIN_STAGE_BYTES = 32 * PM_CHAIN_LDA * 2;   // >= the 64 KiB of the 16 partial tiles that reuse it

// One unit of the forward chain: z = in W^T + b, a = act(z).
struct PmChainFwd {
  PmWLoc<bf16_t> W;      // [n_out, n_in], version max(t - tau_fwd, 0) of the unit (ring slot read in place)
  int64_t boff;          // offset of the bias inside the unit
  const bf16_t* in;      // [M, n_in]: the staged batch or the previous unit's a
  bf16_t* z;             // [M, n_out] pre-activation (kept for the backward pass)
  bf16_t* a;             // [M, n_out]
  int32_t n_in, n_out, act;
  int32_t in_shared;     // 1: `in` is produced inside this launch (polled in place)
};
// One unit of the data-gradient chain: dz_prev = (dz W_bkwd) * act_prev'(z_prev).
struct PmChainBwd {
  PmWLoc<bf16_t> W;      // [n_out, n_in], the backward weights of the unit (corrected buffer or ring slot)
  const bf16_t* dz;      // [M, n_out]
  const bf16_t* zprev;   // [M, n_in] pre-activation of the unit below (forward pass)
  bf16_t* dzprev;        // [M, n_in]
  int32_t n_in, n_out, act_prev;
  int32_t dz_shared;     // 1: dz is produced inside this launch
};

// Every pointer of these kernels comes out of a table, so the compiler cannot know that it points to device
// memory and would use flat loads - which count as LDS traffic too, so that every wait for an LDS read would also
// wait for the weights requested a tile ahead.  All accesses to device memory therefore go through
// global-address-space pointers.
#define PM_CHAIN_G __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ const T PM_CHAIN_G* pm_chain_g(const T* p) {
  return (const T PM_CHAIN_G*)p;
}
template <class T>
__device__ __forceinline__ T PM_CHAIN_G* pm_chain_g(T* p) {
  return (T PM_CHAIN_G*)p;
}

// A value read from LDS sits in vector registers even when every lane reads the same word; these move it to
// scalar registers (the unit tables are the same for the whole block).
__device__ __forceinline__ int pm_chain_uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <class T>
__device__ __forceinline__ T* pm_chain_uni(T* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<T*>(((unsigned long long)hi << 32) | lo);
}

typedef unsigned int pm_chain_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int pm_chain_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 pm_chain_ldg16(const bf16_t* p) {
  const pm_chain_u32x4 v = *pm_chain_g(reinterpret_cast<const pm_chain_u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ pm_bf16x8 pm_chain_as_frag(uint4 v) {
  union { uint4 u; pm_bf16x8 f; } x;
  x.u = v;
  return x.f;
}

constexpr unsigned long long PM_CHAIN_EMPTY = ~0ull;    // "not written yet"

__device__ __forceinline__ void pm_chain_st8_shared(bf16_t* p, float a, float b, float c, float d) {
  unsigned long long v = (unsigned long long)pm_pack_bf16(a, b) | ((unsigned long long)pm_pack_bf16(c, d) << 32);
  if (v == PM_CHAIN_EMPTY) v = PM_CHAIN_EMPTY - 1;     // four NaNs stay four NaNs, but not the "empty" word
  __hip_atomic_store(pm_chain_g(reinterpret_cast<unsigned long long*>(p)), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void pm_chain_st8_plain(bf16_t* p, float a, float b, float c, float d) {
  pm_chain_u32x2 v;
  v.x = pm_pack_bf16(a, b);
  v.y = pm_pack_bf16(c, d);
  *pm_chain_g(reinterpret_cast<pm_chain_u32x2*>(p)) = v;
}

// Rows i0 .. i0 + 31, columns k0 .. k0 + kp - 1 (kp a multiple of 64, at most PM_CHAIN_KP) of src [*, K] into the
// LDS panel At [32][PM_CHAIN_LDA].  The panel is 32 * kp / 4 words of 8 bytes; thread x takes words x, x + 1024, ...
// (word -> row word / (kp / 4), columns 4 (word % (kp / 4)) ...).  shared: other blocks of this launch may still be
// writing src (see the head of this file).  Ends with a block barrier.
__device__ __forceinline__ void pm_chain_stage(const bf16_t* src, int K, int i0, int k0, int kp, bool shared,
                                               bf16_t* At, PmStepHdr* hdr) {
  const int wpr = kp >> 2, nw = 32 * wpr, ldw = K >> 2;
  const unsigned long long PM_CHAIN_G* base = pm_chain_g(reinterpret_cast<const unsigned long long*>(src + (int64_t)i0 * K + k0));
  // word x + 1024 from word x: q rows down and r words to the right, with a carry into the next row
  const int q = PM_CHAIN_NT / wpr, r = PM_CHAIN_NT - q * wpr;
  const int row0 = (int)threadIdx.x / wpr, col0 = (int)threadIdx.x - row0 * wpr;
  // f(j, offset of word j in src, offset of word j in At, whether this thread has a word j).  The loads below are
  // issued for every j, at offset 0 where the thread has no such word: eight requests in flight, one wait.
  auto walk = [&](auto f) __attribute__((always_inline)) {
    int col = col0, go = row0 * ldw + col0, lo = row0 * PM_CHAIN_LDA + 4 * col0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      f(j, go, lo, (int)threadIdx.x + PM_CHAIN_NT * j < nw);
      col += r; go += q * ldw + r; lo += q * PM_CHAIN_LDA + 4 * r;
      if (col >= wpr) { col -= wpr; go += ldw - wpr; lo += PM_CHAIN_LDA - 4 * wpr; }
    }
  };
  unsigned long long w[8];
  if (!shared) {
    walk([&](int j, int go, int, bool mine) __attribute__((always_inline)) { w[j] = base[mine ? go : 0]; });
  } else {
    unsigned spins = 0;
    bool gave_up = false;
    // one word first
    {
      const unsigned long long PM_CHAIN_G* p0 = base + ((int)threadIdx.x < nw ? row0 * ldw + col0 : 0);
      while ((w[0] = __hip_atomic_load(p0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) == PM_CHAIN_EMPTY) {
        ++spins;
        if (((spins & 255u) == 0 && __hip_atomic_load(pm_chain_g(&hdr->chain_err), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) ||
            spins > PM_CHAIN_SPINS) {
          gave_up = true;
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
    }
    // then the rest, and again whatever is not there yet
    walk([&](int j, int go, int, bool mine) __attribute__((always_inline)) {
      if (j > 0) w[j] = __hip_atomic_load(base + (mine ? go : 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    });
    while (!gave_up) {
      bool miss = false;
      walk([&](int j, int, int, bool) __attribute__((always_inline)) { miss |= w[j] == PM_CHAIN_EMPTY; });
      if (!miss) break;
      ++spins;
      if (((spins & 255u) == 0 && __hip_atomic_load(pm_chain_g(&hdr->chain_err), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) ||
          spins > PM_CHAIN_SPINS) {
        gave_up = true;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
      walk([&](int j, int go, int, bool mine) __attribute__((always_inline)) {
        if (w[j] == PM_CHAIN_EMPTY) w[j] = __hip_atomic_load(base + (mine ? go : 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      });
    }
    if (gave_up && spins > PM_CHAIN_SPINS)
      __hip_atomic_store(pm_chain_g(&hdr->chain_err), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  walk([&](int j, int, int lo, bool mine) __attribute__((always_inline)) {
    if (mine) *reinterpret_cast<unsigned long long*>(At + lo) = w[j];
  });
  __syncthreads();
}

// tile t of a unit with tiles_i x tiles_j tiles -> (row tile, column tile).  Blocks with the same id mod 8
// share an XCD: when the column tiles divide by 8, XCD k takes the k-th eighth of them for all row tiles, so
// the rows of W a column tile needs are fetched into one L2 only.
__device__ __forceinline__ void pm_chain_tile(int t, int tiles_i, int tiles_j, int nblk, int* rt, int* ct) {
  if ((tiles_j & 7) == 0 && (nblk & 7) == 0) {
    const int per_xcd = (tiles_j >> 3) * tiles_i;          // tiles of one XCD's share
    const int x = t & 7, q = t >> 3;                        // q < per_xcd when the grid covers the unit in one round
    if (q < per_xcd) {
      *ct = x * (tiles_j >> 3) + q / tiles_i;
      *rt = q % tiles_i;
      return;
    }
  }
  *rt = t % tiles_i;
  *ct = t / tiles_i;
}

// Four 16-byte pieces of a weight slice per lane.  A wave's slice is fetched line by line - consecutive lanes take
// consecutive pieces of a row - and parked in the wave's own LDS region, from where the lanes read the operand
// layout of the matrix instruction: a lane-per-row pattern would look up 4 to 8 times as many cache lines per
// request, and the vector memory pipeline of the compute unit (one line per clock) was what a tile waited for.
struct PmChainW4 {
  uint4 a, b, c, d;
};
// forward: rows j0 .. j0 + 31 of W, 64 columns (128 bytes = 8 pieces per row): piece 64 i + lane -> row 8 i + lane / 8
__device__ __forceinline__ PmChainW4 pm_chain_ld_wf(const bf16_t* slice, int ld, int lane) {
  const bf16_t* p = slice + (int64_t)(lane >> 3) * ld + 8 * (lane & 7);
  return PmChainW4{pm_chain_ldg16(p), pm_chain_ldg16(p + (int64_t)8 * ld), pm_chain_ldg16(p + (int64_t)16 * ld),
                   pm_chain_ldg16(p + (int64_t)24 * ld)};
}
// backward: rows k .. k + 63 of W, 32 columns (64 bytes = 4 pieces per row): piece 64 i + lane -> row 16 i + lane / 4
__device__ __forceinline__ PmChainW4 pm_chain_ld_wb(const bf16_t* slice, int ld, int lane) {
  const bf16_t* p = slice + (int64_t)(lane >> 2) * ld + 8 * (lane & 3);
  return PmChainW4{pm_chain_ldg16(p), pm_chain_ldg16(p + (int64_t)16 * ld), pm_chain_ldg16(p + (int64_t)32 * ld),
                   pm_chain_ldg16(p + (int64_t)48 * ld)};
}

// One work item of a block: tile t of unit u.  The item after (u, t) is the block's next tile of the same unit,
// else its first tile of the next unit that has one for this block ({-1, 0} stands before the first item,
// {n, 0} after the last).
struct PmChainItem {
  int u, t;
};
template <class Tab, class NT>
__device__ __forceinline__ PmChainItem pm_chain_next(const Tab* tabs, int n, int tiles_i, PmChainItem it, NT ntiles_of) {
  if (it.u >= 0 && it.u < n && it.t + (int)gridDim.x < pm_chain_uni(ntiles_of(tabs[it.u])) * tiles_i) return PmChainItem{it.u, it.t + (int)gridDim.x};
  for (int u = it.u + 1; u < n; ++u)
    if ((int)blockIdx.x < pm_chain_uni(ntiles_of(tabs[u])) * tiles_i) return PmChainItem{u, (int)blockIdx.x};
  return PmChainItem{n, 0};
}
__device__ __forceinline__ void pm_chain_rt_ct(int t, int tiles_i, int tiles_j, int* rt, int* ct) {
  if (tiles_i * tiles_j <= (int)gridDim.x) pm_chain_tile(t, tiles_i, tiles_j, (int)gridDim.x, rt, ct);
  else { *rt = t % tiles_i; *ct = t / tiles_i; }
}

// ---------------------------------------------------------------------------------------------
// forward chain: units tab[0 .. n - 1]
// ---------------------------------------------------------------------------------------------
struct PmChainFwdR {       // a unit with its ring slot resolved
  const bf16_t* W;
  const bf16_t* bias;
  const bf16_t* in;
  bf16_t* z;
  bf16_t* a;
  int32_t n_in, n_out, act, in_shared;
};

__global__ __launch_bounds__(PM_CHAIN_NT) void pm_chain_fwd_kernel(const PmChainFwd* __restrict__ tab, int n, int M,
                                                                  PmStepHdr* hdr) {
  // the staged input panel; once the products are done the same memory holds the partial tiles of the 16 waves
  __shared__ __attribute__((aligned(16))) unsigned char stage_mem[PM_CHAIN_STAGE_BYTES];
  constexpr int WF = 72;                                   // LDS row stride of a parked weight slice (64 columns + pad), elements
  __shared__ __attribute__((aligned(16))) bf16_t wt[16][32 * WF];   // per wave: 32 weight rows x 64 contraction columns
  __shared__ PmChainFwdR tabs[PM_CHAIN_MAX_UNITS];
  bf16_t* At = reinterpret_cast<bf16_t*>(stage_mem);
  bf16_t* mine = wt[threadIdx.x >> 6];
  float (*red)[32 * 32] = reinterpret_cast<float (*)[32 * 32]>(stage_mem);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int lr = lane & 31, kg = lane >> 5;
  const int tiles_i = M >> 5;
  if ((int)threadIdx.x < n) {
    const PmChainFwd L = tab[threadIdx.x];
    const bf16_t* W = L.W.get();
    tabs[threadIdx.x] = PmChainFwdR{W, W + L.boff, L.in, L.z, L.a, L.n_in, L.n_out, L.act, L.in_shared};
  }
  __syncthreads();
  auto tiles_j_of = [](const PmChainFwdR& L) { return L.n_out >> 5; };
  // What a tile needs from memory that no other block produces - the first weight slice of this wave and the bias
  // entry of this thread's output column - is requested one tile ahead.  It lives in two register sets that swap
  // roles from tile to tile (the tile loop below is written out twice): copying a set would wait for its loads.
  auto request = [&](PmChainItem it, PmChainW4& w, bf16_t& b) __attribute__((always_inline)) {
    if (it.u >= n) return;
    const PmChainFwdR& T = tabs[it.u];
    const int n_in = pm_chain_uni(T.n_in), n_out = pm_chain_uni(T.n_out);
    int rt, ct;
    pm_chain_rt_ct(it.t, tiles_i, n_out >> 5, &rt, &ct);
    const int j0 = ct << 5;
    if (wave < (n_in >> 6)) w = pm_chain_ld_wf(pm_chain_uni(T.W) + (int64_t)j0 * n_in + wave * 64, n_in, lane);
    b = pm_chain_g(pm_chain_uni(T.bias))[j0 + (threadIdx.x & 31)];     // (raw bits: converting here would wait for the load)
  };
  PmChainItem it = pm_chain_next(tabs, n, tiles_i, PmChainItem{-1, 0}, tiles_j_of);
  // one tile: products with the weights in (w0, b0), the next tile's request into (w1, b1)
  auto tile = [&](const PmChainW4& w0, const bf16_t& b0, PmChainW4& w1, bf16_t& b1) __attribute__((always_inline)) {
    const PmChainFwdR& T = tabs[it.u];
    const PmChainFwdR L{pm_chain_uni(T.W), pm_chain_uni(T.bias), pm_chain_uni(T.in), pm_chain_uni(T.z), pm_chain_uni(T.a),
                        pm_chain_uni(T.n_in), pm_chain_uni(T.n_out), pm_chain_uni(T.act), pm_chain_uni(T.in_shared)};
    const int K = L.n_in;
    int rt, ct;
    pm_chain_rt_ct(it.t, tiles_i, L.n_out >> 5, &rt, &ct);
    const int i0 = rt << 5, j0 = ct << 5;
    const bf16_t* wtile = L.W + (int64_t)j0 * K;
    pm_f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const PmChainItem nxt = pm_chain_next(tabs, n, tiles_i, it, tiles_j_of);
    const bf16_t* ap = At + lr * PM_CHAIN_LDA + wave * 64 + 8 * kg;
    // park a fetched slice in this wave's LDS region (a wave's LDS accesses complete in program order: no barrier
    // inside the wave) ...
    auto park = [&](const PmChainW4& w) __attribute__((always_inline)) {
      uint4* dst = reinterpret_cast<uint4*>(mine + (lane >> 3) * WF + 8 * (lane & 7));
      dst[0] = w.a; dst[WF] = w.b; dst[2 * WF] = w.c; dst[3 * WF] = w.d;      // (8 rows = 8 WF elements = WF uint4)
    };
    // ... and multiply: lane (row lr, half kg) takes columns 16 ks + 8 kg .. + 7 of both operands
    const bf16_t* wp = mine + lr * WF + 8 * kg;
    auto products = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_chain_as_frag(*reinterpret_cast<const uint4*>(ap + 16 * ks)),
                                                      pm_chain_as_frag(*reinterpret_cast<const uint4*>(wp + 16 * ks)), acc, 0, 0, 0);
    };
    // first panel: its weight slice came ahead
    const bool first_active = wave < (min(PM_CHAIN_KP, K) >> 6);
    if (first_active) park(w0);
    pm_chain_stage(L.in, K, i0, 0, min(PM_CHAIN_KP, K), L.in_shared != 0, At, hdr);
    request(nxt, w1, b1);                 // the next tile's weights travel while this one is computed
    if (first_active) products();
    __syncthreads();                      // the panel has been read: the next panel, or the partial tiles, may overwrite it
    for (int k0 = PM_CHAIN_KP; k0 < K; k0 += PM_CHAIN_KP) {
      const int kp = min(PM_CHAIN_KP, K - k0);
      PmChainW4 wx;
      if (wave < (kp >> 6)) wx = pm_chain_ld_wf(wtile + k0 + wave * 64, K, lane);
      pm_chain_stage(L.in, K, i0, k0, kp, L.in_shared != 0, At, hdr);
      if (wave < (kp >> 6)) {
        park(wx);
        products();
      }
      __syncthreads();
    }
    // accumulator value v of lane l: row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32
#pragma unroll
    for (int v = 0; v < 16; ++v) red[wave][(8 * (v >> 2) + 4 * kg + (v & 3)) * 32 + lr] = acc[v];
    __syncthreads();
    // thread e sums output element e = (row e / 32, column e % 32)
    const int e = threadIdx.x;
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) s += red[w][e];
    const float zz = s + bf16_to_f32(b0);
    const float aa = pm_act_fwd(zz, L.act);
    __syncthreads();                                      // every partial has been read: reuse the buffer
    red[0][e] = zz;
    red[1][e] = aa;
    __syncthreads();
    if (e < 256) {                                        // four consecutive columns of a row: one 8-byte store
      const int r = e >> 3, c4 = (e & 7) << 2;
      const int64_t o = (int64_t)(i0 + r) * L.n_out + j0 + c4;
      const float* pz = &red[0][r * 32 + c4];
      const float* pa = &red[1][r * 32 + c4];
      pm_chain_st8_plain(L.z + o, pz[0], pz[1], pz[2], pz[3]);
      pm_chain_st8_shared(L.a + o, pa[0], pa[1], pa[2], pa[3]);
    }
    __syncthreads();                                      // the buffer is free for the next tile
    it = nxt;
  };
  PmChainW4 wA, wB;
  bf16_t bA = 0, bB = 0;
  request(it, wA, bA);
  while (it.u < n) {
    tile(wA, bA, wB, bB);
    if (it.u >= n) break;
    tile(wB, bB, wA, bA);
  }
}

// ---------------------------------------------------------------------------------------------
// data-gradient chain: units tab[0 .. n - 1] in execution order (top of the chain first)
// ---------------------------------------------------------------------------------------------
struct PmChainBwdR {
  const bf16_t* W;
  const bf16_t* dz;
  const bf16_t* zprev;
  bf16_t* dzprev;
  int32_t n_in, n_out, act_prev, dz_shared;
};

__global__ __launch_bounds__(PM_CHAIN_NT) void pm_chain_bwd_kernel(const PmChainBwd* __restrict__ tab, int n, int M,
                                                                  PmStepHdr* hdr) {
  constexpr int WS = 40;                                    // LDS row stride of a weight slice (32 columns + pad), elements
  __shared__ __attribute__((aligned(16))) unsigned char stage_mem[PM_CHAIN_STAGE_BYTES];   // input panel, then partial tiles
  __shared__ __attribute__((aligned(16))) bf16_t wt[16][64 * WS];   // per wave: 64 contraction rows x 32 output columns
  __shared__ PmChainBwdR tabs[PM_CHAIN_MAX_UNITS];
  bf16_t* At = reinterpret_cast<bf16_t*>(stage_mem);
  float (*red)[32 * 32] = reinterpret_cast<float (*)[32 * 32]>(stage_mem);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int lr = lane & 31, kg = lane >> 5;
  const int tiles_i = M >> 5;
  bf16_t* mine = wt[wave];
  if ((int)threadIdx.x < n) {
    const PmChainBwd L = tab[threadIdx.x];
    tabs[threadIdx.x] = PmChainBwdR{L.W.get(), L.dz, L.zprev, L.dzprev, L.n_in, L.n_out, L.act_prev, L.dz_shared};
  }
  __syncthreads();
  auto tiles_j_of = [](const PmChainBwdR& L) { return L.n_in >> 5; };
  // Requested one tile ahead, into one of two register sets that swap roles from tile to tile: this wave's first
  // weight slice (contraction rows wave * 64 + lane, 32 columns from j0: 64 contiguous bytes per row) and this
  // thread's entry of the stored pre-activation below (raw bits, converted where it is used).
  auto request = [&](PmChainItem it, PmChainW4& w, bf16_t& z) __attribute__((always_inline)) {
    if (it.u >= n) return;
    const PmChainBwdR& T = tabs[it.u];
    const int J = pm_chain_uni(T.n_in), K = pm_chain_uni(T.n_out);
    int rt, ct;
    pm_chain_rt_ct(it.t, tiles_i, J >> 5, &rt, &ct);
    const int i0 = rt << 5, j0 = ct << 5;
    if (wave < (K >> 6)) w = pm_chain_ld_wb(pm_chain_uni(T.W) + (int64_t)(wave * 64) * J + j0, J, lane);
    if (pm_chain_uni(T.act_prev))
      z = pm_chain_g(pm_chain_uni(T.zprev))[(int64_t)(i0 + ((int)threadIdx.x >> 5)) * J + j0 + ((int)threadIdx.x & 31)];
  };
  PmChainItem it = pm_chain_next(tabs, n, tiles_i, PmChainItem{-1, 0}, tiles_j_of);
  auto tile = [&](const PmChainW4& w0, const bf16_t& z0, PmChainW4& w1, bf16_t& z1) __attribute__((always_inline)) {
    const PmChainBwdR& T = tabs[it.u];
    const PmChainBwdR L{pm_chain_uni(T.W), pm_chain_uni(T.dz), pm_chain_uni(T.zprev), pm_chain_uni(T.dzprev),
                        pm_chain_uni(T.n_in), pm_chain_uni(T.n_out), pm_chain_uni(T.act_prev), pm_chain_uni(T.dz_shared)};
    const int K = L.n_out, J = L.n_in;
    int rt, ct;
    pm_chain_rt_ct(it.t, tiles_i, J >> 5, &rt, &ct);
    const int i0 = rt << 5, j0 = ct << 5;
    const bf16_t* wtile = L.W + j0;
    pm_f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const PmChainItem nxt = pm_chain_next(tabs, n, tiles_i, it, tiles_j_of);
    const bf16_t* ap = At + lr * PM_CHAIN_LDA + wave * 64 + 8 * kg;
    // park the slice [k][j] in this wave's LDS region (a wave's LDS accesses complete in program order: no barrier
    // inside the wave)
    auto park = [&](const PmChainW4& w) __attribute__((always_inline)) {
      uint4* dst = reinterpret_cast<uint4*>(mine + (lane >> 2) * WS + 8 * (lane & 3));
      dst[0] = w.a; dst[2 * WS] = w.b; dst[4 * WS] = w.c; dst[6 * WS] = w.d;      // (16 rows = 16 WS elements = 2 WS uint4)
    };
    // ... and read it back transposed: in each group of 16 lanes, lane g16 supplies the address of 4 consecutive
    // columns of one contraction row and receives, for the column given by its index in the group, 4 consecutive rows
    auto products = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int g = lane >> 4, g16 = lane & 15;
        const bf16_t* p = mine + (ks * 16 + 8 * (g >> 1) + (g16 >> 2)) * WS + 16 * (g & 1) + 4 * (g16 & 3);
        typedef pm_v4s __attribute__((address_space(3))) * lds_v4s;
        union { pm_bf16x8 v; pm_v4s h[2]; } b;
        b.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
        b.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 4 * WS));
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pm_chain_as_frag(*reinterpret_cast<const uint4*>(ap + ks * 16)), b.v, acc, 0, 0, 0);
      }
    };
    const bool first_active = wave < (min(PM_CHAIN_KP, K) >> 6);
    if (first_active) park(w0);
    pm_chain_stage(L.dz, K, i0, 0, min(PM_CHAIN_KP, K), L.dz_shared != 0, At, hdr);
    request(nxt, w1, z1);
    if (first_active) products();
    __syncthreads();
    for (int k0 = PM_CHAIN_KP; k0 < K; k0 += PM_CHAIN_KP) {
      const int kp = min(PM_CHAIN_KP, K - k0);
      PmChainW4 wx;
      if (wave < (kp >> 6)) wx = pm_chain_ld_wb(wtile + (int64_t)(k0 + wave * 64) * J, J, lane);
      pm_chain_stage(L.dz, K, i0, k0, kp, L.dz_shared != 0, At, hdr);
      if (wave < (kp >> 6)) {
        park(wx);
        products();
      }
      __syncthreads();
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) red[wave][(8 * (v >> 2) + 4 * kg + (v & 3)) * 32 + lr] = acc[v];
    __syncthreads();
    const int e = threadIdx.x;
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) s += red[w][e];
    if (L.act_prev) s *= pm_act_bwd(bf16_to_f32(z0), L.act_prev);
    __syncthreads();
    red[0][e] = s;
    __syncthreads();
    if (e < 256) {
      const int r = e >> 3, c4 = (e & 7) << 2;
      const float* pd = &red[0][r * 32 + c4];
      pm_chain_st8_shared(L.dzprev + (int64_t)(i0 + r) * J + j0 + c4, pd[0], pd[1], pd[2], pd[3]);
    }
    __syncthreads();
    it = nxt;
  };
  PmChainW4 wA, wB;
  bf16_t zA = 0, zB = 0;
  request(it, wA, zA);
  while (it.u < n) {
    tile(wA, zA, wB, zB);
    if (it.u >= n) break;
    tile(wB, zB, wA, zA);
  }
}
