// Host runtime and C ABI of the PipeMare step library (see include/pipemare.h).
// gfx950 only.  The library owns no device memory: everything lives in the caller's arena.
#include "../../include/pipemare.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <climits>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "pm_common.hpp"
#include "pm_elem.hpp"
#include "pm_gemm_mfma.hpp"
#include "pm_update.hpp"
#include "pm_chain.hpp"
#include "pm_transformer.hpp"
#include "pm_conv.hpp"

namespace {

thread_local std::string g_err;

pm_status fail(pm_status s, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return s;
}

#define PM_HIP(call)                                                                           \
  do {                                                                                         \
    hipError_t e_ = (call);                                                                    \
    if (e_ != hipSuccess) return fail(PM_EHIP, "%s: %s", #call, hipGetErrorString(e_));        \
  } while (0)

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// Integer inverse-CDF table of one stage's delay (App. "Hogwild! asynchrony": exponential, truncated):
// X ~ Exp(mean) truncated to [0, tau_max + 1), delay = floor(X);
// T[k] = min(floor(2^32 P(delay <= k)), 2^32 - 1), P(delay <= k) = (1 - e^{-(k+1)/mean}) / (1 - e^{-(tau_max+1)/mean}).
// mean <= 0: the delay is always 0.
inline void delay_thresholds(double mean, int tau_max, uint32_t* T) {
  if (mean <= 0.0) {
    for (int k = 0; k < tau_max; ++k) T[k] = 0xFFFFFFFFu;
    return;
  }
  const double norm = 1.0 - std::exp(-(double)(tau_max + 1) / mean);
  for (int k = 0; k < tau_max; ++k) {
    const double v = std::floor((1.0 - std::exp(-(double)(k + 1) / mean)) / norm * 4294967296.0);
    T[k] = v >= 4294967295.0 ? 0xFFFFFFFFu : (uint32_t)v;
  }
}

struct Unit {
  pm_layer_desc d;
  int64_t nw;        // values of the first part: W (n_out * n_in), embedding table, or LayerNorm gain
  int64_t nb;        // values of the second part (bias); 0 for an embedding
  int64_t boff;      // offset of the second part inside the unit (nw rounded up to 8 elements)
  int64_t n;         // boff + nb
  int64_t n_pad;     // n rounded up to PM_CHUNK
  int64_t off;       // element offset in the flat arrays
  int64_t ring_off;  // element offset in the ring
  int32_t tau_f, tau_b, R;
  double gamma;
  int32_t corr;      // tau_f - tau_b when T2 applies, else 0
  // recomputation (chain only): delay of the weights that rebuild this unit's activations in the
  // backward pass, the coefficient of their correction when the unit keeps a corrected copy of its own
  // (0: the copy would equal the corrected backward weights, or no correction applies), and the
  // unit's place in its segment
  int32_t tau_r = 0, corr_r = 0;
  bool seg_first = false, seg_last = false;
  int ld_in, ld_out; // leading dimensions of the activation matrices (multiples of 8)
  // activation buffers (byte offsets into the arena)
  size_t z_off, a_off, dz_off, z32_off;
};

struct Layout {
  std::vector<Unit> units;
  int64_t n_flat = 0;     // padded element count of the flat arrays
  int64_t n_real = 0;     // true parameter count
  int64_t ring_elems = 0;
  int64_t n_chunks = 0;
  size_t esz = 4;         // bytes per element of the compute dtype
  // byte offsets
  size_t w_off, g_off, v_off, s_off, d_off, ub_off, ur_off, cdf_off, ring_off, chunk_off, ls_off, ld_off, hdr_off, probs_off, x_off;
  size_t chain_f_off, chain_b_off;                         // unit tables of the chained launches
  size_t act_begin, act_end, total;
  // Transformer activations (byte offsets; see launch_tfm).  Per layer: index [layer]
  struct TfmLayer {
    size_t x, mu1, rs1, n1, q, k, v, lse, o, h, mu2, rs2, n2, z1, f;
    size_t dzq, dzk, dzv, dzo, dz1, dz2;   // d loss / d (output of Wq, Wk, Wv, Wo, W1, W2), kept until the weight gradients
  };
  std::vector<TfmLayer> tl;
  // CNN activations per convolution unit (byte offsets), all [B, Ho, Wo, Cout] in the compute dtype
  struct ConvBuf {
    PmConvGeom g;
    size_t z, y, da, dz, dy;
  };
  std::vector<ConvBuf> cv;
  size_t r_x, r_pool, r_logits, r_dlogits, r_dpool, r_wscratch, r_ascratch;
  size_t t_xf, t_muf, t_rsf, t_nf, t_logits, t_dlogits;      // final LayerNorm and head
  size_t t_dx, t_dn, t_do;                                   // backward scratch, reused by every layer
  size_t t_pos, t_zero;                                      // positions fp32 [S, d]; zero-region table
  size_t t_fuse, t_ublocks;                                  // update in the weight-gradient epilogue: problem table of that launch, blocks left to the update pass
  size_t t_wprobs, t_wtiles, t_wsegs;                        // grouped weight-gradient launch: problems (2 sets), tiles per XCD, segments
  int n_zero = 0;
  int64_t zero_max = 0;
  bool recompute = false;   // the backward pass rebuilds the activations inside each segment
  bool has_ur = false;      // some unit keeps corrected recompute weights of its own
};

pm_status validate(int32_t P, int32_t L, const pm_layer_desc* layers, const int32_t* tau_fwd,
                   const int32_t* tau_bkwd, const pm_opts* o) {
  if (P < 1 || L < 1 || !layers || !tau_fwd || !o) return fail(PM_EINVAL, "P, L >= 1 and non-NULL arrays required");
  if (o->dtype != PM_F32 && o->dtype != PM_BF16) return fail(PM_EINVAL, "dtype must be PM_F32 or PM_BF16");
  if (o->opt != PM_OPT_SGDM && o->opt != PM_OPT_ADAMW) return fail(PM_EINVAL, "unknown optimizer");
  if (o->loss != PM_LOSS_MSE && o->loss != PM_LOSS_XENT) return fail(PM_EINVAL, "unknown loss");
  if (o->microbatch < 1 || o->n_microbatches < 1) return fail(PM_EINVAL, "microbatch and n_microbatches must be >= 1");
  if (!(o->D > 0.0 && o->D <= 1.0)) return fail(PM_EINVAL, "D must be in (0, 1]");
  if (o->sync_warmup_steps < 0) return fail(PM_EINVAL, "sync_warmup_steps must be >= 0");
  if (o->clip_norm < 0.0 || o->weight_decay < 0.0) return fail(PM_EINVAL, "clip_norm and weight_decay must be >= 0");
  if (o->arch < PM_ARCH_CHAIN || o->arch > PM_ARCH_RESNET) return fail(PM_EINVAL, "unknown architecture");
  int prev_stage = 1;
  for (int l = 0; l < L; ++l) {
    const pm_layer_desc& d = layers[l];
    if (d.kind < PM_LINEAR || d.kind > PM_CONV3X3) return fail(PM_EINVAL, "unit %d: unknown kind", l);
    if (o->arch == PM_ARCH_CHAIN && d.kind != PM_LINEAR) return fail(PM_EINVAL, "unit %d: a chain holds Linear units only", l);
    if (o->arch == PM_ARCH_TRANSFORMER && d.kind == PM_CONV3X3) return fail(PM_EINVAL, "unit %d: convolutions need PM_ARCH_RESNET", l);
    if (d.n_in < 1 || d.n_out < 1) return fail(PM_EINVAL, "unit %d: sizes must be positive", l);
    if (d.act < PM_ACT_NONE || d.act > PM_ACT_GELU) return fail(PM_EINVAL, "unit %d: unknown activation", l);
    if (d.stage < 1 || d.stage > P) return fail(PM_EINVAL, "unit %d: stage %d outside 1..%d", l, d.stage, P);
    if (d.stage < prev_stage) return fail(PM_EINVAL, "unit %d: stages must be non-decreasing along the chain", l);
    prev_stage = d.stage;
    if (o->arch == PM_ARCH_CHAIN && l > 0 && layers[l - 1].n_out != d.n_in) return fail(PM_EINVAL, "unit %d: n_in %d does not chain with previous n_out %d", l, d.n_in, layers[l - 1].n_out);
  }
  if (o->arch == PM_ARCH_RESNET) {
    if (o->loss != PM_LOSS_XENT) return fail(PM_EINVAL, "the CNN is trained with cross-entropy (PM_LOSS_XENT)");
    if (L < 4 || (L % 2)) return fail(PM_EINVAL, "a CNN has 2 * blocks + 2 units, got %d", L);
    if (o->image_size < 4 || (o->image_size % 4)) return fail(PM_EINVAL, "image_size must be a positive multiple of 4");
    for (int l = 0; l < L - 1; ++l) {
      if (layers[l].kind != PM_CONV3X3) return fail(PM_EINVAL, "unit %d must be a 3x3 convolution", l);
      if (layers[l].n_out & 7) return fail(PM_EINVAL, "unit %d: channel count %d must be a multiple of 8", l, layers[l].n_out);
      if (layers[l].n_out > 256 || (layers[l].n_out & (layers[l].n_out - 1))) return fail(PM_EINVAL, "unit %d: channel count %d must be a power of two up to 256", l, layers[l].n_out);
      if (layers[l].act != PM_ACT_RELU) return fail(PM_EINVAL, "unit %d: convolutions are followed by ReLU", l);
      if (l > 0 && layers[l].n_in != layers[l - 1].n_out) return fail(PM_EINVAL, "unit %d: n_in %d does not chain with previous n_out %d", l, layers[l].n_in, layers[l - 1].n_out);
      if (l > 0 && (l % 2) == 0 && layers[l].n_in != layers[l].n_out) return fail(PM_EINVAL, "unit %d: the second convolution of a block keeps the channel count", l);
      if (l > 0 && (l % 2) == 1 && layers[l].n_out != layers[l].n_in && layers[l].n_out != 2 * layers[l].n_in)
        return fail(PM_EINVAL, "unit %d: the first convolution of a block keeps or doubles the channel count", l);
    }
    int strides = 0;
    for (int l = 1; l < L - 1; l += 2) strides += layers[l].n_out == 2 * layers[l].n_in;
    if ((o->image_size >> strides) < 1 || (o->image_size % (1 << strides))) return fail(PM_EINVAL, "image_size %d does not survive %d halvings", o->image_size, strides);
    if (layers[L - 1].kind != PM_LINEAR || layers[L - 1].n_in != layers[L - 2].n_out) return fail(PM_EINVAL, "the last unit must be the classifier on the pooled channels");
  }
  if (o->arch == PM_ARCH_TRANSFORMER) {
    if (o->loss != PM_LOSS_XENT) return fail(PM_EINVAL, "the Transformer is trained with token cross-entropy (PM_LOSS_XENT)");
    if (L < 11 || (L - 3) % 8) return fail(PM_EINVAL, "a Transformer has 8 * n_layers + 3 units, got %d", L);
    if (o->n_heads < 1 || o->seq_len < 1) return fail(PM_EINVAL, "n_heads and seq_len must be >= 1");
    const int V = layers[0].n_in, d = layers[0].n_out, nl = (L - 3) / 8;
    auto is = [&](int l, int kind, int n_in, int n_out) {
      return layers[l].kind == kind && layers[l].n_in == n_in && layers[l].n_out == n_out;
    };
    if (layers[0].kind != PM_EMBED) return fail(PM_EINVAL, "unit 0 must be the embedding");
    if (d % o->n_heads || (d & 7)) return fail(PM_EINVAL, "width %d must be a multiple of 8 and of n_heads %d", d, o->n_heads);
    const int dff = layers[7].n_out;
    if (dff & 7) return fail(PM_EINVAL, "feed-forward width %d must be a multiple of 8", dff);
    for (int b = 0; b < nl; ++b) {
      const int u = 1 + 8 * b;
      const bool ok = is(u, PM_LAYERNORM, d, d) && is(u + 1, PM_LINEAR, d, d) && is(u + 2, PM_LINEAR, d, d) &&
                      is(u + 3, PM_LINEAR, d, d) && is(u + 4, PM_LINEAR, d, d) && is(u + 5, PM_LAYERNORM, d, d) &&
                      is(u + 6, PM_LINEAR, d, dff) && is(u + 7, PM_LINEAR, dff, d);
      if (!ok) return fail(PM_EINVAL, "layer %d: units must be ln1, Wq, Wk, Wv, Wo, ln2, W1 (d -> d_ff), W2 (d_ff -> d)", b);
      for (int j = 0; j < 8; ++j)
        if (j != 6 && layers[u + j].act != PM_ACT_NONE) return fail(PM_EINVAL, "unit %d: only the first feed-forward matrix has an activation", u + j);
    }
    if (!is(L - 2, PM_LAYERNORM, d, d) || !is(L - 1, PM_LINEAR, d, V)) return fail(PM_EINVAL, "the last two units must be the final LayerNorm and the output head (d -> vocabulary)");
    if (d > 1024) return fail(PM_EINVAL, "LayerNorm kernels support widths up to 1024");
    const int dh = d / o->n_heads;
    const bool mfma_attn = o->dtype == PM_BF16 && pm_attn_mfma_fits(o->seq_len, dh);
    if (!mfma_attn && !pm_attn_plain_fits(o->seq_len, dh))
      return fail(PM_EINVAL, "attention: outside bf16 / head size 64 / seq_len multiple of 32, the head size must be 4, 8, 16, 32 or 64 and seq_len * (head size + 1) <= 8192");
  }
  for (int i = 0; i < P; ++i) {
    if (tau_fwd[i] < 0) return fail(PM_EINVAL, "tau_fwd[%d] < 0", i);
    if (tau_bkwd && (tau_bkwd[i] < 0 || tau_bkwd[i] > tau_fwd[i])) return fail(PM_EINVAL, "need 0 <= tau_bkwd[%d] <= tau_fwd[%d]", i, i);
  }
  if (o->update_placement < 0 || o->update_placement > 2) return fail(PM_EINVAL, "update_placement must be 0 (automatic), 1 (separate pass) or 2 (weight-gradient launch)");
  if (o->stochastic_delays) {
    if (o->tau_max < 0 || o->tau_max > 65535) return fail(PM_EINVAL, "tau_max must be in 0..65535");
    if (o->tau_recomp) return fail(PM_EINVAL, "stochastic delays and recomputation are not combined");
  }
  if (o->tau_recomp) {
    if (o->segment_size < 1) return fail(PM_EINVAL, "recomputation needs segment_size >= 1 (stages per segment)");
    for (int i = 0; i < P; ++i) {
      const int tb = tau_bkwd ? tau_bkwd[i] : 0;
      if (o->tau_recomp[i] < tb || o->tau_recomp[i] > tau_fwd[i])
        return fail(PM_EINVAL, "need tau_bkwd[%d] <= tau_recomp[%d] <= tau_fwd[%d]", i, i, i);
    }
  }
  return PM_OK;
}

void make_layout(int32_t L, const pm_layer_desc* layers, const int32_t* tau_fwd, const int32_t* tau_bkwd,
                 const pm_opts* o, Layout& lay) {
  lay.units.resize(L);
  lay.esz = o->dtype == PM_BF16 ? 2 : 4;
  int64_t off = 0, roff = 0, real = 0;
  for (int l = 0; l < L; ++l) {
    Unit& u = lay.units[l];
    u.d = layers[l];
    if (u.d.kind == PM_LAYERNORM) { u.nw = u.d.n_out; u.nb = u.d.n_out; }
    else if (u.d.kind == PM_EMBED) { u.nw = (int64_t)u.d.n_in * u.d.n_out; u.nb = 0; }
    else if (u.d.kind == PM_CONV3X3) { u.nw = (int64_t)u.d.n_out * 9 * u.d.n_in; u.nb = 2 * (int64_t)u.d.n_out; }
    else { u.nw = (int64_t)u.d.n_out * u.d.n_in; u.nb = u.d.n_out; }
    u.boff = round_up(u.nw, 8);
    u.n = u.boff + u.nb;
    u.n_pad = round_up(u.n, PM_CHUNK);
    u.off = off;
    u.ring_off = roff;
    u.tau_f = tau_fwd[u.d.stage - 1];
    u.tau_b = tau_bkwd ? tau_bkwd[u.d.stage - 1] : 0;
    u.R = (o->stochastic_delays ? o->tau_max : u.tau_f) + 1;
    // stochastic delays: both passes read the drawn version, so there is nothing to correct
    const int dd = o->stochastic_delays ? 0 : u.tau_f - u.tau_b;
    // nothing flows through an embedding to earlier units: its backward weights are never read
    u.corr = (o->t2_enabled && dd > 0 && u.d.kind != PM_EMBED) ? dd : 0;
    if (o->gamma_override) u.gamma = o->gamma_override[u.d.stage - 1];
    else u.gamma = dd > 0 ? std::pow(o->D, 1.0 / dd) : 0.0;
    u.tau_r = u.tau_b;
    u.corr_r = 0;
    if (o->tau_recomp) {
      lay.recompute = true;
      u.tau_r = o->tau_recomp[u.d.stage - 1];
      const int dr = u.tau_f - u.tau_r;
      const int cr = (o->t2_enabled && dr > 0) ? dr : 0;
      // same delay and same coefficient as the backward weights: those are read instead
      if (cr > 0 && !(u.tau_r == u.tau_b && cr == u.corr)) { u.corr_r = cr; lay.has_ur = true; }
      const int seg = (u.d.stage - 1) / o->segment_size;
      u.seg_first = l == 0 || (layers[l - 1].stage - 1) / o->segment_size != seg;
      u.seg_last = l == L - 1 || (layers[l + 1].stage - 1) / o->segment_size != seg;
    }
    u.ld_in = (int)round_up(u.d.n_in, 8);
    u.ld_out = (int)round_up(u.d.n_out, 8);
    off += u.n_pad;
    roff += u.n_pad * u.R;
    real += u.nw + u.nb;
  }
  lay.n_flat = off;
  lay.n_real = real;
  lay.ring_elems = roff;
  lay.n_chunks = off / PM_CHUNK;
  size_t p = 0;
  auto take = [&](size_t bytes) { size_t at = p; p = (size_t)round_up((int64_t)(p + bytes), PM_ALIGN); return at; };
  lay.w_off = take(lay.n_flat * 4);
  lay.g_off = take(lay.n_flat * 4);
  lay.v_off = take(lay.n_flat * 4);
  lay.s_off = take(o->opt == PM_OPT_ADAMW ? lay.n_flat * 4 : 0);
  lay.d_off = take(lay.n_flat * 4);
  lay.ub_off = take(lay.n_flat * lay.esz);
  lay.ur_off = take(lay.has_ur ? lay.n_flat * lay.esz : 0);
  {
    int P = 0;
    for (int l = 0; l < L; ++l) P = std::max(P, (int)layers[l].stage);
    lay.cdf_off = take(o->stochastic_delays ? sizeof(uint32_t) * (size_t)P * (size_t)o->tau_max : 0);
  }
  lay.ring_off = take(lay.ring_elems * lay.esz);
  lay.chunk_off = take(lay.n_chunks * 4);
  lay.ls_off = take(sizeof(PmLayerStatic) * L);
  lay.ld_off = take(sizeof(PmLayerStep) * L * 2);
  lay.hdr_off = take(sizeof(PmStepHdr));
  lay.probs_off = take(sizeof(PmGemmProb<PmEpiBwdWeight>) * 2 * L);
  lay.chain_f_off = take(sizeof(PmChainFwd) * L);
  lay.chain_b_off = take(sizeof(PmChainBwd) * L);
  const int M = o->microbatch;
  lay.act_begin = p;
  if (o->arch == PM_ARCH_TRANSFORMER) {
    const size_t Tk = (size_t)M * o->seq_len, d = lay.units[0].d.n_out, dff = lay.units[7].d.n_out;
    const size_t ldV = (size_t)round_up(lay.units[0].d.n_in, 8), e = lay.esz;
    const int nl = (L - 3) / 8;
    lay.x_off = 0;
    lay.tl.resize(nl);
    for (auto& b : lay.tl) {
      b.x = take(Tk * d * 4); b.mu1 = take(Tk * 4); b.rs1 = take(Tk * 4); b.n1 = take(Tk * d * e);
      b.q = take(Tk * d * e); b.k = take(Tk * d * e); b.v = take(Tk * d * e);
      b.lse = take(Tk * o->n_heads * 4); b.o = take(Tk * d * e);
      b.h = take(Tk * d * 4); b.mu2 = take(Tk * 4); b.rs2 = take(Tk * 4); b.n2 = take(Tk * d * e);
      b.z1 = take(Tk * dff * e); b.f = take(Tk * dff * e);
      b.dzq = take(Tk * d * e); b.dzk = take(Tk * d * e); b.dzv = take(Tk * d * e); b.dzo = take(Tk * d * e);
      b.dz1 = take(Tk * dff * e); b.dz2 = take(Tk * d * e);
    }
    lay.t_xf = take(Tk * d * 4); lay.t_muf = take(Tk * 4); lay.t_rsf = take(Tk * 4); lay.t_nf = take(Tk * d * e);
    lay.t_logits = take(Tk * ldV * 4); lay.t_dlogits = take(Tk * ldV * e);
    lay.t_dx = take(Tk * d * 4); lay.t_dn = take(Tk * d * 4); lay.t_do = take(Tk * d * e);
    lay.t_pos = take((size_t)o->seq_len * d * 4);
    lay.t_fuse = take(sizeof(PmGemmProb<PmEpiBwdWeightUpd>) * L);
    lay.t_ublocks = take(sizeof(int32_t) * (size_t)lay.n_chunks * (PM_CHUNK / 1024));
    lay.t_wprobs = take(sizeof(PmGemmProb<PmEpiBwdWeight>) * 2 * L);
    lay.t_wtiles = take(sizeof(int32_t) * 8);
    lay.t_wsegs = take(sizeof(PmXcdSeg) * 8 * (size_t)(L + 8));
    // gradient regions that are accumulated with atomics and therefore cleared at the start of a
    // minibatch: the embedding table and every LayerNorm
    lay.n_zero = 0;
    lay.zero_max = 0;
    for (int l = 0; l < L; ++l)
      if (lay.units[l].d.kind != PM_LINEAR) { lay.n_zero += 1; lay.zero_max = std::max(lay.zero_max, lay.units[l].n_pad); }
    lay.t_zero = take(sizeof(int64_t) * 2 * lay.n_zero);
  } else if (o->arch == PM_ARCH_RESNET) {
    const size_t e = lay.esz;
    const int nconv = L - 1;
    lay.x_off = 0;
    lay.cv.resize(nconv);
    int H = o->image_size;
    lay.r_x = take((size_t)M * H * H * lay.units[0].d.n_in * e);
    for (int u = 0; u < nconv; ++u) {
      Layout::ConvBuf& b = lay.cv[u];
      const pm_layer_desc& dd = lay.units[u].d;
      const int stride = (u > 0 && (u % 2) == 1 && dd.n_out == 2 * dd.n_in) ? 2 : 1;
      b.g = PmConvGeom{M, H, H, dd.n_in, dd.n_out, stride, (H - 1) / stride + 1, (H - 1) / stride + 1};
      H = b.g.Ho;
      const size_t n = (size_t)M * H * H * dd.n_out * e;
      b.z = take(n); b.y = take(n); b.da = take(n); b.dz = take(n); b.dy = take(n);
    }
    const int C = lay.units[L - 2].d.n_out, ncls = lay.units[L - 1].d.n_out;
    lay.r_pool = take((size_t)M * C * e);
    lay.r_logits = take((size_t)M * round_up(ncls, 8) * 4);
    lay.r_dlogits = take((size_t)M * round_up(ncls, 8) * e);
    lay.r_dpool = take((size_t)M * C * e);
    size_t ws = 0;
    for (int u = 0; u < nconv; ++u)
      ws = std::max(ws, o->dtype == PM_BF16 ? pm_conv_wgrad_scratch_elems<bf16_t>(lay.cv[u].g)
                                            : pm_conv_wgrad_scratch_elems<float>(lay.cv[u].g));
    lay.r_wscratch = take(ws * 4);
    lay.r_ascratch = take((size_t)PM_CONV_AFFINE_MAX_BLOCKS * 2 * 256 * 4);     // per-block channel sums of the affine backward
    lay.n_zero = nconv;
    lay.zero_max = 0;
    for (int u = 0; u < nconv; ++u) lay.zero_max = std::max(lay.zero_max, lay.units[u].n_pad);
    lay.t_zero = take(sizeof(int64_t) * 2 * lay.n_zero);
  } else {
    lay.x_off = take((size_t)M * lay.units[0].ld_in * lay.esz);
    for (int l = 0; l < L; ++l) {
      Unit& u = lay.units[l];
      const size_t e = (size_t)M * u.ld_out;
      u.z_off = take(e * lay.esz);
      u.a_off = take(e * lay.esz);
      u.dz_off = take(e * lay.esz);
      u.z32_off = (l == L - 1) ? take(e * 4) : 0;
    }
  }
  lay.act_end = p;
  lay.total = p;
}

}  // namespace

constexpr size_t PM_MAX_GRAPHS = 64;   // captured step graphs kept per context

struct pm_ctx {
  int32_t P, L;
  pm_opts o;
  pm_lr_sched sched;
  std::vector<double> gamma_override;
  std::vector<int32_t> tau_f, tau_b, tau_r;
  Layout lay;
  char* arena;
  hipStream_t stream;
  int64_t t_host = 0;      // completed optimizer steps
  int32_t micro = 0;       // microbatches accumulated in the current minibatch
  bool diverged = false;
  float last_loss = 0.f;
  // captured steps: one graph per (x, y) batch-buffer pair seen, oldest dropped beyond PM_MAX_GRAPHS
  struct StepGraph {
    const void* x;
    const void* y;
    hipGraph_t graph;
    hipGraphExec_t exec;
  };
  std::vector<StepGraph> graphs;
  // all weight-gradient products as one grouped MFMA launch (problem tables live in the arena)
  bool dw_grouped = false;
  bool fuse_upd = false;         // the grouped weight-gradient launch applies the update of its units' weight matrices
  int upd_nblocks = 0;           // blocks left to the update pass then
  int64_t upd_fused_params = 0;  // parameters updated in the epilogues
  int dw_maxI = 0, dw_maxJ = 0;
  int dw_nprob = 0, dw_ntiles = 0;   // Transformer: problems and grid size (8 x the longest XCD list) of the grouped launch
  int dw_max_segs = 0;
  bool dw_aligned = false;           // no tile of the grouped launch needs a bounds test
  int dw_tile = 128;                 // block tile of the grouped launch (128 or 256)
  // MLP chain with few rows: units 0 .. chain_nf - 1 run forward as one chained launch, the data gradients of
  // units chain_hb .. 1 as another (0: the launch-per-product path)
  int chain_nf = 0, chain_hb = 0, chain_grid = 0;
  int64_t chain_fill16 = 0;   // 16-byte words from the first unit's z to the last unit's dz (filled before every chained pass)
  // overlap of the update of step t with the forward of step t+1 (second stream owned by the library)
  bool overlap = false;
  int32_t min_tau_f = 0;
  hipStream_t stream_b = nullptr;
  hipEvent_t ev_bwd = nullptr, ev_upd = nullptr;
  bool upd_pending = false;    // an update is (possibly) still running on stream_b
  int last_par = 0;            // step-table set used by the most recent step
  // optional per-phase timing (host-side event objects only)
  std::vector<hipEvent_t> prof_ev;   // 4 per step: start, after forward+loss, after backward, after update
  int32_t prof_cap = 0, prof_n = 0;
  bool prof_on = false;
  // per-class kernel time of the first steps of a profiling pass: an event pair around every launch of a
  // matrix / convolution product (class 0) and of an attention-core kernel (class 1)
  std::vector<hipEvent_t> cls_ev;    // begin, end, begin, end, ...
  std::vector<int8_t> cls_tag;       // class of each pair
  int32_t cls_cap = 0;               // steps that record class spans
  double cls_ms[2] = {0.0, 0.0};     // result of the last pass: mean milliseconds per step
  int32_t cls_steps = 0;

  template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(arena + off); }
  PmStepHdr* hdr() const { return at<PmStepHdr>(lay.hdr_off); }
  PmLayerStatic* ls() const { return at<PmLayerStatic>(lay.ls_off); }
  PmLayerStep* ld(int par) const { return at<PmLayerStep>(lay.ld_off) + (size_t)par * L; }
  int par() const { return overlap ? (int)(t_host & 1) : 0; }   // which step-table set the current step uses
};

namespace {

PmSchedDev sched_dev(const pm_ctx* c) {
  PmSchedDev s;
  s.kind = c->sched.kind;
  s.base = c->sched.base;
  s.init = c->sched.init;
  s.factor = c->sched.factor;
  s.interval = c->sched.interval;
  s.K = c->sched.K;
  s.t1_enabled = c->o.t1_enabled;
  s.beta1 = c->o.beta1;
  s.beta2 = c->o.beta2;
  s.gscale0 = 1.0 / c->o.n_microbatches;
  s.sync_warmup = c->o.sync_warmup_steps;
  s.stoch = c->o.stochastic_delays ? 1 : 0;
  s.tau_max = c->o.tau_max;
  s.P = c->P;
  s.seed = c->o.delay_seed;
  s.cdf = c->o.stochastic_delays ? c->at<uint32_t>(c->lay.cdf_off) : nullptr;
  return s;
}

inline void prof_mark(pm_ctx* c, int which) {
  if (c->prof_on && c->prof_n < c->prof_cap) (void)hipEventRecord(c->prof_ev[(size_t)c->prof_n * 4 + which], c->stream);
}

// Event pair around the launches of one kernel class while a profiling pass records classes.
struct ProfSpan {
  pm_ctx* c;
  bool on;
  ProfSpan(pm_ctx* ctx, int cls) : c(ctx), on(ctx->prof_on && ctx->prof_n < ctx->cls_cap) {
    if (!on) return;
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) { on = false; return; }
    (void)hipEventRecord(e, c->stream);
    c->cls_ev.push_back(e);
    c->cls_tag.push_back((int8_t)cls);
  }
  ~ProfSpan() {
    if (!on) return;
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) {          // drop the unmatched begin marker
      (void)hipEventDestroy(c->cls_ev.back());
      c->cls_ev.pop_back();
      c->cls_tag.pop_back();
      return;
    }
    (void)hipEventRecord(e, c->stream);
    c->cls_ev.push_back(e);
  }
  ProfSpan(const ProfSpan&) = delete;
  ProfSpan& operator=(const ProfSpan&) = delete;
};
constexpr int PM_CLS_GEMM = 0, PM_CLS_ATTN = 1;

// ---- kernel launches of one microbatch / one update, templated on the compute dtype -------------
template <typename T>
pm_status launch_update(pm_ctx* c, hipStream_t st, int par, bool all_params = false) {
  const Layout& lay = c->lay;
  if (c->o.clip_norm > 0.0) {
    int blocks = (int)std::min<int64_t>(2048, (lay.n_flat / 4 + 255) / 256);
    hipLaunchKernelGGL(pm_sumsq_kernel, dim3(blocks), dim3(256), 0, st, c->at<float>(lay.g_off), lay.n_flat,
                       &c->hdr()->gnorm2[par]);
    hipLaunchKernelGGL(pm_clip_scale_kernel, dim3(1), dim3(1), 0, st, c->hdr(), (float)c->o.clip_norm, par);
  }
  prof_mark(c, 2);
  PmUpdArgs<T> a;
  a.g = c->at<float>(lay.g_off);
  a.w = c->at<float>(lay.w_off);
  a.v = c->at<float>(lay.v_off);
  a.s = c->at<float>(lay.s_off);
  a.d = c->at<float>(lay.d_off);
  a.ring = c->at<T>(lay.ring_off);
  a.ub = c->at<T>(lay.ub_off);
  a.ur = lay.has_ur ? c->at<T>(lay.ur_off) : nullptr;
  a.chunk_layer = c->at<int32_t>(lay.chunk_off);
  a.ls = c->ls();
  a.ld = c->ld(par);
  a.hdr = c->hdr();
  a.par = par;
  a.beta1 = (float)c->o.beta1;
  a.beta2 = (float)c->o.beta2;
  a.eps = (float)c->o.eps;
  a.wd = (float)c->o.weight_decay;
  // Streams of up to a few times the 256 MB last-level cache are partly still resident from the
  // previous step (w, v, delta written at step t are read at t+1): cached accesses win there
  // (measured 6.4 vs 5.6 TB/s at 0.5 GB).  Beyond that nothing survives a step and non-temporal
  // accesses with one group of four elements per thread are ahead (see PmAcc).
  const bool nontemporal = (size_t)lay.n_flat * 32 > ((size_t)1 << 30);
  // the parameters that the weight-gradient epilogues of this step have already updated are left out
  // (not when the gradients came from the caller: pm_apply_update)
  const bool rest_only = c->fuse_upd && !all_params;
  a.blocks = rest_only ? c->at<int32_t>(lay.t_ublocks) : nullptr;
  const dim3 grid(rest_only ? (unsigned)c->upd_nblocks
                            : (unsigned)(lay.n_chunks * (PM_CHUNK / (nontemporal ? PmAcc<2>::PER_BLOCK : PmAcc<1>::PER_BLOCK)))), blk(256);
  if (grid.x == 0) { prof_mark(c, 3); return PM_OK; }
#define PM_UPD(OPT, VAR) hipLaunchKernelGGL((pm_fused_update_kernel<T, OPT, VAR>), grid, blk, 0, st, a)
  if (c->o.opt == PM_OPT_SGDM) {
    if (nontemporal) PM_UPD(0, 2); else PM_UPD(0, 1);
  } else {
    if (nontemporal) PM_UPD(1, 2); else PM_UPD(1, 1);
  }
#undef PM_UPD
  prof_mark(c, 3);
  PM_HIP(hipGetLastError());
  return PM_OK;
}

void launch_prologue(pm_ctx* c, int par) {
  hipLaunchKernelGGL(pm_prologue_kernel, dim3(1), dim3(256), 0, c->stream, c->hdr(), c->ls(), c->ld(par), c->L,
                     sched_dev(c), par);
}

// Make the caller's stream wait for an update that may still run on the library's second stream.
pm_status quiesce(pm_ctx* c) {
  if (c->upd_pending) {
    PM_HIP(hipStreamWaitEvent(c->stream, c->ev_upd, 0));
    c->upd_pending = false;
  }
  return PM_OK;
}

template <typename T, class Epi>
void launch_gemm_on(hipStream_t st, int I, int J, int K, const T* A, int64_t sai, int64_t sak, PmWLoc<T> B, int64_t sbj,
                    int64_t sbk, const Epi& epi, const PmPrefetch* pf = nullptr) {
  if constexpr (sizeof(T) == 2) {
    if (pm_mfma_gemm_try(st, I, J, K, A, sai, sak, B, sbj, sbk, epi, pf)) return;
  }
  dim3 grid((J + 15) / 16, (I + 15) / 16);
  hipLaunchKernelGGL((pm_gemm_plain_kernel<T, T, Epi>), grid, dim3(256), 0, st, I, J, K, A, sai, sak, B, sbj, sbk, epi);
}

// Bias gradient db = column sums of dz as its own launch (when the GEMM does not fuse it).
template <typename T>
void launch_bias_grad(hipStream_t st, const T* dz, float* db, int M, int N, int ld, int accumulate) {
  if (M > 512) {
    if (!accumulate) hipLaunchKernelGGL(pm_zero_f32_kernel, dim3((N + 255) / 256), dim3(256), 0, st, db, (int64_t)N);
    hipLaunchKernelGGL((pm_bias_grad_chunked_kernel<T>), dim3((N + 63) / 64, (M + 255) / 256), dim3(256), 0, st, dz, db,
                       M, N, ld);
  } else {
    hipLaunchKernelGGL((pm_bias_grad_kernel<T>), dim3((N + 63) / 64), dim3(256), 0, st, dz, db, M, N, ld, accumulate);
  }
}

template <typename T, class Epi>
void launch_gemm(pm_ctx* c, int I, int J, int K, const T* A, int64_t sai, int64_t sak, PmWLoc<T> B, int64_t sbj,
                 int64_t sbk, const Epi& epi, const PmPrefetch* pf = nullptr) {
  ProfSpan span(c, PM_CLS_GEMM);
  launch_gemm_on<T>(c->stream, I, J, K, A, sai, sak, B, sbj, sbk, epi, pf);
}

// What the extra blocks of a small product should read ahead: the weight matrix W [n_out, n_in] of a
// later product of the chain.  forward: the consumer is Z = A W^T (its column tiles are rows of W);
// else the data gradient dA = dZ W (its column tiles are column ranges of W).
template <typename T>
PmPrefetch prefetch_of(const PmWLoc<T>& W, int n_out, int n_in, bool forward) {
  PmPrefetch pf{nullptr, nullptr, 0, 0, 0, 0, 0, 0};
  if (sizeof(T) != 2) return pf;
  const int tiles = ((forward ? n_out : n_in) + 31) / 32;       // the consumer's column tiles (32 wide)
  if (tiles % 8) return pf;
  pf.base = reinterpret_cast<const unsigned char*>(W.base);
  pf.slot = W.slot;
  pf.stride_bytes = W.stride * (int64_t)sizeof(T);
  pf.rows = n_out;
  pf.row_bytes = n_in * (int)sizeof(T);
  pf.ld_bytes = (int64_t)n_in * sizeof(T);
  pf.by_rows = forward ? 1 : 0;
  pf.share = forward ? tiles / 8 * 32 : tiles / 8 * 32 * (int)sizeof(T);
  return pf;
}

// Forward on the tau_fwd-stale ring slots, loss, backward on the corrected weights.
template <typename T>
pm_status launch_fwd_bwd(pm_ctx* c, const void* x_dev, const void* y_dev, int accumulate, int par) {
  const Layout& lay = c->lay;
  hipStream_t st = c->stream;
  const int M = c->o.microbatch, L = c->L;
  T* ring = c->at<T>(lay.ring_off);
  T* ub = c->at<T>(lay.ub_off);
  float* g = c->at<float>(lay.g_off);
  const Unit& u0 = lay.units[0];
  prof_mark(c, 0);
  const bool chained = sizeof(T) == 2 && c->chain_grid > 0 && par == 0;
  {
    // one launch: block 0 also refreshes the slot / step-size table at the start of a minibatch
    const int64_t tot = std::max<int64_t>((int64_t)M * u0.ld_in, chained ? c->chain_fill16 : 0);
    hipLaunchKernelGGL((pm_begin_step_kernel<T>), dim3((unsigned)std::min<int64_t>(1024, (tot + 255) / 256)), dim3(256),
                       0, st, (const float*)x_dev, c->at<T>(lay.x_off), M, u0.d.n_in, u0.ld_in, c->hdr(), c->ls(),
                       c->ld(par), accumulate ? 0 : L, sched_dev(c), par,
                       chained ? c->at<uint4>(lay.units[0].z_off) : nullptr, chained ? c->chain_fill16 : 0);
  }
  if (chained && c->chain_nf >= 2) {
    ProfSpan span(c, PM_CLS_GEMM);
    hipLaunchKernelGGL(pm_chain_fwd_kernel, dim3(c->chain_grid), dim3(PM_CHAIN_NT), 0, st, c->at<PmChainFwd>(lay.chain_f_off),
                       c->chain_nf, M, c->hdr());
  }
  const int fwd_first = chained && c->chain_nf >= 2 ? c->chain_nf : 0;
  // ---- forward: unit l reads W (and b) of version max(t - tau_fwd, 0) in place from its ring slot
  for (int l = fwd_first; l < L; ++l) {
    const Unit& u = lay.units[l];
    const T* a_in = l == 0 ? c->at<T>(lay.x_off) : c->at<T>(lay.units[l - 1].a_off);
    PmWLoc<T> W{ring + u.ring_off, &c->ld(par)[l].fwd_slot, u.n_pad};
    PmEpiFwd<T> epi;
    epi.bias = PmWLoc<T>{ring + u.ring_off + u.boff, &c->ld(par)[l].fwd_slot, u.n_pad};
    epi.z = (l == L - 1) ? nullptr : c->at<T>(u.z_off);
    epi.a = (l == L - 1) ? nullptr : c->at<T>(u.a_off);
    epi.z32 = (l == L - 1) ? c->at<float>(u.z32_off) : nullptr;
    epi.ld = u.ld_out;
    epi.act = u.d.act;
    epi.b_ = nullptr;
    // while this product runs, its idle blocks read ahead the next unit's forward weights
    PmPrefetch pf{nullptr, nullptr, 0, 0, 0, 0, 0, 0};
    if (l + 1 < L) {
      const Unit& un = lay.units[l + 1];
      pf = prefetch_of<T>(PmWLoc<T>{ring + un.ring_off, &c->ld(par)[l + 1].fwd_slot, un.n_pad}, un.d.n_out, un.d.n_in, true);
    }
    // Z[M, n_out] = A[M, n_in] . W[n_out, n_in]^T
    launch_gemm<T>(c, M, u.d.n_out, u.d.n_in, a_in, u.ld_in, 1, W, u.d.n_in, 1, epi, &pf);
  }
  // ---- loss and d(loss)/d(z_last)   (the last unit's activation must be PM_ACT_NONE)
  {
    const Unit& u = lay.units[L - 1];
    if (c->o.loss == PM_LOSS_XENT)
      pm_xent_launch<T>(st, c->at<float>(u.z32_off), (const int32_t*)y_dev, c->at<T>(u.dz_off), M, u.d.n_out, u.ld_out,
                        c->hdr());
    else {
      const int64_t tot = (int64_t)M * u.ld_out;
      hipLaunchKernelGGL((pm_mse_kernel<T>), dim3((unsigned)std::min<int64_t>(256, (tot + 255) / 256)), dim3(256), 0, st,
                         c->at<float>(u.z32_off), (const float*)y_dev, c->at<T>(u.dz_off), M, u.d.n_out, u.ld_out,
                         c->hdr());
    }
  }
  prof_mark(c, 1);
  // The backward needs what the previous step's update produced (corrected weights, or version t
  // itself when tau_bkwd = 0) and will overwrite the gradient buffer that update reads.
  {
    pm_status qs = quiesce(c);
    if (qs != PM_OK) return qs;
  }
  // ---- backward, data-gradient chain: da_in[M, n_in] = dz . W_bkwd, fused with act'(z_prev).
  // W_bkwd = corrected buffer when the T2 coefficient is non-zero, else version max(t - tau_bkwd, 0).
  // The first unit needs none (its backward weights never enter any gradient).
  auto bwd_data = [&](int l) {
    const Unit& u = lay.units[l];
    const Unit& up = lay.units[l - 1];
    const T* dz = c->at<T>(u.dz_off);
    PmWLoc<T> Wb = u.corr ? PmWLoc<T>{ub + u.off, nullptr, 0}
                          : PmWLoc<T>{ring + u.ring_off, &c->ld(par)[l].bkwd_slot, u.n_pad};
    PmEpiBwdData<T> ed{c->at<T>(up.z_off), c->at<T>(up.dz_off), up.ld_out, up.d.act};
    // idle blocks read ahead the backward weights of the unit below (the next product of the chain)
    PmPrefetch pf{nullptr, nullptr, 0, 0, 0, 0, 0, 0};
    if (l >= 2) {
      const PmWLoc<T> Wn = up.corr ? PmWLoc<T>{ub + up.off, nullptr, 0}
                                   : PmWLoc<T>{ring + up.ring_off, &c->ld(par)[l - 1].bkwd_slot, up.n_pad};
      pf = prefetch_of<T>(Wn, up.d.n_out, up.d.n_in, false);
    }
    launch_gemm<T>(c, M, u.d.n_in, u.d.n_out, dz, u.ld_out, 1, Wb, 1, u.d.n_in, ed, &pf);
  };
  if (!lay.recompute) {
    const int hb = chained && c->chain_hb >= 2 ? c->chain_hb : 0;
    for (int l = L - 1; l > hb; --l) bwd_data(l);
    if (hb) {
      ProfSpan span(c, PM_CLS_GEMM);
      hipLaunchKernelGGL(pm_chain_bwd_kernel, dim3(c->chain_grid), dim3(PM_CHAIN_NT), 0, st, c->at<PmChainBwd>(lay.chain_b_off),
                         hb, M, c->hdr());
    }
  } else {
    // Recomputation (App. on recompute): the forward pass is taken to have kept only the input of
    // every segment; before a segment's backward its pre-activations and inner inputs are rebuilt
    // from that input with the weights u_recomp = version max(t - tau_recomp, 0), corrected by
    // (tau_fwd - tau_recomp) delta_t ("T2 for Recompute").  The rebuilt values overwrite the forward's
    // in place - except a segment's output, which is the next segment's kept input.  The head needs
    // no pre-activation (no activation function) and is not recomputed.
    // (The product that crosses a segment boundary multiplies by act'(z) of the earlier segment's
    // last unit, a rebuilt value: it waits until that segment has been recomputed.)
    T* ur = lay.has_ur ? c->at<T>(lay.ur_off) : nullptr;
    int hi = L - 1, pending = -1;
    while (hi >= 0) {
      int lo = hi;
      while (!lay.units[lo].seg_first) --lo;
      for (int l = lo; l <= hi; ++l) {
        if (l == L - 1) continue;
        const Unit& u = lay.units[l];
        const T* a_in = l == 0 ? c->at<T>(lay.x_off) : c->at<T>(lay.units[l - 1].a_off);
        const T* base;
        const int32_t* slot;
        if (u.corr_r) { base = ur + u.off; slot = nullptr; }                       // own corrected copy
        else if (u.tau_r == u.tau_b && u.corr) { base = ub + u.off; slot = nullptr; }   // same as the backward weights
        else { base = ring + u.ring_off; slot = &c->ld(par)[l].rec_slot; }          // plain version, read in place
        PmWLoc<T> W{base, slot, slot ? u.n_pad : 0};
        PmEpiFwd<T> epi;
        epi.bias = PmWLoc<T>{base + u.boff, slot, slot ? u.n_pad : 0};
        epi.z = c->at<T>(u.z_off);
        epi.a = l == hi ? nullptr : c->at<T>(u.a_off);
        epi.z32 = nullptr;
        epi.ld = u.ld_out;
        epi.act = u.d.act;
        epi.b_ = nullptr;
        launch_gemm<T>(c, M, u.d.n_out, u.d.n_in, a_in, u.ld_in, 1, W, u.d.n_in, 1, epi);
      }
      if (pending >= 1) bwd_data(pending);
      for (int l = hi; l > lo; --l) bwd_data(l);
      pending = lo;
      hi = lo - 1;
    }
  }
  // ---- weight gradients from the stored forward activations: dW[n_out, n_in] = dz^T . a_in,
  // db = column sums of dz.  They depend only on stored tensors, so all units go out as ONE
  // grouped launch (bias gradients fused) when every unit fits the MFMA kernel.
  bool grouped = false;
  if constexpr (sizeof(T) == 2) {
    if (c->dw_grouped) {
      ProfSpan span(c, PM_CLS_GEMM);
      const auto* tab = c->at<PmGemmProb<PmEpiBwdWeight>>(lay.probs_off) + (accumulate ? L : 0);
      dim3 grid((c->dw_maxJ + 63) / 64, (c->dw_maxI + 63) / 64, L);
      if (M <= 128)
        hipLaunchKernelGGL((pm_gemm_mfma_grouped_kernel<PmCfgShortK, false, false, PmEpiBwdWeight>), grid, dim3(256), 0,
                           st, tab);
      else
        hipLaunchKernelGGL((pm_gemm_mfma_grouped_kernel<PmCfgMid, false, false, PmEpiBwdWeight>), grid, dim3(256), 0, st,
                           tab);
      grouped = true;
    }
  }
  if (!grouped) {
    for (int l = L - 1; l >= 0; --l) {
      const Unit& u = lay.units[l];
      const T* a_in = l == 0 ? c->at<T>(lay.x_off) : c->at<T>(lay.units[l - 1].a_off);
      const T* dz = c->at<T>(u.dz_off);
      PmEpiBwdWeight ew{g + u.off, u.d.n_in, accumulate, nullptr};
      launch_gemm<T>(c, u.d.n_out, u.d.n_in, M, dz, 1, u.ld_out, PmWLoc<T>{a_in, nullptr, 0}, 1, u.ld_in, ew);
      launch_bias_grad<T>(st, dz, g + u.off + u.boff, M, u.d.n_out, u.ld_out, accumulate);
    }
  }
  PM_HIP(hipGetLastError());
  return PM_OK;
}


// ---------------------------------------------------------------------------------------------
// Fine-grained pre-LN causal Transformer: one microbatch forward on the tau_fwd-stale ring slots,
// token cross-entropy, backward on the corrected weights.  Residual stream and its gradient fp32;
// GEMM operands in the compute dtype.  A backward kernel reads a weight only where a gradient
// flows through it (Linear: dz . W; LayerNorm: dy * gain); weight gradients use stored forward
// activations (Sec. 2.1).
// ---------------------------------------------------------------------------------------------
template <typename T>
pm_status launch_tfm(pm_ctx* c, const void* x_dev, const void* y_dev, int accumulate, int par) {
  const Layout& lay = c->lay;
  hipStream_t st = c->stream;
  const int L = c->L, nl = (L - 3) / 8;
  const int B = c->o.microbatch, S = c->o.seq_len, H = c->o.n_heads;
  const int Tk = B * S, V = lay.units[0].d.n_in, d = lay.units[0].d.n_out, dff = lay.units[7].d.n_out, dh = d / H;
  const int ldV = (int)round_up(V, 8);
  T* ring = c->at<T>(lay.ring_off);
  T* ub = c->at<T>(lay.ub_off);
  float* g = c->at<float>(lay.g_off);
  PmLayerStep* tab = c->ld(par);
  const int32_t* tokens = (const int32_t*)x_dev;
  auto U = [&](int u) -> const Unit& { return lay.units[u]; };
  auto Wf = [&](int u, int64_t extra) { return PmWLoc<T>{ring + U(u).ring_off + extra, &tab[u].fwd_slot, U(u).n_pad}; };
  auto Wb = [&](int u, int64_t extra) {
    return U(u).corr ? PmWLoc<T>{ub + U(u).off + extra, nullptr, 0}
                     : PmWLoc<T>{ring + U(u).ring_off + extra, &tab[u].bkwd_slot, U(u).n_pad};
  };
  // the weights that rebuild unit u's activations in a recomputing backward pass: the unit's own corrected
  // copy, the corrected backward weights where delay and coefficient coincide, else the plain version
  // max(t - tau_recomp, 0) read in place from the ring
  T* ur = lay.has_ur ? c->at<T>(lay.ur_off) : nullptr;
  auto Wr = [&](int u, int64_t extra) {
    if (U(u).corr_r) return PmWLoc<T>{ur + U(u).off + extra, nullptr, 0};
    if (U(u).tau_r == U(u).tau_b && U(u).corr) return PmWLoc<T>{ub + U(u).off + extra, nullptr, 0};
    return PmWLoc<T>{ring + U(u).ring_off + extra, &tab[u].rec_slot, U(u).n_pad};
  };
  bool rebuilding = false;     // the forward helpers below read Wr instead of Wf while a segment is rebuilt
  auto Wx = [&](int u, int64_t extra) { return rebuilding ? Wr(u, extra) : Wf(u, extra); };
  // z = a_in W_fwd^T + b (optional), a = act(z)
  auto lin_fwd = [&](int u, const T* a_in, int n_in, int n_out, T* z, T* a, int act) {
    PmEpiFwd<T> epi;
    epi.bias = Wx(u, U(u).boff);
    epi.z = z; epi.a = a; epi.z32 = nullptr; epi.ld = n_out; epi.act = act; epi.b_ = nullptr;
    launch_gemm<T>(c, Tk, n_out, n_in, a_in, n_in, 1, Wx(u, 0), n_in, 1, epi);
  };
  // out = res + a_in W_fwd^T + b   (fp32 residual stream)
  auto lin_fwd_res = [&](int u, const T* a_in, int n_in, int n_out, const float* res, float* out) {
    PmEpiFwdRes<T> epi;
    epi.bias = Wx(u, U(u).boff);
    epi.res = res; epi.out = out; epi.ld = n_out; epi.b_ = nullptr;
    launch_gemm<T>(c, Tk, n_out, n_in, a_in, n_in, 1, Wx(u, 0), n_in, 1, epi);
  };
  // dW = dz^T a_in, db = column sums of dz
  auto wgrad = [&](int u, const T* dz, int ld_dz, const T* a_in, int n_out, int n_in) {
    PmEpiBwdWeight ew{g + U(u).off, n_in, accumulate, nullptr};
    launch_gemm<T>(c, n_out, n_in, Tk, dz, 1, ld_dz, PmWLoc<T>{a_in, nullptr, 0}, 1, n_in, ew);
    launch_bias_grad<T>(st, dz, g + U(u).off + U(u).boff, Tk, n_out, ld_dz, accumulate);
  };
  // fp32 out (+)= dz W_bkwd
  auto dgrad_f32 = [&](int u, const T* dz, int ld_dz, int n_out, int n_in, float* out, int acc) {
    PmEpiF32 e{out, n_in, acc};
    launch_gemm<T>(c, Tk, n_in, n_out, dz, ld_dz, 1, Wb(u, 0), 1, n_in, e);
  };
  // out = (dz W_bkwd) * act'(zprev) in the compute dtype
  auto dgrad_t = [&](int u, const T* dz, int n_out, int n_in, const T* zprev, int act, T* out) {
    PmEpiBwdData<T> e{zprev, out, n_in, act};
    launch_gemm<T>(c, Tk, n_in, n_out, dz, n_out, 1, Wb(u, 0), 1, n_in, e);
  };
  // query, key and value projections of units u+1 .. u+3 (same input): one launch when the shapes suit
  auto qkv_fwd = [&](int u, const T* n1, T* q, T* k, T* v) {
    if constexpr (sizeof(T) == 2) {
      T* outs[3] = {q, k, v};
      PmGemmProb<PmEpiFwd<T>> pr[3];
      for (int p = 0; p < 3; ++p) {
        PmEpiFwd<T> epi;
        epi.bias = Wf(u + 1 + p, U(u + 1 + p).boff);
        epi.z = nullptr; epi.a = outs[p]; epi.z32 = nullptr; epi.ld = d; epi.act = PM_ACT_NONE; epi.b_ = nullptr;
        pr[p] = PmGemmProb<PmEpiFwd<T>>{Tk, d, d, n1, d, Wf(u + 1 + p, 0), d, epi};
      }
      ProfSpan span(c, PM_CLS_GEMM);
      if (pm_gemm_multi3_try(st, pr)) return;
    }
    lin_fwd(u + 1, n1, d, d, nullptr, q, PM_ACT_NONE);
    lin_fwd(u + 2, n1, d, d, nullptr, k, PM_ACT_NONE);
    lin_fwd(u + 3, n1, d, d, nullptr, v, PM_ACT_NONE);
  };
  // out = dzq Wq + dzk Wk + dzv Wv (backward weights): one product over the concatenated contraction
  auto qkv_dgrad = [&](int u, const T* dzq, const T* dzk, const T* dzv, float* out) {
    if constexpr (sizeof(T) == 2) {
      const T* const A[3] = {dzq, dzk, dzv};
      const PmWLoc<T> Bw[3] = {Wb(u + 1, 0), Wb(u + 2, 0), Wb(u + 3, 0)};
      PmEpiF32 e{out, d, 0};
      ProfSpan span(c, PM_CLS_GEMM);
      if (pm_gemm_kseg3_try(st, Tk, d, d, A, d, Bw, d, e)) return;
    }
    dgrad_f32(u + 1, dzq, d, d, d, out, 0);
    dgrad_f32(u + 2, dzk, d, d, d, out, 1);
    dgrad_f32(u + 3, dzv, d, d, d, out, 1);
  };
  auto ln_fwd = [&](int u, const float* x, T* out, float* mu, float* rs) {
    pm_ln_fwd_launch<T>(st, x, Wx(u, 0), (int)U(u).boff, out, mu, rs, Tk, d);
  };
  auto ln_bwd = [&](int u, const float* dy, const float* x, const float* mu, const float* rs, const float* dx_res,
                    float* dx_out, T* dx_t) {
    pm_ln_bwd_launch<T>(st, dy, x, mu, rs, Wb(u, 0), dx_res, dx_out, dx_t, g + U(u).off, g + U(u).off + U(u).boff, Tk, d);
  };
  auto F = [&](size_t off) { return c->at<float>(off); };
  auto TT = [&](size_t off) { return c->at<T>(off); };
  // Behind a ReLU the pre-activation need not be kept: the derivative mask of z is the mask of a = relu(z).
  // The first feed-forward product then writes one output instead of two.
  auto ff_keeps_z = [&](int u6) { return U(u6).d.act != PM_ACT_RELU; };
  auto ff_mask_src = [&](const Layout::TfmLayer& b, int u6) { return ff_keeps_z(u6) ? TT(b.z1) : TT(b.f); };

  prof_mark(c, 0);
  hipLaunchKernelGGL(pm_begin_tokens_kernel, dim3(1), dim3(256), 0, st, c->hdr(), c->ls(), tab, accumulate ? 0 : L,
                     sched_dev(c), par);
  // ---- forward
  float* x0 = F(nl ? lay.tl[0].x : lay.t_xf);
  auto embed_fwd = [&]() {
    const int64_t tot = (int64_t)Tk * d;
    hipLaunchKernelGGL((pm_embed_fwd_kernel<T>), dim3((unsigned)std::min<int64_t>(4096, (tot + 255) / 256)), dim3(256), 0,
                       st, tokens, Wx(0, 0), F(lay.t_pos), x0, Tk, S, d, V);
  };
  auto attn_fwd = [&](const Layout::TfmLayer& b) {
    ProfSpan span(c, PM_CLS_ATTN);
    return pm_attn_fwd_launch<T>(st, B, S, H, dh, TT(b.q), TT(b.k), TT(b.v), TT(b.o), F(b.lse));
  };
  embed_fwd();
  for (int l = 0; l < nl; ++l) {
    const Layout::TfmLayer& b = lay.tl[l];
    const int u = 1 + 8 * l;
    float* x = F(b.x);
    float* y = F(l + 1 < nl ? lay.tl[l + 1].x : lay.t_xf);
    ln_fwd(u, x, TT(b.n1), F(b.mu1), F(b.rs1));
    qkv_fwd(u, TT(b.n1), TT(b.q), TT(b.k), TT(b.v));
    if (!attn_fwd(b)) return fail(PM_EINVAL, "attention shape not supported");
    lin_fwd_res(u + 4, TT(b.o), d, d, x, F(b.h));
    ln_fwd(u + 5, F(b.h), TT(b.n2), F(b.mu2), F(b.rs2));
    lin_fwd(u + 6, TT(b.n2), d, dff, ff_keeps_z(u + 6) ? TT(b.z1) : nullptr, TT(b.f), U(u + 6).d.act);
    lin_fwd_res(u + 7, TT(b.f), dff, d, F(b.h), y);
  }
  ln_fwd(L - 2, F(lay.t_xf), TT(lay.t_nf), F(lay.t_muf), F(lay.t_rsf));
  {
    PmEpiFwd<T> epi;
    epi.bias = Wf(L - 1, U(L - 1).boff);
    epi.z = nullptr; epi.a = nullptr; epi.z32 = F(lay.t_logits); epi.ld = ldV; epi.act = PM_ACT_NONE; epi.b_ = nullptr;
    launch_gemm<T>(c, Tk, V, d, TT(lay.t_nf), d, 1, Wf(L - 1, 0), d, 1, epi);
  }
  pm_xent_launch<T>(st, F(lay.t_logits), (const int32_t*)y_dev, TT(lay.t_dlogits), Tk, V, ldV, c->hdr());
  prof_mark(c, 1);
  {
    pm_status qs = quiesce(c);
    if (qs != PM_OK) return qs;
  }
  // ---- backward
  if (!accumulate && lay.n_zero > 0) {
    const unsigned bx = (unsigned)std::max<int64_t>(1, std::min<int64_t>(1024, lay.zero_max / 4 / 256));
    hipLaunchKernelGGL(pm_zero_regions_kernel, dim3(bx, lay.n_zero), dim3(256), 0, st, g, c->at<int64_t>(lay.t_zero));
  }
  float* dx = F(lay.t_dx);
  float* dn = F(lay.t_dn);
  // Weight gradients depend only on stored tensors (dz of the unit, its forward input).  On the MFMA
  // path they are deferred: every unit's dz stays in a buffer of its own and ONE grouped launch at the
  // end computes all dW and db.  Otherwise each unit's products go out as they become available.
  const bool grouped = c->dw_grouped;
  auto wg = [&](int u, const T* dz, int ld_dz, const T* a_in, int n_out, int n_in) {
    if (!grouped) wgrad(u, dz, ld_dz, a_in, n_out, n_in);
  };
  // Recomputation (App. on recompute; "T2 for Recompute"): the forward pass is taken to have kept only the
  // tensors that cross a segment boundary.  Units are walked backwards; on entering a segment, all its units
  // first run again in order with the weights Wr, overwriting their outputs in place.  At that moment every
  // later segment has finished its backward pass, and no earlier one has been rebuilt: so a unit - in the
  // rebuild and in its backward alike - sees rebuilt tensors exactly where the producer sits in its own segment
  // and the kept forward tensors where it sits in an earlier one.  Weight gradients go out as soon as their unit
  // is reached (their inputs may be overwritten by an earlier segment's rebuild).  The head is not rebuilt (the
  // loss gradient comes from the forward pass).
  auto seg_of = [&](int u) { return (U(u).d.stage - 1) / c->o.segment_size; };
  auto rebuild_unit = [&](int u) -> bool {
    if (u == 0) { embed_fwd(); return true; }
    if (u == L - 2) { ln_fwd(u, F(lay.t_xf), TT(lay.t_nf), F(lay.t_muf), F(lay.t_rsf)); return true; }
    const int l = (u - 1) / 8, j = (u - 1) % 8, u0 = 1 + 8 * l;
    const Layout::TfmLayer& b = lay.tl[l];
    switch (j) {
      case 0: ln_fwd(u, F(b.x), TT(b.n1), F(b.mu1), F(b.rs1)); break;
      case 1: lin_fwd(u, TT(b.n1), d, d, nullptr, TT(b.q), PM_ACT_NONE); break;
      case 2: lin_fwd(u, TT(b.n1), d, d, nullptr, TT(b.k), PM_ACT_NONE); break;
      case 3: lin_fwd(u, TT(b.n1), d, d, nullptr, TT(b.v), PM_ACT_NONE); break;
      case 4:
        if (!attn_fwd(b)) return false;
        lin_fwd_res(u, TT(b.o), d, d, F(b.x), F(b.h));
        break;
      case 5: ln_fwd(u, F(b.h), TT(b.n2), F(b.mu2), F(b.rs2)); break;
      case 6: lin_fwd(u, TT(b.n2), d, dff, ff_keeps_z(u) ? TT(b.z1) : nullptr, TT(b.f), U(u).d.act); break;
      default: lin_fwd_res(u0 + 7, TT(b.f), dff, d, F(b.h), F(l + 1 < nl ? lay.tl[l + 1].x : lay.t_xf)); break;
    }
    return true;
  };
  auto enter = [&](int u) -> bool {       // called before the backward of unit u
    if (!lay.recompute || (u < L - 1 && seg_of(u) == seg_of(u + 1))) return true;
    int lo = u;
    while (lo > 0 && seg_of(lo - 1) == seg_of(u)) --lo;
    rebuilding = true;
    bool ok = true;
    for (int v = lo; v <= u && ok; ++v)
      if (v != L - 1) ok = rebuild_unit(v);
    rebuilding = false;
    return ok;
  };
#define PM_ENTER(u) do { if (!enter(u)) return fail(PM_EINVAL, "attention shape not supported"); } while (0)
  PM_ENTER(L - 1);
  wg(L - 1, TT(lay.t_dlogits), ldV, TT(lay.t_nf), V, d);
  // The data gradient through the vocabulary projection: Tk x d outputs (few tiles) over a contraction of V.
  // When 256 x 256 tiles of it cover at most half the chip, the contraction is cut into two halves that run
  // side by side on such tiles; the second half's output goes to the (still unused) buffer of dx and the
  // LayerNorm backward that consumes the gradient adds the two.
  const float* dn2 = nullptr;
  bool head_split = false;
  if constexpr (sizeof(T) == 2) {
    const int t256 = (Tk / 256) * (d / 256);
    if (Tk % 256 == 0 && d % 256 == 0 && V % 128 == 0 && V >= 16384 && ldV == V && 2 * t256 <= 256 && 2 * t256 >= 128) {
      const int Kh = V / 2;
      const T* dl = TT(lay.t_dlogits);
      const PmWLoc<T> W = Wb(L - 1, 0);
      PmGemmProb<PmEpiF32> p0{Tk, d, Kh, dl, ldV, W, d, PmEpiF32{dn, d, 0}};
      PmWLoc<T> W1 = W;
      W1.base += (int64_t)Kh * d;
      PmGemmProb<PmEpiF32> p1{Tk, d, Kh, dl + Kh, ldV, W1, d, PmEpiF32{dx, d, 0}};
      ProfSpan span(c, PM_CLS_GEMM);
      hipLaunchKernelGGL((pm_gemm_big_khalves_kernel<PmBig256, true, false, PmEpiF32>), dim3(2 * t256), dim3(PmBig256::NT), 0, st,
                         p0, p1, Tk / 256, d / 256);
      dn2 = dx;
      head_split = true;
    }
  }
  if (!head_split) dgrad_f32(L - 1, TT(lay.t_dlogits), ldV, V, d, dn, 0);
  PM_ENTER(L - 2);
  pm_ln_bwd_launch<T>(st, dn, F(lay.t_xf), F(lay.t_muf), F(lay.t_rsf), Wb(L - 2, 0), nullptr, dx, nl ? TT(lay.tl[nl - 1].dz2) : nullptr,
                      g + U(L - 2).off, g + U(L - 2).off + U(L - 2).boff, Tk, d, dn2);
  for (int l = nl - 1; l >= 0; --l) {
    const Layout::TfmLayer& b = lay.tl[l];
    const int u = 1 + 8 * l;
    // y = h + f W2^T + b2.  The activation derivative of the first feed-forward matrix rides on this product
    // unless a segment boundary separates the two: then it waits for the rebuilt pre-activations.
    const bool split_act = lay.recompute && seg_of(u + 6) != seg_of(u + 7) && U(u + 6).d.act != PM_ACT_NONE;
    PM_ENTER(u + 7);
    wg(u + 7, TT(b.dz2), d, TT(b.f), d, dff);
    dgrad_t(u + 7, TT(b.dz2), d, dff, ff_mask_src(b, u + 6), split_act ? (int)PM_ACT_NONE : U(u + 6).d.act, TT(b.dz1));
    PM_ENTER(u + 6);
    if (split_act) {
      const int64_t tot = (int64_t)Tk * dff;
      hipLaunchKernelGGL((pm_act_bwd_apply_kernel<T>), dim3((unsigned)std::min<int64_t>(4096, (tot / 4 + 255) / 256)), dim3(256), 0,
                         st, TT(b.dz1), ff_mask_src(b, u + 6), U(u + 6).d.act, tot);
    }
    wg(u + 6, TT(b.dz1), dff, TT(b.n2), dff, d);
    dgrad_f32(u + 6, TT(b.dz1), dff, dff, d, dn, 0);
    PM_ENTER(u + 5);
    ln_bwd(u + 5, dn, F(b.h), F(b.mu2), F(b.rs2), dx, dx, TT(b.dzo));          // dx is now d loss / d h
    // h = x + o Wo^T + bo
    PM_ENTER(u + 4);
    wg(u + 4, TT(b.dzo), d, TT(b.o), d, d);
    dgrad_t(u + 4, TT(b.dzo), d, d, nullptr, PM_ACT_NONE, TT(lay.t_do));
    {
      ProfSpan span(c, PM_CLS_ATTN);
      if (!pm_attn_bwd_launch<T>(st, B, S, H, dh, TT(b.q), TT(b.k), TT(b.v), TT(b.o), TT(lay.t_do), F(b.lse), TT(b.dzq),
                                 TT(b.dzk), TT(b.dzv)))
        return fail(PM_EINVAL, "attention shape not supported");
    }
    PM_ENTER(u + 3);
    wg(u + 3, TT(b.dzv), d, TT(b.n1), d, d);
    PM_ENTER(u + 2);
    wg(u + 2, TT(b.dzk), d, TT(b.n1), d, d);
    PM_ENTER(u + 1);
    wg(u + 1, TT(b.dzq), d, TT(b.n1), d, d);
    qkv_dgrad(u, TT(b.dzq), TT(b.dzk), TT(b.dzv), dn);
    PM_ENTER(u);
    ln_bwd(u, dn, F(b.x), F(b.mu1), F(b.rs1), dx, dx, l ? TT(lay.tl[l - 1].dz2) : nullptr);   // dx is now d loss / d x
  }
#undef PM_ENTER
  if constexpr (sizeof(T) == 2) {
    if (grouped) {
      ProfSpan span(c, PM_CLS_GEMM);
      const auto* tab = c->at<PmGemmProb<PmEpiBwdWeight>>(lay.t_wprobs) + (accumulate ? c->dw_nprob : 0);
      if (c->fuse_upd && c->dw_tile == 256)
        hipLaunchKernelGGL((pm_gemm_big_grouped_kernel<PmBig256, false, false, false, PmEpiBwdWeightUpd>), dim3(c->dw_ntiles),
                           dim3(PmBig256::NT), 0, st, c->at<PmGemmProb<PmEpiBwdWeightUpd>>(lay.t_fuse),
                           c->at<PmXcdSeg>(lay.t_wsegs), c->at<int32_t>(lay.t_wtiles), c->dw_max_segs);
      else if (c->fuse_upd)
        hipLaunchKernelGGL((pm_gemm_big_grouped_kernel<PmBig128, false, false, false, PmEpiBwdWeightUpd>), dim3(c->dw_ntiles),
                           dim3(PmBig128::NT), 0, st, c->at<PmGemmProb<PmEpiBwdWeightUpd>>(lay.t_fuse),
                           c->at<PmXcdSeg>(lay.t_wsegs), c->at<int32_t>(lay.t_wtiles), c->dw_max_segs);
      else if (c->dw_tile == 256)
        hipLaunchKernelGGL((pm_gemm_big_grouped_kernel<PmBig256, false, false, false, PmEpiBwdWeight>), dim3(c->dw_ntiles),
                           dim3(PmBig256::NT), 0, st, tab, c->at<PmXcdSeg>(lay.t_wsegs), c->at<int32_t>(lay.t_wtiles),
                           c->dw_max_segs);
      else if (c->dw_aligned)
        hipLaunchKernelGGL((pm_gemm_big_grouped_kernel<PmBig128, false, false, false, PmEpiBwdWeight>), dim3(c->dw_ntiles),
                           dim3(PmBig128::NT), 0, st, tab, c->at<PmXcdSeg>(lay.t_wsegs), c->at<int32_t>(lay.t_wtiles),
                           c->dw_max_segs);
      else
        hipLaunchKernelGGL((pm_gemm_big_grouped_kernel<PmBig128, false, false, true, PmEpiBwdWeight>), dim3(c->dw_ntiles),
                           dim3(PmBig128::NT), 0, st, tab, c->at<PmXcdSeg>(lay.t_wsegs), c->at<int32_t>(lay.t_wtiles),
                           c->dw_max_segs);
    }
  }
  {
    const int64_t tot = (int64_t)Tk * d;
    hipLaunchKernelGGL(pm_embed_bwd_kernel, dim3((unsigned)std::min<int64_t>(4096, (tot + 255) / 256)), dim3(256), 0, st,
                       tokens, dx, g + U(0).off, Tk, d, V);
  }
  PM_HIP(hipGetLastError());
  return PM_OK;
}

// ---------------------------------------------------------------------------------------------
// ResNet-shaped CNN: one microbatch forward on the tau_fwd-stale ring slots, cross-entropy, backward
// on the corrected weights.  Unit u < L - 1 is a 3x3 convolution with folded affine and ReLU;
// units (1, 2), (3, 4), ... form residual blocks; the last unit is the classifier on the pooled map.
// ---------------------------------------------------------------------------------------------
template <typename T>
pm_status launch_resnet(pm_ctx* c, const void* x_dev, const void* y_dev, int accumulate, int par) {
  const Layout& lay = c->lay;
  hipStream_t st = c->stream;
  const int L = c->L, nconv = L - 1, B = c->o.microbatch;
  T* ring = c->at<T>(lay.ring_off);
  T* ub = c->at<T>(lay.ub_off);
  float* g = c->at<float>(lay.g_off);
  PmLayerStep* tab = c->ld(par);
  auto U = [&](int u) -> const Unit& { return lay.units[u]; };
  auto Wf = [&](int u, int64_t extra) { return PmWLoc<T>{ring + U(u).ring_off + extra, &tab[u].fwd_slot, U(u).n_pad}; };
  auto Wb = [&](int u, int64_t extra) {
    return U(u).corr ? PmWLoc<T>{ub + U(u).off + extra, nullptr, 0}
                     : PmWLoc<T>{ring + U(u).ring_off + extra, &tab[u].bkwd_slot, U(u).n_pad};
  };
  T* ur = lay.has_ur ? c->at<T>(lay.ur_off) : nullptr;
  auto Wr = [&](int u, int64_t extra) {       // the weights that rebuild unit u's activations (see launch_tfm)
    if (U(u).corr_r) return PmWLoc<T>{ur + U(u).off + extra, nullptr, 0};
    if (U(u).tau_r == U(u).tau_b && U(u).corr) return PmWLoc<T>{ub + U(u).off + extra, nullptr, 0};
    return PmWLoc<T>{ring + U(u).ring_off + extra, &tab[u].rec_slot, U(u).n_pad};
  };
  auto TT = [&](size_t off) { return c->at<T>(off); };
  const int fc = L - 1, C = U(fc).d.n_in, ncls = U(fc).d.n_out, ldc = (int)round_up(ncls, 8);
  const PmConvGeom& gl = lay.cv[nconv - 1].g;
  const int HW = gl.Ho * gl.Wo;

  prof_mark(c, 0);
  hipLaunchKernelGGL(pm_begin_tokens_kernel, dim3(1), dim3(256), 0, st, c->hdr(), c->ls(), tab, accumulate ? 0 : L,
                     sched_dev(c), par);
  {
    const PmConvGeom& g0 = lay.cv[0].g;
    const int64_t tot = (int64_t)B * g0.H * g0.W * g0.Cin;
    hipLaunchKernelGGL((pm_image_stage_kernel<T>), dim3((unsigned)std::min<int64_t>(2048, (tot + 255) / 256)), dim3(256), 0, st,
                       (const float*)x_dev, TT(lay.r_x), B, g0.Cin, g0.H, g0.W);
  }
  // ---- forward
  auto input_of = [&](int u) { return u == 0 ? TT(lay.r_x) : TT(lay.cv[u - 1].y); };
  auto conv_fwd = [&](int u, PmWLoc<T> W) {
    const Layout::ConvBuf& b = lay.cv[u];
    PmShortcut<T> sc{nullptr, 0, 0, 0, 1};
    if (u >= 2 && (u % 2) == 0) {                     // second convolution of a block: add the block input
      const PmConvGeom& g1 = lay.cv[u - 1].g;         // geometry of the block's first convolution
      sc = PmShortcut<T>{input_of(u - 1), g1.H, g1.W, g1.Cin, g1.stride};
    }
    ProfSpan span(c, PM_CLS_GEMM);
    pm_conv_fwd_launch<T>(st, b.g, input_of(u), W, sc, TT(b.z), TT(b.y));
  };
  for (int u = 0; u < nconv; ++u) conv_fwd(u, Wf(u, 0));
  pm_pool_fwd_launch<T>(st, TT(lay.cv[nconv - 1].y), TT(lay.r_pool), B, HW, C);
  {
    PmEpiFwd<T> epi;
    epi.bias = Wf(fc, U(fc).boff);
    epi.z = nullptr; epi.a = nullptr; epi.z32 = c->at<float>(lay.r_logits); epi.ld = ldc; epi.act = PM_ACT_NONE; epi.b_ = nullptr;
    launch_gemm<T>(c, B, ncls, C, TT(lay.r_pool), C, 1, Wf(fc, 0), C, 1, epi);
  }
  pm_xent_launch<T>(st, c->at<float>(lay.r_logits), (const int32_t*)y_dev, TT(lay.r_dlogits), B, ncls, ldc, c->hdr());
  prof_mark(c, 1);
  {
    pm_status qs = quiesce(c);
    if (qs != PM_OK) return qs;
  }
  // ---- backward
  if (!accumulate) {
    const unsigned bx = (unsigned)std::max<int64_t>(1, std::min<int64_t>(64, lay.zero_max / 4 / 256));
    hipLaunchKernelGGL(pm_zero_regions_kernel, dim3(bx, lay.n_zero), dim3(256), 0, st, g, c->at<int64_t>(lay.t_zero));
  }
  // Recomputation: on entering a segment (walking the units backwards) its convolutions run again in order with
  // the weights Wr, overwriting their outputs in place; a unit then sees rebuilt tensors where the producer sits in
  // its own segment and kept forward tensors where it sits in an earlier one (see launch_tfm).  The classifier is
  // not rebuilt; its pooled input is, when the last convolution shares its segment.
  auto seg_of = [&](int u) { return (U(u).d.stage - 1) / c->o.segment_size; };
  auto enter = [&](int u) {                 // called before the backward of unit u
    if (!lay.recompute || (u < L - 1 && seg_of(u) == seg_of(u + 1))) return;
    int lo = u;
    while (lo > 0 && seg_of(lo - 1) == seg_of(u)) --lo;
    for (int v = lo; v <= u; ++v)
      if (v < nconv) conv_fwd(v, Wr(v, 0));
    if (u == fc && lo <= nconv - 1) pm_pool_fwd_launch<T>(st, TT(lay.cv[nconv - 1].y), TT(lay.r_pool), B, HW, C);
  };
  enter(fc);
  {
    PmEpiBwdWeight ew{g + U(fc).off, C, accumulate, nullptr};
    launch_gemm<T>(c, ncls, C, B, TT(lay.r_dlogits), 1, ldc, PmWLoc<T>{TT(lay.r_pool), nullptr, 0}, 1, C, ew);
    launch_bias_grad<T>(st, TT(lay.r_dlogits), g + U(fc).off + U(fc).boff, B, ncls, ldc, accumulate);
    PmEpiBwdData<T> ed{nullptr, TT(lay.r_dpool), C, PM_ACT_NONE};
    launch_gemm<T>(c, B, C, ncls, TT(lay.r_dlogits), ldc, 1, Wb(fc, 0), 1, C, ed);
    const int64_t tot = (int64_t)B * HW * C;
    hipLaunchKernelGGL((pm_pool_bwd_kernel<T>), dim3((unsigned)std::min<int64_t>(2048, (tot + 255) / 256)), dim3(256), 0, st,
                       TT(lay.r_dpool), TT(lay.cv[nconv - 1].dy), B, HW, C);
  }
  for (int u = nconv - 1; u >= 0; --u) {
    enter(u);
    const Layout::ConvBuf& b = lay.cv[u];
    const int64_t nw = U(u).nw, tot = (int64_t)B * b.g.Ho * b.g.Wo * b.g.Cout;
    // the per-channel sums of the affine backward ride on the weight gradient's reduce launch when it has one
    PmReduceJob sums{nullptr, 0, 0, nullptr, 1};
    float* apart = pm_conv_wgrad_has_reduce<T>(b.g) ? c->at<float>(lay.r_ascratch) : nullptr;
    if (!pm_conv_affine_bwd_launch<T>(st, TT(b.dy), TT(b.y), TT(b.z), Wb(u, nw), TT(b.da), TT(b.dz), g + U(u).off + nw,
                                      g + U(u).off + nw + b.g.Cout, tot, b.g.Cout, apart, &sums))
      return fail(PM_EINVAL, "unit %d: channel count not supported", u);
    // the reduce that ends the weight gradient rides on the data gradient's launch (none for the first layer)
    PmReducePending pend{};
    ProfSpan span(c, PM_CLS_GEMM);      // weight gradient and data gradient of this convolution
    pm_conv_wgrad_launch<T>(st, b.g, TT(b.dz), input_of(u), g + U(u).off, accumulate, c->at<float>(lay.r_wscratch), sums,
                            u > 0 ? &pend : nullptr);
    if (u == 0) break;
    PmShortcutBwd<T> sb{nullptr, 0, 0, 0, 1};
    if ((u % 2) == 1) {                               // first convolution of a block: its input also feeds the shortcut
      const PmConvGeom& g2 = lay.cv[u + 1].g;
      sb = PmShortcutBwd<T>{TT(lay.cv[u + 1].da), g2.Ho, g2.Wo, g2.Cout, b.g.stride};
    }
    pm_conv_dgrad_launch<T>(st, b.g, TT(b.dz), Wb(u, 0), sb, TT(lay.cv[u - 1].dy), &pend);
  }
  PM_HIP(hipGetLastError());
  return PM_OK;
}

template <typename T>
pm_status enqueue_step(pm_ctx* c, const void* x, const void* y, bool first_micro, bool last_micro) {
  const int par = c->par();
  c->last_par = par;
  // The forward of step t reads versions <= t - 1 when every effective tau_fwd is >= 1, i.e. nothing
  // the still-running update of step t-1 (which writes version t) touches: that asynchrony of the
  // method is what lets the two overlap.  A zero delay (GPipe mode, synchronous warm-up) needs
  // version t itself, so then the forward waits.
  const bool fwd_independent = c->min_tau_f >= 1 && c->t_host >= c->o.sync_warmup_steps;
  if (!fwd_independent) {
    pm_status qs = quiesce(c);
    if (qs != PM_OK) return qs;
  }
  pm_status s = c->o.arch == PM_ARCH_TRANSFORMER ? launch_tfm<T>(c, x, y, first_micro ? 0 : 1, par)
                : c->o.arch == PM_ARCH_RESNET    ? launch_resnet<T>(c, x, y, first_micro ? 0 : 1, par)
                                                 : launch_fwd_bwd<T>(c, x, y, first_micro ? 0 : 1, par);
  if (s != PM_OK) return s;
  if (last_micro) {
    if (c->overlap && !c->prof_on) {
      PM_HIP(hipEventRecord(c->ev_bwd, c->stream));
      PM_HIP(hipStreamWaitEvent(c->stream_b, c->ev_bwd, 0));
      s = launch_update<T>(c, c->stream_b, par);
      PM_HIP(hipEventRecord(c->ev_upd, c->stream_b));
      c->upd_pending = true;
    } else {
      s = launch_update<T>(c, c->stream, par);
    }
    if (c->prof_on && c->prof_n < c->prof_cap) c->prof_n += 1;
  }
  return s;
}

pm_status enqueue_step_dt(pm_ctx* c, const void* x, const void* y, bool first_micro, bool last_micro) {
  return c->o.dtype == PM_BF16 ? enqueue_step<bf16_t>(c, x, y, first_micro, last_micro)
                               : enqueue_step<float>(c, x, y, first_micro, last_micro);
}

pm_status check_unit(pm_ctx* c, int32_t layer, size_t n) {
  if (!c) return fail(PM_EINVAL, "NULL context");
  if (layer < 0 || layer >= c->L) return fail(PM_EINVAL, "unit index %d outside 0..%d", layer, c->L - 1);
  const Unit& u = c->lay.units[layer];
  if ((int64_t)n != u.nw + u.nb) return fail(PM_EINVAL, "unit %d holds %lld values, caller said %zu", layer, (long long)(u.nw + u.nb), n);
  return PM_OK;
}

}  // namespace

namespace {
template <typename T>
pm_status linear_fwd_t(hipStream_t st, int M, int n_in, int n_out, const void* x, const void* W, const void* b, int act,
                       void* z, void* a) {
  PmEpiFwd<T> epi;
  epi.bias = PmWLoc<T>{(const T*)b, nullptr, 0};
  epi.z = (T*)z; epi.a = (T*)a; epi.z32 = nullptr; epi.ld = n_out; epi.act = act; epi.b_ = nullptr;
  launch_gemm_on<T>(st, M, n_out, n_in, (const T*)x, n_in, 1, PmWLoc<T>{(const T*)W, nullptr, 0}, n_in, 1, epi);
  PM_HIP(hipGetLastError());
  return PM_OK;
}
template <typename T>
pm_status linear_bwd_data_t(hipStream_t st, int M, int n_in, int n_out, const void* dz, const void* W, const void* zprev,
                            int act_prev, void* dzprev) {
  PmEpiBwdData<T> epi{(const T*)zprev, (T*)dzprev, n_in, act_prev};
  launch_gemm_on<T>(st, M, n_in, n_out, (const T*)dz, n_out, 1, PmWLoc<T>{(const T*)W, nullptr, 0}, 1, n_in, epi);
  PM_HIP(hipGetLastError());
  return PM_OK;
}
template <typename T>
pm_status linear_bwd_weight_t(hipStream_t st, int M, int n_in, int n_out, const void* dz, const void* a, float* dW,
                              float* db, int accumulate) {
  // the MFMA kernels produce the bias gradient themselves (column sums of the dz tile in LDS)
  // (for few rows; with many rows the column sums would sit on the critical path of the blocks
  // that own them, and a chunked reduction over the whole chip is faster)
  bool fused_db = false;
  if constexpr (sizeof(T) == 2) fused_db = M <= 512 && pm_mfma_takes(n_out, n_in, M, dz, 1, n_out, a, 0, 1, n_in);
  PmEpiBwdWeight epi{dW, n_in, accumulate, fused_db ? db : nullptr};
  launch_gemm_on<T>(st, n_out, n_in, M, (const T*)dz, 1, n_out, PmWLoc<T>{(const T*)a, nullptr, 0}, 1, n_in, epi);
  if (db && !fused_db) launch_bias_grad<T>(st, (const T*)dz, db, M, n_out, n_out, accumulate);
  PM_HIP(hipGetLastError());
  return PM_OK;
}
pm_status check_linear(int32_t dtype, int32_t M, int32_t n_in, int32_t n_out, int32_t act) {
  if (dtype != PM_F32 && dtype != PM_BF16) return fail(PM_EINVAL, "dtype must be PM_F32 or PM_BF16");
  if (M < 1 || n_in < 1 || n_out < 1) return fail(PM_EINVAL, "sizes must be positive");
  if (act < PM_ACT_NONE || act > PM_ACT_GELU) return fail(PM_EINVAL, "unknown activation");
  if (dtype == PM_BF16 && ((n_in | n_out) & 7)) return fail(PM_EINVAL, "bf16 primitives need n_in and n_out to be multiples of 8");
  return PM_OK;
}
}  // namespace

extern "C" {

const char* pm_status_str(pm_status s) {
  switch (s) {
    case PM_OK: return "PM_OK";
    case PM_EINVAL: return "PM_EINVAL";
    case PM_ENOMEM: return "PM_ENOMEM";
    case PM_EHIP: return "PM_EHIP";
    case PM_ESTATE: return "PM_ESTATE";
    case PM_EDIVERGED: return "PM_EDIVERGED";
  }
  return "PM_?";
}

const char* pm_last_error(void) { return g_err.c_str(); }

pm_status pm_delays(int32_t P, int32_t N, int32_t method, int32_t* tau_fwd, int32_t* tau_bkwd) {
  if (P < 1 || N < 1 || !tau_fwd || !tau_bkwd) return fail(PM_EINVAL, "P, N >= 1 and output arrays required");
  if (method < PM_METHOD_PIPEMARE || method > PM_METHOD_GPIPE) return fail(PM_EINVAL, "unknown method");
  for (int32_t i = 1; i <= P; ++i) {
    const int32_t num = 2 * (P - i) + 1;
    const int32_t tf = method == PM_METHOD_GPIPE ? 0 : (num + N - 1) / N;
    tau_fwd[i - 1] = tf;
    tau_bkwd[i - 1] = method == PM_METHOD_PIPEDREAM ? tf : 0;
  }
  return PM_OK;
}

pm_status pm_delay_thresholds(double mean, int32_t tau_max, uint32_t* thresholds) {
  if (tau_max < 0 || (tau_max > 0 && !thresholds)) return fail(PM_EINVAL, "tau_max >= 0 and an output array required");
  delay_thresholds(mean, tau_max, thresholds);
  return PM_OK;
}

pm_status pm_stochastic_delays(int32_t P, const int32_t* mean_tau, int32_t tau_max, uint64_t seed, int64_t t,
                               int32_t* tau_out) {
  if (P < 1 || !mean_tau || tau_max < 0 || t < 0 || !tau_out) return fail(PM_EINVAL, "P >= 1, tau_max >= 0, t >= 0 and arrays required");
  std::vector<uint32_t> T((size_t)std::max(tau_max, 1));
  for (int32_t i = 1; i <= P; ++i) {
    delay_thresholds((double)mean_tau[i - 1], tau_max, T.data());
    tau_out[i - 1] = pm_delay_from_u32(pm_counter_u32(seed, t, i, P), T.data(), tau_max);
  }
  return PM_OK;
}

pm_status pm_recompute_delays(int32_t P, int32_t S, int32_t N, const int32_t* tau_bkwd, int32_t* tau_recomp) {
  if (P < 1 || S < 1 || N < 1 || !tau_recomp) return fail(PM_EINVAL, "P, S, N >= 1 and an output array required");
  for (int32_t i = 1; i <= P; ++i) {
    const int32_t first = ((i - 1) / S) * S + 1;                 // first stage of i's segment
    const int32_t size = std::min(S, P - first + 1);             // stages in that segment
    const int32_t j = i - first + 1;                             // i's position in it
    tau_recomp[i - 1] = (tau_bkwd ? tau_bkwd[i - 1] : 0) + (2 * (size - j) + N - 1) / N;
  }
  return PM_OK;
}

pm_status pm_slots(int32_t tau_fwd, int32_t tau_bkwd, int64_t t, int32_t* fwd_slot, int32_t* bkwd_slot,
                   int32_t* write_slot) {
  if (tau_fwd < 0 || tau_bkwd < 0 || tau_bkwd > tau_fwd || t < 0) return fail(PM_EINVAL, "need 0 <= tau_bkwd <= tau_fwd and t >= 0");
  const int64_t R = (int64_t)tau_fwd + 1;
  const int64_t vf = t - tau_fwd > 0 ? t - tau_fwd : 0;
  const int64_t vb = t - tau_bkwd > 0 ? t - tau_bkwd : 0;
  if (fwd_slot) *fwd_slot = (int32_t)(vf % R);
  if (bkwd_slot) *bkwd_slot = (int32_t)(vb % R);
  if (write_slot) *write_slot = (int32_t)((t + 1) % R);
  return PM_OK;
}

pm_status pm_t1_lr(const pm_lr_sched* s, int32_t tau, int64_t k, int32_t t1_enabled, double* lr) {
  if (!s || !lr || k < 0 || tau < 0) return fail(PM_EINVAL, "bad argument");
  double a;
  switch (s->kind) {
    case PM_LR_CONST: a = s->base; break;
    case PM_LR_STEP:
      if (s->interval < 1) return fail(PM_EINVAL, "interval must be >= 1");
      a = s->base * std::pow(s->factor, (double)(k / s->interval));
      break;
    case PM_LR_WARMUP_INVSQRT:
      if (s->interval < 1) return fail(PM_EINVAL, "warmup length must be >= 1");
      if (k < s->interval) a = s->init + (s->base - s->init) * ((double)k / (double)s->interval);
      else a = s->base * std::sqrt((double)s->interval / (double)k);
      break;
    default: return fail(PM_EINVAL, "unknown schedule kind");
  }
  double p = 0.0;
  if (s->K > 0) p = 1.0 - std::fmin((double)k / (double)s->K, 1.0);
  if (t1_enabled && p > 0.0) a /= std::pow((double)(tau > 1 ? tau : 1), p);
  *lr = a;
  return PM_OK;
}

pm_status pm_query_bytes(int32_t P, int32_t L, const pm_layer_desc* layers, const int32_t* tau_fwd,
                         const pm_opts* opts, size_t* out_bytes) {
  if (!out_bytes) return fail(PM_EINVAL, "out_bytes is NULL");
  pm_status s = validate(P, L, layers, tau_fwd, nullptr, opts);
  if (s != PM_OK) return s;
  Layout lay;
  make_layout(L, layers, tau_fwd, nullptr, opts, lay);
  *out_bytes = lay.total;
  return PM_OK;
}

pm_status pm_create(int32_t P, int32_t L, const pm_layer_desc* layers, const int32_t* tau_fwd,
                    const int32_t* tau_bkwd, const pm_lr_sched* sched, const pm_opts* opts,
                    const float* const* init_weights_host, void* device_arena, size_t arena_bytes,
                    void* hip_stream, pm_ctx** out) {
  if (!out) return fail(PM_EINVAL, "out is NULL");
  *out = nullptr;
  if (!tau_bkwd || !sched || !init_weights_host || !device_arena) return fail(PM_EINVAL, "NULL argument");
  pm_status s = validate(P, L, layers, tau_fwd, tau_bkwd, opts);
  if (s != PM_OK) return s;
  if (layers[L - 1].act != PM_ACT_NONE) return fail(PM_EINVAL, "the last unit feeds the loss and must have no activation");
  if (sched->kind < PM_LR_CONST || sched->kind > PM_LR_WARMUP_INVSQRT) return fail(PM_EINVAL, "unknown schedule kind");
  if (sched->kind != PM_LR_CONST && sched->interval < 1) return fail(PM_EINVAL, "schedule interval must be >= 1");
  if (sched->K < 0) return fail(PM_EINVAL, "K must be >= 0");
  if (((uintptr_t)device_arena) % PM_ALIGN) return fail(PM_EINVAL, "arena must be %d-byte aligned", PM_ALIGN);
  for (int l = 0; l < L; ++l)
    if (!init_weights_host[l]) return fail(PM_EINVAL, "init_weights_host[%d] is NULL", l);
  if (L > 65535) return fail(PM_EINVAL, "too many units");
  if (opts->use_graph && !hip_stream) return fail(PM_EINVAL, "use_graph needs a stream of its own: the default stream cannot be captured");

  pm_ctx* c = new pm_ctx();
  c->P = P;
  c->L = L;
  c->o = *opts;
  c->sched = *sched;
  if (opts->gamma_override) {
    c->gamma_override.assign(opts->gamma_override, opts->gamma_override + P);
    c->o.gamma_override = c->gamma_override.data();
  }
  c->tau_f.assign(tau_fwd, tau_fwd + P);
  c->tau_b.assign(tau_bkwd, tau_bkwd + P);
  if (opts->tau_recomp) {
    c->tau_r.assign(opts->tau_recomp, opts->tau_recomp + P);
    c->o.tau_recomp = c->tau_r.data();
  }
  make_layout(L, layers, tau_fwd, tau_bkwd, &c->o, c->lay);
  const Layout& lay = c->lay;
  if (arena_bytes < lay.total) {
    delete c;
    return fail(PM_ENOMEM, "arena has %zu bytes, %zu needed", arena_bytes, lay.total);
  }
  c->arena = (char*)device_arena;
  c->stream = (hipStream_t)hip_stream;
  c->min_tau_f = opts->stochastic_delays ? 0 : *std::min_element(c->tau_f.begin(), c->tau_f.end());   // a drawn delay can be 0
  c->overlap = opts->overlap_update != 0 && opts->use_graph == 0;
  if (c->overlap) {
    // host-side objects only; default priority
    if (hipStreamCreateWithFlags(&c->stream_b, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_bwd, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_upd, hipEventDisableTiming) != hipSuccess) {
      if (c->ev_bwd) (void)hipEventDestroy(c->ev_bwd);
      if (c->stream_b) (void)hipStreamDestroy(c->stream_b);
      delete c;
      return fail(PM_EHIP, "could not create the second stream for overlap_update");
    }
  }

  // host images of the static tables and the packed initial weights
  std::vector<float> w0((size_t)lay.n_flat, 0.f);
  std::vector<int32_t> chunk_layer((size_t)lay.n_chunks);
  std::vector<PmLayerStatic> ls(L);
  for (int l = 0; l < L; ++l) {
    const Unit& u = lay.units[l];
    std::memcpy(&w0[u.off], init_weights_host[l], sizeof(float) * u.nw);
    if (u.nb) std::memcpy(&w0[u.off + u.boff], init_weights_host[l] + u.nw, sizeof(float) * u.nb);
    for (int64_t ch = u.off / PM_CHUNK; ch < (u.off + u.n_pad) / PM_CHUNK; ++ch) chunk_layer[ch] = l;
    PmLayerStatic& S = ls[l];
    S.off = u.off; S.n_pad = u.n_pad; S.ring_off = u.ring_off; S.R = u.R; S.tau_f = u.tau_f; S.tau_b = u.tau_b;
    S.stage = u.d.stage; S.gamma = (float)u.gamma; S.corr = (float)u.corr;
    S.tau_r = u.tau_r; S.corr_r = (float)u.corr_r;
  }
  hipStream_t st = c->stream;
  auto bail = [&](hipError_t e, const char* what) {
    delete c;
    return fail(PM_EHIP, "%s: %s", what, hipGetErrorString(e));
  };
  hipError_t e;
  // zero everything except the ring (which the init kernel fills): optimizer state, delta, grads,
  // tables, header, activations (their pad columns must stay zero)
  if ((e = hipMemsetAsync(c->arena + lay.g_off, 0, lay.ub_off - lay.g_off, st)) != hipSuccess) return bail(e, "memset state");
  if ((e = hipMemsetAsync(c->arena + lay.chunk_off, 0, lay.total - lay.chunk_off, st)) != hipSuccess) return bail(e, "memset tables");
  if ((e = hipMemcpyAsync(c->arena + lay.w_off, w0.data(), w0.size() * 4, hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy weights");
  if ((e = hipMemcpyAsync(c->arena + lay.chunk_off, chunk_layer.data(), chunk_layer.size() * 4, hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy chunk table");
  if ((e = hipMemcpyAsync(c->arena + lay.ls_off, ls.data(), ls.size() * sizeof(PmLayerStatic), hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy unit table");
  std::vector<uint32_t> cdf;
  if (c->o.stochastic_delays && c->o.tau_max > 0) {
    cdf.resize((size_t)P * c->o.tau_max);
    for (int i = 0; i < P; ++i) delay_thresholds((double)tau_fwd[i], c->o.tau_max, &cdf[(size_t)i * c->o.tau_max]);
    if ((e = hipMemcpyAsync(c->arena + lay.cdf_off, cdf.data(), cdf.size() * 4, hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy delay table");
  }
  std::vector<PmGemmProb<PmEpiBwdWeight>> probs;
  std::vector<float> pos;
  std::vector<int64_t> zero_tab;
  if (c->o.arch == PM_ARCH_TRANSFORMER) {
    // fixed sinusoidal positions pos[s, 2i] = sin(s / 10000^(2i/d)), pos[s, 2i+1] = cos(same)
    const int S = c->o.seq_len, d = lay.units[0].d.n_out;
    pos.resize((size_t)S * d);
    for (int sidx = 0; sidx < S; ++sidx)
      for (int j = 0; j < d; ++j) {
        const double ang = (double)sidx / std::pow(10000.0, (double)(j & ~1) / (double)d);
        pos[(size_t)sidx * d + j] = (float)((j & 1) ? std::cos(ang) : std::sin(ang));
      }
    for (int l = 0; l < L; ++l)
      if (lay.units[l].d.kind != PM_LINEAR) { zero_tab.push_back(lay.units[l].off); zero_tab.push_back(lay.units[l].n_pad); }
    if ((e = hipMemcpyAsync(c->arena + lay.t_pos, pos.data(), pos.size() * 4, hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy positions");
    if ((e = hipMemcpyAsync(c->arena + lay.t_zero, zero_tab.data(), zero_tab.size() * 8, hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy region table");
    if (c->o.dtype == PM_BF16) {
      // grouped weight-gradient launch: one problem per Linear unit, largest first
      const int nl = (L - 3) / 8, Tk = c->o.microbatch * S, V = lay.units[0].d.n_in;
      const int ldV = (int)round_up(V, 8);
      float* g = c->at<float>(lay.g_off);
      struct WP { int u; const bf16_t* dz; int ld_dz; const bf16_t* a_in; };
      std::vector<WP> wp;
      wp.push_back({L - 1, c->at<bf16_t>(lay.t_dlogits), ldV, c->at<bf16_t>(lay.t_nf)});
      for (int l = 0; l < nl; ++l) {
        const Layout::TfmLayer& b = lay.tl[l];
        const int u = 1 + 8 * l;
        wp.push_back({u + 1, c->at<bf16_t>(b.dzq), d, c->at<bf16_t>(b.n1)});
        wp.push_back({u + 2, c->at<bf16_t>(b.dzk), d, c->at<bf16_t>(b.n1)});
        wp.push_back({u + 3, c->at<bf16_t>(b.dzv), d, c->at<bf16_t>(b.n1)});
        wp.push_back({u + 4, c->at<bf16_t>(b.dzo), d, c->at<bf16_t>(b.o)});
        wp.push_back({u + 6, c->at<bf16_t>(b.dz1), lay.units[u + 6].d.n_out, c->at<bf16_t>(b.n2)});
        wp.push_back({u + 7, c->at<bf16_t>(b.dz2), d, c->at<bf16_t>(b.f)});
      }
      // 256 x 256 block tiles (half the LDS traffic per MFMA) when every problem is a whole number of
      // them and there are enough to balance 256 compute units; else 128 x 128
      int TB = 256;
      {
        int64_t t256 = 0;
        for (const WP& w : wp) {
          const pm_layer_desc& dd = lay.units[w.u].d;
          if (!pm_big_aligned<PmBig256>(dd.n_out, dd.n_in, Tk)) TB = 128;
          t256 += (int64_t)((dd.n_out + 255) / 256) * ((dd.n_in + 255) / 256);
        }
        if (t256 < 256) TB = 128;
      }
      auto tiles_of = [&](const WP& w) {
        const pm_layer_desc& dd = lay.units[w.u].d;
        return (int64_t)((dd.n_out + TB - 1) / TB) * ((dd.n_in + TB - 1) / TB);
      };
      std::stable_sort(wp.begin(), wp.end(), [&](const WP& a, const WP& b) { return tiles_of(a) > tiles_of(b); });
      const int np = (int)wp.size();
      probs.resize((size_t)2 * np);
      bool fits = true, aligned = true;
      for (int i = 0; i < np; ++i) {
        const Unit& u = lay.units[wp[i].u];
        fits = fits && pm_mfma_fits(u.d.n_out, u.d.n_in, Tk, wp[i].dz, 1, wp[i].ld_dz, wp[i].a_in, 0, 1, u.d.n_in);
        aligned = aligned && pm_big_aligned<PmBig128>(u.d.n_out, u.d.n_in, Tk);
        for (int acc = 0; acc < 2; ++acc) {
          PmGemmProb<PmEpiBwdWeight>& pr = probs[(size_t)acc * np + i];
          pr.I = u.d.n_out; pr.J = u.d.n_in; pr.K = Tk;
          pr.A = wp[i].dz; pr.lda = wp[i].ld_dz;
          pr.B = PmWLoc<bf16_t>{wp[i].a_in, nullptr, 0}; pr.ldb = u.d.n_in;
          pr.epi = PmEpiBwdWeight{g + u.off, u.d.n_in, acc, g + u.off + u.boff};
        }
      }
      // Work lists per XCD (largest problems first, each to the least loaded XCD).  A problem with more
      // than 1/8 of all tiles is cut into ranges of whole 8-row tile panels spread over all XCDs.
      int64_t total_tiles = 0;
      for (int i = 0; i < np; ++i) total_tiles += tiles_of(wp[i]);
      const int max_segs = np + 8;
      std::vector<PmXcdSeg> segs((size_t)8 * max_segs, PmXcdSeg{0, 0, INT32_MAX, 0});
      int32_t load[8] = {0, 0, 0, 0, 0, 0, 0, 0}, nseg[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      auto push = [&](int x, int prob, int tile0, int count) {
        segs[(size_t)x * max_segs + nseg[x]] = PmXcdSeg{prob, tile0, load[x], 0};
        nseg[x] += 1;
        load[x] += count;
      };
      for (int i = 0; i < np; ++i) {
        const pm_layer_desc& dd = lay.units[wp[i].u].d;
        const int ti = (dd.n_out + TB - 1) / TB, tj = (dd.n_in + TB - 1) / TB;
        if ((int64_t)ti * tj * 8 > total_tiles && ti >= 16) {
          const int panels = (ti + 7) / 8;                       // panels of 8 tile rows (the body's walking order)
          int p0 = 0;
          for (int x = 0; x < 8; ++x) {
            const int p1 = (int)((int64_t)panels * (x + 1) / 8);
            if (p1 > p0) {
              const int r0 = p0 * 8, r1 = std::min(p1 * 8, ti);
              push(x, i, r0 * tj, (r1 - r0) * tj);
            }
            p0 = p1;
          }
        } else {
          int best = 0;
          for (int x = 1; x < 8; ++x)
            if (load[x] < load[best]) best = x;
          push(best, i, 0, ti * tj);
        }
      }
      const int32_t longest = *std::max_element(load, load + 8);
      c->dw_grouped = fits && !lay.recompute;   // a recomputing backward needs each weight gradient at its unit's turn
      c->dw_aligned = aligned;
      c->dw_tile = TB;
      c->dw_nprob = np;
      c->dw_ntiles = longest * 8;
      c->dw_max_segs = max_segs;
      if ((e = hipMemcpyAsync(c->arena + lay.t_wprobs, probs.data(), probs.size() * sizeof(probs[0]), hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy problem table");
      if ((e = hipMemcpyAsync(c->arena + lay.t_wtiles, load, sizeof load, hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy tile table");
      if ((e = hipMemcpyAsync(c->arena + lay.t_wsegs, segs.data(), segs.size() * sizeof(PmXcdSeg), hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy segment table");
      // The update inside the weight-gradient epilogue: possible when the gradient a tile holds is final (one
      // microbatch per step, no clipping by the global norm) and the grouped launch runs last with whole tiles.
      std::vector<PmGemmProb<PmEpiBwdWeightUpd>> fprobs;
      std::vector<int32_t> ublocks;
      const bool nontemporal = (size_t)lay.n_flat * 32 > ((size_t)1 << 30);          // as in launch_update
      // (measured: 15.0 -> 14.9 ms per step on the 12-layer workload, whose 8.6 GB of state leave the caches between
      // steps; 1.99 against 1.99 - 2.01 ms on the 6-layer one, whose pass is cache assisted: hence the default)
      const bool in_launch = c->o.update_placement == 2 || (c->o.update_placement == 0 && nontemporal);
      if (in_launch && c->dw_grouped && aligned && c->o.n_microbatches == 1 && c->o.clip_norm <= 0.0 &&
          !c->overlap && !lay.has_ur) {
        const int per_block = nontemporal ? PmAcc<2>::PER_BLOCK : PmAcc<1>::PER_BLOCK;
        std::vector<char> fused((size_t)(lay.n_flat / per_block), 0);
        fprobs.resize(np);
        for (int i = 0; i < np; ++i) {
          const Unit& u = lay.units[wp[i].u];
          const PmGemmProb<PmEpiBwdWeight>& p0 = probs[i];
          PmGemmProb<PmEpiBwdWeightUpd>& pr = fprobs[i];
          pr.I = p0.I; pr.J = p0.J; pr.K = p0.K; pr.A = p0.A; pr.lda = p0.lda; pr.B = p0.B; pr.ldb = p0.ldb;
          PmEpiBwdWeightUpd& ep = pr.epi;
          std::memset(&ep, 0, sizeof ep);
          ep.g = p0.epi.g; ep.ld = p0.epi.ld; ep.db = p0.epi.db;
          ep.f.w = c->at<float>(lay.w_off) + u.off;
          ep.f.v = c->at<float>(lay.v_off) + u.off;
          ep.f.s = c->at<float>(lay.s_off) + u.off;
          ep.f.d = c->at<float>(lay.d_off) + u.off;
          ep.f.ring = c->at<bf16_t>(lay.ring_off) + u.ring_off;
          ep.f.ub = c->at<bf16_t>(lay.ub_off) + u.off;
          ep.f.step = c->ld(0) + wp[i].u;
          ep.f.hdr = c->hdr();
          ep.f.n_pad = u.n_pad;
          ep.f.gamma = (float)u.gamma; ep.f.beta1 = (float)c->o.beta1; ep.f.beta2 = (float)c->o.beta2;
          ep.f.eps = (float)c->o.eps; ep.f.wd = (float)c->o.weight_decay;
          ep.f.opt = c->o.opt == PM_OPT_SGDM ? 0 : 1;
          ep.f.has_ub = u.corr != 0.0 ? 1 : 0;
          ep.f.tau_b = u.tau_b;
          // whole update blocks inside the matrix belong to the epilogue; the matrix is a whole number of tiles,
          // hence of blocks (128 x 128 elements per tile at least)
          const int64_t nw = (int64_t)u.d.n_out * u.d.n_in;
          for (int64_t b = u.off / per_block; b < (u.off + nw) / per_block; ++b) fused[(size_t)b] = 1;
          c->upd_fused_params += nw;
        }
        for (size_t b = 0; b < fused.size(); ++b)
          if (!fused[b]) ublocks.push_back((int32_t)b);
        c->fuse_upd = true;
        c->upd_nblocks = (int)ublocks.size();
        if ((e = hipMemcpyAsync(c->arena + lay.t_fuse, fprobs.data(), fprobs.size() * sizeof(fprobs[0]), hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy fused problem table");
        if (!ublocks.empty() && (e = hipMemcpyAsync(c->arena + lay.t_ublocks, ublocks.data(), ublocks.size() * 4, hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy block list");
      }
      if ((e = hipStreamSynchronize(st)) != hipSuccess) return bail(e, "synchronise after tables");   // host tables go out of scope
      probs.clear();
    }
  }
  if (c->o.arch == PM_ARCH_RESNET) {
    for (int l = 0; l < L - 1; ++l) { zero_tab.push_back(lay.units[l].off); zero_tab.push_back(lay.units[l].n_pad); }
    if ((e = hipMemcpyAsync(c->arena + lay.t_zero, zero_tab.data(), zero_tab.size() * 8, hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy region table");
  }
  if (c->o.dtype == PM_BF16 && c->o.arch == PM_ARCH_CHAIN) {
    // weight-gradient problem tables (first microbatch: overwrite, later ones: accumulate)
    const int M = c->o.microbatch;
    float* g = c->at<float>(lay.g_off);
    bool fits = true;
    probs.resize((size_t)2 * L);
    for (int acc = 0; acc < 2; ++acc)
      for (int l = 0; l < L; ++l) {
        const Unit& u = lay.units[l];
        const bf16_t* a_in = l == 0 ? c->at<bf16_t>(lay.x_off) : c->at<bf16_t>(lay.units[l - 1].a_off);
        const bf16_t* dz = c->at<bf16_t>(u.dz_off);
        fits = fits && pm_mfma_fits(u.d.n_out, u.d.n_in, M, dz, 1, u.ld_out, a_in, 0, 1, u.ld_in);
        PmGemmProb<PmEpiBwdWeight>& pr = probs[(size_t)acc * L + l];
        pr.I = u.d.n_out; pr.J = u.d.n_in; pr.K = M;
        pr.A = dz; pr.lda = u.ld_out;
        pr.B = PmWLoc<bf16_t>{a_in, nullptr, 0}; pr.ldb = u.ld_in;
        pr.epi = PmEpiBwdWeight{g + u.off, u.d.n_in, acc, g + u.off + u.boff};
        c->dw_maxI = std::max(c->dw_maxI, (int)u.d.n_out);
        c->dw_maxJ = std::max(c->dw_maxJ, (int)u.d.n_in);
      }
    c->dw_grouped = fits;
    if ((e = hipMemcpyAsync(c->arena + lay.probs_off, probs.data(), probs.size() * sizeof(probs[0]), hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy problem table");
    // chained launches (see pm_chain.hpp): few rows, no recomputation, one step-table set
    std::vector<PmChainFwd> cf;
    std::vector<PmChainBwd> cb;
    if (c->o.chained_launches && M % 32 == 0 && M <= 32 * PM_CHAIN_MAX_ROW_TILES && !lay.recompute && !c->overlap) {
      bf16_t* ring = c->at<bf16_t>(lay.ring_off);
      bf16_t* ub = c->at<bf16_t>(lay.ub_off);
      const PmLayerStep* tab = c->ld(0);
      int nf = 0;
      while (nf < L - 1 && nf < PM_CHAIN_MAX_UNITS && lay.units[nf].d.n_in % 64 == 0 && lay.units[nf].d.n_out % 32 == 0) ++nf;   // (the last unit writes fp32 logits for the loss: not chained)
      int hb = 0;
      while (hb + 1 < L && hb < PM_CHAIN_MAX_UNITS && lay.units[hb + 1].d.n_out % 64 == 0 && lay.units[hb + 1].d.n_in % 32 == 0) ++hb;
      int max_tiles = 0;
      for (int l = 0; l < nf; ++l) {
        const Unit& u = lay.units[l];
        PmChainFwd f;
        f.W = PmWLoc<bf16_t>{ring + u.ring_off, &tab[l].fwd_slot, u.n_pad};
        f.boff = u.boff;
        f.in = l == 0 ? c->at<bf16_t>(lay.x_off) : c->at<bf16_t>(lay.units[l - 1].a_off);
        f.z = c->at<bf16_t>(u.z_off);
        f.a = c->at<bf16_t>(u.a_off);
        f.n_in = u.d.n_in; f.n_out = u.d.n_out; f.act = u.d.act;
        f.in_shared = l > 0;
        cf.push_back(f);
        max_tiles = std::max(max_tiles, (M / 32) * (u.d.n_out / 32));
      }
      for (int l = hb; l >= 1; --l) {
        const Unit& u = lay.units[l];
        const Unit& up = lay.units[l - 1];
        PmChainBwd b;
        b.W = u.corr ? PmWLoc<bf16_t>{ub + u.off, nullptr, 0} : PmWLoc<bf16_t>{ring + u.ring_off, &tab[l].bkwd_slot, u.n_pad};
        b.dz = c->at<bf16_t>(u.dz_off);
        b.zprev = c->at<bf16_t>(up.z_off);
        b.dzprev = c->at<bf16_t>(up.dz_off);
        b.n_in = u.d.n_in; b.n_out = u.d.n_out; b.act_prev = up.d.act;
        b.dz_shared = l < hb;
        cb.push_back(b);
        max_tiles = std::max(max_tiles, (M / 32) * (u.d.n_in / 32));
      }
      int cus = 0, dev = 0;
      if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
      if (cus >= 8 && (nf >= 2 || hb >= 2)) {
        c->chain_nf = nf >= 2 ? nf : 0;
        c->chain_hb = hb >= 2 ? hb : 0;
        // one block per compute unit at most (all blocks must be resident: they wait for each other)
        c->chain_grid = std::max(8, std::min(cus / 8 * 8, (max_tiles + 7) / 8 * 8));
        const Unit& ul = lay.units[L - 1];
        c->chain_fill16 = (int64_t)((ul.dz_off + (size_t)M * ul.ld_out * lay.esz - lay.units[0].z_off + 15) / 16);
        if (!cf.empty() && (e = hipMemcpyAsync(c->arena + lay.chain_f_off, cf.data(), cf.size() * sizeof(cf[0]), hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy chain table");
        if (!cb.empty() && (e = hipMemcpyAsync(c->arena + lay.chain_b_off, cb.data(), cb.size() * sizeof(cb[0]), hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "copy chain table");
        if ((e = hipStreamSynchronize(st)) != hipSuccess) return bail(e, "synchronise after chain tables");
      }
    }
  }
  if (c->o.dtype == PM_BF16)
    hipLaunchKernelGGL((pm_init_ring_kernel<bf16_t>), dim3((unsigned)lay.n_chunks), dim3(256), 0, st,
                       c->at<float>(lay.w_off), c->at<bf16_t>(lay.ring_off), c->at<bf16_t>(lay.ub_off),
                       lay.has_ur ? c->at<bf16_t>(lay.ur_off) : nullptr,
                       c->at<int32_t>(lay.chunk_off), c->ls());
  else
    hipLaunchKernelGGL((pm_init_ring_kernel<float>), dim3((unsigned)lay.n_chunks), dim3(256), 0, st,
                       c->at<float>(lay.w_off), c->at<float>(lay.ring_off), c->at<float>(lay.ub_off),
                       lay.has_ur ? c->at<float>(lay.ur_off) : nullptr,
                       c->at<int32_t>(lay.chunk_off), c->ls());
  if ((e = hipGetLastError()) != hipSuccess) return bail(e, "init kernel");
  if ((e = hipStreamSynchronize(st)) != hipSuccess) return bail(e, "synchronise after init");   // host images go out of scope
  *out = c;
  return PM_OK;
}

pm_status pm_step(pm_ctx* c, const void* x_dev, const void* y_dev, float* loss_out_host) {
  if (!c || !x_dev || !y_dev) return fail(PM_EINVAL, "NULL argument");
  if (c->diverged) return fail(PM_EDIVERGED, "a non-finite weight was produced at an earlier step");
  const bool first = c->micro == 0;
  const bool last = c->micro + 1 == c->o.n_microbatches;
  pm_status s = PM_OK;
  if (c->o.use_graph && c->o.n_microbatches == 1 && !c->prof_on) {
    // All slot and step-size values are read from the device table inside the kernels, so one graph
    // serves every step that uses the same batch buffers; a caller cycling through a few resident
    // batches gets one graph per buffer pair.
    hipGraphExec_t exec = nullptr;
    for (const pm_ctx::StepGraph& sg : c->graphs)
      if (sg.x == x_dev && sg.y == y_dev) exec = sg.exec;
    if (!exec) {
      if (c->graphs.size() >= PM_MAX_GRAPHS) {
        (void)hipGraphExecDestroy(c->graphs.front().exec);
        (void)hipGraphDestroy(c->graphs.front().graph);
        c->graphs.erase(c->graphs.begin());
      }
      hipGraph_t graph = nullptr;
      PM_HIP(hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
      s = enqueue_step_dt(c, x_dev, y_dev, true, true);
      hipError_t e = hipStreamEndCapture(c->stream, &graph);
      if (s != PM_OK) {
        if (graph) (void)hipGraphDestroy(graph);
        return s;
      }
      if (e != hipSuccess) return fail(PM_EHIP, "hipStreamEndCapture: %s", hipGetErrorString(e));
      e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
      if (e != hipSuccess) {
        (void)hipGraphDestroy(graph);
        return fail(PM_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e));
      }
      c->graphs.push_back(pm_ctx::StepGraph{x_dev, y_dev, graph, exec});
    }
    PM_HIP(hipGraphLaunch(exec, c->stream));
  } else {
    s = enqueue_step_dt(c, x_dev, y_dev, first, last);
    if (s != PM_OK) return s;
  }
  if (last) { c->micro = 0; c->t_host += 1; } else c->micro += 1;
  if (loss_out_host) {
    PmStepHdr h;
    PM_HIP(hipMemcpyAsync(&h, c->hdr(), sizeof h, hipMemcpyDeviceToHost, c->stream));
    PM_HIP(hipStreamSynchronize(c->stream));
    *loss_out_host = c->last_loss = h.loss;
    if (h.chain_err) return fail(PM_EHIP, "a chained launch gave up waiting for its producers (results of this context are invalid)");
    if (h.diverged) { c->diverged = true; return fail(PM_EDIVERGED, "non-finite weight after step %lld", (long long)h.t_used); }
  }
  return PM_OK;
}

pm_status pm_weights(pm_ctx* c, int32_t layer, float* dst_host, size_t n) { return pm_state(c, 0, layer, dst_host, n); }

pm_status pm_state(pm_ctx* c, int32_t which, int32_t layer, float* dst, size_t n) {
  pm_status s = check_unit(c, layer, n);
  if (s != PM_OK) return s;
  if (!dst) return fail(PM_EINVAL, "dst is NULL");
  if ((s = quiesce(c)) != PM_OK) return s;
  const Layout& lay = c->lay;
  const Unit& u = lay.units[layer];
  size_t base;
  switch (which) {
    case 0: base = lay.w_off; break;
    case 1: base = lay.d_off; break;
    case 2: base = lay.v_off; break;
    case 3: base = lay.ub_off; break;
    case 4: base = lay.g_off; break;
    case 5:
      if (!lay.has_ur) return fail(PM_ESTATE, "this context keeps no corrected recompute weights");
      base = lay.ur_off;
      break;
    default: return fail(PM_EINVAL, "unknown state selector %d", which);
  }
  if ((which == 3 || which == 5) && c->o.dtype == PM_BF16) {
    std::vector<bf16_t> tmp((size_t)u.n);
    PM_HIP(hipMemcpyAsync(tmp.data(), c->at<bf16_t>(base) + u.off, tmp.size() * 2, hipMemcpyDeviceToHost, c->stream));
    PM_HIP(hipStreamSynchronize(c->stream));
    auto widen = [](bf16_t h) { uint32_t b = (uint32_t)h << 16; float f; std::memcpy(&f, &b, 4); return f; };
    for (int64_t i = 0; i < u.nw; ++i) dst[i] = widen(tmp[i]);
    for (int64_t i = 0; i < u.nb; ++i) dst[u.nw + i] = widen(tmp[u.boff + i]);
    return PM_OK;
  }
  const float* src = c->at<float>(base) + u.off;
  PM_HIP(hipMemcpyAsync(dst, src, sizeof(float) * u.nw, hipMemcpyDeviceToHost, c->stream));
  if (u.nb) PM_HIP(hipMemcpyAsync(dst + u.nw, src + u.boff, sizeof(float) * u.nb, hipMemcpyDeviceToHost, c->stream));
  PM_HIP(hipStreamSynchronize(c->stream));
  return PM_OK;
}

pm_status pm_device_step_table(pm_ctx* c, int64_t* t_used, int32_t* fwd_slot, int32_t* bkwd_slot,
                               int32_t* write_slot, float* lr) {
  if (!c) return fail(PM_EINVAL, "NULL context");
  pm_status qs = quiesce(c);
  if (qs != PM_OK) return qs;
  std::vector<PmLayerStep> ld(c->L);
  PmStepHdr h;
  PM_HIP(hipMemcpyAsync(ld.data(), c->ld(c->last_par), sizeof(PmLayerStep) * c->L, hipMemcpyDeviceToHost, c->stream));
  PM_HIP(hipMemcpyAsync(&h, c->hdr(), sizeof h, hipMemcpyDeviceToHost, c->stream));
  PM_HIP(hipStreamSynchronize(c->stream));
  if (t_used) *t_used = h.t_used;
  for (int l = 0; l < c->L; ++l) {
    if (fwd_slot) fwd_slot[l] = ld[l].fwd_slot;
    if (bkwd_slot) bkwd_slot[l] = ld[l].bkwd_slot;
    if (write_slot) write_slot[l] = ld[l].write_slot;
    if (lr) lr[l] = ld[l].lr;
  }
  return PM_OK;
}

pm_status pm_device_recompute_slots(pm_ctx* c, int64_t* t_used, int32_t* rec_slot) {
  if (!c) return fail(PM_EINVAL, "NULL context");
  if (!c->lay.recompute) return fail(PM_ESTATE, "this context does not recompute");
  pm_status qs = quiesce(c);
  if (qs != PM_OK) return qs;
  std::vector<PmLayerStep> ld(c->L);
  PmStepHdr h;
  PM_HIP(hipMemcpyAsync(ld.data(), c->ld(c->last_par), sizeof(PmLayerStep) * c->L, hipMemcpyDeviceToHost, c->stream));
  PM_HIP(hipMemcpyAsync(&h, c->hdr(), sizeof h, hipMemcpyDeviceToHost, c->stream));
  PM_HIP(hipStreamSynchronize(c->stream));
  if (t_used) *t_used = h.t_used;
  if (rec_slot)
    for (int l = 0; l < c->L; ++l) rec_slot[l] = ld[l].rec_slot;
  return PM_OK;
}

pm_status pm_chained_units(pm_ctx* c, int32_t* n_forward, int32_t* n_backward) {
  if (!c) return fail(PM_EINVAL, "NULL context");
  const bool on = c->o.dtype == PM_BF16 && c->chain_grid > 0;
  if (n_forward) *n_forward = on ? c->chain_nf : 0;
  if (n_backward) *n_backward = on ? c->chain_hb : 0;
  return PM_OK;
}

pm_status pm_update_split(pm_ctx* c, int64_t* n_epilogue, int64_t* n_pass) {
  if (!c) return fail(PM_EINVAL, "NULL context");
  if (n_epilogue) *n_epilogue = c->fuse_upd ? c->upd_fused_params : 0;
  if (n_pass) *n_pass = c->fuse_upd ? c->lay.n_flat - c->upd_fused_params : c->lay.n_flat;
  return PM_OK;
}

pm_status pm_stats(pm_ctx* c, double* loss, double* grad_norm, double* param_norm, int64_t* t) {
  if (!c) return fail(PM_EINVAL, "NULL context");
  pm_status qs = quiesce(c);
  if (qs != PM_OK) return qs;
  const Layout& lay = c->lay;
  if (param_norm) {
    PM_HIP(hipMemsetAsync(&c->hdr()->pnorm2, 0, sizeof(float), c->stream));
    int blocks = (int)std::min<int64_t>(2048, (lay.n_flat / 4 + 255) / 256);
    hipLaunchKernelGGL(pm_sumsq_kernel, dim3(blocks), dim3(256), 0, c->stream, c->at<float>(lay.w_off), lay.n_flat,
                       &c->hdr()->pnorm2);
  }
  PmStepHdr h;
  PM_HIP(hipMemcpyAsync(&h, c->hdr(), sizeof h, hipMemcpyDeviceToHost, c->stream));
  PM_HIP(hipStreamSynchronize(c->stream));
  if (loss) *loss = h.loss;
  if (grad_norm) *grad_norm = c->o.clip_norm > 0.0 ? std::sqrt((double)h.gnorm2[c->last_par]) / c->o.n_microbatches : 0.0;
  if (param_norm) *param_norm = std::sqrt((double)h.pnorm2);
  if (t) *t = h.t_next;
  if (h.chain_err) return fail(PM_EHIP, "a chained launch gave up waiting for its producers (results of this context are invalid)");
  if (h.diverged) { c->diverged = true; return fail(PM_EDIVERGED, "non-finite weight after step %lld", (long long)h.t_used); }
  return PM_OK;
}

pm_status pm_set_grads(pm_ctx* c, int32_t layer, const float* src, size_t n) {
  pm_status s = check_unit(c, layer, n);
  if (s != PM_OK) return s;
  if (!src) return fail(PM_EINVAL, "src is NULL");
  if ((s = quiesce(c)) != PM_OK) return s;
  const Unit& u = c->lay.units[layer];
  float* g = c->at<float>(c->lay.g_off) + u.off;
  PM_HIP(hipMemcpyAsync(g, src, sizeof(float) * u.nw, hipMemcpyHostToDevice, c->stream));
  if (u.nb) PM_HIP(hipMemcpyAsync(g + u.boff, src + u.nw, sizeof(float) * u.nb, hipMemcpyHostToDevice, c->stream));
  PM_HIP(hipStreamSynchronize(c->stream));
  return PM_OK;
}

pm_status pm_apply_update(pm_ctx* c) {
  if (!c) return fail(PM_EINVAL, "NULL context");
  if (c->micro != 0) return fail(PM_ESTATE, "a minibatch is in progress");
  if (c->diverged) return fail(PM_EDIVERGED, "a non-finite weight was produced at an earlier step");
  pm_status s = quiesce(c);
  if (s != PM_OK) return s;
  const int par = c->par();
  c->last_par = par;
  launch_prologue(c, par);
  s = c->o.dtype == PM_BF16 ? launch_update<bf16_t>(c, c->stream, par, true) : launch_update<float>(c, c->stream, par, true);
  if (s == PM_OK) c->t_host += 1;
  return s;
}


pm_status pm_linear_fwd(void* stream, int32_t dtype, int32_t M, int32_t n_in, int32_t n_out, const void* x_dev,
                        const void* W_dev, const void* b_dev, int32_t act, void* z_dev, void* a_dev) {
  pm_status s = check_linear(dtype, M, n_in, n_out, act);
  if (s != PM_OK) return s;
  if (!x_dev || !W_dev || !b_dev || (!z_dev && !a_dev)) return fail(PM_EINVAL, "NULL argument");
  return dtype == PM_BF16 ? linear_fwd_t<bf16_t>((hipStream_t)stream, M, n_in, n_out, x_dev, W_dev, b_dev, act, z_dev, a_dev)
                          : linear_fwd_t<float>((hipStream_t)stream, M, n_in, n_out, x_dev, W_dev, b_dev, act, z_dev, a_dev);
}

pm_status pm_linear_bwd_data(void* stream, int32_t dtype, int32_t M, int32_t n_in, int32_t n_out, const void* dz_dev,
                             const void* W_dev, const void* zprev_dev, int32_t act_prev, void* dzprev_dev) {
  pm_status s = check_linear(dtype, M, n_in, n_out, act_prev);
  if (s != PM_OK) return s;
  if (!dz_dev || !W_dev || !zprev_dev || !dzprev_dev) return fail(PM_EINVAL, "NULL argument");
  return dtype == PM_BF16 ? linear_bwd_data_t<bf16_t>((hipStream_t)stream, M, n_in, n_out, dz_dev, W_dev, zprev_dev, act_prev, dzprev_dev)
                          : linear_bwd_data_t<float>((hipStream_t)stream, M, n_in, n_out, dz_dev, W_dev, zprev_dev, act_prev, dzprev_dev);
}

pm_status pm_linear_bwd_weight(void* stream, int32_t dtype, int32_t M, int32_t n_in, int32_t n_out, const void* dz_dev,
                               const void* a_dev, float* dW_dev, float* db_dev, int32_t accumulate) {
  pm_status s = check_linear(dtype, M, n_in, n_out, 0);
  if (s != PM_OK) return s;
  if (!dz_dev || !a_dev || !dW_dev) return fail(PM_EINVAL, "NULL argument");
  return dtype == PM_BF16 ? linear_bwd_weight_t<bf16_t>((hipStream_t)stream, M, n_in, n_out, dz_dev, a_dev, dW_dev, db_dev, accumulate)
                          : linear_bwd_weight_t<float>((hipStream_t)stream, M, n_in, n_out, dz_dev, a_dev, dW_dev, db_dev, accumulate);
}

pm_status pm_layernorm_fwd(void* stream, int32_t dtype, int32_t rows, int32_t d, const float* x_dev, const void* gain_dev,
                           const void* bias_dev, void* y_dev, float* mean_dev, float* rstd_dev) {
  if (dtype != PM_F32 && dtype != PM_BF16) return fail(PM_EINVAL, "dtype must be PM_F32 or PM_BF16");
  if (rows < 1 || d < 4 || d > 1024 || (d & 3)) return fail(PM_EINVAL, "need rows >= 1 and d a multiple of 4 in 4..1024");
  if (!x_dev || !gain_dev || !bias_dev || !y_dev || !mean_dev || !rstd_dev) return fail(PM_EINVAL, "NULL argument");
  hipStream_t st = (hipStream_t)stream;
  if (dtype == PM_BF16) {
    const bf16_t* gp = (const bf16_t*)gain_dev;
    if (((const bf16_t*)bias_dev - gp) & 3) return fail(PM_EINVAL, "bias must lie a multiple of 4 elements after the gain");
    pm_ln_fwd_launch<bf16_t>(st, x_dev, PmWLoc<bf16_t>{gp, nullptr, 0}, (int)((const bf16_t*)bias_dev - gp), (bf16_t*)y_dev,
                             mean_dev, rstd_dev, rows, d);
  } else {
    const float* gp = (const float*)gain_dev;
    if (((const float*)bias_dev - gp) & 3) return fail(PM_EINVAL, "bias must lie a multiple of 4 elements after the gain");
    pm_ln_fwd_launch<float>(st, x_dev, PmWLoc<float>{gp, nullptr, 0}, (int)((const float*)bias_dev - gp), (float*)y_dev,
                            mean_dev, rstd_dev, rows, d);
  }
  PM_HIP(hipGetLastError());
  return PM_OK;
}

pm_status pm_layernorm_bwd(void* stream, int32_t dtype, int32_t rows, int32_t d, const float* dy_dev, const float* x_dev,
                           const float* mean_dev, const float* rstd_dev, const void* gain_bkwd_dev,
                           const float* dx_res_dev, float* dx_dev, void* dx_t_dev, float* dgain_dev, float* dbias_dev) {
  if (dtype != PM_F32 && dtype != PM_BF16) return fail(PM_EINVAL, "dtype must be PM_F32 or PM_BF16");
  if (rows < 1 || d < 4 || d > 1024 || (d & 3)) return fail(PM_EINVAL, "need rows >= 1 and d a multiple of 4 in 4..1024");
  if (!dy_dev || !x_dev || !mean_dev || !rstd_dev || !gain_bkwd_dev || !dx_dev || !dgain_dev || !dbias_dev)
    return fail(PM_EINVAL, "NULL argument");
  hipStream_t st = (hipStream_t)stream;
  if (dtype == PM_BF16)
    pm_ln_bwd_launch<bf16_t>(st, dy_dev, x_dev, mean_dev, rstd_dev, PmWLoc<bf16_t>{(const bf16_t*)gain_bkwd_dev, nullptr, 0},
                             dx_res_dev, dx_dev, (bf16_t*)dx_t_dev, dgain_dev, dbias_dev, rows, d);
  else
    pm_ln_bwd_launch<float>(st, dy_dev, x_dev, mean_dev, rstd_dev, PmWLoc<float>{(const float*)gain_bkwd_dev, nullptr, 0},
                            dx_res_dev, dx_dev, (float*)dx_t_dev, dgain_dev, dbias_dev, rows, d);
  PM_HIP(hipGetLastError());
  return PM_OK;
}

pm_status pm_attention_fwd(void* stream, int32_t dtype, int32_t B, int32_t S, int32_t H, int32_t dh, const void* q_dev,
                           const void* k_dev, const void* v_dev, void* o_dev, float* lse_dev) {
  if (dtype != PM_F32 && dtype != PM_BF16) return fail(PM_EINVAL, "dtype must be PM_F32 or PM_BF16");
  if (B < 1 || S < 1 || H < 1 || dh < 1) return fail(PM_EINVAL, "sizes must be positive");
  if (!q_dev || !k_dev || !v_dev || !o_dev || !lse_dev) return fail(PM_EINVAL, "NULL argument");
  hipStream_t st = (hipStream_t)stream;
  const bool ok = dtype == PM_BF16
      ? pm_attn_fwd_launch<bf16_t>(st, B, S, H, dh, (const bf16_t*)q_dev, (const bf16_t*)k_dev, (const bf16_t*)v_dev, (bf16_t*)o_dev, lse_dev)
      : pm_attn_fwd_launch<float>(st, B, S, H, dh, (const float*)q_dev, (const float*)k_dev, (const float*)v_dev, (float*)o_dev, lse_dev);
  if (!ok) return fail(PM_EINVAL, "attention shape (S %d, head size %d) not supported for this dtype", S, dh);
  PM_HIP(hipGetLastError());
  return PM_OK;
}

pm_status pm_attention_bwd(void* stream, int32_t dtype, int32_t B, int32_t S, int32_t H, int32_t dh, const void* q_dev,
                           const void* k_dev, const void* v_dev, const void* o_dev, const void* do_dev,
                           const float* lse_dev, void* dq_dev, void* dk_dev, void* dv_dev) {
  if (dtype != PM_F32 && dtype != PM_BF16) return fail(PM_EINVAL, "dtype must be PM_F32 or PM_BF16");
  if (B < 1 || S < 1 || H < 1 || dh < 1) return fail(PM_EINVAL, "sizes must be positive");
  if (!q_dev || !k_dev || !v_dev || !o_dev || !do_dev || !lse_dev || !dq_dev || !dk_dev || !dv_dev) return fail(PM_EINVAL, "NULL argument");
  hipStream_t st = (hipStream_t)stream;
  const bool ok = dtype == PM_BF16
      ? pm_attn_bwd_launch<bf16_t>(st, B, S, H, dh, (const bf16_t*)q_dev, (const bf16_t*)k_dev, (const bf16_t*)v_dev, (const bf16_t*)o_dev,
                                   (const bf16_t*)do_dev, lse_dev, (bf16_t*)dq_dev, (bf16_t*)dk_dev, (bf16_t*)dv_dev)
      : pm_attn_bwd_launch<float>(st, B, S, H, dh, (const float*)q_dev, (const float*)k_dev, (const float*)v_dev, (const float*)o_dev,
                                  (const float*)do_dev, lse_dev, (float*)dq_dev, (float*)dk_dev, (float*)dv_dev);
  if (!ok) return fail(PM_EINVAL, "attention shape (S %d, head size %d) not supported for this dtype", S, dh);
  PM_HIP(hipGetLastError());
  return PM_OK;
}

namespace {
pm_status check_conv(int32_t dtype, int32_t B, int32_t H, int32_t W, int32_t Cin, int32_t Cout, int32_t stride) {
  if (dtype != PM_F32 && dtype != PM_BF16) return fail(PM_EINVAL, "dtype must be PM_F32 or PM_BF16");
  if (B < 1 || H < 1 || W < 1 || Cin < 1 || Cout < 1) return fail(PM_EINVAL, "sizes must be positive");
  if (stride != 1 && stride != 2) return fail(PM_EINVAL, "stride must be 1 or 2");
  if (Cout & 7) return fail(PM_EINVAL, "C_out must be a multiple of 8");
  return PM_OK;
}
PmConvGeom conv_geom(int B, int H, int W, int Cin, int Cout, int stride) {
  return PmConvGeom{B, H, W, Cin, Cout, stride, (H - 1) / stride + 1, (W - 1) / stride + 1};
}
}  // namespace

pm_status pm_conv3x3_fwd(void* stream, int32_t dtype, int32_t B, int32_t H, int32_t W, int32_t C_in, int32_t C_out,
                         int32_t stride, const void* x_dev, const void* params_dev, void* z_dev, void* y_dev) {
  pm_status s = check_conv(dtype, B, H, W, C_in, C_out, stride);
  if (s != PM_OK) return s;
  if (!x_dev || !params_dev || !z_dev || !y_dev) return fail(PM_EINVAL, "NULL argument");
  const PmConvGeom g = conv_geom(B, H, W, C_in, C_out, stride);
  hipStream_t st = (hipStream_t)stream;
  if (dtype == PM_BF16)
    pm_conv_fwd_launch<bf16_t>(st, g, (const bf16_t*)x_dev, PmWLoc<bf16_t>{(const bf16_t*)params_dev, nullptr, 0},
                               PmShortcut<bf16_t>{nullptr, 0, 0, 0, 1}, (bf16_t*)z_dev, (bf16_t*)y_dev);
  else
    pm_conv_fwd_launch<float>(st, g, (const float*)x_dev, PmWLoc<float>{(const float*)params_dev, nullptr, 0},
                              PmShortcut<float>{nullptr, 0, 0, 0, 1}, (float*)z_dev, (float*)y_dev);
  PM_HIP(hipGetLastError());
  return PM_OK;
}

pm_status pm_conv3x3_bwd_data(void* stream, int32_t dtype, int32_t B, int32_t H, int32_t W, int32_t C_in, int32_t C_out,
                              int32_t stride, const void* dz_dev, const void* params_dev, void* dx_dev) {
  pm_status s = check_conv(dtype, B, H, W, C_in, C_out, stride);
  if (s != PM_OK) return s;
  if (!dz_dev || !params_dev || !dx_dev) return fail(PM_EINVAL, "NULL argument");
  const PmConvGeom g = conv_geom(B, H, W, C_in, C_out, stride);
  hipStream_t st = (hipStream_t)stream;
  if (dtype == PM_BF16)
    pm_conv_dgrad_launch<bf16_t>(st, g, (const bf16_t*)dz_dev, PmWLoc<bf16_t>{(const bf16_t*)params_dev, nullptr, 0},
                                 PmShortcutBwd<bf16_t>{nullptr, 0, 0, 0, 1}, (bf16_t*)dx_dev);
  else
    pm_conv_dgrad_launch<float>(st, g, (const float*)dz_dev, PmWLoc<float>{(const float*)params_dev, nullptr, 0},
                                PmShortcutBwd<float>{nullptr, 0, 0, 0, 1}, (float*)dx_dev);
  PM_HIP(hipGetLastError());
  return PM_OK;
}

pm_status pm_conv3x3_bwd_weight_scratch(int32_t dtype, int32_t B, int32_t H, int32_t W, int32_t C_in, int32_t C_out,
                                        int32_t stride, size_t* out_bytes) {
  pm_status s = check_conv(dtype, B, H, W, C_in, C_out, stride);
  if (s != PM_OK) return s;
  if (!out_bytes) return fail(PM_EINVAL, "out_bytes is NULL");
  const PmConvGeom g = conv_geom(B, H, W, C_in, C_out, stride);
  *out_bytes = 4 * (dtype == PM_BF16 ? pm_conv_wgrad_scratch_elems<bf16_t>(g) : pm_conv_wgrad_scratch_elems<float>(g));
  return PM_OK;
}

pm_status pm_conv3x3_bwd_weight(void* stream, int32_t dtype, int32_t B, int32_t H, int32_t W, int32_t C_in, int32_t C_out,
                                int32_t stride, const void* dz_dev, const void* x_dev, float* dW_dev, void* scratch_dev,
                                size_t scratch_bytes) {
  pm_status s = check_conv(dtype, B, H, W, C_in, C_out, stride);
  if (s != PM_OK) return s;
  if (!dz_dev || !x_dev || !dW_dev) return fail(PM_EINVAL, "NULL argument");
  const PmConvGeom g = conv_geom(B, H, W, C_in, C_out, stride);
  const size_t need = 4 * (dtype == PM_BF16 ? pm_conv_wgrad_scratch_elems<bf16_t>(g) : pm_conv_wgrad_scratch_elems<float>(g));
  if (need && (!scratch_dev || scratch_bytes < need)) return fail(PM_ENOMEM, "scratch has %zu bytes, %zu needed", scratch_bytes, need);
  hipStream_t st = (hipStream_t)stream;
  if (dtype == PM_BF16) pm_conv_wgrad_launch<bf16_t>(st, g, (const bf16_t*)dz_dev, (const bf16_t*)x_dev, dW_dev, 0, (float*)scratch_dev);
  else pm_conv_wgrad_launch<float>(st, g, (const float*)dz_dev, (const float*)x_dev, dW_dev, 0, (float*)scratch_dev);
  PM_HIP(hipGetLastError());
  return PM_OK;
}

namespace {
pm_status profile_begin(pm_ctx* c, int32_t max_steps, bool classes);
}
// ---- the entry point that allocates nothing: the weight gradient of a convolution with its per-block
// partial results in a fixed device array of this library instead of a caller-provided workspace.
// Every GPU the library runs on holds its own copy of the array (at its own address) until the process
// ends; host code reaches it only through the address looked up once per device below.
constexpr size_t PM_STATIC_SCRATCH_BYTES = (size_t)16 << 20;
static __device__ __align__(256) unsigned char pm_static_scratch[PM_STATIC_SCRATCH_BYTES];

namespace {
constexpr int PM_MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[PM_MAX_DEVICES] = {};

// device address of pm_static_scratch on the current device (looked up on the first call per device)
pm_status static_scratch(void** out) {
  int dev = -1;
  PM_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= PM_MAX_DEVICES) return fail(PM_EINVAL, "device index %d outside 0..%d", dev, PM_MAX_DEVICES - 1);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    PM_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(pm_static_scratch)));
    if (!p) return fail(PM_EHIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return PM_OK;
}
}  // namespace

pm_status pm_static_scratch_bytes(size_t* out_bytes) {
  if (!out_bytes) return fail(PM_EINVAL, "out_bytes is NULL");
  *out_bytes = PM_STATIC_SCRATCH_BYTES;
  return PM_OK;
}

pm_status pm_conv3x3_bwd_weight_static(void* stream, int32_t dtype, int32_t B, int32_t H, int32_t W, int32_t C_in,
                                       int32_t C_out, int32_t stride, const void* dz_dev, const void* x_dev,
                                       float* dW_dev) {
  pm_status s = check_conv(dtype, B, H, W, C_in, C_out, stride);
  if (s != PM_OK) return s;
  if (!dz_dev || !x_dev || !dW_dev) return fail(PM_EINVAL, "NULL argument");
  const PmConvGeom g = conv_geom(B, H, W, C_in, C_out, stride);
  const size_t need = 4 * (dtype == PM_BF16 ? pm_conv_wgrad_scratch_elems<bf16_t>(g) : pm_conv_wgrad_scratch_elems<float>(g));
  if (need > PM_STATIC_SCRATCH_BYTES)
    return fail(PM_ENOMEM, "this shape needs %zu bytes of partial results, the built-in scratch holds %zu: use "
                           "pm_conv3x3_bwd_weight with a workspace", need, PM_STATIC_SCRATCH_BYTES);
  void* scratch = nullptr;
  if ((s = static_scratch(&scratch)) != PM_OK) return s;
  // every block of the kernels writes all of its slice of the partial results before the reduce reads
  // it, so nothing left by an earlier call needs clearing
  hipStream_t st = (hipStream_t)stream;
  if (dtype == PM_BF16) pm_conv_wgrad_launch<bf16_t>(st, g, (const bf16_t*)dz_dev, (const bf16_t*)x_dev, dW_dev, 0, (float*)scratch);
  else pm_conv_wgrad_launch<float>(st, g, (const float*)dz_dev, (const float*)x_dev, dW_dev, 0, (float*)scratch);
  PM_HIP(hipGetLastError());
  return PM_OK;
}

pm_status pm_profile_begin(pm_ctx* c, int32_t max_steps) { return profile_begin(c, max_steps, false); }
pm_status pm_profile_begin_classes(pm_ctx* c, int32_t max_steps) {
  if (max_steps > 64) return fail(PM_EINVAL, "a pass that records kernel classes takes at most 64 steps");
  return profile_begin(c, max_steps, true);
}
namespace {
pm_status profile_begin(pm_ctx* c, int32_t max_steps, bool classes) {
  if (!c || max_steps < 1 || max_steps > 65536) return fail(PM_EINVAL, "need a context and 1 <= max_steps <= 65536");
  if (c->o.n_microbatches != 1) return fail(PM_ESTATE, "phase timing supports n_microbatches = 1 only");
  {
    pm_status qs = quiesce(c);
    if (qs != PM_OK) return qs;
  }
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  c->prof_ev.assign((size_t)max_steps * 4, nullptr);
  for (auto& e : c->prof_ev) PM_HIP(hipEventCreate(&e));
  c->prof_cap = max_steps;
  c->prof_n = 0;
  c->prof_on = true;
  for (hipEvent_t e : c->cls_ev) (void)hipEventDestroy(e);
  c->cls_ev.clear();
  c->cls_tag.clear();
  c->cls_cap = classes ? max_steps : 0;
  if (classes) {
    c->cls_ms[0] = c->cls_ms[1] = 0.0;
    c->cls_steps = 0;
  }
  return PM_OK;
}
}  // namespace

pm_status pm_profile_end(pm_ctx* c, double* fwd_ms, double* bwd_ms, double* update_ms, int32_t* n_steps) {
  if (!c) return fail(PM_EINVAL, "NULL context");
  if (!c->prof_on) return fail(PM_ESTATE, "pm_profile_begin was not called");
  PM_HIP(hipStreamSynchronize(c->stream));
  double acc[3] = {0, 0, 0};
  for (int i = 0; i < c->prof_n; ++i)
    for (int k = 0; k < 3; ++k) {
      float ms = 0.f;
      PM_HIP(hipEventElapsedTime(&ms, c->prof_ev[(size_t)i * 4 + k], c->prof_ev[(size_t)i * 4 + k + 1]));
      acc[k] += ms;
    }
  const double inv = c->prof_n ? 1.0 / c->prof_n : 0.0;
  if (fwd_ms) *fwd_ms = acc[0] * inv;
  if (bwd_ms) *bwd_ms = acc[1] * inv;
  if (update_ms) *update_ms = acc[2] * inv;
  if (n_steps) *n_steps = c->prof_n;
  if (c->cls_cap > 0) {
    double cls[2] = {0.0, 0.0};
    for (size_t i = 0; i + 1 < c->cls_ev.size(); i += 2) {
      float ms = 0.f;
      PM_HIP(hipEventElapsedTime(&ms, c->cls_ev[i], c->cls_ev[i + 1]));
      cls[c->cls_tag[i / 2]] += ms;
    }
    c->cls_steps = std::min(c->prof_n, c->cls_cap);
    for (int k = 0; k < 2; ++k) c->cls_ms[k] = c->cls_steps ? cls[k] / c->cls_steps : 0.0;
    for (hipEvent_t e : c->cls_ev) (void)hipEventDestroy(e);
    c->cls_ev.clear();
    c->cls_tag.clear();
    c->cls_cap = 0;
  }
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  c->prof_ev.clear();
  c->prof_on = false;
  c->prof_cap = c->prof_n = 0;
  return PM_OK;
}

pm_status pm_profile_classes(pm_ctx* c, double* product_ms, double* attention_ms, int32_t* n_steps) {
  if (!c) return fail(PM_EINVAL, "NULL context");
  if (c->prof_on) return fail(PM_ESTATE, "a profiling pass is still open: call pm_profile_end first");
  if (product_ms) *product_ms = c->cls_ms[0];
  if (attention_ms) *attention_ms = c->cls_ms[1];
  if (n_steps) *n_steps = c->cls_steps;
  return PM_OK;
}

pm_status pm_synchronize(pm_ctx* c) {
  if (!c) return fail(PM_EINVAL, "NULL context");
  PM_HIP(hipStreamSynchronize(c->stream));
  if (c->stream_b) PM_HIP(hipStreamSynchronize(c->stream_b));
  c->upd_pending = false;
  return PM_OK;
}

// ---- checkpoint / resume: header + the state arrays as they lie in the arena
namespace {
struct CkptHdr {
  uint64_t magic;
  uint32_t version, esz;
  int32_t L, P, opt, has_ur;
  int64_t n_flat, ring_elems;
  int64_t t;
  int32_t diverged;
  float last_loss;
};
constexpr uint64_t CKPT_MAGIC = 0x50697065'4d617265ull;   // "PipeMare"

struct CkptSeg { size_t off, bytes; };
std::vector<CkptSeg> ckpt_segments(const pm_ctx* c) {
  const Layout& lay = c->lay;
  const size_t f32 = (size_t)lay.n_flat * 4, cd = (size_t)lay.n_flat * lay.esz;
  std::vector<CkptSeg> v{{lay.w_off, f32}, {lay.v_off, f32}};
  if (c->o.opt == PM_OPT_ADAMW) v.push_back({lay.s_off, f32});
  v.push_back({lay.d_off, f32});
  v.push_back({lay.ub_off, cd});
  if (lay.has_ur) v.push_back({lay.ur_off, cd});
  v.push_back({lay.ring_off, (size_t)lay.ring_elems * lay.esz});
  return v;
}
CkptHdr ckpt_header(const pm_ctx* c) {
  CkptHdr h{};
  h.magic = CKPT_MAGIC;
  h.version = 1;
  h.esz = (uint32_t)c->lay.esz;
  h.L = c->L;
  h.P = c->P;
  h.opt = c->o.opt;
  h.has_ur = c->lay.has_ur ? 1 : 0;
  h.n_flat = c->lay.n_flat;
  h.ring_elems = c->lay.ring_elems;
  h.t = c->t_host;
  h.diverged = c->diverged ? 1 : 0;
  h.last_loss = c->last_loss;
  return h;
}
}  // namespace

pm_status pm_checkpoint_bytes(pm_ctx* c, size_t* bytes) {
  if (!c || !bytes) return fail(PM_EINVAL, "NULL argument");
  size_t n = sizeof(CkptHdr);
  for (const CkptSeg& sgm : ckpt_segments(c)) n += sgm.bytes;
  *bytes = n;
  return PM_OK;
}

pm_status pm_checkpoint_save(pm_ctx* c, void* dst, size_t bytes) {
  size_t need = 0;
  pm_status s = pm_checkpoint_bytes(c, &need);
  if (s != PM_OK) return s;
  if (!dst || bytes < need) return fail(PM_EINVAL, "checkpoint buffer: need %zu bytes", need);
  if (c->micro != 0) return fail(PM_ESTATE, "checkpoint in the middle of a minibatch");
  if ((s = pm_synchronize(c)) != PM_OK) return s;
  char* p = static_cast<char*>(dst);
  const CkptHdr h = ckpt_header(c);
  std::memcpy(p, &h, sizeof h);
  p += sizeof h;
  for (const CkptSeg& sgm : ckpt_segments(c)) {
    PM_HIP(hipMemcpy(p, c->arena + sgm.off, sgm.bytes, hipMemcpyDeviceToHost));
    p += sgm.bytes;
  }
  return PM_OK;
}

pm_status pm_checkpoint_load(pm_ctx* c, const void* src, size_t bytes) {
  size_t need = 0;
  pm_status s = pm_checkpoint_bytes(c, &need);
  if (s != PM_OK) return s;
  if (!src || bytes < need) return fail(PM_EINVAL, "checkpoint image: need %zu bytes", need);
  const char* p = static_cast<const char*>(src);
  CkptHdr h;
  std::memcpy(&h, p, sizeof h);
  const CkptHdr w = ckpt_header(c);
  if (h.magic != CKPT_MAGIC || h.version != w.version || h.esz != w.esz || h.L != w.L || h.P != w.P || h.opt != w.opt ||
      h.has_ur != w.has_ur || h.n_flat != w.n_flat || h.ring_elems != w.ring_elems || h.t < 0)
    return fail(PM_EINVAL, "checkpoint image does not match this context");
  if ((s = pm_synchronize(c)) != PM_OK) return s;
  p += sizeof h;
  for (const CkptSeg& sgm : ckpt_segments(c)) {
    PM_HIP(hipMemcpy(c->arena + sgm.off, p, sgm.bytes, hipMemcpyHostToDevice));
    p += sgm.bytes;
  }
  // the device step counter; the step table is rebuilt from it by the first kernel of the next step
  PmStepHdr dh;
  PM_HIP(hipMemcpy(&dh, c->hdr(), sizeof dh, hipMemcpyDeviceToHost));
  dh.t_next = h.t;
  dh.t_used = h.t > 0 ? h.t - 1 : 0;
  dh.diverged = h.diverged;
  dh.loss = 0.f;
  PM_HIP(hipMemcpy(c->hdr(), &dh, sizeof dh, hipMemcpyHostToDevice));
  c->t_host = h.t;
  c->micro = 0;
  c->diverged = h.diverged != 0;
  c->last_loss = h.last_loss;
  c->upd_pending = false;
  return PM_OK;
}

void pm_destroy(pm_ctx* c) {
  if (!c) return;
  if (c->stream_b) {
    (void)hipStreamSynchronize(c->stream_b);
    (void)hipStreamDestroy(c->stream_b);
  }
  if (c->ev_bwd) (void)hipEventDestroy(c->ev_bwd);
  if (c->ev_upd) (void)hipEventDestroy(c->ev_upd);
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->cls_ev) (void)hipEventDestroy(e);
  for (const pm_ctx::StepGraph& sg : c->graphs) {
    (void)hipGraphExecDestroy(sg.exec);
    (void)hipGraphDestroy(sg.graph);
  }
  delete c;
}

}  // extern "C"
