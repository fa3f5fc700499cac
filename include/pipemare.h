/*
 * pipemare.h — C ABI of the MI355X (gfx950) PipeMare training-step library.
 *
 * One context executes asynchronous pipeline-parallel training of a network of weight units
 * (a chain of Linear + bias + activation units, or a fine-grained pre-LN causal Transformer made of
 * embedding, LayerNorm and Linear units) as a delay-faithful single-GPU run of all P pipeline stages:
 * forward with weights that are tau_fwd,i optimizer steps old, read in place from a
 * device-resident ring of weight versions; backward with discrepancy-corrected weights; one
 * fused update pass (learning-rate rescheduling, optimizer, delta accumulator, ring and
 * corrected-weight write-back).
 *
 * Conventions for every entry point
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP device memory on the
 *     GPU that was current when pm_create was called.
 *   - The library never allocates or frees device memory: the caller provides one arena
 *     (pm_query_bytes tells how large) and owns it, the HIP stream and the batch buffers.
 *   - All GPU work is enqueued on the stream given to pm_create (plus, with overlap_update, the
 *     fused update on a second stream the library creates).  Only pm_weights, pm_state, pm_stats,
 *     pm_device_step_table, pm_set_grads, pm_synchronize, pm_profile_end and pm_step with a
 *     non-NULL loss pointer wait for it.
 *   - Errors are return codes (never exceptions, never abort); a NULL context gives PM_EINVAL.
 *   - A context is not re-entrant: one thread, one stream.
 */
#ifndef PIPEMARE_H_
#define PIPEMARE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pm_ctx pm_ctx;

typedef enum {
  PM_OK = 0,
  PM_EINVAL = 1,    /* bad argument (shape chain, delays, NULL, misaligned pointer, ...) */
  PM_ENOMEM = 2,    /* arena smaller than pm_query_bytes reports */
  PM_EHIP = 3,      /* a HIP runtime call failed; pm_last_error() has the text */
  PM_ESTATE = 4,    /* call not valid in the current state (e.g. mid-minibatch) */
  PM_EDIVERGED = 5  /* a non-finite weight was produced (sticky; training can diverge by design
                       of the experiment, cf. the stability analysis of Sec. 3.1) */
} pm_status;

typedef enum {
  PM_LINEAR = 0,     /* W [n_out, n_in] row-major + bias [n_out] */
  PM_EMBED = 1,      /* table E [n_in = vocabulary, n_out = width], no bias */
  PM_LAYERNORM = 2,  /* gain [n_out] + bias [n_out] over rows of width n_in = n_out, eps 1e-5 */
  PM_CONV3X3 = 3     /* 3x3 convolution, zero padding 1: W [n_out][3][3][n_in] + per-channel scale [n_out] and
                        shift [n_out] (a folded normalisation); stride 2 where n_out = 2 n_in, else 1 */
} pm_layer_kind;
typedef enum {
  PM_ARCH_CHAIN = 0,       /* Linear units in sequence, unit l feeds unit l+1 */
  PM_ARCH_TRANSFORMER = 1, /* embed | per layer: ln1, Wq, Wk, Wv, Wo, ln2, W1, W2 | final ln, head (see pm_opts) */
  PM_ARCH_RESNET = 2       /* conv | blocks of two convs with parameter-free shortcuts | pool, classifier (see pm_opts) */
} pm_arch;
typedef enum { PM_ACT_NONE = 0, PM_ACT_RELU = 1, PM_ACT_GELU = 2 /* exact erf form */ } pm_act;
typedef enum { PM_METHOD_PIPEMARE = 0, PM_METHOD_PIPEDREAM = 1, PM_METHOD_GPIPE = 2 } pm_method;
typedef enum { PM_LR_CONST = 0, PM_LR_STEP = 1, PM_LR_WARMUP_INVSQRT = 2 } pm_lr_kind;
typedef enum { PM_OPT_SGDM = 0, PM_OPT_ADAMW = 1 } pm_opt_kind;
typedef enum { PM_F32 = 0, PM_BF16 = 1 /* bf16 compute + ring, fp32 master/optimizer state */ } pm_dtype;
typedef enum { PM_LOSS_MSE = 0, PM_LOSS_XENT = 1 } pm_loss_kind;

/* One weight unit.  Linear: y = act(x W^T + b), W is n_out x n_in row-major.  Weight and bias always
 * share a pipeline stage (Sec. 4.1, "Pipeline Stages"); `stage` is 1-based and non-decreasing in
 * topological order; several consecutive units may share a stage (a LayerNorm normally rides in the
 * stage of the matrix that consumes it).  Packed host layout of a unit's values, used by
 * init_weights_host, pm_weights, pm_state and pm_set_grads: [W | b] (Linear), [E] (embedding),
 * [gain | bias] (LayerNorm), [W | scale | shift] (convolution). */
typedef struct {
  int32_t kind;   /* pm_layer_kind */
  int32_t n_in;
  int32_t n_out;
  int32_t act;    /* pm_act */
  int32_t stage;  /* 1..P */
} pm_layer_desc;

/* Synchronous base schedule alpha_{k,base} (Sec. 3.1) and the T1 annealing length K (in steps).
 *   CONST:           base
 *   STEP:            base * factor^floor(k / interval)
 *   WARMUP_INVSQRT:  linear init -> base over `interval` steps, then base * sqrt(interval / k)
 * K = 0 disables the rescheduling exponent (p_k = 0). */
typedef struct {
  int32_t kind;       /* pm_lr_kind */
  double base;
  double init;
  double factor;
  int64_t interval;
  int64_t K;
} pm_lr_sched;

typedef struct {
  int32_t opt;               /* pm_opt_kind */
  double beta1;              /* SGD momentum beta (App. B.3 form), or Adam beta1 */
  double beta2;              /* Adam beta2 */
  double eps;                /* Adam epsilon */
  double weight_decay;       /* SGD: added to the gradient (L2); AdamW: decoupled */
  double clip_norm;          /* > 0: scale gradients so their global L2 norm is at most this */
  double D;                  /* T2 decay, gamma_i = D^(1/(tau_fwd,i - tau_bkwd,i)) (Sec. 3.2) */
  const double* gamma_override; /* host, P entries or NULL: per-stage gamma_i given directly */
  int32_t t1_enabled;        /* 0: every stage uses alpha_{k,base} */
  int32_t t2_enabled;        /* 0: backward reads the plain version t - tau_bkwd,i */
  int32_t n_microbatches;    /* N >= 1: pm_step accumulates N calls, then updates (Sec. 2.1) */
  int32_t dtype;             /* pm_dtype */
  int32_t loss;              /* pm_loss_kind */
  int32_t microbatch;        /* rows M of every batch given to pm_step */
  int32_t use_graph;         /* 1: replay the step as a captured HIP graph after the first call with a given pair
                                of batch buffers (one graph per (x_dev, y_dev) pair, up to 64 pairs kept) */
  int64_t sync_warmup_steps; /* E_w >= 0: the first E_w optimizer steps run synchronously (all delays 0,
                                base step size, no correction: the warm-up of PipeMareW, Sec. 4), then
                                the delays apply and the T1 step counter starts from 0 */
  int32_t overlap_update;    /* 1: run the fused update of step t on a second stream owned by the library,
                                concurrently with the forward of step t+1 (which, with tau_fwd >= 1
                                everywhere, reads only versions <= t-1: the method's own asynchrony).
                                Ignored with use_graph.  The caller's stream being idle then no longer
                                implies the last update has finished: pm_synchronize or any read-back
                                call waits for it. */
  int32_t arch;              /* pm_arch.  PM_ARCH_TRANSFORMER: the L = 8*n_layers + 3 units must be, in order,
                                EMBED(vocab, d) | n_layers x { LAYERNORM(d), LINEAR(d,d) q, LINEAR(d,d) k, LINEAR(d,d) v,
                                LINEAR(d,d) o, LAYERNORM(d), LINEAR(d,d_ff) with act, LINEAR(d_ff,d) } | LAYERNORM(d),
                                LINEAR(d,vocab).  Pre-LN residual blocks, causal attention, fixed sinusoidal positions,
                                untied output head, mean token cross-entropy (loss must be PM_LOSS_XENT).  `microbatch`
                                counts sequences; pm_step takes int32 token ids [microbatch, seq_len] as x and the
                                int32 next-token targets of the same shape as y. */
  int32_t n_heads;           /* Transformer: attention heads (d % n_heads == 0) */
  int32_t seq_len;           /* Transformer: tokens per sequence */
  int32_t image_size;        /* PM_ARCH_RESNET: input images are 3 x image_size x image_size (a multiple of 4).  The
                                L = 2 * blocks + 2 units must be CONV3X3(c0_in -> c) | blocks x { CONV3X3(a -> b),
                                CONV3X3(b -> b) } with b = a or b = 2a (then stride 2 and the shortcut takes every
                                second pixel, new channels zero) | LINEAR(last b -> classes).  y = relu(scale * conv(x)
                                + shift [+ shortcut(block input)]); global average pool before the classifier;
                                cross-entropy (loss must be PM_LOSS_XENT).  Channel counts multiples of 8.  pm_step
                                takes fp32 images [microbatch, c0_in, image_size, image_size] (NCHW) as x and int32
                                labels [microbatch] as y. */
  const int32_t* tau_recomp; /* host, P entries or NULL.  Non-NULL turns on recomputation (all architectures; App.
                                "Statistical efficiency and recompute"): the forward pass is taken to keep only the
                                tensors that enter a segment of `segment_size` consecutive stages from an earlier
                                one; the backward pass rebuilds the activations inside a segment from those with the
                                weights of version max(t - tau_recomp,i, 0), corrected - when t2_enabled - by
                                (tau_fwd,i - tau_recomp,i) delta_t ("T2 for Recompute").  A unit's backward (and the
                                rebuild itself) uses the rebuilt value of a tensor produced in the unit's own
                                segment and the kept forward value of one produced in an earlier segment; a
                                weight-free operator (attention core, residual add, pooling) belongs to the unit
                                that consumes its result; the loss gradient comes from the forward pass.  Needs
                                tau_bkwd,i <= tau_recomp,i <= tau_fwd,i.  pm_recompute_delays gives the delays of
                                PipeMare Recompute. */
  int32_t segment_size;      /* stages per segment (>= 1) when tau_recomp is given; the last segment may be shorter */
  int32_t stochastic_delays; /* 1: Hogwild-style stochastic delays (App. "Hogwild! asynchrony"): at every optimizer step
                                each stage i draws a delay from the exponential distribution with mean tau_fwd[i-1]
                                truncated at tau_max, and BOTH passes read that version of the stage's weights (no
                                forward/backward discrepancy, so T2 does not apply and tau_bkwd is ignored); T1 keeps
                                dividing by the mean tau_fwd[i-1].  Every ring then has tau_max + 1 slots.  The draw is
                                a pure function of (delay_seed, step, stage): see pm_stochastic_delays.  Not combined
                                with recomputation. */
  int32_t tau_max;           /* stochastic delays: largest delay, 0 .. 65535 */
  uint64_t delay_seed;       /* stochastic delays: seed of the counter-based generator */
  int32_t chained_launches;  /* 1 (PM_ARCH_CHAIN, bf16, at most 128 rows, a multiple of 32, unit widths multiples of
                                64): the forward products of all such units (Sec. 2.1: one per stage, each waiting
                                for the one before) run as ONE persistent launch whose blocks pass the activations
                                to each other through device memory, likewise the data-gradient products.  Same
                                results up to the order of the fp32 partial sums.  0 (default): one launch per
                                product, which measures slightly faster on the 16-layer MLP workload.  Ignored
                                for other shapes, with recomputation and with overlap_update. */
  int32_t update_placement;  /* Where the update of Sec. 2.1 / 3.1 / 3.2 is applied to the weight matrices of a bf16
                                Transformer whose weight gradients come out of one grouped launch with whole tiles
                                (one microbatch per step, no clipping, no recomputation, no overlap_update).
                                2: in that launch - a block that has stored the gradients of its tile applies the
                                update to those parameters at once, and the update pass covers only the remaining
                                ones (biases, LayerNorm, embedding); the gradient of a weight matrix is not read
                                back from memory.  1: always the separate pass over all parameters.  0 (default):
                                2 where the parameter state is too large to stay cached from step to step (the
                                regime in which it measures faster), else 1.  Same arithmetic per parameter either
                                way; pm_state still returns the gradient; pm_update_split tells what applies. */
} pm_opts;

const char* pm_status_str(pm_status s);
/* Text of the last failure on this thread ("" if none).  Host pointer owned by the library. */
const char* pm_last_error(void);

/* Per-stage delays of Table 1 for stages i = 1..P with N microbatches per minibatch:
 * tau_fwd,i = ceil((2(P-i)+1)/N); tau_bkwd,i = 0 (PipeMare) | tau_fwd,i (PipeDream); both 0 for
 * GPipe.  Host arrays of P entries each (index i-1).  PM_EINVAL if P < 1 or N < 1. */
pm_status pm_delays(int32_t P, int32_t N, int32_t method, int32_t* tau_fwd, int32_t* tau_bkwd);

/* Stochastic delays (App. "Hogwild! asynchrony"): integer inverse-CDF table of one stage's delay.
 * X ~ Exp(mean) truncated to [0, tau_max + 1), delay = floor(X) in 0..tau_max;
 * thresholds[k] = min(floor(2^32 P(delay <= k)), 2^32 - 1) for k = 0..tau_max-1 (host array, out);
 * a 32-bit draw r gives delay = #{k : r > thresholds[k]}.  mean <= 0: always 0. */
pm_status pm_delay_thresholds(double mean, int32_t tau_max, uint32_t* thresholds);

/* The delays all P stages draw at optimizer step t: stage i (1-based) takes output number t * P + i
 * of the SplitMix64 generator started at `seed` (upper 32 bits) through the table of mean
 * mean_tau[i-1].  Pure host integer function, identical to what the device computes.
 * mean_tau: host, P entries; tau_out: host, P entries (out). */
pm_status pm_stochastic_delays(int32_t P, const int32_t* mean_tau, int32_t tau_max, uint64_t seed, int64_t t,
                               int32_t* tau_out);

/* Recompute delays of PipeMare Recompute (App. "Trade compute for memory via PipeMare Recompute"): with the P
 * stages cut into segments of S consecutive stages (the last may be shorter), the j-th stage of a segment of S'
 * stages recomputes 2 (S' - j) microbatch slots before its backward pass:
 * tau_recomp,i = tau_bkwd,i + ceil(2 (S' - j) / N).  tau_bkwd: host, P entries, or NULL for all zero;
 * tau_recomp: host, P entries (out).  PM_EINVAL if P, S or N < 1. */
pm_status pm_recompute_delays(int32_t P, int32_t S, int32_t N, const int32_t* tau_bkwd, int32_t* tau_recomp);

/* Ring-slot arithmetic for one stage at optimizer step t (Sec. 2.1 delayed reads; the ring of
 * R = tau_fwd + 1 slots is this library's stand-in for the paper's queue of stale weights):
 * version read forward max(t - tau_fwd, 0), backward max(t - tau_bkwd, 0), written t + 1;
 * slot = version mod R.  Pure host integer function. */
pm_status pm_slots(int32_t tau_fwd, int32_t tau_bkwd, int64_t t,
                   int32_t* fwd_slot, int32_t* bkwd_slot, int32_t* write_slot);

/* T1 step size alpha_{k,i} = alpha_{k,base} / max(tau_i,1)^{p_k}, p_k = 1 - min(k/K,1) (Sec. 3.1),
 * computed on the host in double precision. */
pm_status pm_t1_lr(const pm_lr_sched* sched, int32_t tau, int64_t k, int32_t t1_enabled, double* lr);

/* Bytes of device arena pm_create needs for this configuration: fp32 master weights, gradients, optimizer
 * moments and the delta accumulator of Sec. 3.2 (the "+33 % / +25 %" of weight-plus-optimizer memory the
 * paper quotes for T2), the corrected backward weights, the ring of tau_fwd,i + 1 weight versions per
 * stage (sum_i |w_i| (tau_fwd,i + 1) values: what a delay-faithful run on ONE device costs; on a real
 * pipeline the delayed weights are simply the ones in memory, Sec. 2.2), activations and small tables.
 * Same argument rules as pm_create; *out_bytes host, out. */
pm_status pm_query_bytes(int32_t P, int32_t L, const pm_layer_desc* layers, const int32_t* tau_fwd,
                         const pm_opts* opts, size_t* out_bytes);

/* Build a context for the recurrence of Sec. 2.1, w_{t+1} = w_t - alpha grad f_t(u_fwd,t, u_bkwd,t) with
 * (u_fwd,t)_i = (w_{t - tau_fwd,i})_i and (u_bkwd,t)_i = (w_{t - tau_bkwd,i})_i (delays as in Sec. 2.2 /
 * Table 1: pm_delays), the step sizes of T1 (Sec. 3.1: sched, sched->K, opts->t1_enabled) and the
 * corrected backward weights of T2 (Sec. 3.2: opts->D or gamma_override, opts->t2_enabled).
 *   P, L               stages and weight units; layers[L] host
 *   tau_fwd, tau_bkwd  host, P entries, 0 <= tau_bkwd,i <= tau_fwd,i
 *   init_weights_host  L host pointers, unit l in its packed layout (see pm_layer_desc), fp32
 *   device_arena       device, 256-byte aligned, arena_bytes >= pm_query_bytes
 *   hip_stream         hipStream_t (NULL = default stream)
 * Every ring slot starts as w_0, delta_0 = v_0 = 0, corrected weights = w_0.
 * On success *out owns only host memory; release with pm_destroy. */
pm_status pm_create(int32_t P, int32_t L, const pm_layer_desc* layers,
                    const int32_t* tau_fwd, const int32_t* tau_bkwd,
                    const pm_lr_sched* sched, const pm_opts* opts,
                    const float* const* init_weights_host,
                    void* device_arena, size_t arena_bytes, void* hip_stream, pm_ctx** out);

/* One microbatch through all stages (forward on stale weights, loss, backward on corrected
 * weights); after the N-th microbatch of a minibatch also the fused update (Sec. 2.1 recurrence,
 * T1, T2).  Chain: x_dev device fp32 [microbatch, n_in of unit 0] row-major, y_dev device fp32
 * [microbatch, n_out of last unit] (MSE) or int32 [microbatch] labels (cross-entropy).
 * Transformer: x_dev, y_dev device int32 [microbatch, seq_len] (ids outside the vocabulary are
 * clamped on input and contribute no loss as targets).
 * loss_out_host: NULL, or host float that receives this microbatch's mean loss (forces a
 * stream synchronisation).  Returns PM_EDIVERGED once a non-finite weight has been seen by a
 * synchronising call. */
pm_status pm_step(pm_ctx* ctx, const void* x_dev, const void* y_dev, float* loss_out_host);

/* fp32 master weights of unit `layer` - the current iterate w_t of the recurrence of Sec. 2.1 after the t
 * optimizer steps completed so far, not any delayed version - into host memory in the unit's packed
 * layout; n must equal the unit's value count.  Synchronises the stream. */
pm_status pm_weights(pm_ctx* ctx, int32_t layer, float* dst_host, size_t n);

/* Same layout for the delta accumulator (which = 1), the optimizer's first state v or m
 * (which = 2), the corrected backward weights currently stored (which = 3, widened to fp32), the
 * gradient buffer (which = 4) and the corrected recompute weights (which = 5; PM_ESTATE if the
 * context keeps none: they exist only for units whose recompute delay or coefficient differs
 * from the backward one). */
pm_status pm_state(pm_ctx* ctx, int32_t which, int32_t layer, float* dst_host, size_t n);

/* What the kernels of the most recent step actually used, read back from the device-resident
 * step table: per unit the forward / backward / write slot and the step size.  Host arrays of L
 * entries (any may be NULL); *t_used receives that step's index.  Synchronises. */
pm_status pm_device_step_table(pm_ctx* ctx, int64_t* t_used, int32_t* fwd_slot, int32_t* bkwd_slot,
                               int32_t* write_slot, float* lr);

/* With recomputation: per unit the ring slot (max(t - tau_recomp, 0)) mod R of the most recent
 * step, from the device-resident step table (host array of L entries, may be NULL).
 * PM_ESTATE without recomputation.  Synchronises. */
pm_status pm_device_recompute_slots(pm_ctx* ctx, int64_t* t_used, int32_t* rec_slot);

/* How many units the chained launches of this context cover (see pm_opts.chained_launches): units 0 ..
 * *n_forward - 1 run forward as one launch, the data-gradient products of units *n_backward .. 1 as one launch;
 * 0 = that direction keeps one launch per product (option off, or the shapes do not qualify).  Either output may
 * be NULL.  No device work. */
pm_status pm_chained_units(pm_ctx* ctx, int32_t* n_forward, int32_t* n_backward);

/* Where the update of Sec. 2.1 / 3 is applied in this context (see pm_opts.update_placement): *n_epilogue
 * parameters (weight matrices) are updated in the epilogues of the grouped weight-gradient launch, *n_pass
 * parameters (padding included) by the update pass that follows; *n_epilogue = 0 when the separate pass covers
 * everything.  Either output may be NULL.  No device work. */
pm_status pm_update_split(pm_ctx* ctx, int64_t* n_epilogue, int64_t* n_pass);

/* Running numbers: mean loss of the most recent MICROBATCH (with n_microbatches > 1 not the mean over the
 * minibatch), global L2 norm of the averaged minibatch gradient of the last update (only when clipping
 * is on, else 0; App. C's clipping threshold acts on it), L2 norm of the master weights w_t (the quantity
 * whose blow-up marks the divergence studied in Sec. 3.1), number t of completed optimizer steps.  Any
 * output may be NULL.  Synchronises both streams, so a divergence flagged by an overlapped update is seen
 * here at once, while pm_step's loss read-back (caller's stream only) may report it one step late. */
pm_status pm_stats(pm_ctx* ctx, double* loss, double* grad_norm, double* param_norm, int64_t* t);

/* Testing / benchmarking of the update pass in isolation (the T1/T2/optimizer/write-back part of
 * the step without a model): overwrite unit `layer`'s gradient buffer from host fp32 [W | b], and
 * run exactly the update of one optimizer step on whatever the gradient buffers hold. */
pm_status pm_set_grads(pm_ctx* ctx, int32_t layer, const float* src_host, size_t n);
pm_status pm_apply_update(pm_ctx* ctx);

/* Per-phase GPU timing of pm_step with HIP events recorded on the context's stream (host-side
 * event objects; no device memory).  Between begin and end every pm_step runs eagerly (a captured
 * graph is bypassed) and records four events: start, after forward + loss, after backward, after
 * the fused update.  pm_profile_end synchronises and returns the mean milliseconds per step of
 * the three phases over the steps recorded (at most max_steps).  n_microbatches must be 1. */
pm_status pm_profile_begin(pm_ctx* ctx, int32_t max_steps);
pm_status pm_profile_end(pm_ctx* ctx, double* fwd_ms, double* bwd_ms, double* update_ms, int32_t* n_steps);
/* A profiling pass (ended by pm_profile_end like the one above) of at most 64 steps that ALSO brackets every
 * launch of a stage's matrix or convolution product (forward, data gradient, weight gradient: the products
 * of Sec. 2.1's per-stage forward and backward) and every attention-core launch with an event pair - two
 * stream markers per launch, which is why the phase times are better taken from a plain pass.
 * pm_profile_classes returns, for the last such pass that has ended, the mean milliseconds per step summed
 * over each class and the number of steps measured (zeros if there was none).  Any output may be NULL.
 * PM_ESTATE while a pass is open. */
pm_status pm_profile_begin_classes(pm_ctx* ctx, int32_t max_steps);
pm_status pm_profile_classes(pm_ctx* ctx, double* product_ms, double* attention_ms, int32_t* n_steps);

/* The three matrix products of one Linear unit as stand-alone primitives (the per-stage forward
 * and the two halves of the per-stage backward of Sec. 2.1), on plain device matrices, for
 * kernel-level tests and roofline measurement.  All matrices row-major and dense (leading
 * dimension = width); element type bf16 (raw 16-bit) or fp32 per `dtype`; bf16 needs n_in and
 * n_out to be multiples of 8 and 16-byte aligned pointers.  Asynchronous on `stream`.
 *   fwd:        z = x W^T + b,  a = act(z)          x[M,n_in] W[n_out,n_in] b[n_out] -> z, a [M,n_out] (either may be NULL)
 *   bwd_data:   dzprev = (dz W) * act_prev'(zprev)  dz[M,n_out] W[n_out,n_in] zprev[M,n_in] -> dzprev[M,n_in]
 *   bwd_weight: dW = dz^T a, db = column sums of dz a[M,n_in] -> dW fp32 [n_out,n_in], db fp32 [n_out] (db may be NULL);
 *               accumulate != 0 adds to the existing contents. */
pm_status pm_linear_fwd(void* stream, int32_t dtype, int32_t M, int32_t n_in, int32_t n_out,
                        const void* x_dev, const void* W_dev, const void* b_dev, int32_t act,
                        void* z_dev, void* a_dev);
pm_status pm_linear_bwd_data(void* stream, int32_t dtype, int32_t M, int32_t n_in, int32_t n_out,
                             const void* dz_dev, const void* W_dev, const void* zprev_dev,
                             int32_t act_prev, void* dzprev_dev);
pm_status pm_linear_bwd_weight(void* stream, int32_t dtype, int32_t M, int32_t n_in, int32_t n_out,
                               const void* dz_dev, const void* a_dev, float* dW_dev, float* db_dev,
                               int32_t accumulate);

/* Weight-free and vector-weight operators of the Transformer stages as stand-alone primitives for
 * kernel-level tests and measurement.  rows = tokens, row r = sequence r / S, position r % S.
 * Element type of the "T" matrices per `dtype` (bf16 raw 16-bit, or fp32); d a multiple of 4 up to 1024.
 *   layernorm_fwd: y = (x - mean) * rstd * gain + bias        x fp32 [rows,d], gain/bias T [d] -> y T [rows,d],
 *                  mean, rstd fp32 [rows]
 *   layernorm_bwd: dx = (dx_res or 0) + rstd (dxh - mean(dxh) - xhat mean(dxh xhat)), dxh = dy * gain_bkwd
 *                  (the gain of the BACKWARD weights, Sec. 2.1); dgain += sum dy xhat, dbias += sum dy
 *                  dy fp32 [rows,d]; dx fp32 (may alias dx_res); dx_t T copy of dx or NULL; dgain, dbias fp32 [d]
 *                  are added to (caller zeroes them)
 *   attention_fwd: causal softmax(q k^T / sqrt(dh)) v per (sequence, head); q, k, v, o T [B*S, H*dh], head h in
 *                  columns h*dh..; lse fp32 [B, H, S] receives log-sum-exp of the scaled scores
 *   attention_bwd: gradients dq, dk, dv T [B*S, H*dh] from do, recomputing probabilities from q, k, lse */
pm_status pm_layernorm_fwd(void* stream, int32_t dtype, int32_t rows, int32_t d, const float* x_dev,
                           const void* gain_dev, const void* bias_dev, void* y_dev, float* mean_dev, float* rstd_dev);
pm_status pm_layernorm_bwd(void* stream, int32_t dtype, int32_t rows, int32_t d, const float* dy_dev,
                           const float* x_dev, const float* mean_dev, const float* rstd_dev,
                           const void* gain_bkwd_dev, const float* dx_res_dev, float* dx_dev, void* dx_t_dev,
                           float* dgain_dev, float* dbias_dev);
pm_status pm_attention_fwd(void* stream, int32_t dtype, int32_t B, int32_t S, int32_t H, int32_t dh,
                           const void* q_dev, const void* k_dev, const void* v_dev, void* o_dev, float* lse_dev);
pm_status pm_attention_bwd(void* stream, int32_t dtype, int32_t B, int32_t S, int32_t H, int32_t dh,
                           const void* q_dev, const void* k_dev, const void* v_dev, const void* o_dev,
                           const void* do_dev, const float* lse_dev, void* dq_dev, void* dk_dev, void* dv_dev);

/* The three products of one 3x3 convolution unit (zero padding 1, stride 1 or 2) as stand-alone
 * primitives for kernel-level tests and measurement.  Tensors NHWC in the element type of `dtype`;
 * params = [W (C_out x 3 x 3 x C_in) | scale (C_out) | shift (C_out)].  bf16 with C_in and C_out multiples
 * of 16 (at most 64) runs as implicit GEMM on MFMA, anything else on plain kernels.  C_out a multiple of 8.
 *   fwd:        z = conv(x, W); y = relu(scale * z + shift)     x [B,H,W,C_in] -> z, y [B,Ho,Wo,C_out], Ho = (H-1)/stride+1
 *   bwd_data:   dx = transposed convolution of dz with W        dz [B,Ho,Wo,C_out] -> dx [B,H,W,C_in]
 *   bwd_weight: dW (fp32 [C_out][3][3][C_in]) = correlation of dz with x; overwritten.  The MFMA path reduces per-block
 *               partial results through a caller-provided device workspace of pm_conv3x3_bwd_weight_scratch bytes
 *               (0 for shapes on the plain path; PM_ENOMEM if the workspace is too small). */
pm_status pm_conv3x3_fwd(void* stream, int32_t dtype, int32_t B, int32_t H, int32_t W, int32_t C_in, int32_t C_out,
                         int32_t stride, const void* x_dev, const void* params_dev, void* z_dev, void* y_dev);
pm_status pm_conv3x3_bwd_data(void* stream, int32_t dtype, int32_t B, int32_t H, int32_t W, int32_t C_in, int32_t C_out,
                              int32_t stride, const void* dz_dev, const void* params_dev, void* dx_dev);
pm_status pm_conv3x3_bwd_weight_scratch(int32_t dtype, int32_t B, int32_t H, int32_t W, int32_t C_in, int32_t C_out,
                                        int32_t stride, size_t* out_bytes);
pm_status pm_conv3x3_bwd_weight(void* stream, int32_t dtype, int32_t B, int32_t H, int32_t W, int32_t C_in, int32_t C_out,
                                int32_t stride, const void* dz_dev, const void* x_dev, float* dW_dev, void* scratch_dev,
                                size_t scratch_bytes);

/* pm_conv3x3_bwd_weight for callers that cannot allocate device memory or bring a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the per-block partial results go
 * to a fixed array inside the library (pm_static_scratch_bytes: 16 MiB, held once per GPU the library runs
 * on until the process ends) instead of a caller-provided workspace.  Same arguments, layouts and results as
 * pm_conv3x3_bwd_weight otherwise (dW overwritten).  Calls no allocating routine.  A shape whose partial
 * results exceed the array (pm_conv3x3_bwd_weight_scratch reports the need) is rejected with PM_ENOMEM and
 * nothing is launched.  The device current in the calling thread must be the one the pointers and the
 * stream belong to; the first call on a device looks up the array's address there (make one call before
 * capturing a graph).  All calls on one GPU share the array: two calls whose kernels overlap in time (on
 * different streams) race; calls on one stream are ordered. */
pm_status pm_static_scratch_bytes(size_t* out_bytes);
pm_status pm_conv3x3_bwd_weight_static(void* stream, int32_t dtype, int32_t B, int32_t H, int32_t W, int32_t C_in,
                                       int32_t C_out, int32_t stride, const void* dz_dev, const void* x_dev,
                                       float* dW_dev);

/* Waits for everything the context has enqueued, on the caller's stream and on the library's
 * second stream (overlap_update). */
pm_status pm_synchronize(pm_ctx* ctx);

/* Checkpoint / resume of the training state (the paper's method has none of its own; the state of
 * the recurrences of Sec. 2 and Sec. 3.2 is what must survive): step counter, fp32 master weights,
 * optimizer moments, delta accumulator, every ring slot, the corrected backward (and recompute) weights.
 * pm_checkpoint_bytes: size in bytes of the image (host, out).
 * pm_checkpoint_save: writes the image to dst_host (host memory, caller-owned, `bytes` as returned above;
 *   PM_EINVAL if smaller).  PM_ESTATE in the middle of a minibatch.  Synchronises.
 * pm_checkpoint_load: restores a context created with the SAME layers, delays, dtype and options from an
 *   image (PM_EINVAL if the image does not match the context's layout or is truncated).  The next
 *   pm_step continues bit-identically to the run that saved.  Synchronises. */
pm_status pm_checkpoint_bytes(pm_ctx* ctx, size_t* bytes);
pm_status pm_checkpoint_save(pm_ctx* ctx, void* dst_host, size_t bytes);
pm_status pm_checkpoint_load(pm_ctx* ctx, const void* src_host, size_t bytes);

/* Frees host state only; the arena stays the caller's. */
void pm_destroy(pm_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* PIPEMARE_H_ */
