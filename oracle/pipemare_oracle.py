"""Plain fp64 CPU oracle for the PipeMare asynchronous pipeline-parallel training step.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file: it is for
tests, the smoke check and the benchmark's CPU-baseline leg.  It shares no code with the
HIP library and is deliberately slow and literal: explicit, version-indexed weight
histories (never a ring buffer), no fusion, no blocking, NumPy fp64 throughout.

What it computes, with the paper passages it follows:
  * delay model  w_{t+1} = w_t - alpha * grad f_t(u_fwd,t, u_bkwd,t) with per-stage delayed
    reads (u_fwd,t)_i = (w_{t - tau_fwd,i})_i, (u_bkwd,t)_i = (w_{t - tau_bkwd,i})_i      [Sec. 2.1]
  * per-method delays tau_fwd,i = ceil((2(P-i)+1)/N), tau_bkwd,i = 0 | tau_fwd,i | 0      [Sec. 2.2, Table 1]
  * T1 learning-rate rescheduling alpha_{k,i} = alpha_{k,base} / tau_i^{p_k},
    p_k = 1 - min(k/K, 1)                                                                 [Sec. 3.1, T1]
  * T2 discrepancy correction u_bkwd = w_{t-tau_bkwd} - (tau_fwd - tau_bkwd) * delta_t,
    delta_{t+1} = gamma*delta_t + (1-gamma)(w_{t+1}-w_t), gamma = D^{1/(tau_fwd-tau_bkwd)} [Sec. 3.2, T2]
  * SGD with momentum in the paper's form v <- beta v - alpha g, w <- w + v               [App. B.3]
  * AdamW (decoupled weight decay) as the Transformer experiments' base optimizer         [App. C, Transformer table]
  * backpropagation with two weight sets: forward with u_fwd, data-gradient path with u_bkwd [Sec. 2.1]
  * recomputation: activations inside a segment of stages are rebuilt in the backward pass from the
    segment's stored input with a third weight set (u_recomp,t)_i = (w_{t - tau_recomp,i})_i, corrected
    like u_bkwd: minus (tau_fwd,i - tau_recomp,i) * delta_t       [App. "Statistical efficiency and recompute"]
    with tau_recomp,i = tau_bkwd,i + ceil(2 (S - j) / N) for the j-th of the S stages of a segment
                                                                  [App. "PipeMare Recompute"]

  * Hogwild-style stochastic delays: every step draws a delay per stage from an exponential
    distribution truncated at tau_max, stages differing in its mean; T1 uses the mean  [App. "Hogwild! asynchrony"]

Readings where the paper is silent (documented in the design notes of the repository):
versions before step 0 clamp to w_0; stages are 1-based; tau_i in T1 is tau_fwd,i and
max(tau_i,1) is used so that tau=0 gives scale 1; step counter k is 0-based; delta_0 = v_0 = 0;
tau_fwd == tau_bkwd gives correction coefficient 0; the correction always uses the
current delta_t.

Pins (tests/test_oracle_*.py): synchronous special case vs autograd + textbook optimizers,
equal-delay special case, the stability threshold of Lemma 1 from both sides, the
momentum and T2 characteristic polynomials as annihilators of the oracle's trajectory,
T1 closed form, delay tables, hand-worked scalar recurrences (incl. the l2 term and the global
gradient-norm clip, each also against torch's own routine), finite differences and an
autograd construction of the two-weight gradient.
Parity unpinned: the T2 correction with tau_bkwd > 0, and the recompute correction with
tau_recomp > 0 (in both the paper's text uses the current delta_t while its appendix polynomials
correspond to a delayed delta; the text is followed and pinned against the polynomial derived from it); the inverse-square-root tail of the warmup
schedule (the paper only gives the warmup part).
"""
from __future__ import annotations

import math
from typing import Callable, List, Sequence

import numpy as np

try:  # erf for exact GELU
    from scipy.special import erf as _erf
except Exception:  # pragma: no cover
    _erf = np.vectorize(math.erf)


# --------------------------------------------------------------------------- delays (Sec. 2.2)
def pipeline_delays(P: int, N: int = 1, method: str = "pipemare"):
    """Per-stage (tau_fwd, tau_bkwd) lists for stages i = 1..P (returned 0-indexed by i-1)."""
    if P < 1 or N < 1:
        raise ValueError("P >= 1 and N >= 1 required")
    if method == "gpipe":
        return [0] * P, [0] * P
    tau_fwd = [-((-(2 * (P - i) + 1)) // N) for i in range(1, P + 1)]   # integer ceiling
    if method == "pipemare":
        return tau_fwd, [0] * P
    if method == "pipedream":
        return tau_fwd, list(tau_fwd)
    raise ValueError(method)


def recompute_delays(P: int, S: int, N: int = 1, tau_bkwd=None):
    """tau_recomp per stage (index i-1) when the P stages are cut into segments of S consecutive stages
    (the last one may be shorter): the j-th stage of a segment with S' stages recomputes 2 (S' - j)
    microbatch slots before its backward pass (App. "PipeMare Recompute"), i.e.
    tau_recomp,i = tau_bkwd,i + ceil(2 (S' - j) / N)."""
    if P < 1 or S < 1 or N < 1:
        raise ValueError("P, S, N >= 1 required")
    tb = [0] * P if tau_bkwd is None else list(tau_bkwd)
    out = []
    for i in range(1, P + 1):
        first = ((i - 1) // S) * S + 1
        size = min(S, P - first + 1)
        j = i - first + 1
        out.append(tb[i - 1] + -((-2 * (size - j)) // N))
    return out


def segment_starts(P: int, S: int):
    """First stage (1-based) of every segment."""
    return list(range(1, P + 1, S))


# --------------------------------------------------------------------------- stochastic delays (App. "Hogwild! asynchrony")
_M64 = (1 << 64) - 1


def counter_u32(seed: int, t: int, i: int, P: int) -> int:
    """32 random bits for (step t, stage i of P), a pure function of its arguments: output number
    t*P + i of the SplitMix64 generator (Steele, Lea, Flood 2014) started at `seed`, upper half."""
    z = (seed + (t * P + i) * 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    z ^= z >> 31
    return z >> 32


def delay_thresholds(mean: float, tau_max: int):
    """Integer inverse-CDF table of the delay of one stage: X ~ Exp(mean) truncated to [0, tau_max + 1),
    delay = floor(X) in {0..tau_max}.  P(delay <= k) = (1 - e^{-(k+1)/mean}) / (1 - e^{-(tau_max+1)/mean});
    T[k] = min(floor(2^32 P(delay <= k)), 2^32 - 1) for k = 0..tau_max-1.  mean <= 0: always delay 0."""
    if tau_max < 0:
        raise ValueError("tau_max >= 0 required")
    if mean <= 0:
        return [0xFFFFFFFF] * tau_max
    norm = 1.0 - math.exp(-(tau_max + 1) / mean)
    return [min(int(math.floor((1.0 - math.exp(-(k + 1) / mean)) / norm * 4294967296.0)), 0xFFFFFFFF)
            for k in range(tau_max)]


def delay_from_u32(r: int, thresholds) -> int:
    """delay = number of table entries the draw exceeds (the table is non-decreasing)."""
    return sum(1 for T in thresholds if r > T)


def stochastic_delay(seed: int, t: int, i: int, P: int, thresholds) -> int:
    """Delay of stage i (1-based) at step t."""
    return delay_from_u32(counter_u32(seed, t, i, P), thresholds)


def gpipe_utilization(N: int, P: int) -> float:
    """Fraction of busy stages for fill-and-drain pipelining (Sec. 2.2)."""
    return N / (N + P - 1)


def pipedream_stash_elems(sizes: Sequence[int], tau_fwd: Sequence[int]) -> int:
    """Extra weight copies kept by weight stashing: sum_i |w_i| * tau_fwd,i (Sec. 2.2)."""
    return int(sum(n * t for n, t in zip(sizes, tau_fwd)))


# --------------------------------------------------------------------------- T1 (Sec. 3.1)
def t1_exponent(k: int, K: int) -> float:
    """p_k = 1 - min(k/K, 1); K = 0 means no rescheduling (p = 0)."""
    if K <= 0:
        return 0.0
    return 1.0 - min(k / K, 1.0)


def t1_lr(alpha_base: float, tau: int, k: int, K: int) -> float:
    """alpha_{k,i} = alpha_{k,base} / tau_i^{p_k}, with tau_i = 0 treated as 1."""
    return alpha_base / (float(max(tau, 1)) ** t1_exponent(k, K))


def base_lr(sched: dict, k: int) -> float:
    """The synchronous schedule alpha_{k,base}.

    {"kind": "const", "base": a}
    {"kind": "step", "base": a, "factor": f, "interval": S}      a * f^floor(k/S)   (ResNet-style drops)
    {"kind": "warmup_invsqrt", "base": a_max, "init": a0, "warmup": W}
        linear from a0 to a_max over W steps, then a_max*sqrt(W/k)  (Transformer-style)
    """
    kind = sched["kind"]
    if kind == "const":
        return float(sched["base"])
    if kind == "step":
        return float(sched["base"]) * float(sched["factor"]) ** (k // int(sched["interval"]))
    if kind == "warmup_invsqrt":
        W = int(sched["warmup"])
        a0, a1 = float(sched["init"]), float(sched["base"])
        if k < W:
            return a0 + (a1 - a0) * (k / W)
        return a1 * math.sqrt(W / k) if k > 0 else a1
    raise ValueError(kind)


# --------------------------------------------------------------------------- T2 (Sec. 3.2)
def t2_gamma(D: float, tau_fwd: int, tau_bkwd: int) -> float:
    """gamma_i = D^{1/(tau_fwd,i - tau_bkwd,i)}; no discrepancy -> 0 (value unused)."""
    d = tau_fwd - tau_bkwd
    return float(D) ** (1.0 / d) if d > 0 else 0.0


def t2_decay_from_gamma(gamma: float, tau_fwd: int, tau_bkwd: int) -> float:
    """D = gamma^(tau_fwd - tau_bkwd) (App. B, end of the T2 analysis)."""
    return gamma ** (tau_fwd - tau_bkwd)


# --------------------------------------------------------------------------- models
class QuadraticModel:
    """The paper's one-dimensional analysis model, one scalar weight per stage.

    grad_i = (lam + Delta) * u_fwd,i - Delta * u_bkwd,i - eta_t   (Sec. 3.2; Delta = 0 gives Sec. 3's model)
    With recomputation (App. "Statistical efficiency and recompute") a third term with sensitivity Phi:
    grad_i = (lam + Delta) * u_fwd,i - (Delta - Phi) * u_bkwd,i - Phi * u_recomp,i - eta_t.
    The 'batch' passed to the step is the noise sample eta_t (scalar or per-stage array).
    """

    def __init__(self, n_stages: int, lam: float = 1.0, Delta: float = 0.0, Phi: float = 0.0):
        self.n = n_stages
        self.lam, self.Delta, self.Phi = float(lam), float(Delta), float(Phi)

    def loss_and_grads(self, u_fwd, u_bkwd, eta, u_recomp=None, checkpoints=None):
        eta = np.broadcast_to(np.asarray(0.0 if eta is None else eta, dtype=np.float64), (self.n,))
        u_r = u_bkwd if u_recomp is None else u_recomp
        grads = [(self.lam + self.Delta) * u_fwd[i] - (self.Delta - self.Phi) * u_bkwd[i] - self.Phi * u_r[i] - eta[i]
                 for i in range(self.n)]
        loss = 0.5 * self.lam * float(sum(np.sum(u ** 2) for u in u_fwd))
        return loss, grads


def _act(z, kind):
    if kind == "none":
        return z
    if kind == "relu":
        return np.maximum(z, 0.0)
    if kind == "gelu":   # exact (erf) form
        return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))
    raise ValueError(kind)


def _act_grad(z, kind):
    if kind == "none":
        return np.ones_like(z)
    if kind == "relu":
        return (z > 0.0).astype(z.dtype)
    if kind == "gelu":
        return 0.5 * (1.0 + _erf(z / math.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)
    raise ValueError(kind)


class MLPModel:
    """Chain of Linear(+bias)+activation layers with an MSE or softmax cross-entropy loss.

    Layer l has a packed parameter vector [W (n_out x n_in row-major) | b (n_out)].
    loss_and_grads(u_fwd, u_bkwd, (x, y)) returns the gradient that backpropagation produces
    when the forward pass uses u_fwd and the backward pass uses u_bkwd (Sec. 2.1): activations
    and activation-derivative masks come from the forward pass; the only place the backward
    pass reads a weight is the data-gradient product dz @ W, which uses u_bkwd.
    """

    def __init__(self, layers, loss="mse"):
        # layers: sequence of objects with n_in, n_out, act
        self.layers = list(layers)
        self.loss_kind = loss

    def unpack(self, p, l):
        L = self.layers[l]
        nw = L.n_out * L.n_in
        return p[:nw].reshape(L.n_out, L.n_in), p[nw:nw + L.n_out]

    def forward(self, params, x):
        a = np.asarray(x, dtype=np.float64)
        acts, zs = [a], []
        for l, L in enumerate(self.layers):
            W, b = self.unpack(params[l], l)
            z = a @ W.T + b
            a = _act(z, L.act)
            zs.append(z)
            acts.append(a)
        return acts, zs

    @staticmethod
    def loss_and_dout(out, y, loss):
        M = out.shape[0]
        if loss == "mse":       # mean over every output element
            y = np.asarray(y, dtype=np.float64).reshape(out.shape)
            diff = out - y
            return float(np.mean(diff ** 2)), 2.0 * diff / diff.size
        if loss == "xent":      # mean over rows of -log softmax[label]
            y = np.asarray(y).astype(np.int64)
            zmax = out.max(axis=1, keepdims=True)
            e = np.exp(out - zmax)
            p = e / e.sum(axis=1, keepdims=True)
            lse = np.log(e.sum(axis=1)) + zmax[:, 0]
            val = float(np.mean(lse - out[np.arange(M), y]))
            d = p.copy()
            d[np.arange(M), y] -= 1.0
            return val, d / M
        raise ValueError(loss)

    def loss_and_grads(self, u_fwd, u_bkwd, batch, u_recomp=None, checkpoints=None):
        """checkpoints (with u_recomp): indices of the layers whose INPUT the forward pass keeps (the
        first layer of every segment; 0 is always one).  Everything else the backward pass needs -
        the inputs and pre-activations of the layers inside a segment - is rebuilt from the segment's
        kept input with the weights u_recomp.  The loss and its gradient come from the forward pass."""
        x, y = batch
        acts, zs = self.forward(u_fwd, x)
        loss, da = self.loss_and_dout(acts[-1], y, self.loss_kind)
        if u_recomp is not None:
            cps = sorted(set([0] + [int(c) for c in (checkpoints or [])]))
            nL = len(self.layers)
            acts_r, zs_r = list(acts), list(zs)
            for si, s0 in enumerate(cps):
                s1 = cps[si + 1] if si + 1 < len(cps) else nL
                a = acts[s0]                                   # kept by the forward pass
                for l in range(s0, s1):
                    W, b = self.unpack(u_recomp[l], l)
                    acts_r[l] = a
                    zs_r[l] = a @ W.T + b
                    a = _act(zs_r[l], self.layers[l].act)
            acts, zs = acts_r, zs_r
        grads = [None] * len(self.layers)
        for l in range(len(self.layers) - 1, -1, -1):
            L = self.layers[l]
            dz = da * _act_grad(zs[l], L.act)
            dW = dz.T @ acts[l]
            db = dz.sum(axis=0)
            grads[l] = np.concatenate([dW.ravel(), db])
            Wb, _ = self.unpack(u_bkwd[l], l)
            da = dz @ Wb
        return loss, grads


# --------------------------------------------------------------------------- the recurrence
class PipeMareOracle:
    """Delayed-gradient recurrence over explicit weight histories.

    model          object with loss_and_grads(u_fwd, u_bkwd, batch) -> (loss, [grad per unit])
    w0             list of initial parameter vectors, one per weight unit
    stage_of_unit  1-based pipeline stage of every unit
    tau_fwd/bkwd   per-stage delays, index i-1 for stage i
    opt            dict: kind "sgdm" | "adamw"; beta (sgdm); beta1, beta2, eps (adamw);
                   weight_decay; clip_norm (0 = off); D; gamma_override (list per stage or None);
                   K; t1 (bool); t2 (bool); sched (dict for base_lr); N (microbatches);
                   sync_warmup (int E_w >= 0): the first E_w steps run synchronously (all delays 0,
                   base step size: "PipeMareW", Sec. 4), after which the delays apply and the T1
                   counter starts at 0; delta keeps accumulating during the warm-up;
                   tau_recomp (list per stage, or None = no recomputation) and segment (stages per
                   segment): the backward pass rebuilds activations with u_recomp (see the header);
                   stochastic (None, or dict(tau_max, seed)): Hogwild-style delays - at every step each
                   stage i draws a delay from the exponential with mean tau_fwd,i truncated at tau_max,
                   and both passes read that version of its weights (no forward/backward discrepancy,
                   hence no T2); T1 keeps dividing by the mean tau_fwd,i; tau_bkwd is ignored
    keep_history   True keeps every version; False drops versions no delay can reach any more
                   (still indexed by absolute version number).
    """

    def __init__(self, model, w0, stage_of_unit, tau_fwd, tau_bkwd, opt, keep_history=False):
        self.model = model
        self.U = len(w0)
        self.stage = [int(s) for s in stage_of_unit]
        self.tau_fwd = [int(t) for t in tau_fwd]
        self.tau_bkwd = [int(t) for t in tau_bkwd]
        for tf, tb in zip(self.tau_fwd, self.tau_bkwd):
            if tb < 0 or tb > tf:
                raise ValueError("need 0 <= tau_bkwd <= tau_fwd")
        o = dict(kind="sgdm", beta=0.0, beta1=0.9, beta2=0.98, eps=1e-8, weight_decay=0.0,
                 clip_norm=0.0, D=1.0, gamma_override=None, K=0, t1=True, t2=True,
                 sched=dict(kind="const", base=0.1), N=1, sync_warmup=0, tau_recomp=None, segment=0,
                 stochastic=None)
        o.update(opt)
        self.opt = o
        self.stoch = None
        if o["stochastic"] is not None:
            if o["tau_recomp"] is not None:
                raise ValueError("stochastic delays and recomputation are not combined")
            tm, P_ = int(o["stochastic"]["tau_max"]), len(self.tau_fwd)
            self.stoch = dict(tau_max=tm, seed=int(o["stochastic"]["seed"]),
                              tables=[delay_thresholds(float(m), tm) for m in self.tau_fwd])
            self.last_delays = [0] * P_
        self.tau_recomp = None
        self.checkpoints = None
        if o["tau_recomp"] is not None:
            self.tau_recomp = [int(t) for t in o["tau_recomp"]]
            for tf, tb, tr in zip(self.tau_fwd, self.tau_bkwd, self.tau_recomp):
                if tr < tb or tr > tf:
                    raise ValueError("need tau_bkwd <= tau_recomp <= tau_fwd")
            if int(o["segment"]) < 1:
                raise ValueError("recomputation needs segment >= 1 (stages per segment)")
            starts = set(segment_starts(len(self.tau_fwd), int(o["segment"])))
            # a unit opens a segment if it is the first unit of a stage that opens one
            self.checkpoints = [u for u in range(self.U)
                                if self.stage[u] in starts and (u == 0 or self.stage[u - 1] != self.stage[u])]
        self.keep_history = keep_history
        self.t = 0
        self.hist = [{0: np.array(w, dtype=np.float64).copy()} for w in w0]
        self.delta = [np.zeros_like(h[0]) for h in self.hist]
        self.v = [np.zeros_like(h[0]) for h in self.hist]      # momentum / Adam first moment
        self.s = [np.zeros_like(h[0]) for h in self.hist]      # Adam second moment
        self.last_lr = [0.0] * self.U
        self.last_versions = [(0, 0)] * self.U
        self.last_grads = None          # the gradients the most recent update consumed (after averaging and clipping)

    # -- helpers
    def _tf(self, u): return self.tau_fwd[self.stage[u] - 1]
    def _tb(self, u): return self.tau_bkwd[self.stage[u] - 1]

    def gamma(self, u):
        go = self.opt["gamma_override"]
        if go is not None:
            return float(go[self.stage[u] - 1])
        return t2_gamma(self.opt["D"], self._tf(u), self._tb(u))

    def weights(self, u=None):
        if u is None:
            return [h[self.t] for h in self.hist]
        return self.hist[u][self.t]

    def read_versions(self, t=None):
        """(forward version, backward version) per unit at step t: max(t - tau, 0); the current
        version t for both during the synchronous warm-up."""
        t = self.t if t is None else t
        if t < self.opt["sync_warmup"]:
            return [(t, t)] * self.U
        if self.stoch is not None:
            P_ = len(self.tau_fwd)
            d = [stochastic_delay(self.stoch["seed"], t, i, P_, self.stoch["tables"][i - 1]) for i in range(1, P_ + 1)]
            self.last_delays = d
            return [(max(t - d[self.stage[u] - 1], 0),) * 2 for u in range(self.U)]
        return [(max(t - self._tf(u), 0), max(t - self._tb(u), 0)) for u in range(self.U)]

    # -- one optimizer step
    def step(self, batch):
        """One minibatch.  `batch` is a single microbatch, or a list of N microbatches whose
        gradients are averaged (all computed with the same delayed weights, Sec. 2.1)."""
        o, t = self.opt, self.t
        warm = t < o["sync_warmup"]
        vers = self.read_versions(t)
        self.last_versions = vers
        u_fwd = [self.hist[u][vers[u][0]] for u in range(self.U)]
        u_bkwd = []
        for u in range(self.U):
            base = self.hist[u][vers[u][1]]
            d = self._tf(u) - self._tb(u)
            if o["t2"] and d > 0 and not warm and self.stoch is None:
                base = base - d * self.delta[u]
            u_bkwd.append(base)
        extra = {}
        if self.tau_recomp is not None:
            u_rec = []
            for u in range(self.U):
                tr = 0 if warm else self.tau_recomp[self.stage[u] - 1]
                base = self.hist[u][max(t - tr, 0)]
                d = self._tf(u) - tr
                if o["t2"] and d > 0 and not warm:
                    base = base - d * self.delta[u]
                u_rec.append(base)
            extra = dict(u_recomp=u_rec, checkpoints=self.checkpoints)

        mbs = batch if isinstance(batch, list) else [batch]
        loss, grads = 0.0, None
        for mb in mbs:
            l_, g_ = self.model.loss_and_grads(u_fwd, u_bkwd, mb, **extra)
            loss += l_ / len(mbs)
            g_ = [np.asarray(g, dtype=np.float64) / len(mbs) for g in g_]
            grads = g_ if grads is None else [a + b for a, b in zip(grads, g_)]

        if o["clip_norm"] > 0.0:
            gn = math.sqrt(sum(float(np.sum(g * g)) for g in grads))
            scale = min(1.0, o["clip_norm"] / gn) if gn > 0.0 else 1.0
            grads = [g * scale for g in grads]

        self.last_grads = grads
        a_base = base_lr(o["sched"], t)
        for u in range(self.U):
            w = self.hist[u][t]
            lr = t1_lr(a_base, self._tf(u), t - o["sync_warmup"], o["K"]) if (o["t1"] and not warm) else a_base
            self.last_lr[u] = lr
            g = grads[u]
            if o["kind"] == "sgdm":
                g = g + o["weight_decay"] * w
                self.v[u] = o["beta"] * self.v[u] - lr * g
                w_new = w + self.v[u]
            elif o["kind"] == "adamw":
                b1, b2 = o["beta1"], o["beta2"]
                self.v[u] = b1 * self.v[u] + (1.0 - b1) * g
                self.s[u] = b2 * self.s[u] + (1.0 - b2) * g * g
                mhat = self.v[u] / (1.0 - b1 ** (t + 1))
                shat = self.s[u] / (1.0 - b2 ** (t + 1))
                w_new = w - lr * (mhat / (np.sqrt(shat) + o["eps"]) + o["weight_decay"] * w)
            else:
                raise ValueError(o["kind"])
            gam = self.gamma(u)
            self.delta[u] = gam * self.delta[u] + (1.0 - gam) * (w_new - w)
            self.hist[u][t + 1] = w_new
            if not self.keep_history:
                oldest = t + 1 - (self._tf(u) if self.stoch is None else self.stoch["tau_max"])
                for ver in [k for k in self.hist[u] if k < oldest]:
                    del self.hist[u][ver]
        self.t = t + 1
        return loss
