"""fp64 CPU oracle model: fine-grained pre-LN Transformer (decoder-style, causal) with the
two-weight backward of asynchronous pipeline parallelism.

TEST INFRASTRUCTURE ONLY (same rules as pipemare_oracle.py: nothing in the product path may
import it; it shares no code with the HIP library).

It plugs into pipemare_oracle.PipeMareOracle as `model`: loss_and_grads(u_fwd, u_bkwd, batch)
returns the gradient that backpropagation produces when the forward pass uses the weights
u_fwd and the backward pass uses u_bkwd (Sec. 2.1); with u_recomp the activations inside every
segment of stages are rebuilt in the backward pass with a third weight set (App. "Statistical
efficiency and recompute"; see loss_and_grads).  Activations, normalisation statistics,
attention probabilities and activation-derivative masks come from the forward pass; the
backward pass reads a weight only where a gradient flows *through* it to earlier layers:
  * Linear:     dA = dZ @ W_bkwd                (dW = dZ^T A and db use stored activations)
  * LayerNorm:  d(xhat) = dY * gain_bkwd        (d gain, d bias use the stored xhat)
  * Embedding:  nothing earlier, so u_bkwd is unused
Weight-free operators (attention core, softmax, residual adds, positions) have one gradient.

Weight units, in topological order (the paper's partition rule: weight + bias of a layer are one
unit; Sec. 4.1 "Pipeline Stages"), each a packed fp64 vector:
  unit 0                     embedding            [E (vocab x d)]
  per layer, 8 units         ln1 [g | b], Wq, Wk, Wv, Wo, ln2 [g | b], W1, W2   (Linear: [W (out x in) | b])
  last 2 units               final ln [g | b], head [W (vocab x d) | b]
The stage of every unit is the caller's choice (a LayerNorm normally shares its consumer's stage).

Architecture readings (the paper names only "12-layer Transformer"; the workload text fixes the
sizes): pre-LN, causal mask, sinusoidal (weight-free) positions, untied output head, ReLU
feed-forward, no dropout, no label smoothing, LayerNorm eps 1e-5, loss = mean token cross-entropy.
"""
from __future__ import annotations

import math

import numpy as np

LN_EPS = 1e-5


def sinusoidal_positions(S: int, d: int) -> np.ndarray:
    """pos[s, 2i] = sin(s / 10000^(2i/d)), pos[s, 2i+1] = cos(s / 10000^(2i/d))."""
    pos = np.zeros((S, d))
    s = np.arange(S)[:, None]
    i = np.arange(0, d, 2)[None, :]
    ang = s / np.power(10000.0, i / d)
    pos[:, 0::2] = np.sin(ang)
    pos[:, 1::2] = np.cos(ang)
    return pos


def _ln_fwd(x, g, b):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xhat = (x - mu) * rstd
    return xhat * g + b, xhat, rstd


def _ln_bwd(dy, xhat, rstd, g_bkwd):
    """Returns (dx through the backward gain, d gain, d bias)."""
    dg = (dy * xhat).sum(axis=0)
    db = dy.sum(axis=0)
    dxh = dy * g_bkwd
    dx = rstd * (dxh - dxh.mean(axis=-1, keepdims=True) - xhat * (dxh * xhat).mean(axis=-1, keepdims=True))
    return dx, dg, db


class TransformerModel:
    def __init__(self, n_layers: int, d_model: int, n_heads: int, d_ff: int, vocab: int, seq: int):
        assert d_model % n_heads == 0
        self.nl, self.d, self.h, self.dff, self.V, self.S = n_layers, d_model, n_heads, d_ff, vocab, seq
        self.dh = d_model // n_heads
        self.pos = sinusoidal_positions(seq, d_model)
        self.n_units = 1 + 8 * n_layers + 2

    # ---- unit bookkeeping
    def unit_sizes(self):
        d, dff, V = self.d, self.dff, self.V
        sizes = [V * d]
        for _ in range(self.nl):
            sizes += [2 * d, d * d + d, d * d + d, d * d + d, d * d + d, 2 * d, dff * d + dff, d * dff + d]
        sizes += [2 * d, V * d + V]
        return sizes

    @staticmethod
    def _lin(p, n_out, n_in):
        return p[:n_out * n_in].reshape(n_out, n_in), p[n_out * n_in:n_out * n_in + n_out]

    def _ln(self, p):
        return p[:self.d], p[self.d:2 * self.d]

    def _attention_fwd(self, q, k, v, B):
        S, H, dh = self.S, self.h, self.dh
        q4 = q.reshape(B, S, H, dh).transpose(0, 2, 1, 3)
        k4 = k.reshape(B, S, H, dh).transpose(0, 2, 1, 3)
        v4 = v.reshape(B, S, H, dh).transpose(0, 2, 1, 3)
        sc = q4 @ k4.transpose(0, 1, 3, 2) / math.sqrt(dh)
        mask = np.triu(np.ones((S, S), dtype=bool), k=1)
        sc = np.where(mask, -np.inf, sc)
        sc = sc - sc.max(axis=-1, keepdims=True)
        p = np.exp(sc)
        p = p / p.sum(axis=-1, keepdims=True)
        o4 = p @ v4
        return o4.transpose(0, 2, 1, 3).reshape(B * S, H * dh), (q4, k4, v4, p)

    def _attention_bwd(self, do, cache, B):
        S, H, dh = self.S, self.h, self.dh
        q4, k4, v4, p = cache
        do4 = do.reshape(B, S, H, dh).transpose(0, 2, 1, 3)
        dv4 = p.transpose(0, 1, 3, 2) @ do4
        dp = do4 @ v4.transpose(0, 1, 3, 2)
        ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
        ds = ds / math.sqrt(dh)
        dq4 = ds @ k4
        dk4 = ds.transpose(0, 1, 3, 2) @ q4
        back = lambda t: t.transpose(0, 2, 1, 3).reshape(B * S, H * dh)
        return back(dq4), back(dk4), back(dv4)

    # ---- one weight unit's share of the forward pass (with the weight-free operators that ride in its stage)
    def _unit_forward(self, u, p, get, B):
        """Tensors unit u produces from the tensors it reads through get(name).  Residual stream into layer l:
        x{l}; inside layer l: xh1_, rs1_, n1_ (ln1) | q_ | k_ | v_ | o_, att_ (attention core: it rides with the
        output projection, the unit that consumes it), h_ (Wo) | xh2_, rs2_, n2_ (ln2) | z1_, f_ (W1) |
        x{l+1} (W2); then xhf, rsf, nf (final ln).  The head is not a producer here (its logits feed the loss)."""
        d, dff, V = self.d, self.dff, self.V
        if u == 0:
            E = p.reshape(V, d)
            return {"x0": E[get("tokens").reshape(-1)] + np.tile(self.pos, (B, 1))}
        if u == 1 + 8 * self.nl:
            gf, bf = self._ln(p)
            nf, xhf, rsf = _ln_fwd(get(f"x{self.nl}"), gf, bf)
            return {"nf": nf, "xhf": xhf, "rsf": rsf}
        l, j = divmod(u - 1, 8)
        t = lambda name: f"{name}_{l}"
        if j == 0:
            g1, b1 = self._ln(p)
            n1, xh1, rs1 = _ln_fwd(get(f"x{l}"), g1, b1)
            return {t("n1"): n1, t("xh1"): xh1, t("rs1"): rs1}
        if j in (1, 2, 3):
            W, b = self._lin(p, d, d)
            return {t("qkv"[j - 1]): get(t("n1")) @ W.T + b}
        if j == 4:
            o, acache = self._attention_fwd(get(t("q")), get(t("k")), get(t("v")), B)
            Wo, bo = self._lin(p, d, d)
            return {t("o"): o, t("att"): acache, t("h"): get(f"x{l}") + o @ Wo.T + bo}
        if j == 5:
            g2, b2 = self._ln(p)
            n2, xh2, rs2 = _ln_fwd(get(t("h")), g2, b2)
            return {t("n2"): n2, t("xh2"): xh2, t("rs2"): rs2}
        if j == 6:
            W1, bb1 = self._lin(p, dff, d)
            z1 = get(t("n2")) @ W1.T + bb1
            return {t("z1"): z1, t("f"): np.maximum(z1, 0.0)}
        W2, bb2 = self._lin(p, d, dff)
        return {f"x{l + 1}": get(t("h")) + get(t("f")) @ W2.T + bb2}

    # ---- the two-weight gradient (three-weight with recomputation)
    def loss_and_grads(self, u_fwd, u_bkwd, batch, u_recomp=None, checkpoints=None):
        """checkpoints (with u_recomp): indices of the units that open a segment (0 is always one).  The forward
        pass is taken to keep only the tensors that cross a segment boundary; in the backward pass every
        segment's units first run again, in order, with the weights u_recomp - reading kept forward tensors
        where the producer sits in an earlier segment and rebuilt ones where it sits in the same segment -
        and a unit's backward then uses, for every stored tensor it needs, the rebuilt value if that tensor was
        produced in the unit's own segment and the kept forward value otherwise.  The loss and its gradient
        come from the forward pass (the head is not rebuilt).  Data gradients use u_bkwd as always."""
        tokens, targets = batch
        tokens = np.asarray(tokens).astype(np.int64)
        targets = np.asarray(targets).astype(np.int64).reshape(-1)
        B = tokens.shape[0]
        d, dff, V, S = self.d, self.dff, self.V, self.S
        T = B * S
        F, Bk = u_fwd, u_bkwd
        nU = self.n_units
        uf = 1 + 8 * self.nl
        grads = [None] * nU

        # ---------------- forward with u_fwd
        fwd = {"tokens": tokens}
        for u in range(nU - 1):
            fwd.update(self._unit_forward(u, F[u], fwd.__getitem__, B))
        Wh, bh = self._lin(F[uf + 1], V, d)
        logits = fwd["nf"] @ Wh.T + bh
        zmax = logits.max(axis=1, keepdims=True)
        ex = np.exp(logits - zmax)
        prob = ex / ex.sum(axis=1, keepdims=True)
        loss = float(np.mean(np.log(ex.sum(axis=1)) + zmax[:, 0] - logits[np.arange(T), targets]))

        # ---------------- recomputation: every segment's units again with u_recomp
        if u_recomp is None:
            def view(c, name):
                return fwd[name]
        else:
            cps = sorted(set([0] + [int(c) for c in (checkpoints or [])]))
            seg_of = [sum(1 for c in cps if c <= u) - 1 for u in range(nU)]
            rebuilt = [dict() for _ in cps]
            for u in range(nU - 1):
                mine = rebuilt[seg_of[u]]
                mine.update(self._unit_forward(
                    u, u_recomp[u], lambda name, mine=mine: mine[name] if name in mine else fwd[name], B))

            def view(c, name):
                mine = rebuilt[seg_of[c]]
                return mine[name] if name in mine else fwd[name]

        # ---------------- backward: stored (or rebuilt) quantities, weights from u_bkwd on the data path
        dlog = prob
        dlog[np.arange(T), targets] -= 1.0
        dlog = dlog / T
        grads[uf + 1] = np.concatenate([(dlog.T @ view(uf + 1, "nf")).ravel(), dlog.sum(axis=0)])
        Wh_b, _ = self._lin(Bk[uf + 1], V, d)
        dnf = dlog @ Wh_b
        gf_b, _ = self._ln(Bk[uf])
        dx, dg, db = _ln_bwd(dnf, view(uf, "xhf"), view(uf, "rsf"), gf_b)
        grads[uf] = np.concatenate([dg, db])
        for l in range(self.nl - 1, -1, -1):
            u = 1 + 8 * l
            t = lambda name: f"{name}_{l}"
            # y = h + f W2^T + b
            grads[u + 7] = np.concatenate([(dx.T @ view(u + 7, t("f"))).ravel(), dx.sum(axis=0)])
            W2_b, _ = self._lin(Bk[u + 7], d, dff)
            df = dx @ W2_b
            dz1 = df * (view(u + 6, t("z1")) > 0.0)
            grads[u + 6] = np.concatenate([(dz1.T @ view(u + 6, t("n2"))).ravel(), dz1.sum(axis=0)])
            W1_b, _ = self._lin(Bk[u + 6], dff, d)
            dn2 = dz1 @ W1_b
            g2_b, _ = self._ln(Bk[u + 5])
            dh_ln, dg, db = _ln_bwd(dn2, view(u + 5, t("xh2")), view(u + 5, t("rs2")), g2_b)
            grads[u + 5] = np.concatenate([dg, db])
            dh = dx + dh_ln
            # h = x + o Wo^T + b
            grads[u + 4] = np.concatenate([(dh.T @ view(u + 4, t("o"))).ravel(), dh.sum(axis=0)])
            Wo_b, _ = self._lin(Bk[u + 4], d, d)
            do = dh @ Wo_b
            dq, dk, dv = self._attention_bwd(do, view(u + 4, t("att")), B)
            grads[u + 1] = np.concatenate([(dq.T @ view(u + 1, t("n1"))).ravel(), dq.sum(axis=0)])
            grads[u + 2] = np.concatenate([(dk.T @ view(u + 2, t("n1"))).ravel(), dk.sum(axis=0)])
            grads[u + 3] = np.concatenate([(dv.T @ view(u + 3, t("n1"))).ravel(), dv.sum(axis=0)])
            Wq_b, _ = self._lin(Bk[u + 1], d, d)
            Wk_b, _ = self._lin(Bk[u + 2], d, d)
            Wv_b, _ = self._lin(Bk[u + 3], d, d)
            dn1 = dq @ Wq_b + dk @ Wk_b + dv @ Wv_b
            g1_b, _ = self._ln(Bk[u])
            dx_ln, dg, db = _ln_bwd(dn1, view(u, t("xh1")), view(u, t("rs1")), g1_b)
            grads[u] = np.concatenate([dg, db])
            dx = dh + dx_ln
        dE = np.zeros((V, d))
        np.add.at(dE, tokens.reshape(-1), dx)
        grads[0] = dE.ravel()
        return loss, grads
