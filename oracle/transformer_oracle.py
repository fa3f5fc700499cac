"""fp64 CPU oracle model: fine-grained pre-LN Transformer (decoder-style, causal) with the
two-weight backward of asynchronous pipeline parallelism.

TEST INFRASTRUCTURE ONLY (same rules as pipemare_oracle.py: nothing in the product path may
import it; it shares no code with the HIP library).

It plugs into pipemare_oracle.PipeMareOracle as `model`: loss_and_grads(u_fwd, u_bkwd, batch)
returns the gradient that backpropagation produces when the forward pass uses the weights
u_fwd and the backward pass uses u_bkwd (Sec. 2.1).  Activations, normalisation statistics,
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

    # ---- the two-weight gradient
    def loss_and_grads(self, u_fwd, u_bkwd, batch):
        tokens, targets = batch
        tokens = np.asarray(tokens).astype(np.int64)
        targets = np.asarray(targets).astype(np.int64).reshape(-1)
        B = tokens.shape[0]
        d, dff, V, S = self.d, self.dff, self.V, self.S
        T = B * S
        F, Bk = u_fwd, u_bkwd
        grads = [None] * self.n_units

        # ---------------- forward with u_fwd
        E = F[0].reshape(V, d)
        x = E[tokens.reshape(-1)] + np.tile(self.pos, (B, 1))
        saved = []
        for l in range(self.nl):
            u = 1 + 8 * l
            g1, b1 = self._ln(F[u])
            n1, xh1, rs1 = _ln_fwd(x, g1, b1)
            Wq, bq = self._lin(F[u + 1], d, d)
            Wk, bk = self._lin(F[u + 2], d, d)
            Wv, bv = self._lin(F[u + 3], d, d)
            q, k, v = n1 @ Wq.T + bq, n1 @ Wk.T + bk, n1 @ Wv.T + bv
            o, acache = self._attention_fwd(q, k, v, B)
            Wo, bo = self._lin(F[u + 4], d, d)
            h = x + o @ Wo.T + bo
            g2, b2 = self._ln(F[u + 5])
            n2, xh2, rs2 = _ln_fwd(h, g2, b2)
            W1, bb1 = self._lin(F[u + 6], dff, d)
            z1 = n2 @ W1.T + bb1
            f = np.maximum(z1, 0.0)
            W2, bb2 = self._lin(F[u + 7], d, dff)
            y = h + f @ W2.T + bb2
            saved.append((xh1, rs1, n1, acache, o, xh2, rs2, n2, z1, f))
            x = y
        uf = 1 + 8 * self.nl
        gf, bf = self._ln(F[uf])
        nf, xhf, rsf = _ln_fwd(x, gf, bf)
        Wh, bh = self._lin(F[uf + 1], V, d)
        logits = nf @ Wh.T + bh
        zmax = logits.max(axis=1, keepdims=True)
        ex = np.exp(logits - zmax)
        prob = ex / ex.sum(axis=1, keepdims=True)
        loss = float(np.mean(np.log(ex.sum(axis=1)) + zmax[:, 0] - logits[np.arange(T), targets]))

        # ---------------- backward: stored forward quantities, weights from u_bkwd on the data path
        dlog = prob
        dlog[np.arange(T), targets] -= 1.0
        dlog = dlog / T
        grads[uf + 1] = np.concatenate([(dlog.T @ nf).ravel(), dlog.sum(axis=0)])
        Wh_b, _ = self._lin(Bk[uf + 1], V, d)
        dnf = dlog @ Wh_b
        gf_b, _ = self._ln(Bk[uf])
        dx, dg, db = _ln_bwd(dnf, xhf, rsf, gf_b)
        grads[uf] = np.concatenate([dg, db])
        for l in range(self.nl - 1, -1, -1):
            u = 1 + 8 * l
            xh1, rs1, n1, acache, o, xh2, rs2, n2, z1, f = saved[l]
            # y = h + f W2^T + b
            grads[u + 7] = np.concatenate([(dx.T @ f).ravel(), dx.sum(axis=0)])
            W2_b, _ = self._lin(Bk[u + 7], d, dff)
            df = dx @ W2_b
            dz1 = df * (z1 > 0.0)
            grads[u + 6] = np.concatenate([(dz1.T @ n2).ravel(), dz1.sum(axis=0)])
            W1_b, _ = self._lin(Bk[u + 6], dff, d)
            dn2 = dz1 @ W1_b
            g2_b, _ = self._ln(Bk[u + 5])
            dh_ln, dg, db = _ln_bwd(dn2, xh2, rs2, g2_b)
            grads[u + 5] = np.concatenate([dg, db])
            dh = dx + dh_ln
            # h = x + o Wo^T + b
            grads[u + 4] = np.concatenate([(dh.T @ o).ravel(), dh.sum(axis=0)])
            Wo_b, _ = self._lin(Bk[u + 4], d, d)
            do = dh @ Wo_b
            dq, dk, dv = self._attention_bwd(do, acache, B)
            grads[u + 1] = np.concatenate([(dq.T @ n1).ravel(), dq.sum(axis=0)])
            grads[u + 2] = np.concatenate([(dk.T @ n1).ravel(), dk.sum(axis=0)])
            grads[u + 3] = np.concatenate([(dv.T @ n1).ravel(), dv.sum(axis=0)])
            Wq_b, _ = self._lin(Bk[u + 1], d, d)
            Wk_b, _ = self._lin(Bk[u + 2], d, d)
            Wv_b, _ = self._lin(Bk[u + 3], d, d)
            dn1 = dq @ Wq_b + dk @ Wk_b + dv @ Wv_b
            g1_b, _ = self._ln(Bk[u])
            dx_ln, dg, db = _ln_bwd(dn1, xh1, rs1, g1_b)
            grads[u] = np.concatenate([dg, db])
            dx = dh + dx_ln
        dE = np.zeros((V, d))
        np.add.at(dE, tokens.reshape(-1), dx)
        grads[0] = dE.ravel()
        return loss, grads
