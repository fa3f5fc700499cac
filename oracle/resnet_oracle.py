"""fp64 CPU oracle model: ResNet-20-shaped CNN with the two-weight backward of asynchronous
pipeline parallelism.

TEST INFRASTRUCTURE ONLY (same rules as pipemare_oracle.py: nothing in the product path may
import it; it shares no code with the HIP library).

It plugs into pipemare_oracle.PipeMareOracle as `model`: loss_and_grads(u_fwd, u_bkwd, batch)
returns the gradient backpropagation produces when the forward pass uses the weights u_fwd and the
backward pass uses u_bkwd (Sec. 2.1); with u_recomp the activations inside every segment of stages are
rebuilt in the backward pass with a third weight set (see loss_and_grads).  Activations, pre-activations
and ReLU masks come from the forward pass; the backward pass reads a weight only where a gradient flows *through* it:
  * convolution:        d(input) = transposed convolution of dz with W_bkwd   (dW uses the stored input)
  * per-channel affine: dz = da * scale_bkwd        (d scale = sum da * z_stored, d shift = sum da)
  * fully connected:    d(input) = dlogits @ W_bkwd

Architecture (the paper trains ResNet50; the workload text asks for the CIFAR ResNet-20 shape of
its reference [He et al. 2016], one pipeline stage per 3x3 convolution, batch normalisation folded
to a per-channel affine):
  conv0 3 -> 16, then 3 groups of n blocks with 16, 32, 64 channels on 32x32, 16x16, 8x8 maps; a block
  is y = relu(affine2(conv2(relu(affine1(conv1(x))))) + shortcut(x)); the first convolution of groups
  2 and 3 has stride 2 and their shortcut is parameter-free: every second pixel, new channels zero
  (the input's channels come first); global average pool; fully connected 64 -> classes; softmax
  cross-entropy, mean over the batch.  All convolutions 3x3, zero padding 1, no bias (the affine's
  shift plays that role).
Weight units in topological order, each a packed fp64 vector:
  conv unit  [W (C_out x 3 x 3 x C_in, row-major, i.e. tap-major then input channel) | scale (C_out) | shift (C_out)]
  last unit  [W (classes x 64) | b (classes)]
Images are NCHW on input ([B, 3, H, W]); internally NHWC.
"""
from __future__ import annotations

import numpy as np


def conv_specs(n_blocks: int):
    """(C_in, C_out, stride) of every convolution in order."""
    specs = [(3, 16, 1)]
    c = 16
    for g in range(3):
        for b in range(n_blocks):
            if g > 0 and b == 0:
                specs += [(c, 2 * c, 2), (2 * c, 2 * c, 1)]
                c *= 2
            else:
                specs += [(c, c, 1), (c, c, 1)]
    return specs


def _im2col(x, stride):
    """x [B, H, W, C] -> patches [B, Ho, Wo, 9 * C] (tap-major: tap = 3 * dy + dx, then channel), pad 1."""
    B, H, W, C = x.shape
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    xp = np.zeros((B, H + 2, W + 2, C))
    xp[:, 1:H + 1, 1:W + 1, :] = x
    cols = np.empty((B, Ho, Wo, 9, C))
    for dy in range(3):
        for dx in range(3):
            cols[:, :, :, 3 * dy + dx, :] = xp[:, dy:dy + stride * (Ho - 1) + 1:stride, dx:dx + stride * (Wo - 1) + 1:stride, :]
    return cols.reshape(B, Ho, Wo, 9 * C)


def _col2im(dcols, shape, stride):
    """Adjoint of _im2col: scatter-add patch gradients back onto the (unpadded) input."""
    B, H, W, C = shape
    Ho, Wo = dcols.shape[1], dcols.shape[2]
    d5 = dcols.reshape(B, Ho, Wo, 9, C)
    dxp = np.zeros((B, H + 2, W + 2, C))
    for dy in range(3):
        for dx in range(3):
            dxp[:, dy:dy + stride * (Ho - 1) + 1:stride, dx:dx + stride * (Wo - 1) + 1:stride, :] += d5[:, :, :, 3 * dy + dx, :]
    return dxp[:, 1:H + 1, 1:W + 1, :]


def _shortcut(x, c_out, stride):
    if stride == 1 and x.shape[3] == c_out:
        return x
    y = np.zeros((x.shape[0], (x.shape[1] - 1) // stride + 1, (x.shape[2] - 1) // stride + 1, c_out))
    y[:, :, :, :x.shape[3]] = x[:, ::stride, ::stride, :]
    return y


def _shortcut_bwd(dy, in_shape, stride):
    if stride == 1 and in_shape[3] == dy.shape[3]:
        return dy
    dx = np.zeros(in_shape)
    dx[:, ::stride, ::stride, :] = dy[:, :, :, :in_shape[3]]
    return dx


class ResNetModel:
    def __init__(self, n_blocks: int = 3, n_classes: int = 10, image: int = 32):
        self.nb, self.ncls, self.image = n_blocks, n_classes, image
        self.specs = conv_specs(n_blocks)
        self.n_units = len(self.specs) + 1

    def unit_sizes(self):
        return [co * 9 * ci + 2 * co for ci, co, _ in self.specs] + [self.ncls * 64 + self.ncls]

    def _conv_unit(self, p, u):
        ci, co, _ = self.specs[u]
        nw = co * 9 * ci
        return p[:nw].reshape(co, 9 * ci), p[nw:nw + co], p[nw + co:nw + 2 * co]

    def _in_name(self, u):
        return "img" if u == 0 else f"y{u - 1}"

    def _conv_forward(self, u, p, get):
        """Convolution unit u from the tensors it reads through get(name): its input (the image or the
        previous unit's output) and, for the second convolution of a block, the block's input (shortcut).
        z = conv(inp), a = s z + t (+ shortcut), y = relu(a)."""
        ci, co, stride = self.specs[u]
        W, s, t = self._conv_unit(p, u)
        z = _im2col(get(self._in_name(u)), stride) @ W.T
        a = z * s + t
        if u >= 2 and (u - 1) % 2 == 1:          # second convolution of a block: add the shortcut of the block input
            _, _, stride_block = self.specs[u - 1]
            a = a + _shortcut(get(self._in_name(u - 1)), co, stride_block)
        return {f"z{u}": z, f"y{u}": np.maximum(a, 0.0)}

    def loss_and_grads(self, u_fwd, u_bkwd, batch, u_recomp=None, checkpoints=None):
        """checkpoints (with u_recomp): indices of the units that open a segment (0 is always one).  The forward
        pass is taken to keep only the tensors that cross a segment boundary; in the backward pass every
        segment's convolution units first run again, in order, with the weights u_recomp - reading kept
        forward tensors where the producer sits in an earlier segment and rebuilt ones where it sits in the
        same segment - and a unit's backward then uses, for every stored tensor it needs (its input, its
        pre-activation z, its output's ReLU mask), the rebuilt value if that tensor was produced in the unit's
        own segment and the kept forward value otherwise (App. "Statistical efficiency and recompute").  The
        classifier is not rebuilt (loss and its gradient come from the forward pass); its pooled input follows
        the same rule.  Data gradients use u_bkwd as always."""
        x, labels = batch
        x = np.transpose(np.asarray(x, dtype=np.float64), (0, 2, 3, 1))        # NCHW -> NHWC
        labels = np.asarray(labels).astype(np.int64).reshape(-1)
        B = x.shape[0]
        F, Bk = u_fwd, u_bkwd
        nconv = len(self.specs)

        # ---------------- forward with u_fwd
        fwd = {"img": x}
        for u in range(nconv):
            fwd.update(self._conv_forward(u, F[u], fwd.__getitem__))
        last = f"y{nconv - 1}"
        pooled = fwd[last].mean(axis=(1, 2))                                    # [B, 64]
        nfc = self.ncls * 64
        Wf, bf = F[nconv][:nfc].reshape(self.ncls, 64), F[nconv][nfc:]
        logits = pooled @ Wf.T + bf
        zmax = logits.max(axis=1, keepdims=True)
        ex = np.exp(logits - zmax)
        prob = ex / ex.sum(axis=1, keepdims=True)
        loss = float(np.mean(np.log(ex.sum(axis=1)) + zmax[:, 0] - logits[np.arange(B), labels]))

        # ---------------- recomputation: every segment's units again with u_recomp
        if u_recomp is None:
            def view(c, name):
                return fwd[name]
        else:
            cps = sorted(set([0] + [int(c) for c in (checkpoints or [])]))
            seg_of = [sum(1 for c in cps if c <= u) - 1 for u in range(nconv + 1)]
            rebuilt = [dict() for _ in cps]
            for u in range(nconv):
                mine = rebuilt[seg_of[u]]
                mine.update(self._conv_forward(u, u_recomp[u], lambda name, mine=mine: mine[name] if name in mine else fwd[name]))

            def view(c, name):
                mine = rebuilt[seg_of[c]]
                return mine[name] if name in mine else fwd[name]

        # ---------------- backward: stored (or rebuilt) quantities, weights from u_bkwd on the data path
        grads = [None] * self.n_units
        dlog = prob
        dlog[np.arange(B), labels] -= 1.0
        dlog = dlog / B
        y_last = view(nconv, last)
        grads[nconv] = np.concatenate([(dlog.T @ y_last.mean(axis=(1, 2))).ravel(), dlog.sum(axis=0)])
        Wf_b = Bk[nconv][:nfc].reshape(self.ncls, 64)
        dpool = dlog @ Wf_b
        hw = y_last.shape[1] * y_last.shape[2]
        dy = np.broadcast_to(dpool[:, None, None, :] / hw, y_last.shape).copy()
        pending_shortcut = None        # gradient that reaches a block's input through its shortcut
        for u in range(nconv - 1, -1, -1):
            ci, co, stride = self.specs[u]
            W_b, s_b, _ = self._conv_unit(Bk[u], u)
            da = dy * (view(u, f"y{u}") > 0.0)
            if u >= 2 and (u - 1) % 2 == 1:          # second convolution of a block: da also feeds the shortcut
                pending_shortcut = da
            ds = (da * view(u, f"z{u}")).sum(axis=(0, 1, 2))
            dt = da.sum(axis=(0, 1, 2))
            dz = da * s_b
            dz2 = dz.reshape(-1, co)
            inp = view(u, self._in_name(u))
            cols = _im2col(inp, stride)
            dW = dz2.T @ cols.reshape(-1, 9 * ci)
            grads[u] = np.concatenate([dW.ravel(), ds, dt])
            if u == 0:
                break
            dcols = (dz2 @ W_b).reshape(cols.shape)
            dy = _col2im(dcols, inp.shape, stride)
            if (u - 1) % 2 == 0:                      # first convolution of a block: its input is the block input
                dy = dy + _shortcut_bwd(pending_shortcut, inp.shape, stride)
        return loss, grads
