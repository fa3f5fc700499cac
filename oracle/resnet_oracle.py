"""fp64 CPU oracle model: ResNet-20-shaped CNN with the two-weight backward of asynchronous
pipeline parallelism.

TEST INFRASTRUCTURE ONLY (same rules as pipemare_oracle.py: nothing in the product path may
import it; it shares no code with the HIP library).

It plugs into pipemare_oracle.PipeMareOracle as `model`: loss_and_grads(u_fwd, u_bkwd, batch)
returns the gradient backpropagation produces when the forward pass uses the weights u_fwd and the
backward pass uses u_bkwd (Sec. 2.1).  Activations, pre-activations and ReLU masks come from the
forward pass; the backward pass reads a weight only where a gradient flows *through* it:
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

    def loss_and_grads(self, u_fwd, u_bkwd, batch):
        x, labels = batch
        x = np.transpose(np.asarray(x, dtype=np.float64), (0, 2, 3, 1))        # NCHW -> NHWC
        labels = np.asarray(labels).astype(np.int64).reshape(-1)
        B = x.shape[0]
        F, Bk = u_fwd, u_bkwd
        nconv = len(self.specs)

        # ---------------- forward with u_fwd.  conv u: z = conv(inp), a = s z + t (+ shortcut), y = relu(a)
        inp, cols, zs, ys = [None] * nconv, [None] * nconv, [None] * nconv, [None] * nconv
        cur = x
        block_in = None
        for u in range(nconv):
            ci, co, stride = self.specs[u]
            W, s, t = self._conv_unit(F[u], u)
            inp[u] = cur
            cols[u] = _im2col(cur, stride)
            z = cols[u] @ W.T
            a = z * s + t
            if u >= 1 and (u - 1) % 2 == 0:          # first convolution of a block
                block_in = cur
            if u >= 2 and (u - 1) % 2 == 1:          # second convolution of a block: add the shortcut
                c_in_block, _, stride_block = self.specs[u - 1]
                a = a + _shortcut(block_in, co, stride_block)
            zs[u] = z
            ys[u] = np.maximum(a, 0.0)
            cur = ys[u]
        pooled = cur.mean(axis=(1, 2))                                          # [B, 64]
        nfc = self.ncls * 64
        Wf, bf = F[nconv][:nfc].reshape(self.ncls, 64), F[nconv][nfc:]
        logits = pooled @ Wf.T + bf
        zmax = logits.max(axis=1, keepdims=True)
        ex = np.exp(logits - zmax)
        prob = ex / ex.sum(axis=1, keepdims=True)
        loss = float(np.mean(np.log(ex.sum(axis=1)) + zmax[:, 0] - logits[np.arange(B), labels]))

        # ---------------- backward: stored forward quantities, weights from u_bkwd on the data path
        grads = [None] * self.n_units
        dlog = prob
        dlog[np.arange(B), labels] -= 1.0
        dlog = dlog / B
        grads[nconv] = np.concatenate([(dlog.T @ pooled).ravel(), dlog.sum(axis=0)])
        Wf_b = Bk[nconv][:nfc].reshape(self.ncls, 64)
        dpool = dlog @ Wf_b
        hw = cur.shape[1] * cur.shape[2]
        dy = np.broadcast_to(dpool[:, None, None, :] / hw, cur.shape).copy()
        pending_shortcut = None        # gradient that reaches a block's input through its shortcut
        for u in range(nconv - 1, -1, -1):
            ci, co, stride = self.specs[u]
            W_b, s_b, _ = self._conv_unit(Bk[u], u)
            da = dy * (ys[u] > 0.0)
            if u >= 2 and (u - 1) % 2 == 1:          # second convolution of a block: da also feeds the shortcut
                pending_shortcut = da
            ds = (da * zs[u]).sum(axis=(0, 1, 2))
            dt = da.sum(axis=(0, 1, 2))
            dz = da * s_b
            dz2 = dz.reshape(-1, co)
            dW = dz2.T @ cols[u].reshape(-1, 9 * ci)
            grads[u] = np.concatenate([dW.ravel(), ds, dt])
            if u == 0:
                break
            dcols = (dz2 @ W_b).reshape(cols[u].shape)
            dy = _col2im(dcols, inp[u].shape, stride)
            if (u - 1) % 2 == 0:                      # first convolution of a block: its input is the block input
                dy = dy + _shortcut_bwd(pending_shortcut, inp[u].shape, stride)
        return loss, grads
