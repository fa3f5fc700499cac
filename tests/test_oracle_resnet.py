"""Pins for the ResNet oracle model: compared with an independent PyTorch (CPU, fp64, autograd)
implementation of the same architecture, in the ordinary and in the two-weight form."""
import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

import workloads as wl
from oracle import pipemare_oracle as po
from oracle.resnet_oracle import ResNetModel, conv_specs


def _setup(seed=0, n_blocks=1, B=3, image=8):
    w = wl.resnet(n_blocks, B, dtype="f32", image=image)
    params = [p.astype(np.float64) for p in wl.init_params(w, seed)]
    model = ResNetModel(n_blocks, 10, image)
    assert [p.size for p in params] == model.unit_sizes()
    x, y = wl.ImageStream(w).batch(0)
    return w, params, model, x, y


def _torch_net(model, Fw, Bw, x, labels, two_weight):
    """Forward values from Fw; with two_weight every place where a gradient flows through a weight
    (convolution input path, affine scale, classifier input path) takes its derivative from Bw:
    f(x, Wb) + (f(x.detach(), Wf) - f(x.detach(), Wb)).detach().  Parameter gradients are collected on
    zero-valued leaves that see detached inputs."""
    leaves = []
    specs = model.specs
    xt = torch.tensor(np.asarray(x, dtype=np.float64))          # NCHW

    def conv(inp, u):
        ci, co, stride = specs[u]
        nw = co * 9 * ci
        unpack = lambda p: torch.tensor(p[:nw].reshape(co, 3, 3, ci)).permute(0, 3, 1, 2).contiguous()   # OIHW
        Wf = unpack(Fw[u])
        sf, tf_ = torch.tensor(Fw[u][nw:nw + co]), torch.tensor(Fw[u][nw + co:])
        Wg = torch.zeros_like(Wf, requires_grad=True)
        sg = torch.zeros_like(sf, requires_grad=True)
        tg = torch.zeros_like(tf_, requires_grad=True)
        leaves.append((u, Wg, sg, tg))
        c = lambda a, W: Fn.conv2d(a, W, stride=stride, padding=1)
        v = lambda s: s.view(1, -1, 1, 1)
        if two_weight:
            Wb = unpack(Bw[u])
            sb = torch.tensor(Bw[u][nw:nw + co])
            z = c(inp, Wb) + (c(inp.detach(), Wf) - c(inp.detach(), Wb)).detach() + c(inp.detach(), Wg)
            return z * v(sb) + (z.detach() * v(sf - sb)) + z.detach() * v(sg) + v(tf_) + v(tg)
        z = c(inp, Wf) + c(inp.detach(), Wg)
        return z * v(sf) + z.detach() * v(sg) + v(tf_) + v(tg)

    def shortcut(a, co, stride):
        if stride == 1 and a.shape[1] == co:
            return a
        a = a[:, :, ::stride, ::stride]
        return Fn.pad(a, (0, 0, 0, 0, 0, co - a.shape[1]))

    cur = torch.relu(conv(xt, 0))
    u = 1
    while u < len(specs):
        ci, co, stride = specs[u]
        y1 = torch.relu(conv(cur, u))
        cur = torch.relu(conv(y1, u + 1) + shortcut(cur, co, stride))
        u += 2
    pooled = cur.mean(dim=(2, 3))
    nconv = len(specs)
    nfc = model.ncls * 64
    Wf = torch.tensor(Fw[nconv][:nfc].reshape(model.ncls, 64))
    bf = torch.tensor(Fw[nconv][nfc:])
    Wg = torch.zeros_like(Wf, requires_grad=True)
    bg = torch.zeros_like(bf, requires_grad=True)
    if two_weight:
        Wb = torch.tensor(Bw[nconv][:nfc].reshape(model.ncls, 64))
        logits = pooled @ Wb.T + (pooled.detach() @ (Wf - Wb).T) + pooled.detach() @ Wg.T + bf + bg
    else:
        logits = pooled @ Wf.T + pooled.detach() @ Wg.T + bf + bg
    loss = Fn.cross_entropy(logits, torch.as_tensor(np.asarray(labels), dtype=torch.long))
    loss.backward()
    grads = {}
    for u, Wg_, sg, tg in leaves:
        grads[u] = np.concatenate([Wg_.grad.permute(0, 2, 3, 1).contiguous().numpy().ravel(), sg.grad.numpy(), tg.grad.numpy()])
    grads[nconv] = np.concatenate([Wg.grad.numpy().ravel(), bg.grad.numpy()])
    return float(loss), grads


def test_conv_specs_resnet20():
    s = conv_specs(3)
    assert len(s) == 19
    assert s[0] == (3, 16, 1) and s[7] == (16, 32, 2) and s[13] == (32, 64, 2) and s[18] == (64, 64, 1)
    w = wl.resnet(3, 128)
    assert w.P == 20 and len(w.layers) == 20
    assert po.pipeline_delays(w.P, 1)[0][0] == 39
    assert sum(wl.n_params(L) for L in w.layers) == sum(ResNetModel(3).unit_sizes())
    assert 0.26e6 < sum(wl.n_params(L) for L in w.layers) < 0.28e6


@pytest.mark.parametrize("n_blocks", [1, 2])
def test_same_weights_equals_autograd(n_blocks):
    """grad f(w, w) is the ordinary gradient (Sec. 2.1)."""
    w, params, model, x, y = _setup(n_blocks=n_blocks)
    loss, grads = model.loss_and_grads(params, params, (x, y))
    tl, tg = _torch_net(model, params, params, x, y, two_weight=False)
    assert loss == pytest.approx(tl, rel=1e-12)
    for u in range(model.n_units):
        assert np.allclose(grads[u], tg[u], rtol=0, atol=1e-12), u


def test_two_weight_gradient_equals_autograd_construction():
    w, params, model, x, y = _setup(seed=5, n_blocks=2)
    rng = np.random.default_rng(1)
    Fw = [p + 0.05 * rng.standard_normal(p.shape) for p in params]
    Bw = [p + 0.05 * rng.standard_normal(p.shape) for p in params]
    loss, grads = model.loss_and_grads(Fw, Bw, (x, y))
    tl, tg = _torch_net(model, Fw, Bw, x, y, two_weight=True)
    assert loss == pytest.approx(tl, rel=1e-12)
    for u in range(model.n_units):
        assert np.allclose(grads[u], tg[u], rtol=0, atol=1e-12), u
    _, g_same = model.loss_and_grads(Fw, Fw, (x, y))
    assert max(np.max(np.abs(a - b)) for a, b in zip(grads, g_same)) > 1e-4      # the backward weights matter
    # ... except the kernel of the first convolution, which nothing flows through (its scale does
    # matter: dz = da * scale_bkwd enters its own weight gradient)
    b0 = Bw[0].copy()
    b0[:16 * 27] += 1.0
    Bw2 = [b0] + Bw[1:]
    _, g2 = model.loss_and_grads(Fw, Bw2, (x, y))
    assert all(np.array_equal(a, b) for a, b in zip(grads, g2))


def test_resnet_in_the_recurrence_all_delays_zero_is_momentum_sgd():
    w, params, model, x, y = _setup(n_blocks=1, B=2, image=8)
    o = po.PipeMareOracle(model, params, [L.stage for L in w.layers], [0] * w.P, [0] * w.P,
                          dict(kind="sgdm", beta=0.9, sched=dict(kind="const", base=0.05)))
    tp = [p.copy() for p in params]
    vel = [np.zeros_like(p) for p in params]
    stream = wl.ImageStream(w)
    for k in range(4):
        xb, yb = stream.batch(k)
        o.step((xb, yb))
        _, g = _torch_net(model, tp, None, xb, yb, two_weight=False)
        for u in range(len(tp)):
            vel[u] = 0.9 * vel[u] - 0.05 * g[u]        # App. B.3 form
            tp[u] = tp[u] + vel[u]
    for a, b in zip(o.weights(), tp):
        assert np.allclose(a, b, rtol=0, atol=1e-12)
