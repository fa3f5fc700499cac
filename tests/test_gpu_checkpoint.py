"""Checkpoint / resume through the C ABI: a run that saves after k steps and a fresh context that loads
the image must continue identically (weights, step tables, losses), for every piece of state the
recurrences carry: master weights, optimizer moments, delta, all ring slots, corrected backward and
recompute weights, step counter (T1 window, stochastic-delay counter).  Bit-identical where the step
itself is deterministic; where fp32 atomics order a sum (gradient-norm for clipping, embedding and
LayerNorm gain gradients, the fp32 convolution weight gradient) two runs of the SAME program differ in the last bits, and the comparison
allows exactly that much."""
import numpy as np
import pytest

import workloads as wl
from oracle import pipemare_oracle as po
from pm_testutil import make_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _batches(torch, w, stream_of, k0, k1):
    s = stream_of(w)
    for k in range(k0, k1):
        x, y = s.batch(k)
        yield torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()


CASES = {
    "mlp_f32_sgdm": (lambda: wl.small_mlp(48, 5, 10, "gelu", "xent", "f32", 16), wl.BatchStream,
                     dict(lr=0.05, beta=0.9, D=0.5, K=12)),
    "mlp_bf16_adamw": (lambda: wl.small_mlp(64, 4, 10, "relu", "xent", "bf16", 32), wl.BatchStream,
                       dict(opt="adamw", lr=2e-3, weight_decay=0.01, K=12)),
    "mlp_f32_sgdm_clip": (lambda: wl.small_mlp(48, 4, 10, "gelu", "xent", "f32", 16), wl.BatchStream,
                          dict(lr=0.05, beta=0.9, D=0.5, K=12, clip_norm=0.5, _atomics=True)),
    "mlp_f32_recompute": (lambda: wl.small_mlp(48, 6, 10, "gelu", "xent", "f32", 16), wl.BatchStream,
                          dict(lr=0.05, beta=0.9, D=0.5, K=12, _recompute=2)),
    "mlp_f32_stochastic": (lambda: wl.small_mlp(48, 4, 10, "gelu", "xent", "f32", 16), wl.BatchStream,
                           dict(lr=0.05, beta=0.9, K=12, stochastic=dict(tau_max=9, seed=11))),
    "mlp_f32_sync_warmup": (lambda: wl.small_mlp(48, 4, 10, "gelu", "xent", "f32", 16), wl.BatchStream,
                            dict(lr=0.05, beta=0.9, D=0.5, K=12, sync_warmup=9)),
    "tiny_transformer_f32": (lambda: wl.transformer(2, 32, 4, 64, 61, 8, 3, dtype="f32"), wl.TokenStream,
                             dict(opt="adamw", lr=1e-3, beta=0.9, beta2=0.98, K=12, _atomics=True)),
    "small_resnet_f32": (lambda: wl.resnet(1, 8, dtype="f32", image=8), wl.batch_stream,
                         dict(lr=0.01, beta=0.9, K=12, _atomics=True)),
}


@pytest.mark.parametrize("name", list(CASES))
def test_resume_is_bit_identical(torch_cuda, name):
    torch = torch_cuda
    mk, stream_of, kw = CASES[name]
    kw = dict(kw)
    w = mk()
    params = wl.init_params(w)
    tf, tb = po.pipeline_delays(w.P, 1)
    S = kw.pop("_recompute", 0)
    exact = not kw.pop("_atomics", False)
    if S:
        kw.update(tau_recomp=po.recompute_delays(w.P, S, 1, tb), segment=S)
    k_save, k_end = 7, 15                       # saved inside the T1 window and (where set) past the warm-up switch

    a = make_gpu(w, params, tf, tb, **kw)
    for x, y in _batches(torch, w, stream_of, 0, k_save):
        a.step(x, y)
    image = a.checkpoint()
    assert image.size == __import__("paper_1910_05124_amd").pm_checkpoint_bytes(a.ctx)
    losses_a = [a.step(x, y, want_loss=True) for x, y in _batches(torch, w, stream_of, k_save, k_end)]
    table_a = a.step_table()
    wa = a.weights()

    other = [np.zeros_like(p) + 0.5 for p in params]          # different initial weights: all state must come from the image
    b = make_gpu(w, other, tf, tb, **kw)
    b.restore(image)
    assert b.stats()["t"] == k_save
    losses_b = [b.step(x, y, want_loss=True) for x, y in _batches(torch, w, stream_of, k_save, k_end)]
    table_b = b.step_table()
    wb = b.weights()

    def same(x, y):
        if exact:
            return np.array_equal(x, y)
        return np.allclose(x, y, rtol=1e-4, atol=1e-6 * float(np.max(np.abs(x))))

    assert losses_a == pytest.approx(losses_b, rel=1e-5)          # the loss itself is summed with atomics
    assert table_a[0] == table_b[0] == k_end - 1 and table_a[1:4] == table_b[1:4]      # integers: always exact
    assert np.array_equal(table_a[4], table_b[4])
    for u, (x, y) in enumerate(zip(wa, wb)):
        assert same(x, y), u
    for which in (1, 2, 3):                                      # delta, momentum, corrected backward weights
        for u in range(len(w.layers)):
            assert same(a.state(which, u), b.state(which, u)), (which, u)
    a.close()
    b.close()


def test_checkpoint_rejections(torch_cuda):
    import paper_1910_05124_amd as pm
    torch = torch_cuda
    w = wl.small_mlp(32, 3, 4, "relu", "xent", "f32", 8)
    params = wl.init_params(w)
    tf, tb = po.pipeline_delays(w.P, 1)
    a = make_gpu(w, params, tf, tb, lr=0.05, beta=0.9)
    image = a.checkpoint()
    with pytest.raises(pm.PmError):                              # truncated image
        a.restore(image[:-8])
    bad = image.copy()
    bad[:8] = 0                                                  # wrong magic
    with pytest.raises(pm.PmError):
        a.restore(bad)
    w2 = wl.small_mlp(32, 4, 4, "relu", "xent", "f32", 8)        # another layout
    tf2, tb2 = po.pipeline_delays(w2.P, 1)
    b = make_gpu(w2, wl.init_params(w2), tf2, tb2, lr=0.05, beta=0.9)
    with pytest.raises(pm.PmError):
        b.restore(np.concatenate([image, np.zeros(1 << 20, np.uint8)]))
    # in the middle of a minibatch a checkpoint is refused
    c = make_gpu(w, params, tf, tb, N=2, lr=0.05, beta=0.9)
    x, y = next(_batches(torch, w, wl.BatchStream, 0, 1))
    c.step(x, y)
    with pytest.raises(pm.PmError):
        c.checkpoint()
    c.step(x, y)
    c.checkpoint()
    for g in (a, b, c):
        g.close()
