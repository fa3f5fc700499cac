"""GPU parity under Hogwild-style stochastic delays: every step each stage draws its delay (counter-based
generator, truncated exponential); the ring slots the device kernels used must equal the oracle's
versions bit for bit at every step, and the weights must stay inside the usual bands."""
import numpy as np
import pytest

import workloads as wl
from oracle import pipemare_oracle as po
from pm_testutil import key_bias_entries, make_gpu, make_oracle, max_rel_err

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3}


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _run(torch, w, steps, st, *, gpu_kw=None, stream_of=None, free_running=False, **kw):
    """free_running: no read-back (loss, step table) before the last step, so nothing but the library's own
    event waits orders consecutive steps and an overlapped update really runs beside the next forward."""
    params = wl.init_params(w)
    tf, tb = po.pipeline_delays(w.P, 1)
    stream = (stream_of or wl.batch_stream)(w)
    o = make_oracle(w, params, tf, tb, stochastic=st, **kw)
    R = st["tau_max"] + 1
    warm = kw.get("sync_warmup", 0)
    side = torch.cuda.Stream()
    seen = set()
    with torch.cuda.stream(side):
        g = make_gpu(w, params, tf, tb, stochastic=st, stream=side, **dict(kw, **(gpu_kw or {})))
        x0, y0 = stream.batch(0)
        xd, yd = torch.from_numpy(x0).cuda(), torch.from_numpy(y0).cuda()
        for k in range(steps):
            x, y = stream.batch(k)
            xd.copy_(torch.from_numpy(x))
            yd.copy_(torch.from_numpy(y))
            lo = o.step((x, y))
            if k >= warm:
                seen.update(o.last_delays)
            if free_running and k + 1 < steps:
                g.step(xd, yd)
                continue
            lg = g.step(xd, yd, want_loss=True)
            assert lg == pytest.approx(lo, rel=3e-2 if w.dtype == "bf16" else 1e-4, abs=1e-6)
            t_used, fs, bs, ws, lrs = g.step_table()
            assert t_used == k
            for u, L in enumerate(w.layers):
                vf, vb = o.last_versions[u]
                assert vf == vb
                assert (fs[u], bs[u], ws[u]) == (vf % R, vf % R, (k + 1) % R)          # bit-exact integers
                assert lrs[u] == pytest.approx(o.last_lr[u], rel=2e-7)
    return g, o, seen


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_mlp_stochastic_delays(torch_cuda, dtype):
    w = wl.small_mlp(64, 5, 10, "gelu", "xent", dtype, 32)
    st = dict(tau_max=2 * w.P + 3, seed=2024)
    g, o, seen = _run(torch_cuda, w, 30 if dtype == "f32" else 20, st, lr=0.05 if dtype == "f32" else 0.01, beta=0.9, K=10)
    err, errs = max_rel_err(g.weights(), o.weights())
    assert err < TOL[dtype], errs
    assert len(seen) >= 6 and 0 in seen                # many different delays were really drawn, zero among them
    g.close()


def test_mlp_stochastic_graph_adamw_and_warmup(torch_cuda):
    w = wl.small_mlp(48, 4, 10, "relu", "xent", "f32", 16)
    st = dict(tau_max=11, seed=2**63 + 5)
    g, o, seen = _run(torch_cuda, w, 24, st, gpu_kw=dict(use_graph=True), opt="adamw", lr=2e-3, weight_decay=0.01,
                      clip_norm=0.5, K=6, sync_warmup=3)
    err, errs = max_rel_err(g.weights(), o.weights())
    assert err < TOL["f32"], errs
    g.close()


def test_mlp_stochastic_with_overlapped_update(torch_cuda):
    # a drawn delay can be 0, so the forward may need the newest version: it must wait for the update
    w = wl.small_mlp(64, 4, 10, "gelu", "xent", "f32", 16)
    st = dict(tau_max=4, seed=1)
    g, o, seen = _run(torch_cuda, w, 24, st, gpu_kw=dict(overlap_update=True), free_running=True, lr=0.05, beta=0.9, K=6)
    assert 0 in seen                       # the case this test is about: a step whose forward needs version t itself
    err, errs = max_rel_err(g.weights(), o.weights())
    assert err < TOL["f32"], errs
    g.close()


def test_tau_max_zero_equals_synchronous(torch_cuda):
    w = wl.small_mlp(48, 3, 10, "gelu", "xent", "f32", 16)
    g, o, seen = _run(torch_cuda, w, 10, dict(tau_max=0, seed=9), lr=0.05, beta=0.9, K=0)
    assert seen == {0}
    err, _ = max_rel_err(g.weights(), o.weights())
    assert err < TOL["f32"]
    g.close()


def test_tiny_transformer_stochastic(torch_cuda):
    w = wl.transformer(2, 32, 4, 64, 61, 8, 3, dtype="f32")
    st = dict(tau_max=9, seed=77)
    g, o, seen = _run(torch_cuda, w, 16, st, opt="adamw", lr=1e-3, beta=0.9, beta2=0.98, K=8)
    err, errs = max_rel_err(g.weights(), o.weights(), skip=key_bias_entries(w))
    assert err < TOL["f32"], errs
    g.close()


def test_small_resnet_stochastic(torch_cuda):
    w = wl.resnet(1, 8, dtype="f32", image=8)
    st = dict(tau_max=7, seed=5)
    g, o, seen = _run(torch_cuda, w, 12, st, lr=0.01, beta=0.9, K=6)
    err, errs = max_rel_err(g.weights(), o.weights())
    assert err < TOL["f32"], errs
    g.close()


def test_stochastic_rejections(torch_cuda):
    import paper_1910_05124_amd as pm
    w = wl.small_mlp(32, 3, 4, "relu", "xent", "f32", 8)
    params = wl.init_params(w)
    tf, tb = po.pipeline_delays(w.P, 1)
    with pytest.raises(pm.PmError):
        make_gpu(w, params, tf, tb, stochastic=dict(tau_max=-1, seed=0))
    with pytest.raises(pm.PmError):
        make_gpu(w, params, tf, tb, stochastic=dict(tau_max=4, seed=0), tau_recomp=[0] * w.P, segment=1)
