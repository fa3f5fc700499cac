"""GPU parity of the convolution stages: the three 3x3-convolution products against NumPy fp64, then
whole PipeMare training runs of ResNet-shaped CNNs against the fp64 oracle (slots and step counters
bit-exact, master weights within 1e-5 (fp32) / 2e-3 (bf16) max-relative per unit)."""
import numpy as np
import pytest

import workloads as wl
from oracle import pipemare_oracle as po
from oracle import resnet_oracle as ro
from pm_testutil import make_gpu, make_oracle, max_rel_err

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3}


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [(2, 8, 8, 16, 16, 1), (2, 8, 8, 16, 32, 2), (1, 12, 12, 32, 32, 1), (2, 8, 8, 64, 64, 1),
                                   (2, 8, 8, 32, 64, 2), (3, 6, 6, 3, 16, 1), (5, 16, 16, 16, 16, 1), (2, 10, 6, 48, 16, 1)])
def test_conv_primitives_against_numpy(torch_cuda, dtype, shape):
    import paper_1910_05124_amd as pm
    torch = torch_cuda
    B, H, W, Cin, Cout, stride = shape
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    rng = np.random.default_rng(sum(shape))
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1

    def dev(a):
        return torch.from_numpy(a.astype(np.float32)).cuda().to(tdt).contiguous()

    def host(t):
        return t.float().cpu().numpy().astype(np.float64)

    x = dev(rng.standard_normal((B, H, W, Cin)))
    params = dev(np.concatenate([(rng.standard_normal((Cout, 9 * Cin)) / np.sqrt(9 * Cin)).ravel(),
                                 1.0 + 0.2 * rng.standard_normal(Cout), 0.2 * rng.standard_normal(Cout)]))
    dz = dev(rng.standard_normal((B, Ho, Wo, Cout)))
    z = torch.empty(B, Ho, Wo, Cout, dtype=tdt, device="cuda")
    y = torch.empty_like(z)
    dx = torch.empty(B, H, W, Cin, dtype=tdt, device="cuda")
    dW = torch.full((Cout, 9 * Cin), 7.0, dtype=torch.float32, device="cuda")       # must be overwritten
    st = torch.cuda.current_stream().cuda_stream
    pm.pm_conv3x3_fwd(st, dtype, B, H, W, Cin, Cout, stride, x.data_ptr(), params.data_ptr(), z.data_ptr(), y.data_ptr())
    pm.pm_conv3x3_bwd_data(st, dtype, B, H, W, Cin, Cout, stride, dz.data_ptr(), params.data_ptr(), dx.data_ptr())
    nscr = pm.pm_conv3x3_bwd_weight_scratch(dtype, B, H, W, Cin, Cout, stride)
    scr = torch.empty(max(nscr, 4), dtype=torch.uint8, device="cuda")
    pm.pm_conv3x3_bwd_weight(st, dtype, B, H, W, Cin, Cout, stride, dz.data_ptr(), x.data_ptr(), dW.data_ptr(),
                             scr.data_ptr(), nscr)
    torch.cuda.synchronize()
    X, P, DZ = host(x), host(params), host(dz)
    Wm, sc, sh = P[:Cout * 9 * Cin].reshape(Cout, 9 * Cin), P[Cout * 9 * Cin:Cout * 9 * Cin + Cout], P[Cout * 9 * Cin + Cout:]
    cols = ro._im2col(X, stride)
    z_ref = cols @ Wm.T
    y_ref = np.maximum(z_ref * sc + sh, 0.0)
    dx_ref = ro._col2im((DZ.reshape(-1, Cout) @ Wm).reshape(cols.shape), X.shape, stride)
    dW_ref = DZ.reshape(-1, Cout).T @ cols.reshape(-1, 9 * Cin)
    out_tol = 2.0 ** -8 if dtype == "bf16" else 3e-6
    for got, ref, tol, name in ((host(z), z_ref, out_tol, "z"), (host(y), y_ref, out_tol * 1.5, "y"),
                                (host(dx), dx_ref, out_tol, "dx"), (host(dW), dW_ref, 3e-6, "dW")):
        err = np.max(np.abs(got - ref.reshape(got.shape))) / np.max(np.abs(ref))
        assert err <= tol, (name, err)


def run_pair(torch, w, steps, tau=None, N=1, gpu_kw=None, check_tables=True, **kw):
    params = wl.init_params(w)
    tf, tb = tau if tau is not None else po.pipeline_delays(w.P, N)
    stream = wl.ImageStream(w)
    o = make_oracle(w, params, tf, tb, N=N, **kw)
    g = make_gpu(w, params, tf, tb, N=N, **dict(kw, **(gpu_kw or {})))
    losses = []
    for k in range(steps):
        mbs = [stream.batch(k * N + j) for j in range(N)]
        lo = o.step(mbs if N > 1 else mbs[0])
        lg = 0.0
        for x, y in mbs:
            lg += g.step(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda(), want_loss=True) / N
        losses.append((lo, lg))
        if check_tables:
            t_used, fs, bs, ws, lrs = g.step_table()
            assert t_used == k
            for u, L in enumerate(w.layers):
                R = tf[L.stage - 1] + 1
                vf, vb = o.last_versions[u]
                assert (fs[u], bs[u], ws[u]) == (vf % R, vb % R, (k + 1) % R)
                assert lrs[u] == pytest.approx(o.last_lr[u], rel=2e-7)
    return g, o, losses


@pytest.mark.parametrize("case", ["pipemare_f32", "pipemare_bf16", "t2_off", "pipedream", "gpipe", "adamw_clip",
                                  "microbatches", "two_blocks_bf16"])
def test_small_resnet_modes(torch_cuda, case):
    dtype = "bf16" if case.endswith("bf16") else "f32"
    nb = 2 if case == "two_blocks_bf16" else 1
    w = wl.resnet(nb, 6, dtype=dtype, image=8)
    kw = dict(opt="sgdm", lr=0.02, beta=0.9, D=0.5, K=6)
    tau, N = None, 1
    if case == "t2_off":
        kw["t2"] = False
    elif case == "pipedream":
        tau = po.pipeline_delays(w.P, 1, "pipedream")
    elif case == "gpipe":
        tau = po.pipeline_delays(w.P, 1, "gpipe")
    elif case == "adamw_clip":
        kw = dict(opt="adamw", lr=1e-3, beta=0.9, beta2=0.98, weight_decay=0.01, clip_norm=0.5, D=0.3, K=6)
    elif case == "microbatches":
        N = 2
    g, o, losses = run_pair(torch_cuda, w, 12, tau=tau, N=N, **kw)
    for lo, lg in losses:
        assert lg == pytest.approx(lo, rel=3e-2 if dtype == "bf16" else 1e-4)
    err, errs = max_rel_err(g.weights(), o.weights())
    print(case, "max-rel", err)
    assert err <= TOL[dtype], errs
    g.close()
