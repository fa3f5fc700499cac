"""Full-size parity for the benchmark workload: 16-stage 1024-wide GELU MLP, bf16 compute with fp32
master weights, microbatch 128, PipeMare delays, 500 optimizer steps, in the launch configuration
bench.py times (captured HIP graph on a side stream, staged batch buffers).

The fp64 oracle runs the same 500 steps on the host (a few minutes); master weights of every unit are
compared element by element at steps 1, 10, 100 and 500.  Bound: max over units of
||w_gpu - w_oracle||_inf / ||w_oracle||_inf <= 2e-3.
"""
import time

import numpy as np
import pytest

import workloads as wl
from oracle import pipemare_oracle as po
from pm_testutil import make_gpu, make_oracle, max_rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(1500)
@pytest.mark.parametrize("launch", ["graph", "overlap", "graph_recompute4", "graph_stochastic", "graph_chain"])
def test_config2_bf16_mlp16_500_steps(launch):
    import torch
    w = wl.config(2)
    o_ = w.opt
    params = wl.init_params(w)
    tf, tb = po.pipeline_delays(w.P, 1)
    assert tf == [2 * (16 - i) + 1 for i in range(1, 17)] and tb == [0] * 16
    kw = dict(lr=o_["lr"], beta=o_["beta"], D=o_["D"], K=o_["K"])
    n_steps = w.steps
    if launch == "graph_recompute4":
        # the same workload with recomputation in segments of 4 stages (App. on recompute), 200 steps
        kw.update(tau_recomp=po.recompute_delays(w.P, 4, 1), segment=4)
        assert kw["tau_recomp"] == [6, 4, 2, 0] * 4
        launch, n_steps = "graph", 200
    if launch == "overlap":
        n_steps = 200            # not the default launch mode (and measured slower): a shorter run keeps the suite in budget
    stoch = None
    if launch == "graph_stochastic":
        # the same workload under Hogwild-style stochastic delays (means = the pipeline's delays), 150 steps
        stoch = dict(tau_max=40, seed=20191005)
        kw.update(stochastic=stoch)
        launch, n_steps = "graph", 150
    chain = launch == "graph_chain"
    if chain:
        # the same 500 steps with the forward products of the 16 wide units in ONE persistent launch and 15 of the
        # 16 data-gradient products in another (the 10-column head keeps its own launches; an option of the library)
        launch = "graph"
    stream = wl.BatchStream(w)
    o = make_oracle(w, params, tf, tb, **kw)
    side = torch.cuda.Stream()
    checkpoints = (1, 10, 100, n_steps)
    report = {}
    t0 = time.time()
    with torch.cuda.stream(side):
        g = make_gpu(w, params, tf, tb, use_graph=(launch == "graph"), overlap_update=(launch == "overlap"),
                     stream=side, chained_launches=chain, **kw)
        assert g.chained_units() == ((16, 15) if chain else (0, 0))
        x0, y0 = stream.batch(0)
        xd, yd = torch.from_numpy(x0).cuda(), torch.from_numpy(y0).cuda()
        for k in range(n_steps):
            x, y = stream.batch(k)
            xd.copy_(torch.from_numpy(x))
            yd.copy_(torch.from_numpy(y))
            lo = o.step((x, y))
            lg = g.step(xd, yd, want_loss=(k % 50 == 0 or k + 1 in checkpoints))
            if k % 50 == 0:
                print(f"step {k}: loss oracle {lo:.5f} gpu {lg:.5f}  ({time.time() - t0:.0f}s)", flush=True)
            if k + 1 in checkpoints:
                err, errs = max_rel_err(g.weights(), o.weights())
                move = max(float(np.max(np.abs(a - b.astype(np.float64))) / np.max(np.abs(b))) for a, b in zip(o.weights(), params))
                report[k + 1] = (err, move)
                print(f"after {k + 1} steps: max-rel weight error {err:.3e} (largest unit movement {move:.3f}); per unit {np.round(errs, 5)}", flush=True)
                t_used, fs, bs, ws, lrs = g.step_table()
                assert t_used == k
                for u, L in enumerate(w.layers):
                    R = (tf[L.stage - 1] if stoch is None else stoch["tau_max"]) + 1
                    vf, vb = o.last_versions[u]
                    assert (fs[u], bs[u], ws[u]) == (vf % R, vb % R, (k + 1) % R)
                    assert lrs[u] == pytest.approx(o.last_lr[u], rel=2e-7)
        g.close()
    for n, (err, move) in report.items():
        assert err <= 2e-3, (n, err)
    assert report[n_steps][1] > 0.02          # the weights really moved: the bound is not met vacuously
