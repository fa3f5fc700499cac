"""GPU parity at the edges of the configuration space: the smallest shapes, ragged sizes, deep rings,
degenerate delay tables, many wrap-arounds of a two-slot ring."""
import numpy as np
import pytest

import workloads as wl
from oracle import pipemare_oracle as po
from pm_testutil import make_gpu, make_oracle, max_rel_err
from test_gpu_parity import run_pair, torch_cuda  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3}


def _wl(name, widths, acts, stages, loss, dtype, M, n_classes=0):
    layers = tuple(wl.Layer("linear", widths[j], widths[j + 1], acts[j], stages[j]) for j in range(len(acts)))
    return wl.Workload(name, layers, max(stages), 1, loss, dtype, M, n_classes or widths[-1])


def test_single_unit_single_row(torch_cuda):
    w = _wl("one", [5, 3], ["none"], [1], "mse", "f32", 1)
    g, o, losses = run_pair(torch_cuda, w, 12, check_tables=True, lr=0.05, beta=0.9, K=3)
    assert max_rel_err(g.weights(), o.weights())[0] < TOL["f32"]
    for lo, lg in losses:
        assert lg == pytest.approx(lo, rel=1e-4, abs=1e-7)
    g.close()


def test_ragged_fp32_sizes(torch_cuda):
    w = _wl("ragged", [7, 13, 1, 9, 3], ["relu", "gelu", "relu", "none"], [1, 2, 2, 3], "mse", "f32", 5)
    g, o, _ = run_pair(torch_cuda, w, 20, check_tables=True, lr=0.03, beta=0.8, D=0.4, K=5, weight_decay=0.01)
    assert max_rel_err(g.weights(), o.weights())[0] < TOL["f32"]
    g.close()


def test_deep_thin_pipeline_large_delays(torch_cuda):
    # 48 stages of width 8: tau_fwd up to 95, rings of up to 96 slots, most of the run inside the pipeline fill
    P = 48
    w = _wl("deep", [8] * (P + 1), ["gelu"] * (P - 1) + ["none"], list(range(1, P + 1)), "mse", "f32", 4)
    g, o, _ = run_pair(torch_cuda, w, 110, check_tables=True, lr=0.02, beta=0.9, D=0.1, K=40)
    assert max_rel_err(g.weights(), o.weights())[0] < TOL["f32"]
    g.close()


def test_two_slot_rings_wrap_many_times(torch_cuda):
    # every stage tau_fwd = 1 (R = 2): 60 steps = 30 wrap-arounds; tau_bkwd = 1 on one stage (plain stale read)
    w = _wl("wrap", [16, 16, 16, 4], ["relu", "relu", "none"], [1, 2, 3], "mse", "f32", 8)
    g, o, _ = run_pair(torch_cuda, w, 60, tau=([1, 1, 1], [0, 1, 0]), check_tables=True, lr=0.05, beta=0.9, D=0.5, K=0)
    assert max_rel_err(g.weights(), o.weights())[0] < TOL["f32"]
    g.close()


def test_all_delays_zero_with_microbatches(torch_cuda):
    w = _wl("sync", [12, 12, 5], ["gelu", "none"], [1, 2], "xent", "f32", 6, n_classes=5)
    g, o, _ = run_pair(torch_cuda, w, 15, tau=([0, 0], [0, 0]), N=3, check_tables=True, lr=0.1, beta=0.5, K=4)
    assert max_rel_err(g.weights(), o.weights())[0] < TOL["f32"]
    g.close()


def test_bf16_minimum_width_with_decay_and_clipping(torch_cuda):
    w = _wl("bf8", [8, 8, 8, 8], ["relu", "gelu", "none"], [1, 2, 3], "mse", "bf16", 8)
    g, o, _ = run_pair(torch_cuda, w, 20, check_tables=True, lr=0.01, beta=0.9, D=0.5, K=6, weight_decay=0.05,
                       clip_norm=0.3)
    assert max_rel_err(g.weights(), o.weights())[0] < TOL["bf16"]
    g.close()


def test_t1_annealing_window_edges(torch_cuda):
    # K = 1 (T1 over after the first step) and K far beyond the run (exponent stays near 1)
    w = _wl("t1", [10, 10, 10, 2], ["relu", "relu", "none"], [1, 2, 3], "mse", "f32", 4)
    for K in (1, 10**9):
        g, o, _ = run_pair(torch_cuda, w, 12, check_tables=True, lr=0.05, beta=0.9, D=0.5, K=K)
        assert max_rel_err(g.weights(), o.weights())[0] < TOL["f32"]
        g.close()


def test_full_depth_thin_chain_rings_wrap_twice(torch_cuda):
    """P = 99 stages of width 8 (the stage count of the 12-layer Transformer): tau_fwd = 197 .. 1, rings of
    198 .. 2 slots, 420 steps so that even the deepest ring wraps twice.  A near-identity linear chain
    (W = I + 0.05 N) keeps signal and gradient alive through all 99 units, so every unit's weights move
    by more than 1 % and every delayed read matters.  Slots bit-exact at every step; weights to 1e-5."""
    P = 99
    layers = tuple(wl.Layer("linear", 8, 8 if j < P - 1 else 2, "none", j + 1) for j in range(P))
    w = wl.Workload("deep99", layers, P, 1, "mse", "f32", 8, 2)
    rng = np.random.default_rng(7)
    params = []
    for L in layers:
        W = np.eye(L.n_out, L.n_in) + 0.05 * rng.standard_normal((L.n_out, L.n_in))
        params.append(np.concatenate([W.ravel(), 0.01 * rng.standard_normal(L.n_out)]).astype(np.float32))
    tf, tb = po.pipeline_delays(P, 1)
    assert tf[0] == 197 and tf[-1] == 1
    kw = dict(lr=5e-5, beta=0.9, D=0.1, K=100)
    o = make_oracle(w, params, tf, tb, **kw)
    g = make_gpu(w, params, tf, tb, **kw)
    stream = wl.BatchStream(w)
    seen_slots = [set() for _ in range(P)]
    for k in range(420):
        x, y = stream.batch(k)
        o.step((x, y))
        g.step(torch_cuda.from_numpy(x).cuda(), torch_cuda.from_numpy(y).cuda())
        t_used, fs, bs, ws, lrs = g.step_table()
        assert t_used == k
        for u in range(P):
            R = tf[u] + 1
            vf, vb = o.last_versions[u]
            assert (fs[u], bs[u], ws[u]) == (vf % R, vb % R, (k + 1) % R)
            seen_slots[u].add(fs[u])
    assert len(seen_slots[0]) == 198 and len(seen_slots[-1]) == 2       # every slot of the deepest ring was read
    err, errs = max_rel_err(g.weights(), o.weights())
    move = [float(np.max(np.abs(a - b.astype(np.float64))) / np.max(np.abs(b))) for a, b in zip(o.weights(), params)]
    print("deep99 max-rel", err, "movement min/max", min(move), max(move))
    assert min(move) > 0.005, move
    assert err < TOL["f32"], errs
    g.close()
