"""Pins for the oracle's recomputation path (paper appendices "PipeMare Recompute" and "Statistical
efficiency and recompute"): each check compares the oracle with something that is not the oracle."""
import os

import numpy as np
import pytest
import torch

from oracle import pipemare_oracle as po
import workloads as wl
from test_oracle_pins import _annihilates, _mlp_setup, scalar_oracle, trajectory


# ----------------------------------------------------------------------------- delays
def test_recompute_delay_table():
    # the appendix's example: 16 stages in 4 segments; stage j of a segment recomputes 2 (S - j) slots early
    assert po.recompute_delays(16, 4) == [6, 4, 2, 0] * 4
    assert po.segment_starts(16, 4) == [1, 5, 9, 13]
    # the recomputed-activation buffers of a segment add up to S (S - 1), the S^2 term of the memory model
    for S in (1, 2, 5, 8):
        assert sum(po.recompute_delays(3 * S, S)[:S]) == S * (S - 1)
    # a shorter last segment counts its own length; microbatches divide the slots (ceiling)
    assert po.recompute_delays(5, 2) == [2, 0, 2, 0, 0]
    assert po.recompute_delays(4, 4, N=2) == [3, 2, 1, 0]
    assert po.recompute_delays(4, 4, N=3) == [2, 2, 1, 0]
    # never beyond the forward delay of the same stage (needed for tau_bkwd <= tau_recomp <= tau_fwd)
    for P, S, N in ((16, 4, 1), (99, 8, 1), (20, 20, 1), (7, 3, 2)):
        tf, tb = po.pipeline_delays(P, N)
        tr = po.recompute_delays(P, S, N)
        assert all(b <= r <= f for f, b, r in zip(tf, tb, tr))
    # on top of a non-zero backward delay
    assert po.recompute_delays(4, 2, tau_bkwd=[1, 1, 1, 1]) == [3, 1, 3, 1]


# ----------------------------------------------------------------------------- the quadratic model
def _recomp_poly(tf, tr, alpha, lam, Delta, Phi, gamma):
    """Characteristic polynomial (coefficients high -> low) of the recurrence the appendix states, for
    tau_bkwd = 0 and the correction taken with the current delta_t as in the T2 text:
      w_{t+1} = w_t - a [ (lam+Delta) w_{t-tf} - (Delta-Phi) (w_t - tf d_t) - Phi (w_{t-tr} - (tf-tr) d_t) ],
      d_{t+1} = g d_t + (1-g)(w_{t+1} - w_t).
    Eliminating d (d = (1-g)(E-1)/(E-g) w in the shift operator E) and clearing denominators:
      (E-1)(E-g)E^tf + a(lam+Delta)(E-g) - a(Delta-Phi)E^tf(E-g) + a(Delta-Phi) tf (1-g) E^tf (E-1)
      - a Phi E^{tf-tr}(E-g) + a Phi (tf-tr)(1-g) E^tf (E-1)."""
    P = np.polynomial.polynomial
    wm1, wmg = [-1.0, 1.0], [-gamma, 1.0]
    wpow = lambda n: [0.0] * n + [1.0]
    p = P.polymul(P.polymul(wm1, wmg), wpow(tf))
    p = P.polyadd(p, alpha * (lam + Delta) * np.array(wmg))
    p = P.polysub(p, alpha * (Delta - Phi) * np.array(P.polymul(wpow(tf), wmg)))
    p = P.polyadd(p, alpha * (Delta - Phi) * tf * (1 - gamma) * np.array(P.polymul(wpow(tf), wm1)))
    p = P.polysub(p, alpha * Phi * np.array(P.polymul(wpow(tf - tr), wmg)))
    p = P.polyadd(p, alpha * Phi * (tf - tr) * (1 - gamma) * np.array(P.polymul(wpow(tf), wm1)))
    return np.asarray(p)[::-1]


def _recomp_oracle(tf, tb, tr, lam, Delta, Phi, alpha, t2, D=0.1):
    model = po.QuadraticModel(1, lam, Delta, Phi)
    return po.PipeMareOracle(model, [np.array([1.0])], [1], [tf], [tb], dict(
        sched=dict(kind="const", base=alpha), t1=False, t2=t2, D=D, tau_recomp=[tr], segment=1), keep_history=True)


def test_recompute_polynomial_annihilates_trajectory():
    tf, tr, lam, Delta, Phi, D, alpha = 10, 4, 1.0, 10.0, -5.0, 0.1, 0.004
    gamma = D ** (1.0 / tf)
    coeffs = _recomp_poly(tf, tr, alpha, lam, Delta, Phi, gamma)
    w = trajectory(_recomp_oracle(tf, 0, tr, lam, Delta, Phi, alpha, True, D), 400)[0]
    ok, worst = _annihilates(coeffs, w[tf + 2:], 1e-11)
    assert ok, worst
    # with tau_recomp = 0 the appendix's printed polynomial and the text's recurrence coincide, and with
    # Phi = 0 both fall back to the T2 polynomial of the main text
    from test_oracle_pins import _t2_poly
    assert np.allclose(_recomp_poly(tf, 0, alpha, lam, Delta, 0.0, gamma), _t2_poly(tf, 0, alpha, lam, Delta, gamma))
    w0 = trajectory(_recomp_oracle(tf, 0, 0, lam, Delta, Phi, alpha, True, D), 300)[0]
    assert _annihilates(_recomp_poly(tf, 0, alpha, lam, Delta, Phi, gamma), w0[tf + 2:], 1e-11)[0]
    # mistakes show: a wrong recompute delay, the correction extrapolating the wrong way, Phi dropped
    for bad in (_recomp_poly(tf, tr + 1, alpha, lam, Delta, Phi, gamma),
                _recomp_poly(tf, tr, alpha, lam, Delta, -Phi, gamma),
                _recomp_poly(tf, tr, alpha, lam, Delta, 0.0, gamma)):
        assert _annihilates(bad, w[tf + 2:], 1e-11)[1] > 1e-8          # the right one leaves ~1e-16


def test_recompute_uncorrected_recurrence():
    # T2 off: w_{t+1} = w_t - a [ (lam+Delta) w_{t-tf} - (Delta-Phi) w_{t-tb} - Phi w_{t-tr} ]   (three plain delays)
    tf, tb, tr, lam, Delta, Phi, alpha = 10, 1, 4, 1.0, 10.0, -5.0, 0.003
    w = trajectory(_recomp_oracle(tf, tb, tr, lam, Delta, Phi, alpha, False), 200)[0]
    c = np.zeros(tf + 2)                       # high -> low, degree tf + 1
    c[0], c[1] = 1.0, -1.0
    c[-1] += alpha * (lam + Delta)
    c[tf + 1 - (tf - tb)] -= alpha * (Delta - Phi)
    c[tf + 1 - (tf - tr)] -= alpha * Phi
    ok, worst = _annihilates(c, w[tf + 1:], 1e-12)
    assert ok, worst


def test_correction_widens_the_stable_range_in_the_appendix_setting(golden_dir):
    """The appendix's figure setting (Delta 10, Phi -5, tau_fwd 10, tau_bkwd 1, tau_recomp 4, lam 1, D 0.1):
    discrepancy correction lowers the largest eigenvalue magnitude.  Checked on trajectories: a step size
    at which the uncorrected recurrence blows up and the corrected one decays."""
    g = {}
    for line in open(os.path.join(golden_dir, "recompute_quadratic.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split()
            g[k] = float(v)
    tf, tb, tr = int(g["tau_fwd"]), int(g["tau_bkwd"]), int(g["tau_recomp"])

    def growth(t2, alpha):
        w = np.abs(trajectory(_recomp_oracle(tf, tb, tr, g["lam"], g["Delta"], g["Phi"], alpha, t2, g["D"]), 1500)[0])
        return (w[1300:1500].max() / w[800:1000].max()) ** (1 / 500)

    alphas = np.linspace(0.002, 0.05, 25)
    stable_plain = [a for a in alphas if growth(False, a) < 1.0]
    stable_corr = [a for a in alphas if growth(True, a) < 1.0]
    assert max(stable_corr) > max(stable_plain)
    a_mid = 0.5 * (max(stable_corr) + max(stable_plain))
    assert growth(False, a_mid) > 1.0 > growth(True, a_mid)


# ----------------------------------------------------------------------------- the MLP gradient
def _three_weight_setup(depth=5, seed=7):
    w, params, stream = _mlp_setup("xent", "gelu", width=16, depth=depth, n_out=4, M=9, seed=seed)
    rng = np.random.default_rng(seed + 1)
    u_f = [p + 0.05 * rng.standard_normal(p.shape) for p in params]
    u_b = [p + 0.05 * rng.standard_normal(p.shape) for p in params]
    u_r = [p + 0.05 * rng.standard_normal(p.shape) for p in params]
    return w, u_f, u_b, u_r, stream.batch(0)


def test_three_weight_gradient_against_autograd_construction():
    """Loss and its gradient at the output from the forward pass (u_fwd); inside each segment inputs
    and activation derivatives from a recomputation with u_recomp that starts at the segment's stored
    input; gradients flow through u_bkwd.  Built independently as a linearised backward chain in torch."""
    w, u_f, u_b, u_r, (x, y) = _three_weight_setup()
    model = po.MLPModel(w.layers, w.loss)
    cps = [0, 2, 5]                                     # segments: layers 0-1, 2-4, 5 (the head)
    loss, grads = model.loss_and_grads(u_f, u_b, (x, y), u_recomp=u_r, checkpoints=cps)

    nL = len(w.layers)
    unpack = lambda p, L: (torch.tensor(p[:L.n_out * L.n_in].reshape(L.n_out, L.n_in)), torch.tensor(p[L.n_out * L.n_in:]))
    act = lambda t, L: torch.nn.functional.gelu(t) if L.act == "gelu" else t
    # forward pass with u_fwd: keeps the loss, d loss / d output, and the inputs of layers 0, 2, 5
    a = torch.as_tensor(x, dtype=torch.float64)
    kept = {}
    for l, L in enumerate(w.layers):
        if l in cps:
            kept[l] = a
        W, b = unpack(u_f[l], L)
        a = act(a @ W.T + b, L)
    out = a.clone().requires_grad_(True)
    lt = torch.nn.functional.cross_entropy(out, torch.as_tensor(y, dtype=torch.long))
    dout, = torch.autograd.grad(lt, out)
    assert loss == pytest.approx(float(lt), rel=1e-12)
    # recomputation with u_recomp from the kept inputs; derivative of the activation by autograd
    a_in, dact = [None] * nL, [None] * nL
    for si, s0 in enumerate(cps):
        s1 = cps[si + 1] if si + 1 < len(cps) else nL
        a = kept[s0]
        for l in range(s0, s1):
            L = w.layers[l]
            W, b = unpack(u_r[l], L)
            a_in[l] = a
            z = (a @ W.T + b).clone().requires_grad_(True)
            av = act(z, L)
            dact[l], = torch.autograd.grad(av.sum(), z)
            a = av.detach()
    # linearised backward chain: h_l = dact_l * (h_{l-1} Wb_l^T + a_in_l Wg_l^T + bg_l), gradient of <dout, h_last>
    leaves, h = [], torch.zeros_like(torch.as_tensor(x, dtype=torch.float64))
    for l, L in enumerate(w.layers):
        Wb, _ = unpack(u_b[l], L)
        Wg = torch.zeros(L.n_out, L.n_in, dtype=torch.float64, requires_grad=True)
        bg = torch.zeros(L.n_out, dtype=torch.float64, requires_grad=True)
        h = dact[l] * (h @ Wb.T + a_in[l] @ Wg.T + bg)
        leaves.append((Wg, bg))
    (dout * h).sum().backward()
    for gl, (Wg, bg) in zip(grads, leaves):
        ref = np.concatenate([Wg.grad.numpy().ravel(), bg.grad.numpy()])
        assert np.allclose(gl, ref, rtol=0, atol=1e-13)
    # the three weight sets all matter, and the recompute weights of the head (no activation, input kept) do not
    for other in (model.loss_and_grads(u_f, u_b, (x, y))[1],
                  model.loss_and_grads(u_f, u_b, (x, y), u_recomp=u_f, checkpoints=cps)[1]):
        assert max(np.max(np.abs(p - q)) for p, q in zip(grads, other)) > 1e-5
    u_r2 = u_r[:-1] + [u_r[-1] + 1.0]
    g2 = model.loss_and_grads(u_f, u_b, (x, y), u_recomp=u_r2, checkpoints=cps)[1]
    assert all(np.array_equal(p, q) for p, q in zip(grads, g2))


def test_recompute_with_forward_weights_is_no_recompute():
    w, u_f, u_b, _, (x, y) = _three_weight_setup()
    model = po.MLPModel(w.layers, w.loss)
    l0, g0 = model.loss_and_grads(u_f, u_b, (x, y))
    for cps in ([0], [0, 3], [0, 1, 2, 3, 4, 5]):
        l1, g1 = model.loss_and_grads(u_f, u_b, (x, y), u_recomp=u_f, checkpoints=cps)
        assert l1 == l0 and all(np.allclose(p, q, rtol=0, atol=1e-15) for p, q in zip(g0, g1))


def test_checkpoint_placement_matters_only_through_the_kept_inputs():
    # one segment per layer: every input is kept, so only the pre-activations are recomputed
    w, u_f, u_b, u_r, (x, y) = _three_weight_setup()
    model = po.MLPModel(w.layers, w.loss)
    g_all = model.loss_and_grads(u_f, u_b, (x, y), u_recomp=u_r, checkpoints=list(range(len(w.layers))))[1]
    g_one = model.loss_and_grads(u_f, u_b, (x, y), u_recomp=u_r, checkpoints=[0])[1]
    assert max(np.max(np.abs(p - q)) for p, q in zip(g_all, g_one)) > 1e-6
    # layer 0's gradient input is x either way; its weight gradient differs only through act'(z_recomputed)
    acts, _ = model.forward(u_f, x)
    assert np.array_equal(acts[0], np.asarray(x, dtype=np.float64))


# ----------------------------------------------------------------------------- in the recurrence
def _run(w, params, stream, steps, **opt):
    model = po.MLPModel(w.layers, w.loss)
    stage = [L.stage for L in w.layers]
    P = max(stage)
    tf, tb = po.pipeline_delays(P, 1)
    o = po.PipeMareOracle(model, params, stage, opt.pop("tau_fwd", tf), opt.pop("tau_bkwd", tb), dict(
        kind="sgdm", beta=0.9, sched=dict(kind="const", base=0.05), K=8, D=0.5, **opt))
    for k in range(steps):
        o.step(stream.batch(k))
    return o


def test_recurrence_special_cases():
    w, params, stream = _mlp_setup("xent", "gelu", width=12, depth=5, n_out=3, M=8)
    P = max(L.stage for L in w.layers)
    tf, _ = po.pipeline_delays(P, 1)
    base = _run(w, params, stream, 25)
    # tau_recomp = tau_fwd: the recomputation reproduces the forward pass, whatever the segments
    same = _run(w, params, stream, 25, tau_recomp=tf, segment=2)
    assert all(np.array_equal(a, b) for a, b in zip(base.weights(), same.weights()))
    # the appendix's delays change the trajectory, and T2 changes it again
    tr = po.recompute_delays(P, 2)
    r_on = _run(w, params, stream, 25, tau_recomp=tr, segment=2)
    r_off = _run(w, params, stream, 25, tau_recomp=tr, segment=2, t2=False)
    assert max(np.max(np.abs(a - b)) for a, b in zip(base.weights(), r_on.weights())) > 1e-6
    assert max(np.max(np.abs(a - b)) for a, b in zip(r_off.weights(), r_on.weights())) > 1e-6
    # all delays zero: synchronous training, recomputation is exact
    z = [0] * P
    s0 = _run(w, params, stream, 12, tau_fwd=z, tau_bkwd=z)
    s1 = _run(w, params, stream, 12, tau_fwd=z, tau_bkwd=z, tau_recomp=z, segment=3)
    assert all(np.allclose(a, b, rtol=0, atol=1e-15) for a, b in zip(s0.weights(), s1.weights()))
    # validation
    with pytest.raises(ValueError):
        _run(w, params, stream, 1, tau_recomp=[t + 1 for t in tf], segment=2)
    with pytest.raises(ValueError):
        _run(w, params, stream, 1, tau_recomp=tr, segment=0)


def test_recompute_reads_the_stated_versions():
    """One scalar stage, hand-unrolled: u_recomp,t = w_{t-tr} - (tf - tr) delta_t."""
    tf, tr, lam, Delta, Phi, alpha, D = 3, 1, 1.0, 2.0, 0.5, 0.1, 0.5
    o = _recomp_oracle(tf, 0, tr, lam, Delta, Phi, alpha, True, D)
    w, d, gam = [1.0], 0.0, D ** (1.0 / tf)
    for t in range(12):
        uf = w[max(t - tf, 0)]
        ub = w[t] - tf * d
        ur = w[max(t - tr, 0)] - (tf - tr) * d
        g = (lam + Delta) * uf - (Delta - Phi) * ub - Phi * ur
        w.append(w[t] - alpha * g)
        d = gam * d + (1 - gam) * (w[t + 1] - w[t])
        o.step(None)
        assert o.weights(0)[0] == pytest.approx(w[-1], rel=1e-14)
