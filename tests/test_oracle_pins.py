"""Pins for the CPU oracle: every check compares it with something that is not the oracle.

Closed forms and special cases come from the paper (sections cited per test); the
autograd / torch.optim comparisons use an independent implementation of the textbook
algorithm that the method must reduce to.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import pipemare_oracle as po
import workloads as wl


# ----------------------------------------------------------------------------- helpers
def read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            if ":" in line:
                k, v = line.split(":")
                out[k.strip()] = [float(x) for x in v.split()]
            else:
                k, v = line.split()[:2]
                out[k] = float(v)
    return out


def scalar_oracle(n, tau_fwd, tau_bkwd, lam=1.0, Delta=0.0, w0=1.0, **opt):
    model = po.QuadraticModel(n, lam, Delta)
    return po.PipeMareOracle(model, [np.array([w0])] * n, list(range(1, n + 1)), tau_fwd, tau_bkwd,
                             opt, keep_history=True)


def trajectory(o, steps, eta=None):
    for _ in range(steps):
        o.step(eta)
    return [np.array([o.hist[u][k][0] for k in range(o.t + 1)]) for u in range(o.U)]


# ----------------------------------------------------------------------------- delays (Sec. 2.2, Table 1)
def test_delay_table():
    assert po.pipeline_delays(4, 1) == ([7, 5, 3, 1], [0, 0, 0, 0])
    tf, tb = po.pipeline_delays(16, 1)
    assert tf == [2 * (16 - i) + 1 for i in range(1, 17)] and tb == [0] * 16
    # last stage always ceil(1/N) = 1, first ceil((2P-1)/N)
    for P in (1, 2, 7, 107):
        for N in (1, 2, 3, 8, 19):
            tf, _ = po.pipeline_delays(P, N)
            assert tf[-1] == 1 and tf[0] == math.ceil((2 * P - 1) / N)
            assert all(a >= b for a, b in zip(tf, tf[1:]))
    assert po.pipeline_delays(5, 2, "pipedream") == ([5, 4, 3, 2, 1], [5, 4, 3, 2, 1])
    assert po.pipeline_delays(5, 2, "gpipe") == ([0] * 5, [0] * 5)


def test_paper_utilisation_and_memory_numbers(golden_dir):
    c = read_golden(os.path.join(golden_dir, "paper_constants.txt"))
    assert round(po.gpipe_utilization(16, 107), 2) == c["util_imagenet_resnet50"]
    assert round(po.gpipe_utilization(19, 93), 2) == c["util_iwslt_transformer"]
    assert round(po.gpipe_utilization(round(29000 / 251), 91), 2) == c["util_wmt_transformer"]
    # one extra buffer (delta) on top of (w, g, v) or (w, g, m, s)
    assert round(4 / 3, 2) == c["t2_mem_sgdm"] and round(5 / 4, 2) == c["t2_mem_adam"]
    # PipeDream's stash formula on a toy: sizes 10,20 with tau 3,1
    assert po.pipedream_stash_elems([10, 20], [3, 1]) == 50


# ----------------------------------------------------------------------------- T1 closed form (Sec. 3.1)
def test_t1_closed_form_every_step():
    K = 20
    for tau in (1, 3, 7, 31):
        for k in range(0, 50):
            got = po.t1_lr(0.01, tau, k, K)
            p = 1 - min(k / K, 1)
            assert got == pytest.approx(0.01 * tau ** (-p), rel=1e-15)
        assert po.t1_lr(0.01, tau, 0, K) == pytest.approx(0.01 / tau)
        assert po.t1_lr(0.01, tau, K, K) == 0.01          # exactly the base rate from K on
        assert po.t1_lr(0.01, tau, 10 * K, K) == 0.01
    assert po.t1_lr(0.3, 1, 0, K) == 0.3                   # tau = 1 is never rescaled
    assert po.t1_lr(0.3, 0, 0, K) == 0.3                   # tau = 0 (synchronous) neither
    assert po.t1_lr(0.3, 9, 0, 0) == 0.3                   # K = 0 switches T1 off
    # geometric interpolation: log(lr) is linear in k during the anneal
    l = [math.log(po.t1_lr(1.0, 8, k, 16)) for k in range(17)]
    assert np.allclose(np.diff(l), math.log(8) / 16)


def test_t1_in_the_step_uses_stage_delay_and_step_counter():
    o = scalar_oracle(3, [5, 3, 1], [0, 0, 0], sched=dict(kind="const", base=0.05), K=10, t2=False)
    for k in range(14):
        o.step(None)
        for u, tau in enumerate([5, 3, 1]):
            assert o.last_lr[u] == pytest.approx(0.05 / tau ** (1 - min(k / 10, 1)), rel=1e-15)


def test_base_schedules():
    s = dict(kind="step", base=0.1, factor=0.1, interval=30)
    assert [po.base_lr(s, k) for k in (0, 29, 30, 59, 60)] == pytest.approx([0.1, 0.1, 0.01, 0.01, 0.001])
    s = dict(kind="warmup_invsqrt", base=5e-4, init=1e-7, warmup=8000)
    assert po.base_lr(s, 0) == 1e-7
    assert po.base_lr(s, 4000) == pytest.approx((1e-7 + 5e-4) / 2)
    assert po.base_lr(s, 8000) == pytest.approx(5e-4)
    assert po.base_lr(s, 32000) == pytest.approx(2.5e-4)


# ----------------------------------------------------------------------------- gamma <-> D (Sec. 3.2, App. B)
def test_gamma_and_decay(golden_dir):
    c = read_golden(os.path.join(golden_dir, "paper_constants.txt"))
    assert po.t2_gamma(0.9, 7, 0) == pytest.approx(0.9 ** (1 / 7))
    assert po.t2_gamma(0.25, 2, 0) == pytest.approx(0.5)
    assert po.t2_gamma(0.5, 4, 4) == 0.0
    for tf, tb in ((10, 0), (10, 6), (40, 10)):
        g = po.t2_gamma(0.3, tf, tb)
        assert po.t2_decay_from_gamma(g, tf, tb) == pytest.approx(0.3)
    # gamma = 1 - 2/(tau+1)  ->  D -> exp(-2) ~ 0.135 for the delays of the experiments
    g = 1 - 2 / (40 - 0 + 1)
    assert round(po.t2_decay_from_gamma(g, 40, 0), 3) == c["suggested_D"]
    assert po.t2_decay_from_gamma(1 - 2 / 4001, 4000, 0) == pytest.approx(math.exp(-2), rel=1e-3)


# ----------------------------------------------------------------------------- hand-worked recurrences
def test_hand_worked_recurrences(golden_dir):
    g = read_golden(os.path.join(golden_dir, "scalar_recurrences.txt"))
    tf, tb = po.pipeline_delays(2, 1)
    assert tf == [3, 1]
    o = scalar_oracle(2, tf, tb, sched=dict(kind="const", base=0.1), t1=False, t2=False)
    tr = trajectory(o, 6)
    assert np.allclose(tr[0][1:], g["A.stage1"], atol=1e-12)
    assert np.allclose(tr[1][1:], g["A.stage2"], atol=1e-12)

    o = scalar_oracle(1, [2], [0], Delta=1.0, sched=dict(kind="const", base=0.1), t1=False, t2=True, D=0.25)
    ws, ds = [], []
    for _ in range(4):
        o.step(None)
        ws.append(o.weights(0)[0])
        ds.append(o.delta[0][0])
    assert np.allclose(ws, g["B.w"], atol=1e-12) and np.allclose(ds, g["B.delta"], atol=1e-12)

    o = scalar_oracle(1, [2], [0], sched=dict(kind="const", base=0.2), K=4, beta=0.5, t2=False)
    ws, lrs = [], []
    for _ in range(5):
        o.step(None)
        ws.append(o.weights(0)[0])
        lrs.append(o.last_lr[0])
    assert np.allclose(ws, g["C.w"], atol=2e-9) and np.allclose(lrs, g["C.lr"], atol=2e-9)


# ----------------------------------------------------------------------------- l2 term and clipping (App. C)
def test_sgd_weight_decay_hand_worked_and_torch(golden_dir):
    """The l2 term enters the gradient with the current weights w_t inside v <- beta v - alpha g'
    (App. B.3 form, App. C's l2 settings): a hand-worked delayed trajectory, then equality with
    torch.optim.SGD(weight_decay=...) at zero delay and constant step size."""
    g = read_golden(os.path.join(golden_dir, "scalar_recurrences.txt"))
    o = scalar_oracle(1, [1], [0], sched=dict(kind="const", base=0.1), beta=0.5, weight_decay=0.5, t1=False, t2=False)
    ws = []
    for _ in range(3):
        o.step(None)
        ws.append(o.weights(0)[0])
    assert np.allclose(ws, g["D.w"], atol=1e-12)

    w, params, stream = _mlp_setup("xent", "gelu")
    P = w.P
    model = po.MLPModel(w.layers, w.loss)
    o = po.PipeMareOracle(model, params, [L.stage for L in w.layers], [0] * P, [0] * P,
                          dict(kind="sgdm", beta=0.9, weight_decay=0.05, sched=dict(kind="const", base=0.05), t1=False))
    tp = [torch.tensor(p, dtype=torch.float64, requires_grad=True) for p in params]
    opt = torch.optim.SGD(tp, lr=0.05, momentum=0.9, weight_decay=0.05)
    for k in range(8):
        x, y = stream.batch(k)
        o.step((x, y))
        opt.zero_grad()
        _torch_loss(w, _torch_forward(w, tp, x), y).backward()
        opt.step()
    for a, b in zip(o.weights(), tp):
        assert np.allclose(a, b.detach().numpy(), rtol=0, atol=1e-12)
    # and the decay really moved something: without it the weights differ visibly
    o0 = po.PipeMareOracle(model, params, [L.stage for L in w.layers], [0] * P, [0] * P,
                           dict(kind="sgdm", beta=0.9, sched=dict(kind="const", base=0.05), t1=False))
    for k in range(8):
        o0.step(stream.batch(k))
    assert max(np.max(np.abs(a - b)) for a, b in zip(o.weights(), o0.weights())) > 1e-3


def test_global_norm_clipping_hand_worked_and_torch(golden_dir):
    """One threshold over the gradients of ALL stages, applied to the averaged minibatch gradient
    (App. C, Transformer table): hand-worked two-stage case, then torch's clip_grad_norm_."""
    g = read_golden(os.path.join(golden_dir, "scalar_recurrences.txt"))

    def two_stage(clip, batch=None):
        model = po.QuadraticModel(2, 1.0, 0.0)
        o = po.PipeMareOracle(model, [np.array([3.0]), np.array([4.0])], [1, 2], [0, 0], [0, 0],
                              dict(sched=dict(kind="const", base=0.1), t1=False, t2=False, clip_norm=clip))
        o.step(batch)
        return [o.weights(0)[0], o.weights(1)[0]], o.last_grads

    w1, gr = two_stage(2.5)
    assert np.allclose(w1, g["E.clipped"], atol=1e-14)
    assert np.allclose([gr[0][0], gr[1][0]], [1.5, 2.0], atol=1e-14)       # both scaled by exactly 0.5
    w1, gr = two_stage(10.0)
    assert np.allclose(w1, g["E.unclipped"], atol=1e-14)
    assert np.allclose([gr[0][0], gr[1][0]], [3.0, 4.0], atol=1e-14)
    w1, _ = two_stage(2.5, [np.array([-3.0, -4.0]), np.array([3.0, 4.0])])   # clipped after averaging
    assert np.allclose(w1, g["E.clipped"], atol=1e-14)

    w, params, stream = _mlp_setup("xent", "gelu")
    P = w.P
    model = po.MLPModel(w.layers, w.loss)
    clip = 0.2
    o = po.PipeMareOracle(model, params, [L.stage for L in w.layers], [0] * P, [0] * P,
                          dict(kind="sgdm", beta=0.9, clip_norm=clip, sched=dict(kind="const", base=0.05), t1=False))
    tp = [torch.tensor(p, dtype=torch.float64, requires_grad=True) for p in params]
    opt = torch.optim.SGD(tp, lr=0.05, momentum=0.9)
    clipped_steps = 0
    for k in range(8):
        x, y = stream.batch(k)
        o.step((x, y))
        opt.zero_grad()
        _torch_loss(w, _torch_forward(w, tp, x), y).backward()
        total = float(torch.nn.utils.clip_grad_norm_(tp, clip))
        clipped_steps += total > clip
        opt.step()
    assert clipped_steps >= 4                       # the threshold was active
    for a, b in zip(o.weights(), tp):
        # torch divides by (norm + 1e-6): a relative difference of ~1e-5 in the clipped gradient
        assert np.allclose(a, b.detach().numpy(), rtol=0, atol=2e-6)


# ----------------------------------------------------------------------------- Lemma 1 threshold (Sec. 3.1)
def _amplitude(o, steps):
    tr = trajectory(o, steps)[0]
    return np.max(np.abs(tr[-50:]))


@pytest.mark.parametrize("tau", [0, 1, 5, 10])
def test_lemma1_threshold_both_sides(tau):
    lam = 1.7
    thr = 2.0 / lam * math.sin(math.pi / (4 * tau + 2))
    if tau == 0:
        assert thr == pytest.approx(2.0 / lam)            # textbook gradient-descent bound
    steps = 6000
    stable = scalar_oracle(1, [tau], [tau], lam=lam, sched=dict(kind="const", base=0.98 * thr), t1=False)
    unstable = scalar_oracle(1, [tau], [tau], lam=lam, sched=dict(kind="const", base=1.02 * thr), t1=False)
    assert _amplitude(stable, steps) < 1e-3
    assert _amplitude(unstable, steps) > 1e3
    # an off-by-one in the delay would move the threshold by more than the 2 % margin
    for other in (tau - 1, tau + 1):
        if other >= 0:
            thr_o = 2.0 / lam * math.sin(math.pi / (4 * other + 2))
            assert abs(thr_o / thr - 1) > 0.04


def test_fig2a_setting(golden_dir):
    c = read_golden(os.path.join(golden_dir, "paper_constants.txt"))
    alpha = c["fig2a_alpha"]
    rng = np.random.default_rng(0)
    res = {}
    for tau in (5, 10):
        o = scalar_oracle(1, [tau], [tau], lam=1.0, w0=0.0, sched=dict(kind="const", base=alpha), t1=False)
        for _ in range(1500):
            o.step(rng.standard_normal())
        res[tau] = abs(o.weights(0)[0])
    assert res[10] > 1e6 and res[5] < 50.0


# ----------------------------------------------------------------------------- characteristic polynomials
def _annihilates(coeffs_high_to_low, w, tol):
    """sum_j c_j w_{t+j} = 0 for every t where all indices are past the pipeline fill."""
    c = np.asarray(coeffs_high_to_low)[::-1]          # c[j] multiplies w_{t+j}
    n = len(c)
    res = [abs(np.dot(c, w[t:t + n])) for t in range(0, len(w) - n)]
    return max(res) < tol, max(res)


def test_momentum_polynomial_annihilates_trajectory():
    # App. B.3: p(w) = w^{tau+1} - (1+beta) w^tau + beta w^{tau-1} + alpha*lambda
    tau, beta, alpha, lam = 6, 0.8, 0.03, 1.3
    o = scalar_oracle(1, [tau], [tau], lam=lam, sched=dict(kind="const", base=alpha), beta=beta, t1=False)
    w = trajectory(o, 120)[0]
    coeffs = np.zeros(tau + 2)
    coeffs[0] = 1.0
    coeffs[1] = -(1 + beta)
    coeffs[2] = beta
    coeffs[-1] += alpha * lam
    # the shift-recurrence p(E) w_{t - tau} = 0 holds once real history exists (t >= tau + 1)
    ok, worst = _annihilates(coeffs, w[tau + 1:], 1e-12)
    assert ok, worst
    # and a wrong delay does not satisfy it
    o2 = scalar_oracle(1, [tau + 1], [tau + 1], lam=lam, sched=dict(kind="const", base=alpha), beta=beta, t1=False)
    assert not _annihilates(coeffs, trajectory(o2, 120)[0][tau + 2:], 1e-6)[0]


def _t2_poly(tf, tb, alpha, lam, Delta, gamma):
    """App. B polynomial of the T2-corrected quadratic model, coefficients high -> low."""
    P = np.polynomial.polynomial
    w = [0.0, 1.0]
    wm1 = [-1.0, 1.0]
    wmg = [-gamma, 1.0]
    wpow = lambda n: [0.0] * n + [1.0]
    p = P.polymul(P.polymul(wm1, wmg), wpow(tf))
    p = P.polyadd(p, alpha * (lam + Delta) * np.array(wmg))
    p = P.polysub(p, alpha * Delta * np.array(P.polymul(wpow(tf - tb), wmg)))
    p = P.polyadd(p, alpha * Delta * (tf - tb) * (1 - gamma) * np.array(P.polymul(wpow(tf - tb), wm1)))
    return np.asarray(p)[::-1]


def test_t2_polynomial_annihilates_trajectory_and_spectral_radius():
    # Fig. 3(b) setting scaled to tau_bkwd = 0: tau_fwd = 10, Delta = 5, D = 0.1
    tf, tb, lam, Delta, D, alpha = 10, 0, 1.0, 5.0, 0.1, 0.01
    gamma = D ** (1.0 / (tf - tb))
    coeffs = _t2_poly(tf, tb, alpha, lam, Delta, gamma)
    # printed values of the polynomial and its derivative at 1
    assert np.polyval(coeffs, 1.0) == pytest.approx(alpha * lam * (1 - gamma), rel=1e-12)
    assert np.polyval(np.polyder(coeffs), 1.0) == pytest.approx(alpha * lam + 1 - gamma, rel=1e-12)
    o = scalar_oracle(1, [tf], [tb], lam=lam, Delta=Delta, sched=dict(kind="const", base=alpha),
                      t1=False, t2=True, D=D)
    w = trajectory(o, 400)[0]
    ok, worst = _annihilates(coeffs, w[tf + 2:], 1e-11)
    assert ok, worst
    # growth/decay rate of the trajectory equals the largest root modulus
    rho = max(abs(np.roots(coeffs)))
    o = scalar_oracle(1, [tf], [tb], lam=lam, Delta=Delta, sched=dict(kind="const", base=alpha),
                      t1=False, t2=True, D=D)
    w = np.abs(trajectory(o, 3000)[0])
    env = [w[a:a + 200].max() for a in (1600, 2600)]
    rate = (env[1] / env[0]) ** (1 / 1000)
    assert rate == pytest.approx(rho, rel=2e-4)
    # a sign error in the correction (extrapolating the wrong way) gives another polynomial
    bad = _t2_poly(tf, tb, alpha, lam, -Delta, gamma)
    assert not _annihilates(bad, w[tf + 2:], 1e-6)[0]


def test_t2_off_matches_uncorrected_polynomial():
    # Sec. 3.2 update: w_{t+1} = w_t - a(lam+Delta) w_{t-tf} + a Delta w_{t-tb}
    tf, tb, lam, Delta, alpha = 10, 6, 1.0, 5.0, 0.004
    o = scalar_oracle(1, [tf], [tb], lam=lam, Delta=Delta, sched=dict(kind="const", base=alpha),
                      t1=False, t2=False)
    w = trajectory(o, 200)[0]
    coeffs = np.zeros(tf + 2)
    coeffs[0], coeffs[1] = 1.0, -1.0
    coeffs[-1] += alpha * (lam + Delta)
    coeffs[tf + 1 - (tf - tb)] -= alpha * Delta       # w^{tf - tb} term
    ok, worst = _annihilates(coeffs, w[tf + 1:], 1e-12)
    assert ok, worst


# ----------------------------------------------------------------------------- special cases of the step
def _mlp_setup(loss="xent", act="gelu", width=24, depth=3, n_out=5, M=12, seed=3):
    w = wl.small_mlp(width, depth, n_out, act, loss, "f32", M)
    params = [p.astype(np.float64) for p in wl.init_params(w, seed)]
    stream = wl.BatchStream(w)
    return w, params, stream


def _torch_forward(w, tparams, x):
    a = torch.as_tensor(x, dtype=torch.float64)
    for L, p in zip(w.layers, tparams):
        W = p[:L.n_out * L.n_in].reshape(L.n_out, L.n_in)
        b = p[L.n_out * L.n_in:]
        z = a @ W.T + b
        a = {"none": lambda t: t, "relu": torch.relu,
             "gelu": lambda t: torch.nn.functional.gelu(t, approximate="none")}[L.act](z)
    return a


def _torch_loss(w, out, y):
    if w.loss == "mse":
        return torch.mean((out - torch.as_tensor(y, dtype=torch.float64)) ** 2)
    return torch.nn.functional.cross_entropy(out, torch.as_tensor(y, dtype=torch.long))


@pytest.mark.parametrize("loss,act", [("xent", "gelu"), ("mse", "relu")])
def test_all_delays_zero_is_synchronous_momentum_sgd(loss, act):
    w, params, stream = _mlp_setup(loss, act)
    P = w.P
    model = po.MLPModel(w.layers, w.loss)
    o = po.PipeMareOracle(model, params, [L.stage for L in w.layers], [0] * P, [0] * P,
                          dict(kind="sgdm", beta=0.9, sched=dict(kind="const", base=0.05), K=7, D=0.5))
    tp = [torch.tensor(p, dtype=torch.float64, requires_grad=True) for p in params]
    opt = torch.optim.SGD(tp, lr=0.05, momentum=0.9)     # textbook form; equal for a constant rate
    for k in range(12):
        x, y = stream.batch(k)
        lo = o.step((x, y))
        opt.zero_grad()
        lt = _torch_loss(w, _torch_forward(w, tp, x), y)
        lt.backward()
        opt.step()
        assert lo == pytest.approx(float(lt), rel=1e-11)
    for a, b in zip(o.weights(), tp):
        assert np.allclose(a, b.detach().numpy(), rtol=0, atol=1e-12)


def test_all_delays_zero_adamw_matches_torch():
    w, params, stream = _mlp_setup("xent", "gelu")
    P = w.P
    model = po.MLPModel(w.layers, w.loss)
    o = po.PipeMareOracle(model, params, [L.stage for L in w.layers], [0] * P, [0] * P,
                          dict(kind="adamw", beta1=0.9, beta2=0.98, eps=1e-8, weight_decay=0.01,
                               sched=dict(kind="const", base=2e-3), K=5))
    tp = [torch.tensor(p, dtype=torch.float64, requires_grad=True) for p in params]
    opt = torch.optim.AdamW(tp, lr=2e-3, betas=(0.9, 0.98), eps=1e-8, weight_decay=0.01)
    for k in range(10):
        x, y = stream.batch(k)
        o.step((x, y))
        opt.zero_grad()
        _torch_loss(w, _torch_forward(w, tp, x), y).backward()
        opt.step()
    for a, b in zip(o.weights(), tp):
        # torch applies the decay multiplicatively before the step and divides by sqrt(1-b2^t)
        # inside the denominator: same quantity up to how eps is scaled, hence the 1e-7 band
        assert np.allclose(a, b.detach().numpy(), rtol=0, atol=2e-7)


def test_equal_delays_is_uncorrected_stale_sgd_and_ignores_t2():
    """tau_bkwd = tau_fwd: the correction coefficient vanishes, so T2 on/off and any D agree,
    and the step equals SGD on the gradient taken at the stale weights (autograd)."""
    w, params, stream = _mlp_setup("mse", "relu", n_out=2)
    tf, tb = po.pipeline_delays(w.P, 1, "pipedream")
    stage = [L.stage for L in w.layers]
    model = po.MLPModel(w.layers, w.loss)
    opts = dict(kind="sgdm", beta=0.0, sched=dict(kind="const", base=0.03), t1=False)
    a = po.PipeMareOracle(model, params, stage, tf, tb, dict(opts, t2=True, D=0.3), keep_history=True)
    b = po.PipeMareOracle(model, params, stage, tf, tb, dict(opts, t2=False), keep_history=True)
    hist = [[p.copy()] for p in params]
    for k in range(9):
        x, y = stream.batch(k)
        a.step((x, y))
        b.step((x, y))
        stale = [torch.tensor(hist[u][max(k - tf[stage[u] - 1], 0)], requires_grad=True)
                 for u in range(len(params))]
        _torch_loss(w, _torch_forward(w, stale, x), y).backward()
        for u in range(len(params)):
            hist[u].append(hist[u][-1] - 0.03 * stale[u].grad.numpy())
    for u in range(len(params)):
        assert np.array_equal(a.weights(u), b.weights(u))
        assert np.allclose(a.weights(u), hist[u][-1], rtol=0, atol=1e-13)


def test_zero_discrepancy_coefficient_with_t2_off_reads_plain_stale_weights():
    """T2 off with tau_bkwd = 0: backward uses w_t itself (the paper's uncorrected PipeMare)."""
    o_on = scalar_oracle(1, [4], [0], Delta=2.0, sched=dict(kind="const", base=0.02), t1=False, t2=True, D=0.5)
    o_off = scalar_oracle(1, [4], [0], Delta=2.0, sched=dict(kind="const", base=0.02), t1=False, t2=False)
    a, b = trajectory(o_on, 30)[0], trajectory(o_off, 30)[0]
    # identical for the very first update (delta_0 = 0), different afterwards
    assert a[1] == b[1] and abs(a[10] - b[10]) > 1e-6
    # uncorrected: w_{t+1} = w_t - a(lam+Delta) w_{t-4} + a*Delta*w_t
    for t in range(4, 29):
        assert b[t + 1] == pytest.approx(b[t] - 0.02 * 3.0 * b[t - 4] + 0.02 * 2.0 * b[t], abs=1e-14)


# ----------------------------------------------------------------------------- the two-weight gradient
def test_two_weight_gradient_against_autograd_construction():
    """Forward value from u_fwd, data-gradient path through u_bkwd: build it with autograd by
    computing z = a @ Wb^T + (a @ (Wf - Wb)^T + b_f).detach-on-input so values use Wf while
    d z/d a flows through Wb only."""
    w, params, stream = _mlp_setup("xent", "gelu")
    rng = np.random.default_rng(5)
    u_f = [p + 0.05 * rng.standard_normal(p.shape) for p in params]
    u_b = [p + 0.05 * rng.standard_normal(p.shape) for p in params]
    x, y = stream.batch(0)
    model = po.MLPModel(w.layers, w.loss)
    loss, grads = model.loss_and_grads(u_f, u_b, (x, y))

    a = torch.as_tensor(x, dtype=torch.float64)
    leaves = []
    for L, pf, pb in zip(w.layers, u_f, u_b):
        nw = L.n_out * L.n_in
        Wf = torch.tensor(pf[:nw].reshape(L.n_out, L.n_in))
        Wb = torch.tensor(pb[:nw].reshape(L.n_out, L.n_in))
        Wg = torch.zeros_like(Wf, requires_grad=True)       # receives dz^T a
        bg = torch.tensor(pf[nw:], requires_grad=True)
        # value: a Wf^T + b ; d/da: Wb ; d/dWg: dz^T a
        z = a @ Wb.T + (a.detach() @ (Wf - Wb).T) + a.detach() @ Wg.T + bg
        a = torch.nn.functional.gelu(z) if L.act == "gelu" else z
        leaves.append((Wg, bg))
    lt = torch.nn.functional.cross_entropy(a, torch.as_tensor(y, dtype=torch.long))
    lt.backward()
    assert loss == pytest.approx(float(lt), rel=1e-12)
    for g, (Wg, bg) in zip(grads, leaves):
        ref = np.concatenate([Wg.grad.numpy().ravel(), bg.grad.numpy()])
        assert np.allclose(g, ref, rtol=0, atol=1e-13)
    # the first layer's backward weights never enter any gradient
    u_b2 = [u_b[0] + 1.0] + u_b[1:]
    _, grads2 = model.loss_and_grads(u_f, u_b2, (x, y))
    assert all(np.array_equal(p, q) for p, q in zip(grads, grads2))


@pytest.mark.parametrize("loss,act", [("xent", "gelu"), ("mse", "relu"), ("mse", "none")])
def test_finite_differences_when_weights_agree(loss, act):
    """grad f(w, w) is the ordinary gradient (Sec. 2.1): central differences of the oracle's loss."""
    w, params, stream = _mlp_setup(loss, act, width=8, depth=2, n_out=3, M=5)
    x, y = stream.batch(1)
    model = po.MLPModel(w.layers, w.loss)
    _, grads = model.loss_and_grads(params, params, (x, y))
    rng = np.random.default_rng(0)
    for u in range(len(params)):
        for idx in rng.choice(params[u].size, size=12, replace=False):
            e = 1e-6
            pp = [p.copy() for p in params]
            pm = [p.copy() for p in params]
            pp[u][idx] += e
            pm[u][idx] -= e
            fd = (model.loss_and_grads(pp, pp, (x, y))[0] - model.loss_and_grads(pm, pm, (x, y))[0]) / (2 * e)
            assert grads[u][idx] == pytest.approx(fd, rel=2e-5, abs=1e-8)


# ----------------------------------------------------------------------------- version bookkeeping
def test_read_versions_clamp_and_history_pruning():
    w, params, stream = _mlp_setup("mse", "relu", width=8, depth=3, n_out=1, M=4)
    tf, tb = po.pipeline_delays(w.P, 1)
    stage = [L.stage for L in w.layers]
    model = po.MLPModel(w.layers, w.loss)
    full = po.PipeMareOracle(model, params, stage, tf, tb, dict(sched=dict(kind="const", base=0.01)), keep_history=True)
    lean = po.PipeMareOracle(model, params, stage, tf, tb, dict(sched=dict(kind="const", base=0.01)), keep_history=False)
    for k in range(15):
        x, y = stream.batch(k)
        assert full.read_versions() == [(max(k - tf[s - 1], 0), k) for s in stage]
        full.step((x, y))
        lean.step((x, y))
    for u in range(len(params)):
        assert np.array_equal(full.weights(u), lean.weights(u))
        assert len(lean.hist[u]) == tf[stage[u] - 1] + 1
        assert len(full.hist[u]) == 16


def test_microbatch_accumulation_is_mean_gradient():
    w, params, stream = _mlp_setup("mse", "relu", width=8, depth=2, n_out=2, M=6)
    stage = [L.stage for L in w.layers]
    model = po.MLPModel(w.layers, w.loss)
    o = po.PipeMareOracle(model, params, stage, [0] * w.P, [0] * w.P,
                          dict(sched=dict(kind="const", base=0.1), t1=False))
    (x0, y0), (x1, y1) = stream.batch(0), stream.batch(1)
    o.step([(x0, y0), (x1, y1)])
    # one microbatch of the concatenation has the same mean loss/gradient
    o2 = po.PipeMareOracle(model, params, stage, [0] * w.P, [0] * w.P,
                           dict(sched=dict(kind="const", base=0.1), t1=False))
    o2.step((np.concatenate([x0, x1]), np.concatenate([y0, y1])))
    for u in range(len(params)):
        assert np.allclose(o.weights(u), o2.weights(u), rtol=0, atol=1e-15)


def test_sync_warmup_then_switch():
    """PipeMareW (Sec. 4): E_w synchronous steps equal a zero-delay run with T1/T2 off; afterwards the
    delayed recurrence applies with the T1 counter restarted, reading versions produced during warm-up."""
    w, params, stream = _mlp_setup("mse", "relu", width=8, depth=3, n_out=1, M=4)
    tf, tb = po.pipeline_delays(w.P, 1)
    stage = [L.stage for L in w.layers]
    model = po.MLPModel(w.layers, w.loss)
    Ew = 6
    o = po.PipeMareOracle(model, params, stage, tf, tb, dict(sched=dict(kind="const", base=0.05), beta=0.9, K=5, D=0.5,
                                                             sync_warmup=Ew), keep_history=True)
    sync = po.PipeMareOracle(model, params, stage, [0] * w.P, [0] * w.P,
                             dict(sched=dict(kind="const", base=0.05), beta=0.9, t1=False, t2=False), keep_history=True)
    for k in range(Ew):
        assert o.read_versions() == [(k, k)] * len(params)
        o.step(stream.batch(k)); sync.step(stream.batch(k))
        assert all(lr == 0.05 for lr in o.last_lr)
    for u in range(len(params)):
        assert np.array_equal(o.weights(u), sync.weights(u))
    # first asynchronous step: delayed versions come from the warm-up history, T1 exponent is 1
    assert o.read_versions() == [(max(Ew - tf[s - 1], 0), Ew) for s in stage]
    o.step(stream.batch(Ew))
    for u, s in enumerate(stage):
        assert o.last_lr[u] == pytest.approx(0.05 / max(tf[s - 1], 1))
    o.step(stream.batch(Ew + 1))
    for u, s in enumerate(stage):
        assert o.last_lr[u] == pytest.approx(0.05 / max(tf[s - 1], 1) ** (1 - 1 / 5))
