"""Pins for the oracle's Hogwild-style stochastic delays (paper appendix "Hogwild! asynchrony"): the
counter-based generator against published vectors, the delay table against the closed form of the
truncated exponential, and the recurrence against hand-unrolled and special cases."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import pipemare_oracle as po
from test_oracle_pins import _mlp_setup


def _read(path):
    out = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split(":")
            out[k.strip()] = [int(x) for x in v.split()]
    return out


def test_generator_matches_published_splitmix64_vectors(golden_dir):
    g = _read(os.path.join(golden_dir, "splitmix64.txt"))
    seed = g["seed"][0]
    # output number n of the generator = counter (t, i) with t * P + i = n; upper 32 bits
    for P in (1, 5):
        for n, want in enumerate(g["outputs"], start=1):
            t, i = (n - 1) // P, (n - 1) % P + 1
            assert po.counter_u32(seed, t, i, P) == want >> 32
    # a pure function of its arguments
    assert po.counter_u32(9, 3, 2, 7) == po.counter_u32(9, 3, 2, 7) != po.counter_u32(9, 3, 3, 7)


def _pmf(mean, tau_max):
    # P(k <= X < k + 1 | X < tau_max + 1) for X ~ Exp(mean), written without cancellation in the tail
    return np.array([math.exp(-k / mean) * -math.expm1(-1.0 / mean) / -math.expm1(-(tau_max + 1) / mean)
                     for k in range(tau_max + 1)])


@pytest.mark.parametrize("mean,tau_max", [(3.0, 5), (1.0, 12), (31.0, 40), (7.0, 200), (0.5, 3)])
def test_delay_table_is_the_truncated_exponential(mean, tau_max):
    T = po.delay_thresholds(mean, tau_max)
    assert len(T) == tau_max and all(a <= b for a, b in zip(T, T[1:])) and all(0 <= x <= 0xFFFFFFFF for x in T)
    pmf = _pmf(mean, tau_max)
    # exact probabilities of the integer table: P(delay <= k) = (T[k] + 1) / 2^32
    cdf_tab = np.array([(x + 1) / 2.0 ** 32 for x in T] + [1.0])
    assert np.max(np.abs(cdf_tab - np.cumsum(pmf))) < 2.0 ** -31
    # ratio of neighbouring probabilities is e^{-1/mean} (memorylessness survives truncation)
    assert np.allclose(pmf[1:] / pmf[:-1], math.exp(-1.0 / mean), rtol=1e-9)
    # draws: range, frequencies and mean
    n = 60000
    d = np.array([po.stochastic_delay(123, t, 2, 3, T) for t in range(n)])
    assert d.min() >= 0 and d.max() <= tau_max
    freq = np.bincount(d, minlength=tau_max + 1) / n
    sigma = np.sqrt(pmf * (1 - pmf) / n)
    big = n * pmf >= 50                        # bins where the normal approximation holds; the rest pooled
    assert np.all(np.abs(freq - pmf)[big] < 5 * sigma[big])
    rest = float(pmf[~big].sum())
    assert abs(float(freq[~big].sum()) - rest) < 5 * math.sqrt(rest * (1 - rest) / n) + 1e-9
    mu = float(np.dot(np.arange(tau_max + 1), pmf))
    assert abs(d.mean() - mu) < 5 * math.sqrt(float(np.dot((np.arange(tau_max + 1) - mu) ** 2, pmf)) / n)


def test_delay_table_edge_cases():
    assert po.delay_thresholds(4.0, 0) == []                      # tau_max 0: the delay is always 0
    assert po.delay_from_u32(0xFFFFFFFF, []) == 0
    T = po.delay_thresholds(0.0, 6)                               # zero mean: always 0
    assert all(po.delay_from_u32(r, T) == 0 for r in (0, 1, 0x7FFFFFFF, 0xFFFFFFFF))
    T = po.delay_thresholds(5.0, 6)
    assert po.delay_from_u32(0, T) == 0 and po.delay_from_u32(0xFFFFFFFF, T) == 6
    # boundaries of the integer table: the draw equal to a threshold still belongs to the smaller delay
    assert po.delay_from_u32(T[2], T) == 2 and po.delay_from_u32(T[2] + 1, T) == 3
    # stages draw independently, steps draw independently
    a = [po.stochastic_delay(5, t, 1, 2, T) for t in range(400)]
    b = [po.stochastic_delay(5, t, 2, 2, T) for t in range(400)]
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.2 and abs(np.corrcoef(a[:-1], a[1:])[0, 1]) < 0.2
    with pytest.raises(ValueError):
        po.delay_thresholds(1.0, -1)


def _scalar(tau_mean, tau_max, seed, alpha, lam=1.0, **opt):
    model = po.QuadraticModel(len(tau_mean), lam, 0.0)
    n = len(tau_mean)
    return po.PipeMareOracle(model, [np.array([1.0])] * n, list(range(1, n + 1)), tau_mean, [0] * n, dict(
        sched=dict(kind="const", base=alpha), stochastic=dict(tau_max=tau_max, seed=seed), **opt), keep_history=True)


def test_hand_unrolled_stochastic_recurrence():
    """Two scalar stages: w_{i,t+1} = w_{i,t} - alpha_i lam w_{i, max(t - tau_{i,t}, 0)} with the drawn delays;
    T1 divides by the MEAN delay; T2 plays no role (both passes read the same version)."""
    mean, tau_max, seed, alpha, lam, K = [4, 2], 6, 99, 0.05, 1.3, 10
    o = _scalar(mean, tau_max, seed, alpha, lam, K=K, t1=True, t2=True, D=0.5)
    tabs = [po.delay_thresholds(float(m), tau_max) for m in mean]
    w = [[1.0], [1.0]]
    for t in range(40):
        o.step(None)
        for i in (1, 2):
            tau = po.stochastic_delay(seed, t, i, 2, tabs[i - 1])
            assert o.last_delays[i - 1] == tau and o.last_versions[i - 1] == (max(t - tau, 0),) * 2
            p = 1.0 - min(t / K, 1.0)
            lr = alpha / max(mean[i - 1], 1) ** p
            w[i - 1].append(w[i - 1][t] - lr * lam * w[i - 1][max(t - tau, 0)])
            assert o.weights(i - 1)[0] == pytest.approx(w[i - 1][-1], rel=1e-13)
    assert len(set(o.hist[0][k][0] for k in range(41))) == 41          # it really moved every step


def test_tau_max_zero_is_synchronous_training():
    w, params, stream = _mlp_setup("xent", "gelu", width=12, depth=3, n_out=3, M=8)
    stage = [L.stage for L in w.layers]
    P = max(stage)
    model = po.MLPModel(w.layers, w.loss)
    opt = dict(kind="sgdm", beta=0.9, sched=dict(kind="const", base=0.05), K=0)
    a = po.PipeMareOracle(model, params, stage, [3] * P, [0] * P, dict(opt, stochastic=dict(tau_max=0, seed=1)))
    b = po.PipeMareOracle(model, params, stage, [0] * P, [0] * P, dict(opt))
    for k in range(10):
        a.step(stream.batch(k))
        b.step(stream.batch(k))
    assert all(np.array_equal(x, y) for x, y in zip(a.weights(), b.weights()))


def test_stochastic_training_differs_from_fixed_delays_and_ignores_t2_and_tau_bkwd():
    w, params, stream = _mlp_setup("xent", "gelu", width=12, depth=3, n_out=3, M=8)
    stage = [L.stage for L in w.layers]
    P = max(stage)
    tf, _ = po.pipeline_delays(P, 1)
    model = po.MLPModel(w.layers, w.loss)
    base = dict(kind="sgdm", beta=0.9, sched=dict(kind="const", base=0.05), K=6, D=0.5)

    def run(tb, **extra):
        o = po.PipeMareOracle(model, params, stage, tf, tb, dict(base, **extra))
        for k in range(20):
            o.step(stream.batch(k))
        return o.weights()
    st = dict(tau_max=2 * P, seed=3)
    s1 = run([0] * P, stochastic=st)
    s2 = run(list(tf), stochastic=st, t2=False)
    fixed = run([0] * P)
    assert all(np.array_equal(x, y) for x, y in zip(s1, s2))
    assert max(np.max(np.abs(x - y)) for x, y in zip(s1, fixed)) > 1e-6
    s3 = run([0] * P, stochastic=dict(tau_max=2 * P, seed=4))
    assert max(np.max(np.abs(x - y)) for x, y in zip(s1, s3)) > 1e-6
    with pytest.raises(ValueError):
        run([0] * P, stochastic=st, tau_recomp=[0] * P, segment=1)
