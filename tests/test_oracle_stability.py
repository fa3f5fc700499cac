"""Pins for the stability-analysis functions: the paper's closed forms (Lemma 1, p(1), p'(1), p''(1), the
gamma assignment), its stated findings on the T2 figure's setting, and the oracle's own trajectories."""
import math

import numpy as np
import pytest

from oracle import pipemare_oracle as po
from oracle import stability as stab
from test_oracle_pins import scalar_oracle, trajectory


@pytest.mark.parametrize("tau", [1, 2, 5, 10, 40])
def test_lemma1_threshold_is_the_largest_stable_step(tau):
    lam = 1.7
    a_star = stab.lemma1_threshold(tau, lam)
    found = stab.largest_stable_alpha(lambda a: stab.sgd_delay_polynomial(tau, a, lam))
    assert found == pytest.approx(a_star, rel=1e-6)
    assert stab.spectral_radius(stab.sgd_delay_polynomial(tau, 0.98 * a_star, lam)) < 1.0
    assert stab.spectral_radius(stab.sgd_delay_polynomial(tau, 1.02 * a_star, lam)) > 1.0


def test_printed_values_of_the_t2_polynomial_at_one():
    tf, tb, lam, alpha = 40, 10, 1.3, 0.004
    for Delta in (-7.0, 0.0, 5.0, 60.0):
        for gamma in (0.3, stab.gamma_second_order(tf, tb), stab.gamma_from_D(0.135, tf, tb)):
            c = stab.t2_polynomial(tf, tb, alpha, lam, Delta, gamma)
            assert np.polyval(c, 1.0) == pytest.approx(alpha * lam * (1 - gamma), rel=1e-10)
            assert np.polyval(np.polyder(c), 1.0) == pytest.approx(alpha * lam + 1 - gamma, rel=1e-10)
            d = tf - tb
            want = 2 * tf * (1 - gamma) + 2 - alpha * Delta * d * (1 + gamma - (1 - gamma) * d)
            assert np.polyval(np.polyder(c, 2), 1.0) == pytest.approx(want, rel=1e-9)
    # the assignment gamma = 1 - 2/(tf - tb + 1) removes Delta from the second derivative, and D -> e^-2
    g = stab.gamma_second_order(tf, tb)
    vals = [np.polyval(np.polyder(stab.t2_polynomial(tf, tb, alpha, lam, D_, g), 2), 1.0) for D_ in (-50.0, 0.0, 80.0)]
    assert max(vals) - min(vals) < 1e-9
    assert stab.gamma_second_order(4000, 0) ** 4000 == pytest.approx(math.exp(-2.0), rel=1e-3)


def test_t2_figure_setting_findings():
    """tau_fwd 40, tau_bkwd 10: the correction enlarges the stable range for Delta >= 0 and can shrink it for
    some Delta < 0 (appendix, discussion of the comparison figure)."""
    rows = stab.stability_table(40, 10, [0.0, 1.0, 5.0, 20.0, 100.0])
    for Delta, a0, a1 in rows:
        assert a1 >= a0 * (1 - 1e-9), (Delta, a0, a1)
    assert any(a1 > 1.2 * a0 for _, a0, a1 in rows)
    neg = stab.stability_table(40, 10, [-100.0, -30.0, -10.0, -3.0, -1.0, -0.3])
    assert any(a1 < a0 for _, a0, a1 in neg)
    # Delta = 0: without correction this is Lemma 1 with tau = tau_fwd
    assert rows[0][1] == pytest.approx(stab.lemma1_threshold(40), rel=1e-6)


def test_uncorrected_two_delay_polynomial_reduces():
    # equal delays: the Delta terms cancel and Lemma 1 is back
    for D_ in (-3.0, 4.0):
        a = stab.largest_stable_alpha(lambda x: stab.uncorrected_polynomial(7, 7, x, 1.0, D_))
        assert a == pytest.approx(stab.lemma1_threshold(7), rel=1e-6)
    # the printed and the text reading of the corrected polynomial coincide for tau_bkwd = 0, differ otherwise
    g = 0.8
    assert np.allclose(stab.t2_polynomial(9, 0, 0.01, 1.0, 5.0, g, "printed"), stab.t2_polynomial(9, 0, 0.01, 1.0, 5.0, g, "text"))
    assert not np.allclose(stab.t2_polynomial(9, 3, 0.01, 1.0, 5.0, g, "printed"), stab.t2_polynomial(9, 3, 0.01, 1.0, 5.0, g, "text"))


@pytest.mark.parametrize("t2", [False, True])
def test_threshold_separates_the_oracles_trajectories(t2):
    """The step size found from the polynomial is where the recurrence itself turns from decay to growth."""
    tf, tb, lam, Delta, D = 10, 0, 1.0, 5.0, 0.3
    gamma = stab.gamma_from_D(D, tf, tb)
    poly = (lambda a: stab.t2_polynomial(tf, tb, a, lam, Delta, gamma, "text")) if t2 else \
           (lambda a: stab.uncorrected_polynomial(tf, tb, a, lam, Delta))
    a_star = stab.largest_stable_alpha(poly)

    def growth(alpha):
        o = scalar_oracle(1, [tf], [tb], lam=lam, Delta=Delta, sched=dict(kind="const", base=alpha), t1=False, t2=t2, D=D)
        w = np.abs(trajectory(o, 4000)[0])
        return w[3600:4000].max() / w[2600:3000].max()
    assert growth(0.93 * a_star) < 1.0 < growth(1.07 * a_star)


@pytest.mark.parametrize("tf,tb", [(10, 6), (10, 0), (5, 4), (40, 10), (3, 1)])
def test_lemma2_bound_on_the_stable_range_with_discrepancy(tf, tb):
    """Sec. 3.2, lemma on the discrepancy-dependent update: for Delta > 0 instability sets in at some
    alpha <= min(2 / (Delta (tau_fwd - tau_bkwd)), (2 / lam) sin(pi / (4 tau_fwd + 2)))."""
    lam = 1.0
    for Delta in (0.5, 5.0, 50.0):
        a = stab.largest_stable_alpha(lambda x: stab.uncorrected_polynomial(tf, tb, x, lam, Delta))
        bound = min(2.0 / (Delta * (tf - tb)), stab.lemma1_threshold(tf, lam))
        assert a <= bound * (1 + 1e-6), (Delta, a, bound)


def test_discrepancy_figure_setting():
    """Sec. 3.2 figure, tau_fwd 10, tau_bkwd 6, lam 1: (a) a non-zero Delta makes a step size diverge that
    converges with Delta = 0; (b) with Delta = 5 the discrepancy raises the largest eigenvalue magnitude,
    the correction with D = 0.1 lowers it again, close to the value without discrepancy."""
    tf, tb, lam, Delta, D = 10, 6, 1.0, 5.0, 0.1
    g = stab.gamma_from_D(D, tf, tb)
    for alpha in (0.04, 0.06, 0.08):
        r_none = stab.spectral_radius(stab.uncorrected_polynomial(tf, tb, alpha, lam, 0.0))
        r_disc = stab.spectral_radius(stab.uncorrected_polynomial(tf, tb, alpha, lam, Delta))
        r_corr = stab.spectral_radius(stab.t2_polynomial(tf, tb, alpha, lam, Delta, g))
        assert r_none < 1.0 < r_disc
        assert r_corr < 1.0 and abs(r_corr - r_none) < 0.25 * abs(r_disc - r_none)
    # the same on the recurrence itself (noise-free trajectories of the oracle)
    def growth(Delta_, alpha):
        o = scalar_oracle(1, [tf], [tb], lam=lam, Delta=Delta_, sched=dict(kind="const", base=alpha), t1=False, t2=False)
        w = np.abs(trajectory(o, 1500)[0])
        return w[1300:1500].max() / w[800:1000].max()
    assert growth(0.0, 0.06) < 1.0 < growth(Delta, 0.06)
