"""Stability analysis of the paper's quadratic model: characteristic polynomials of the companion
matrices, their spectral radius, and the largest stable step size.

TEST INFRASTRUCTURE / ANALYSIS ONLY (same rules as pipemare_oracle.py: CPU, fp64 NumPy, nothing in the
product path imports it, no code shared with the HIP library).  `python -m oracle.stability` prints the
data behind the paper's stability figures (largest stable step size against the discrepancy
sensitivity Delta, with and without the T2 correction).

Polynomials (omega = shift operator; a root outside the unit disk means the recurrence diverges):
  * delayed SGD, one delay (Sec. 3.1):              omega^{tau+1} - omega^tau + alpha lam
    Lemma 1: stable iff alpha <= (2 / lam) sin(pi / (4 tau + 2))
  * two delays, no correction (Sec. 3.2):           omega^{tf} (omega - 1) + alpha (lam + Delta) - alpha Delta omega^{tf - tb}
  * T2-corrected (App. B, as printed):
      (omega-1)(omega-gamma) omega^{tf} + alpha (lam+Delta)(omega-gamma) - alpha Delta omega^{tf-tb} (omega-gamma)
      + alpha Delta omega^{tf-tb} (tf-tb)(1-gamma)(omega-1)
    reading "text": the recurrence of the T2 text (correction with the CURRENT delta_t) instead gives
    omega^{tf} in the last term; the two coincide for tb = 0.
  * with recomputation (App. "Statistical efficiency and recompute"): the same with (Delta - Phi) in place of
    Delta plus the two Phi terms for tau_recomp (printed / text readings differ the same way).
Coefficients are returned highest power first (numpy.roots convention).
"""
from __future__ import annotations

import math
from typing import Callable

import numpy as np

_P = np.polynomial.polynomial


def _pw(n):
    return [0.0] * int(n) + [1.0]


def sgd_delay_polynomial(tau: int, alpha: float, lam: float = 1.0):
    c = np.zeros(tau + 2)
    c[0], c[1] = 1.0, -1.0
    c[-1] += alpha * lam
    return c


def lemma1_threshold(tau: int, lam: float = 1.0) -> float:
    """Largest stable step size of delayed SGD on the quadratic model (Lemma 1)."""
    return 2.0 / lam * math.sin(math.pi / (4 * tau + 2))


def uncorrected_polynomial(tf: int, tb: int, alpha: float, lam: float, Delta: float):
    p = _P.polymul([-1.0, 1.0], _pw(tf))
    p = _P.polyadd(p, [alpha * (lam + Delta)])
    p = _P.polysub(p, alpha * Delta * np.array(_pw(tf - tb)))
    return np.asarray(p)[::-1]


def t2_polynomial(tf: int, tb: int, alpha: float, lam: float, Delta: float, gamma: float, reading: str = "printed",
                  tr: int | None = None, Phi: float = 0.0):
    """T2-corrected model; with tr (tau_recomp) and Phi the recompute variant."""
    if reading not in ("printed", "text"):
        raise ValueError(reading)
    wm1, wmg = [-1.0, 1.0], [-gamma, 1.0]
    p = _P.polymul(_P.polymul(wm1, wmg), _pw(tf))
    p = _P.polyadd(p, alpha * (lam + Delta) * np.array(wmg))
    dphi = Delta - Phi
    p = _P.polysub(p, alpha * dphi * np.array(_P.polymul(_pw(tf - tb), wmg)))
    last = tf - tb if reading == "printed" else tf
    p = _P.polyadd(p, alpha * dphi * (tf - tb) * (1 - gamma) * np.array(_P.polymul(_pw(last), wm1)))
    if tr is not None and Phi != 0.0:
        p = _P.polysub(p, alpha * Phi * np.array(_P.polymul(_pw(tf - tr), wmg)))
        last = tf - tr if reading == "printed" else tf
        p = _P.polyadd(p, alpha * Phi * (tf - tr) * (1 - gamma) * np.array(_P.polymul(_pw(last), wm1)))
    return np.asarray(p)[::-1]


def gamma_from_D(D: float, tf: int, tb: int) -> float:
    return D ** (1.0 / (tf - tb))


def gamma_second_order(tf: int, tb: int) -> float:
    """The decay that makes p''(1) independent of Delta (App. B): 1 - 2 / (tf - tb + 1)."""
    return 1.0 - 2.0 / (tf - tb + 1)


def spectral_radius(coeffs) -> float:
    return float(np.max(np.abs(np.roots(np.asarray(coeffs, dtype=np.float64)))))


def largest_stable_alpha(poly_of_alpha: Callable[[float], np.ndarray], hi: float = 4.0, scan: int = 400,
                         iters: int = 60) -> float:
    """sup of the step sizes a such that every step size in (0, a] is stable: geometric scan from
    hi * 2^-40 upwards for the first unstable point, then bisection."""
    grid = hi * 2.0 ** np.linspace(-40.0, 0.0, scan)
    prev = 0.0
    for a in grid:
        if spectral_radius(poly_of_alpha(float(a))) >= 1.0:
            lo, up = prev, float(a)
            for _ in range(iters):
                mid = 0.5 * (lo + up)
                if spectral_radius(poly_of_alpha(mid)) < 1.0:
                    lo = mid
                else:
                    up = mid
            return lo
        prev = float(a)
    return float(hi)


def stability_table(tf: int, tb: int, deltas, lam: float = 1.0, gamma: float | None = None, reading: str = "printed"):
    """Rows (Delta, largest stable alpha without correction, with T2) - the data of the appendix figure
    that compares the two for tau_fwd = 40, tau_bkwd = 10."""
    g = gamma_second_order(tf, tb) if gamma is None else gamma
    rows = []
    for D_ in deltas:
        a0 = largest_stable_alpha(lambda a: uncorrected_polynomial(tf, tb, a, lam, D_))
        a1 = largest_stable_alpha(lambda a: t2_polynomial(tf, tb, a, lam, D_, g, reading))
        rows.append((float(D_), a0, a1))
    return rows


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description="largest stable step size of the quadratic model vs Delta")
    ap.add_argument("--tau-fwd", type=int, default=40)
    ap.add_argument("--tau-bkwd", type=int, default=10)
    ap.add_argument("--lam", type=float, default=1.0)
    ap.add_argument("--reading", choices=["printed", "text"], default="printed")
    ap.add_argument("--deltas", type=float, nargs="*", default=[-100, -30, -10, -3, -1, 0, 1, 3, 10, 30, 100])
    a = ap.parse_args()
    print(f"# tau_fwd {a.tau_fwd} tau_bkwd {a.tau_bkwd} lam {a.lam} gamma {gamma_second_order(a.tau_fwd, a.tau_bkwd):.6f} ({a.reading} polynomial)")
    print("# Delta, largest stable alpha uncorrected, with T2")
    for row in stability_table(a.tau_fwd, a.tau_bkwd, a.deltas, a.lam, None, a.reading):
        print("%g, %.6g, %.6g" % row)
