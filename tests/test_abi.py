"""CPU-only checks of the C-ABI library: it loads, exports what the header declares, and its host
logic (delays, slots, step sizes, validation) matches the oracle.  No kernel is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_1910_05124_amd as pm
from oracle import pipemare_oracle as po
import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "pipemare.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(pm_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(pm.EXPORTS), declared ^ set(pm.EXPORTS)
    for name in declared:
        assert getattr(pm.lib, name) is not None


def test_delays_match_oracle():
    for P in (1, 2, 4, 16, 107):
        for N in (1, 2, 3, 8, 19):
            for method in ("pipemare", "pipedream", "gpipe"):
                assert pm.pm_delays(P, N, method) == po.pipeline_delays(P, N, method)
    with pytest.raises(pm.PmError):
        pm.pm_delays(0, 1)
    with pytest.raises(pm.PmError):
        pm.pm_delays(4, 0)


def test_recompute_delays_match_oracle():
    for P, S, N in ((16, 4, 1), (5, 2, 1), (4, 4, 2), (4, 4, 3), (99, 8, 1), (7, 3, 2), (1, 1, 1), (20, 20, 1)):
        assert pm.pm_recompute_delays(P, S, N) == po.recompute_delays(P, S, N)
    tb = [1, 0, 2, 1, 0]
    assert pm.pm_recompute_delays(5, 3, 1, tb) == po.recompute_delays(5, 3, 1, tb)
    with pytest.raises(pm.PmError):
        pm.pm_recompute_delays(4, 0, 1)


def test_stochastic_delay_tables_and_draws_match_oracle_bit_for_bit():
    for mean, tau_max in ((3.0, 5), (1.0, 12), (31.0, 40), (7.0, 200), (0.5, 3), (0.0, 6), (197.0, 300), (4.0, 0)):
        assert pm.pm_delay_thresholds(mean, tau_max) == po.delay_thresholds(mean, tau_max)
    for P, tau_max, seed in ((4, 9, 7), (16, 40, 2**63 + 11), (99, 250, 0), (1, 0, 5)):
        mean = po.pipeline_delays(P, 1)[0]
        tabs = [po.delay_thresholds(float(m), tau_max) for m in mean]
        for t in list(range(40)) + [10**6, 2**40 + 3]:
            want = [po.stochastic_delay(seed, t, i, P, tabs[i - 1]) for i in range(1, P + 1)]
            assert pm.pm_stochastic_delays(P, mean, tau_max, seed, t) == want
    with pytest.raises(pm.PmError):
        pm.pm_stochastic_delays(3, [1, 1, 1], -1, 0, 0)


def test_slots_brute_force_against_oracle_versions():
    for tf in (0, 1, 2, 7, 31):
        for tb in sorted({0, tf // 2, tf}):
            R = tf + 1
            for t in range(0, 200):
                f, b, w = pm.pm_slots(tf, tb, t)
                vf, vb = max(t - tf, 0), max(t - tb, 0)
                assert (f, b, w) == (vf % R, vb % R, (t + 1) % R)
                # the ring really holds the versions the oracle reads: simulate which version each slot holds
                held = {s: 0 for s in range(R)}
                for tt in range(t):
                    held[(tt + 1) % R] = tt + 1
                assert held[f] == vf and held[b] == vb
                # R = tau_fwd + 1 slots: version t+1 replaces exactly the oldest one, which is the one
                # this step's forward consumed (the update runs after it on the same stream)
                if t >= tf:
                    assert w == f
    with pytest.raises(pm.PmError):
        pm.pm_slots(3, 4, 0)


def test_t1_lr_matches_oracle_closed_form():
    for kind, kw in (("const", dict(base=0.01)), ("step", dict(base=0.1, factor=0.1, interval=30)),
                     ("warmup_invsqrt", dict(base=5e-4, init=1e-7, interval=40))):
        od = dict(kind=kind, **{("warmup" if (k == "interval" and kind == "warmup_invsqrt") else k): v for k, v in kw.items()})
        for K in (0, 20, 200):
            sc = pm.make_sched(kind=kind, K=K, **kw)
            for tau in (0, 1, 5, 31):
                for k in list(range(0, 45)) + [199, 200, 1000]:
                    want = po.t1_lr(po.base_lr(od, k), tau, k, K)
                    assert pm.pm_t1_lr(sc, tau, k) == pytest.approx(want, rel=1e-14)
                    assert pm.pm_t1_lr(sc, tau, k, False) == pytest.approx(po.base_lr(od, k), rel=1e-14)


def _args(layers=None, P=None, tau=None, **o):
    w = wl.config(1)
    layers = layers or w.layers
    P = P or w.P
    tau = tau or pm.pm_delays(P, 1)[0]
    opts = pm.make_opts(dtype="f32", loss="mse", microbatch=16, D=0.9, **o)
    return layers, P, tau, opts


def test_query_bytes_counts_ring_and_state():
    layers, P, tau, opts = _args()
    n = pm.pm_query_bytes(P, layers, tau, opts)
    pad = lambda x: (x + 2047) // 2048 * 2048
    sizes = [pad((L.n_out * L.n_in + 7) // 8 * 8 + L.n_out) for L in layers]
    ring = sum(s * (t + 1) for s, t in zip(sizes, tau))
    flat = sum(sizes)
    assert n >= 4 * (ring + 5 * flat)               # ring + w, g, v, delta, corrected weights (fp32 context)
    assert n < 4 * (ring + 5 * flat) + (1 << 20)


def test_create_rejects_bad_arguments_before_touching_the_gpu():
    w = wl.config(1)
    params = wl.init_params(w)
    sc = pm.make_sched(base=0.01, K=20)
    good = dict(P=w.P, layers=w.layers, tau_fwd=[7, 5, 3, 1], tau_bkwd=[0, 0, 0, 0], sched=sc,
                opts=pm.make_opts(dtype="f32", loss="mse", microbatch=16, D=0.9), init_weights=params,
                arena_ptr=256, arena_bytes=1 << 30, stream=0)

    def bad(**kw):
        a = dict(good)
        a.update(kw)
        with pytest.raises(pm.PmError) as e:
            pm.pm_create(a["P"], a["layers"], a["tau_fwd"], a["tau_bkwd"], a["sched"], a["opts"],
                         a["init_weights"], a["arena_ptr"], a["arena_bytes"], a["stream"])
        return e.value

    assert bad(tau_bkwd=[0, 0, 4, 0]).name == "PM_EINVAL"            # tau_bkwd > tau_fwd
    assert bad(tau_fwd=[7, 5, -3, 1]).name == "PM_EINVAL"
    assert bad(opts=pm.make_opts(dtype="f32", loss="mse", microbatch=16, D=0.0)).name == "PM_EINVAL"
    assert bad(opts=pm.make_opts(dtype="f32", loss="mse", microbatch=0, D=0.5)).name == "PM_EINVAL"
    assert bad(opts=pm.make_opts(dtype="f32", loss="mse", microbatch=16, D=0.5, N=0)).name == "PM_EINVAL"
    odd = pm.make_opts(dtype="f32", loss="mse", microbatch=16, D=0.5)
    odd.update_placement = 3                                          # 0 automatic, 1 separate pass, 2 weight-gradient launch
    assert bad(opts=odd).name == "PM_EINVAL"
    broken = list(w.layers)
    broken[1] = wl.Layer("linear", 32, 64, "relu", 2)                  # does not chain
    assert bad(layers=broken).name == "PM_EINVAL"
    unordered = list(w.layers)
    unordered[2] = wl.Layer("linear", 64, 64, "relu", 1)               # stage goes backwards
    assert bad(layers=unordered).name == "PM_EINVAL"
    assert bad(arena_ptr=260).name == "PM_EINVAL"                      # misaligned arena
    assert bad(arena_bytes=1024).name == "PM_ENOMEM"
    assert bad(sched=pm.make_sched(base=0.01, K=-1)).name == "PM_EINVAL"
    with pytest.raises(pm.PmError):
        pm.pm_step(None, 0, 0)
    with pytest.raises(pm.PmError):
        pm.pm_apply_update(None)
    pm.pm_destroy(None)                                                # no-op


def test_library_shares_the_hip_runtime_pytorch_loaded():
    """The binding imports PyTorch before the library so that both use one copy of the HIP runtime
    (a second copy cannot use PyTorch's device pointers and streams)."""
    import subprocess
    import sys
    code = ("import paper_1910_05124_amd, re\n"
            "libs = {l.split()[-1] for l in open('/proc/self/maps') if re.search(r'libamdhip64', l)}\n"
            "assert len(libs) == 1, libs\n"
            "import torch, os\n"
            "assert os.path.dirname(next(iter(libs))) == os.path.join(os.path.dirname(torch.__file__), 'lib'), libs\n")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True,
                       cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    assert r.returncode == 0, r.stderr
