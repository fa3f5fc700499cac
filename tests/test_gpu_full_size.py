"""Full-size parity of the Transformer and CNN workloads, in the launch configuration bench.py
times (captured HIP graph replayed on a side stream, fixed batch buffers), against the fp64 oracle:
either run on the host in the same process (short runs, every entry of every unit compared), or - for the
full-length runs, which cost the oracle minutes to hours - against the values a committed script stored from
the oracle alone (tests/golden/make_full_size_goldens.py: sampled entries, per-unit norms, and segment sums
that cover every entry).

Checked at every checkpoint: the device step table (ring slots bit-exact, step sizes to fp32
rounding), the mean loss, the gradient the update consumed (per unit relative L2 error), the master
weights (max-relative error per unit, bound 2e-3 for bf16 compute with fp32 master weights) and the
training movement w - w_0 (relative L2, the non-vacuous companion of the weight bound while the
warm-up keeps the step size tiny).  The key-projection biases are left out of the weight checks (their
gradient is identically zero; see pm_testutil.key_bias_entries).
"""
import importlib.util
import os
import time

import numpy as np
import pytest

import workloads as wl
from oracle import pipemare_oracle as po
from pm_testutil import key_bias_entries, make_gpu, make_oracle, max_rel_err

pytestmark = pytest.mark.gpu


def _rel_l2(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / max(np.linalg.norm(b), 1e-300))


def _run(cfg, steps, checkpoints, grad_tol, move_tol, sgdm_lr=None, segment=0):
    """sgdm_lr None: the workload's own optimizer (AdamW on the paper's warm-up schedule, which starts at
    1e-7: together with the T1 division by tau the first steps are smaller than half an fp32 ulp of
    the master weights, so the training movement is reported but not bounded).  sgdm_lr given:
    momentum SGD with that constant base step, T1 annealed over 8 steps, T2 as in the workload: the
    weights of most units move well above fp32 resolution and the movement is bounded too: relative L2 <=
    move_tol beyond the half ulp per step and entry that fp32 master weights may lose (the embedding, in the
    stage whose step size T1 divides by the largest delay, moves by less than an ulp per step)."""
    import torch
    w = wl.config(cfg)
    o_ = w.opt
    params = wl.init_params(w)
    tf, tb = po.pipeline_delays(w.P, 1)
    if sgdm_lr is None and o_["kind"] == "sgdm":
        kw = dict(opt="sgdm", lr=o_["lr"], beta=o_["beta"], D=o_["D"], K=o_["K"], weight_decay=o_["weight_decay"])
    elif sgdm_lr is None:
        kw = dict(opt=o_["kind"], beta=o_["beta"], beta2=o_["beta2"], eps=o_["eps"], D=o_["D"], K=o_["K"],
                  weight_decay=o_["weight_decay"], sched=o_["sched"])
    else:
        kw = dict(opt="sgdm", lr=sgdm_lr, beta=0.9, D=o_["D"], K=8, weight_decay=o_["weight_decay"])
    if segment > 0:        # recomputation in segments of `segment` stages with the delays of PipeMare Recompute
        kw.update(tau_recomp=po.recompute_delays(w.P, segment, 1, tb), segment=segment)
    stream = wl.batch_stream(w)
    o = make_oracle(w, params, tf, tb, **kw)
    skip = key_bias_entries(w)
    side = torch.cuda.Stream()
    t0 = time.time()
    with torch.cuda.stream(side):
        g = make_gpu(w, params, tf, tb, use_graph=True, stream=side, **kw)
        x0, y0 = stream.batch(0)
        xd, yd = torch.from_numpy(x0).cuda(), torch.from_numpy(y0).cuda()
        for k in range(steps):
            x, y = stream.batch(k)
            xd.copy_(torch.from_numpy(x))
            yd.copy_(torch.from_numpy(y))
            lo = o.step((x, y))
            chk = k + 1 in checkpoints
            lg = g.step(xd, yd, want_loss=True)
            if k < 3 or chk or k % 10 == 0:
                print(f"step {k}: loss oracle {lo:.5f} gpu {lg:.5f}  ({time.time() - t0:.0f}s)", flush=True)
            assert lg == pytest.approx(lo, rel=5e-3)
            if not chk:
                continue
            t_used, fs, bs, ws, lrs = g.step_table()
            assert t_used == k
            for u, L in enumerate(w.layers):
                R = tf[L.stage - 1] + 1
                vf, vb = o.last_versions[u]
                assert (fs[u], bs[u], ws[u]) == (vf % R, vb % R, (k + 1) % R)
                assert lrs[u] == pytest.approx(o.last_lr[u], rel=2e-7)
            gerr = []
            for u in range(len(w.layers)):
                gg, go = g.state(4, u), o.last_grads[u]
                if u in skip:                      # compare the matrix part only
                    gg, go = gg[:skip[u].start], go[:skip[u].start]
                gerr.append(_rel_l2(gg, go))
            werr, werrs = max_rel_err(g.weights(), o.weights(), skip=skip)
            merr = []
            for u, (a, b, c) in enumerate(zip(g.weights(), o.weights(), params)):
                a, b, c = a.astype(np.float64), b, c.astype(np.float64)
                if u in skip:
                    a, b, c = a[:skip[u].start], b[:skip[u].start], c[:skip[u].start]
                # (beyond what fp32 master weights cannot hold: half an ulp per step and entry, see _run_golden)
                res = (k + 1) * 2.0 ** -24 * np.linalg.norm(b)
                merr.append(float(max(np.linalg.norm(a - b) - res, 0.0) / max(np.linalg.norm(b - c), 1e-300)))
            print(f"after {k + 1} steps: gradient rel-L2 max {max(gerr):.3e}, weight max-rel {werr:.3e}, "
                  f"movement rel-L2 beyond fp32 resolution max {max(merr):.3e}", flush=True)
            print("   per unit: weight max-rel", np.array2string(np.array(werrs), precision=1, max_line_width=250),
                  "movement rel-L2", np.array2string(np.array(merr), precision=3, max_line_width=250), flush=True)
            # after the first step each side evaluates its gradient at its own, slightly different weights
            assert max(gerr) <= (grad_tol if k == 0 else 4 * grad_tol), np.round(gerr, 4)
            assert werr <= 2e-3, werrs
            if move_tol is not None and k + 1 == steps:       # the first steps are below fp32 resolution (T1 divides by tau)
                assert max(merr) <= move_tol, np.round(merr, 4)
        g.close()


# ------------------------------------------------------------------------------------------------------
# full-length runs against stored oracle values
# ------------------------------------------------------------------------------------------------------
_GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _gold_module():
    spec = importlib.util.spec_from_file_location("make_full_size_goldens", os.path.join(_GOLD, "make_full_size_goldens.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _run_golden(name, *, grad_tol, move_tol, min_move=0.0):
    """Steps the GPU through the run `name` of the golden script and compares, at every stored checkpoint:
    ring slots (bit-exact, against the delay arithmetic of the oracle module) and step sizes; the loss of
    every step; per unit the sampled master weights (max |dw| / max |w| <= 2e-3) and the sampled consumed
    gradient (max |dg| / max |g| <= grad_tol, 4 x after the first step, when each side evaluates the
    gradient at its own slightly different weights); the segment sums of movement and gradient over ALL
    entries; at the last checkpoint the movement w - w_0 on the samples and that the largest unit movement
    exceeds min_move (the weight bound is then not met vacuously).  The movement bound is relative L2 <=
    move_tol beyond what fp32 master weights cannot hold: an increment far below an entry's ulp is lost or
    rounded up to one (a LayerNorm scale of 1.0 in a stage whose step size T1 divides by 197 moves by 1e-9 per
    step, its ulp is 6e-8), so half an ulp per step and entry - steps x 2^-24 x ||w|| over the samples - is
    allowed on top; at least a third of the units must lie above that floor, or the bound would say nothing."""
    import torch
    gm = _gold_module()
    path = os.path.join(_GOLD, f"full_size_{name}.npz")
    assert os.path.exists(path), f"{path} is missing: write it with tests/golden/make_full_size_goldens.py {name}"
    gold = np.load(path)
    cfg, override, steps, checkpoints = gm.RUNS[name]
    assert int(gold["config"]) == cfg and int(gold["steps"]) == steps
    w = wl.config(cfg)
    params = wl.init_params(w)
    tf, tb = po.pipeline_delays(w.P, 1)
    kw = gm.oracle_kwargs(w, override)
    sched = kw.get("sched") or dict(kind="const", base=kw["lr"])
    stream = wl.batch_stream(w)
    skip = key_bias_entries(w)
    side = torch.cuda.Stream()
    t0 = time.time()
    worst = dict(w=0.0, g=0.0)
    with torch.cuda.stream(side):
        g = make_gpu(w, params, tf, tb, use_graph=True, stream=side, **kw)
        # where the update runs by default (pm_opts.update_placement = 0): inside the weight-gradient launch for the
        # weight matrices of the 12-layer workload (state beyond the caches), the separate pass everywhere else
        n_launch, n_pass = g.update_split()
        n_mat = sum(L.n_in * L.n_out for L in w.layers if L.kind == "linear")
        assert n_launch == (n_mat if cfg == 5 else 0) and n_pass > 0, (cfg, n_launch, n_pass)
        x0, y0 = stream.batch(0)
        xd, yd = torch.from_numpy(x0).cuda(), torch.from_numpy(y0).cuda()
        for k in range(steps):
            x, y = stream.batch(k)
            xd.copy_(torch.from_numpy(x))
            yd.copy_(torch.from_numpy(y))
            chk = k + 1 in checkpoints
            lg = g.step(xd, yd, want_loss=True)
            assert lg == pytest.approx(float(gold["loss"][k]), rel=5e-3), k
            if not chk:
                continue
            t_used, fs, bs, ws, lrs = g.step_table()
            assert t_used == k
            for u, L in enumerate(w.layers):
                tau = tf[L.stage - 1]
                R = tau + 1
                assert (fs[u], bs[u], ws[u]) == (max(k - tau, 0) % R, max(k - tb[L.stage - 1], 0) % R, (k + 1) % R)
                assert lrs[u] == pytest.approx(po.t1_lr(po.base_lr(sched, k), tau, k, kw["K"]), rel=2e-7)
            werrs, gerrs, merrs, moves, floored = [], [], [], [], 0
            for u in range(len(w.layers)):
                key = f"k{k + 1}_u{u}_"
                idx, gw, gg = gold[key + "idx"], gold[key + "w"].astype(np.float64), gold[key + "g"].astype(np.float64)
                maxw, maxg, mvnorm, gnorm = gold[key + "scal"]
                W = g.weights(u).astype(np.float64)
                G = g.state(4, u).astype(np.float64)
                w0 = params[u].astype(np.float64)
                keep = np.ones(idx.size, dtype=bool)
                if u in skip:
                    keep = idx < skip[u].start
                    W[skip[u]] = w0[skip[u]]           # (their segment sums hold no movement on the oracle's side)
                    G[skip[u]] = 0.0
                werrs.append(float(np.max(np.abs(W[idx] - gw)[keep]) / maxw))
                gerrs.append(float(np.max(np.abs(G[idx] - gg)[keep]) / max(maxg, 1e-300)))
                mvs = gw - w0[idx]
                res = (k + 1) * 2.0 ** -24 * np.linalg.norm(gw[keep])
                mvn = max(np.linalg.norm(mvs[keep]), 1e-300)
                merrs.append(float(max(np.linalg.norm(((W[idx] - w0[idx]) - mvs)[keep]) - res, 0.0) / mvn))
                floored += bool(move_tol is not None and res > move_tol * mvn)
                moves.append(float(np.max(np.abs(mvs)) / maxw))
                # every entry, through segment sums: |difference of sums| within a share of the absolute sum plus
                # the noise of sqrt(n) independent element errors of the size the element bounds allow
                seg = gold[key + "seg"].astype(np.float64)
                ms, _ = gm.segment_sums(W - w0)
                gs, _ = gm.segment_sums(G)
                seglen = -(-W.size // gm.N_SEG)
                noise_w = 4.0 * np.sqrt(seglen) * 2e-3 * maxw
                noise_g = 4.0 * np.sqrt(seglen) * grad_tol * maxg
                bad_m = np.abs(ms - seg[0]) > 0.05 * seg[1] + noise_w
                bad_g = np.abs(gs - seg[2]) > 0.10 * seg[3] + noise_g
                assert not bad_m.any(), (k + 1, u, "movement segments", np.nonzero(bad_m)[0][:8])
                assert not bad_g.any(), (k + 1, u, "gradient segments", np.nonzero(bad_g)[0][:8])
            worst["w"], worst["g"] = max(worst["w"], max(werrs)), max(worst["g"], max(gerrs))
            print(f"after {k + 1} steps ({time.time() - t0:.0f}s): sampled weight max-rel {max(werrs):.3e}, sampled gradient max-rel "
                  f"{max(gerrs):.3e}, movement rel-L2 beyond fp32 resolution {max(merrs):.3e} ({floored} units below the floor), "
                  f"largest unit movement {max(moves):.3e}", flush=True)
            print("   per unit weight max-rel", np.array2string(np.array(werrs), precision=1, max_line_width=250), flush=True)
            print("   per unit gradient max-rel", np.array2string(np.array(gerrs), precision=1, max_line_width=250), flush=True)
            print("   per unit movement rel-L2", np.array2string(np.array(merrs), precision=2, max_line_width=250), flush=True)
            assert max(werrs) <= 2e-3 + 2.0 ** -23, werrs
            assert max(gerrs) <= (grad_tol if k == 0 else 4 * grad_tol), gerrs
            if k + 1 == steps:
                assert max(moves) >= min_move, moves
                if move_tol is not None:
                    assert max(merrs) <= move_tol, merrs
                    assert 3 * floored <= 2 * len(w.layers), floored
        g.close()
    return worst


@pytest.mark.timeout(900)
def test_config3_transformer6_bf16_live_oracle_sgdm():
    """6 layers, width 512, 8 heads, feed-forward 2048, vocabulary 8192, 32 x 128 tokens, P = 38 (tau_fwd 75 .. 1):
    16 steps of momentum SGD beside the live oracle, EVERY entry of every unit compared."""
    _run(3, 16, (1, 16), grad_tol=3e-2, move_tol=0.05, sgdm_lr=5e-4)


@pytest.mark.timeout(900)
def test_config3_transformer6_bf16_recompute_live_oracle():
    """The same workload with recomputation in segments of 6 stages (tau_recomp = 10, 8, ..., 0 inside every
    segment; "T2 for Recompute"): 8 steps beside the live oracle, every entry compared.  The cuts fall between
    units of a layer (P = 38 = 1 + 6 per layer + 1), so kept and rebuilt tensors mix inside the layers."""
    _run(3, 8, (1, 8), grad_tol=3e-2, move_tol=0.05, sgdm_lr=5e-4, segment=6)


@pytest.mark.timeout(900)
def test_config4_resnet20_bf16_recompute_live_oracle():
    """ResNet-20 shape with recomputation in segments of 4 stages: 12 steps beside the live oracle."""
    _run(4, 12, (1, 12), grad_tol=3e-2, move_tol=0.05, segment=4)


@pytest.mark.timeout(900)
def test_config3_transformer6_bf16_200_steps_adamw():
    """The same workload with its own recipe (AdamW on the paper's warm-up schedule, T1 over 5x the warm-up) for the
    200 steps the measurement plan names: every stage (tau_fwd <= 75) reads genuinely delayed versions for most
    of the run and every ring wraps at least twice."""
    _run_golden("tfm6_adamw", grad_tol=3e-2, move_tol=None)


@pytest.mark.timeout(900)
def test_config4_resnet20_bf16_200_steps():
    """ResNet-20 shape, 128 images of 3x32x32, P = 20 (tau_fwd 39 .. 1), momentum SGD, the full 200 steps."""
    _run_golden("resnet20", grad_tol=3e-2, move_tol=0.05, min_move=0.02)


@pytest.mark.timeout(900)
def test_config5_transformer12_bf16_sgdm_6_steps():
    """12 layers, width 1024, 16 heads, feed-forward 4096, vocabulary 32000, 16 x 512 tokens, P = 99 (tau_fwd 197 .. 1),
    ~217 M parameters, 43 GB ring.  Momentum SGD with a constant base step (the AdamW warm-up from 1e-7 divided by
    tau moves nothing in a handful of steps): 6 steps, so the last three stages (tau_fwd 1, 3, 5) read ring versions
    other than the initial one, the movement is far above fp32 resolution, and gradients are compared entry by
    entry on the samples and through segment sums everywhere."""
    _run_golden("tfm12_sgdm", grad_tol=3e-2, move_tol=0.05, min_move=1e-4)
