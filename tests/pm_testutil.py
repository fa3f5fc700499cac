"""Shared helpers of the GPU parity tests: build the oracle and the HIP context from one workload."""
import numpy as np

from oracle import pipemare_oracle as po
import workloads as wl


def sched_dict(kind="const", base=0.01, init=0.0, factor=1.0, interval=1):
    if kind == "const":
        return dict(kind="const", base=base)
    if kind == "step":
        return dict(kind="step", base=base, factor=factor, interval=interval)
    return dict(kind="warmup_invsqrt", base=base, init=init, warmup=interval)


def make_oracle(w, params, tau_fwd, tau_bkwd, *, opt="sgdm", lr=0.01, beta=0.9, beta2=0.98, eps=1e-8,
                weight_decay=0.0, clip_norm=0.0, D=0.9, K=0, t1=True, t2=True, N=1, sched=None,
                gamma_override=None, model=None, keep_history=False, sync_warmup=0):
    model = model or po.MLPModel(w.layers, w.loss)
    o = dict(kind=opt, beta=beta, beta1=beta, beta2=beta2, eps=eps, weight_decay=weight_decay,
             clip_norm=clip_norm, D=D, K=K, t1=t1, t2=t2, N=N, gamma_override=gamma_override,
             sched=sched or dict(kind="const", base=lr), sync_warmup=sync_warmup)
    return po.PipeMareOracle(model, [p.astype(np.float64) for p in params], [L.stage for L in w.layers],
                             tau_fwd, tau_bkwd, o, keep_history=keep_history)


def make_gpu(w, params, tau_fwd, tau_bkwd, *, opt="sgdm", lr=0.01, beta=0.9, beta2=0.98, eps=1e-8,
             weight_decay=0.0, clip_norm=0.0, D=0.9, K=0, t1=True, t2=True, N=1, sched=None,
             gamma_override=None, use_graph=False, dtype=None, stream=None, sync_warmup=0, overlap_update=False):
    import paper_1910_05124_amd as pm
    s = sched or dict(kind="const", base=lr)
    sc = pm.make_sched(kind=s["kind"], base=s["base"], init=s.get("init", 0.0), factor=s.get("factor", 1.0),
                       interval=s.get("interval", s.get("warmup", 1)), K=K)
    o = pm.make_opts(opt=opt, beta1=beta, beta2=beta2, eps=eps, weight_decay=weight_decay, clip_norm=clip_norm,
                     D=D, gamma_override=gamma_override, t1=t1, t2=t2, N=N, dtype=dtype or w.dtype, loss=w.loss,
                     microbatch=w.microbatch, use_graph=use_graph, sync_warmup=sync_warmup,
                     overlap_update=overlap_update)
    return pm.PipeMare(w.layers, w.P, tau_fwd, tau_bkwd, sc, o, params, stream=stream)


def max_rel_err(gpu_weights, oracle_weights):
    """Per unit ||w_gpu - w_oracle||_inf / ||w_oracle||_inf; returns the max over units and the list."""
    errs = []
    for a, b in zip(gpu_weights, oracle_weights):
        errs.append(float(np.max(np.abs(a.astype(np.float64) - b)) / np.max(np.abs(b))))
    return max(errs), errs


class GivenGrads:
    """Oracle 'model' that returns gradients supplied by the test (for the update pass in isolation)."""

    def loss_and_grads(self, u_fwd, u_bkwd, grads):
        return 0.0, [np.asarray(g, dtype=np.float64) for g in grads]
