"""Writes the stored expected values of the full-size, full-length parity runs (tests/test_gpu_full_size.py).

Calls ONLY the fp64 CPU oracle (oracle/) on the seeded synthetic workloads (workloads/): nothing here comes
from the HIP path.  The oracle needs minutes to hours for these runs (12-layer Transformer: about two minutes
per step on 8 cores), so the GPU tests compare against what this script stored instead of stepping the oracle
beside the GPU:

    python tests/golden/make_full_size_goldens.py tfm6_adamw     # configuration 3, its own AdamW recipe, 200 steps
    python tests/golden/make_full_size_goldens.py resnet20       # configuration 4, 200 steps
    python tests/golden/make_full_size_goldens.py tfm12_sgdm     # configuration 5, momentum SGD, 6 steps

Stored per checkpoint (after k optimizer steps) and weight unit, all from the oracle:
  * sample indices: the entries with the largest |w_k - w_0| and the largest |g|, plus seeded random ones;
    the oracle's weights w_k and consumed gradient g_{k-1} at those entries (the "sampled outputs" of the run);
  * max |w_k|, max |g| and ||w_k - w_0||_2 of the whole unit (the denominators of the error measures);
  * for 256 contiguous segments of the unit: sum and absolute sum of the movement w_k - w_0 and of the gradient
    (a property of EVERY entry: a wrong tile or a dropped block shows up in its segment);
and the mean loss of every step.  Values are fp32 (the bounds they are compared under are >= 1e-5 relative).
"""
import argparse
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import workloads as wl                                   # noqa: E402
from oracle import pipemare_oracle as po                 # noqa: E402
from pm_testutil import make_oracle                      # noqa: E402

N_RANDOM = 510
N_SEG = 256

# name -> (configuration, optimizer keywords (None: the workload's own recipe), steps, checkpoints)
RUNS = {
    "tfm6_adamw": (3, None, 200, (1, 24, 100, 200)),
    "tfm6_sgdm": (3, dict(opt="sgdm", lr=5e-4, beta=0.9, K=8), 100, (1, 16, 100)),
    "resnet20": (4, None, 200, (1, 10, 100, 200)),
    "tfm12_sgdm": (5, dict(opt="sgdm", lr=5e-4, beta=0.9, K=8), 6, (1, 4, 6)),
}


def oracle_kwargs(w, override):
    o_ = w.opt
    if override is not None:
        return dict(override, D=o_["D"], weight_decay=o_["weight_decay"])
    if o_["kind"] == "sgdm":
        return dict(opt="sgdm", lr=o_["lr"], beta=o_["beta"], D=o_["D"], K=o_["K"], weight_decay=o_["weight_decay"])
    return dict(opt=o_["kind"], beta=o_["beta"], beta2=o_["beta2"], eps=o_["eps"], D=o_["D"], K=o_["K"],
                weight_decay=o_["weight_decay"], sched=o_["sched"])


def segment_sums(v, n_seg=N_SEG):
    """(sum, absolute sum) over n_seg contiguous segments of v (the last ones may be shorter or empty)."""
    n = v.size
    seg = -(-n // n_seg)
    pad = np.zeros(seg * n_seg, dtype=np.float64)
    pad[:n] = v
    m = pad.reshape(n_seg, seg)
    return m.sum(axis=1), np.abs(m).sum(axis=1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("run", choices=sorted(RUNS))
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    cfg, override, steps, checkpoints = RUNS[args.run]
    w = wl.config(cfg)
    params = wl.init_params(w)
    tf, tb = po.pipeline_delays(w.P, 1)
    kw = oracle_kwargs(w, override)
    orc = make_oracle(w, params, tf, tb, **kw)
    stream = wl.batch_stream(w)
    rng = np.random.default_rng(20191005)
    U = len(w.layers)
    rand_idx = [np.sort(rng.choice(p.size, size=min(N_RANDOM, p.size), replace=False)) for p in params]
    out = {"steps": np.int64(steps), "checkpoints": np.array(checkpoints, dtype=np.int64), "config": np.int64(cfg)}
    losses = []
    t0 = time.time()
    for k in range(steps):
        losses.append(orc.step(stream.batch(k)))
        print(f"step {k}: loss {losses[-1]:.6f} ({time.time() - t0:.0f} s)", flush=True)
        if k + 1 not in checkpoints:
            continue
        for u in range(U):
            wk = orc.weights(u)
            g = orc.last_grads[u]
            mv = wk - params[u].astype(np.float64)
            idx = np.unique(np.concatenate([rand_idx[u], [int(np.argmax(np.abs(mv))), int(np.argmax(np.abs(g)))]]))
            key = f"k{k + 1}_u{u}_"
            out[key + "idx"] = idx.astype(np.int64)
            out[key + "w"] = wk[idx].astype(np.float32)
            out[key + "g"] = g[idx].astype(np.float32)
            out[key + "scal"] = np.array([np.max(np.abs(wk)), np.max(np.abs(g)), np.linalg.norm(mv), np.linalg.norm(g)],
                                         dtype=np.float64)
            ms, ma = segment_sums(mv)
            gs, ga = segment_sums(g)
            out[key + "seg"] = np.stack([ms, ma, gs, ga]).astype(np.float32)
    out["loss"] = np.array(losses, dtype=np.float64)
    path = args.out or os.path.join(HERE, f"full_size_{args.run}.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
