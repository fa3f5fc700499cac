#!/usr/bin/env python3
"""Benchmark of the PipeMare hot path on one MI355X.

A "step" is one pass of the whole hot path over one microbatch already resident in HBM: slot /
step-size table, forward of all stages on tau_fwd-stale ring weights, loss, backward on corrected
weights, fused update (T1 + optimizer + delta + ring / corrected-weight write-back).

Workload at N=1: the largest single-GPU configuration of the task's list (number 5): the fine-grained
12-layer Transformer, width 1024, 16 heads, feed-forward 4096, vocabulary 32000, 16 sequences of 512
tokens, every weight unit a pipeline stage of its own (P = 99, tau_fwd = 197 .. 1, tau_bkwd = 0),
~217 M parameters, 43 GB ring of weight versions; bf16 compute, fp32 master weights, AdamW.
`--config 1..4` select the other configurations of the list.

Prints ONE JSON line.  `roofline` prices the fused update pass (HBM bound) with its algorithmic bytes:
AdamW 40 B per parameter per step (read g, w, m, s, delta fp32; write w, m, s, delta fp32 + ring slot bf16
+ corrected weights bf16), momentum SGD 32 B.  On the Transformer workloads the weight matrices are updated
inside the grouped weight-gradient launch and the pass of the timed region covers the other parameters
(embedding, biases, LayerNorm); `roofline_all_parameters` then gives the same kernel over every parameter,
from a second context of the same process.  `stage_gemms` prices the stages' matrix products (MFMA
bound) twice: over the summed duration of the product kernels themselves (event pairs around every such
launch) and over the whole forward + backward phase.  `cpu_baseline` times the fp64 NumPy oracle on a
bounded sample of the same workload on the host cores (a reference point, not a target).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 MFMA rate
BYTES_PER_PARAM = {("sgdm", "bf16"): 32, ("adamw", "bf16"): 40, ("sgdm", "f32"): 36, ("adamw", "f32"): 44}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default per workload: 300 / 500 / 200 / 300 / 100)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before (default 20; 10 for config 5)")
    ap.add_argument("--config", type=int, default=5,
                    help="position in the task's list of configurations (1: tiny fp32 MLP, 2: 16-stage bf16 MLP, "
                         "3: 6-layer Transformer, 4: ResNet-20, 5: 12-layer Transformer (default, the headline workload))")
    ap.add_argument("--launch", choices=["graph", "eager", "overlap"], default="graph",
                    help="overlap: eager launches, the update of step t on the library's second stream concurrent "
                         "with the forward of step t+1; graph: replay a captured HIP graph; eager: one stream")
    ap.add_argument("--no-graph", action="store_true", help="same as --launch eager")
    ap.add_argument("--cpu-steps", type=int, default=None,
                    help="oracle steps timed for cpu_baseline (0 = skip; default per workload, about 10-60 s of host work: "
                         "200 / 24 / 8 / 12 / 1)")
    ap.add_argument("--pool", type=int, default=64, help="distinct device-resident microbatches cycled through")
    ap.add_argument("--recompute", type=int, default=0,
                    help="MLP workloads: S > 0 turns on recomputation with segments of S stages (the backward pass "
                         "rebuilds the activations inside each segment with the delayed, corrected recompute weights)")
    ap.add_argument("--stochastic", type=int, default=-1,
                    help="TAU_MAX >= 0 turns on Hogwild-style stochastic delays: every step each stage draws its delay from "
                         "the exponential with the pipeline's delay as mean, truncated at TAU_MAX")
    ap.add_argument("--chain", action="store_true",
                    help="MLP workloads: the chained forward / data-gradient launches instead of one launch per product")
    ap.add_argument("--separate-update", action="store_true",
                    help="Transformer workloads: always the separate update pass over all parameters (default: on the large "
                         "workload the weight matrices are updated inside the grouped weight-gradient launch)")
    ap.add_argument("--single-context", action="store_true",
                    help="skip the second context (separate update pass over all parameters) that the default Transformer "
                         "run adds after the timed region for roofline_all_parameters: keeps a profiler's kernel list to one "
                         "launch configuration")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run three plain device-to-device copies of this many MiB after the timed region "
                         "(a kernel of known traffic to scale rocprofv3's FETCH_SIZE / WRITE_SIZE readings by)")
    args = ap.parse_args()
    if args.steps is None:
        args.steps = {1: 300, 2: 500, 3: 200, 4: 300, 5: 100}.get(args.config, 100)
    if args.warmup is None:
        args.warmup = 10 if args.config == 5 else 20
    if args.cpu_steps is None:
        args.cpu_steps = {1: 200, 2: 24, 3: 8, 4: 12, 5: 1}.get(args.config, 1)
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_1910_05124_amd as pm
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    w = wl.config(args.config)
    o = w.opt
    tau_fwd, tau_bkwd = pm.pm_delays(w.P, w.N, "pipemare")
    stoch = dict(tau_max=args.stochastic, seed=20191005) if args.stochastic >= 0 else None
    tau_recomp = pm.pm_recompute_delays(w.P, args.recompute, w.N, tau_bkwd) if args.recompute > 0 else None
    params = wl.init_params(w)
    n_params = int(sum(p.size for p in params))
    stream_data = wl.batch_stream(w)
    is_tfm = w.arch.get("kind") == "transformer"
    is_cnn = w.arch.get("kind") == "resnet"
    launch = "eager" if args.no_graph else args.launch
    use_graph = launch == "graph"
    side = torch.cuda.Stream()
    sd = o.get("sched") or dict(kind="const", base=o["lr"])
    # Microbatches are resident in HBM before the timed region and handed over by pointer.  A captured
    # graph is bound to its batch buffers and the library keeps one graph per buffer pair, so the pool is
    # no larger than the warm-up (every pair's graph is captured during the untimed steps).
    npool = max(1, min(args.pool, args.warmup, 64)) if use_graph else args.pool
    with torch.cuda.stream(side):
        pool = [stream_data.batch(k) for k in range(npool)]
        xs = [torch.from_numpy(x).cuda() for x, _ in pool]
        ys = [torch.from_numpy(y).cuda() for _, y in pool]

    def measure(placement, steps, timed):
        """One context; `steps` timed steps (if timed), then `steps` eager steps with four events per step, then up
        to 16 with an event pair around every product / attention launch."""
        with torch.cuda.stream(side):
            sched = pm.make_sched(kind=sd["kind"], base=sd["base"], init=sd.get("init", 0.0), factor=sd.get("factor", 1.0),
                                  interval=sd.get("interval", sd.get("warmup", 1)), K=o["K"])
            opts = pm.make_opts(opt=o["kind"], beta1=o["beta"], beta2=o.get("beta2", 0.98), eps=o.get("eps", 1e-8), D=o["D"],
                                weight_decay=o["weight_decay"], t1=True, t2=True,
                                N=w.N, dtype=w.dtype, loss=w.loss, microbatch=w.microbatch, use_graph=use_graph,
                                overlap_update=(launch == "overlap"), arch=w.arch.get("kind", "chain"),
                                n_heads=w.arch.get("n_heads", 0), seq_len=w.arch.get("seq", 0),
                                image_size=w.arch.get("image", 0), tau_recomp=tau_recomp, segment_size=args.recompute,
                                stochastic=stoch, chained_launches=args.chain, update_placement=placement)
            eng = pm.PipeMare(w.layers, w.P, tau_fwd, tau_bkwd, sched, opts, params, stream=side)

            def run(n, base):
                for k in range(n):
                    i = (base + k) % npool
                    eng.step(xs[i], ys[i])

            r = {"split": eng.update_split(), "dt": None}
            run(args.warmup, 0)
            eng.synchronize()
            torch.cuda.synchronize()
            if timed:
                t0 = time.perf_counter()
                run(steps, args.warmup)
                eng.synchronize()          # the caller's stream and the library's second stream
                torch.cuda.synchronize()
                r["dt"] = time.perf_counter() - t0
            r["stats"] = eng.stats(param_norm=True)
            # per-phase kernel time with HIP events on the engine's stream, same steps, eager launches on one
            # stream (no overlap, so the update kernel's duration is its own)
            pm.pm_profile_begin(eng.ctx, steps)
            run(steps, args.warmup + steps)
            r["prof"] = pm.pm_profile_end(eng.ctx)
            # a second, short pass that also brackets every product / attention launch with an event pair
            ncls = max(1, min(steps, 16))
            pm.pm_profile_begin_classes(eng.ctx, ncls)
            run(ncls, args.warmup + 2 * steps)
            pm.pm_profile_end(eng.ctx)
            r["cls"] = pm.pm_profile_classes(eng.ctx)
            eng.close()
        return r

    m = measure("pass" if args.separate_update else "auto", args.steps, True)
    dt, stats, prof, cls = m["dt"], m["stats"], m["prof"], m["cls"]
    n_epilogue, n_pass = m["split"]
    # Where the weight matrices are updated inside the weight-gradient launch, the pass of the timed region covers
    # the remaining parameters only; a second context with the separate pass over ALL parameters gives the pass at
    # the full footprint and the product kernels without the update work inside (a few untimed steps)
    m_sep = measure("pass", max(4, min(args.steps, 20)), False) if (n_epilogue > 0 and not args.single_context) else None
    if args.calib_copy_mib > 0:
        with torch.cuda.stream(side):
            src = torch.ones(args.calib_copy_mib << 20, dtype=torch.uint8, device="cuda")
            dst = torch.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
            side.synchronize()

    ms_per_step = dt / args.steps * 1e3
    steps_per_s = args.steps / dt
    bpp = BYTES_PER_PARAM[(o["kind"], w.dtype)]
    if stoch is not None:
        bpp -= 2 if w.dtype == "bf16" else 4        # no corrected backward weights are written
    upd_s = prof["update_ms"] * 1e-3
    # an embedding has no corrected backward weights (nothing flows through it): one 2- or 4-byte stream less
    esz = 2 if w.dtype == "bf16" else 4
    # parameters the pass covers: all, or - when the weight matrices are updated in the weight-gradient epilogues -
    # the rest (embedding, biases, LayerNorm)
    in_pass = [wl.n_params(L) - (L.n_in * L.n_out if (n_epilogue > 0 and L.kind == "linear") else 0) for L in w.layers]
    assert n_epilogue == 0 or sum(in_pass) == n_params - n_epilogue
    alg_bytes = sum(n * (bpp - (esz if L.kind == "embed" else 0)) for n, L in zip(in_pass, w.layers))
    if tau_recomp is not None:
        # units that keep corrected recompute weights of their own (delay or coefficient differs from the
        # backward weights'): one more stored stream, plus a read of the older ring version when tau_recomp > 0
        for L in w.layers:
            tr, tf_, tb_ = tau_recomp[L.stage - 1], tau_fwd[L.stage - 1], tau_bkwd[L.stage - 1]
            if tf_ - tr > 0 and not (tr == tb_):
                alg_bytes += wl.n_params(L) * esz * (2 if tr > 0 else 1)
    achieved = alg_bytes / upd_s / 1e9 if upd_s > 0 else 0.0
    lin = [L for L in w.layers if L.kind == "linear"]
    if is_tfm:
        a = w.arch
        tokens = w.microbatch * a["seq"]
        # every Linear: forward, data gradient, weight gradient (2 M n_in n_out each); causal attention core:
        # 2 products forward, 4 backward, each S^2 dh flops per (sequence, head) when only the lower triangle counts
        gemm_flops = 6.0 * tokens * sum(L.n_in * L.n_out for L in lin)
        attn_flops = 6.0 * a["seq"] ** 2 * (a["d_model"] // a["n_heads"]) * w.microbatch * a["n_heads"] * a["n_layers"]
        gemm_flops += attn_flops
        if tau_recomp is not None:      # the rebuilt forward: every product but the head, and the attention core's forward third
            gemm_flops += 2.0 * tokens * sum(L.n_in * L.n_out for L in lin[:-1]) + attn_flops / 3.0
        samples = tokens
    elif is_cnn:
        # every convolution: forward, data gradient (not for the first), weight gradient, 2 * pixels_out * C_out * 9 C_in each
        H = w.arch["image"]
        gemm_flops = 0.0
        for u, L in enumerate(w.layers[:-1]):
            if u > 0 and u % 2 == 1 and L.n_out == 2 * L.n_in:
                H //= 2
            gemm_flops += ((3.0 if u > 0 else 2.0) + (1.0 if tau_recomp is not None else 0.0)) * 2.0 * w.microbatch * H * H * L.n_out * 9 * L.n_in
        gemm_flops += 6.0 * w.microbatch * w.layers[-1].n_in * w.layers[-1].n_out
        samples = w.microbatch
    else:
        gemm_flops = 6.0 * w.microbatch * sum(L.n_in * L.n_out for L in lin) - 2.0 * w.microbatch * lin[0].n_in * lin[0].n_out
        samples = w.microbatch
        if tau_recomp is not None:      # the rebuilt forward of every unit but the head
            gemm_flops += 2.0 * w.microbatch * sum(L.n_in * L.n_out for L in lin[:-1])
    gemm_s = (prof["fwd_ms"] + prof["bwd_ms"]) * 1e-3
    kern_s = (cls["product_ms"] + cls["attention_ms"]) * 1e-3      # the product (and attention) kernels alone
    traffic, traffic_src = (measured_traffic(w.name + ("_separate_update" if args.separate_update and is_tfm else ""))
                            if tau_recomp is None and stoch is None else (None, None))
    out = {
        "metric": "async pipeline train steps/s",
        "value": round(steps_per_s, 2),
        "unit": "steps/s",
        "samples_per_s": round(steps_per_s * samples * w.N, 1),
        "samples_unit": "tokens" if is_tfm else "rows",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype if w.dtype != "f32" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.P}-stage {'Transformer' if is_tfm else 'CNN' if is_cnn else 'MLP'}, {len(w.layers)} weight units, {n_params} params, "
                               f"microbatch {w.microbatch}{' x ' + str(w.arch['seq']) + ' tokens' if is_tfm else ''}, "
                               f"PipeMare delays tau_fwd={tau_fwd[0]}..{tau_fwd[-1]}, tau_bkwd=0, "
                               f"{o['kind']} beta {o['beta']}, T1 K={o['K']}, T2 D={o['D']}"
                               + (f", stochastic delays (truncated exponential, tau_max {args.stochastic}; both passes read the drawn version, no T2)"
                                  if stoch is not None else "")
                               + (f", recomputation in segments of {args.recompute} stages (tau_recomp={tau_recomp[0]}..{tau_recomp[-1]})"
                                  if tau_recomp is not None else ""),
                   "launch": launch, "final_loss": round(stats["loss"], 5)},
        "roofline": {"kernel": "pm_fused_update_kernel", "bound": "hbm", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_source": traffic_src, "algorithmic_bytes": alg_bytes,
                     "bytes_per_param": bpp, "params": sum(in_pass), "params_updated_in_weight_gradient_epilogues": n_epilogue,
                     "avg_kernel_ms": round(prof["update_ms"], 5), "launches_timed": prof["n"]},
        "phases_ms": {"forward_loss": round(prof["fwd_ms"], 4), "backward": round(prof["bwd_ms"], 4),
                      "update": round(prof["update_ms"], 4), "note": "serial (non-overlapped) profiling pass"},
        "stage_gemms": {"bound": "mfma", "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "algorithmic_tflop_per_step": round(gemm_flops / 1e12, 5),
                        "kernels_ms_per_step": round(kern_s * 1e3, 4),
                        "kernels_achieved": round(gemm_flops / kern_s / 1e12, 2) if kern_s > 0 else None,
                        "kernels_frac": round(gemm_flops / kern_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 5) if kern_s > 0 else None,
                        "kernels_steps_timed": cls["n"],
                        "phase_achieved": round(gemm_flops / gemm_s / 1e12, 2) if gemm_s > 0 else None,
                        "phase_frac": round(gemm_flops / gemm_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 5) if gemm_s > 0 else None,
                        "note": "flops of the stages' matrix / convolution products (and the attention core; with recomputation also of the rebuilt forward); kernels_*: "
                                "over the summed duration of those kernels alone (HIP event pairs around each launch in "
                                "the eager profiling pass); phase_*: over the whole forward + backward phase (loss, "
                                "LayerNorm, bias-gradient, embedding kernels and launch gaps inside).  Where the products take a few "
                                "microseconds each (configurations 1, 2, 4) the two markers per launch cost more than the kernels: "
                                "read phase_* there"},
    }
    if m_sep is not None:
        # the same quantities from the context whose update pass covers every parameter
        ps, cs = m_sep["prof"], m_sep["cls"]
        all_bytes = sum(wl.n_params(L) * (bpp - (esz if L.kind == "embed" else 0)) for L in w.layers)
        a_all = all_bytes / (ps["update_ms"] * 1e-3) / 1e9 if ps["update_ms"] > 0 else 0.0
        ks = (cs["product_ms"] + cs["attention_ms"]) * 1e-3
        traffic_all, traffic_all_src = measured_traffic(w.name + "_separate_update")
        out["roofline"]["note"] = ("the pass of the timed region: the weight matrices (params_updated_in_weight_gradient_epilogues) are "
                                   "updated by the blocks of the grouped weight-gradient launch, 36 B per parameter there (no "
                                   "gradient read-back); roofline_all_parameters is the same kernel over every parameter")
        out["roofline_all_parameters"] = {
            "kernel": "pm_fused_update_kernel", "bound": "hbm", "achieved": round(a_all, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(a_all / HBM_PEAK_GBS, 4), "traffic": traffic_all, "traffic_source": traffic_all_src,
            "algorithmic_bytes": all_bytes, "bytes_per_param": bpp, "params": n_params,
            "avg_kernel_ms": round(ps["update_ms"], 5), "launches_timed": ps["n"],
            "note": "second context of the same process with pm_opts.update_placement = 1 (untimed for `value`)"}
        out["stage_gemms"]["separate_update"] = {
            "kernels_ms_per_step": round(ks * 1e3, 4),
            "kernels_achieved": round(gemm_flops / ks / 1e12, 2) if ks > 0 else None,
            "kernels_frac": round(gemm_flops / ks / 1e12 / MFMA_BF16_PEAK_TFLOPS, 5) if ks > 0 else None,
            "phases_ms": {"forward_loss": round(ps["fwd_ms"], 4), "backward": round(ps["bwd_ms"], 4), "update": round(ps["update_ms"], 4)},
            "note": "the product kernels without the update work inside the weight-gradient launch (context with the separate pass)"}
    if args.cpu_steps > 0:
        out["cpu_baseline"] = cpu_baseline(w, params, tau_fwd, tau_bkwd, args.cpu_steps, tau_recomp, args.recompute, stoch)
    print(json.dumps(out), flush=True)


def measured_traffic(workload_name):
    """workload_name: the workload, with "_separate_update" appended for the runs whose pass covers every parameter
    of a Transformer.  HBM bytes per launch of the update kernel from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a plain copy) and where
    that number comes from (file and the source revision it was taken at), or (None, None).  Counters
    cannot be collected inside this process, so the figure is not live: the source string says so."""
    name = f"update_traffic_{workload_name}.txt"
    path = os.path.join(ROOT, "profiles", name)
    val, rev = None, "unknown revision"
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("# taken at source revision"):
                    rev = line.split("revision", 1)[1].strip()
                if line.startswith("traffic_bytes_per_launch pm_fused_update_kernel:"):
                    val = int(float(line.split(":")[1]))
    except OSError:
        pass
    return (val, f"profiles/{name} (rocprofv3 counters of a separate run, taken at {rev})") if val is not None else (None, None)


def cpu_baseline(w, params, tau_fwd, tau_bkwd, n_steps, tau_recomp=None, segment=0, stochastic=None):
    """The fp64 NumPy oracle as it stands, timed on the host cores on the first n_steps of the workload."""
    import workloads as wl
    from pm_testutil import make_oracle
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    o = w.opt
    orc = make_oracle(w, params, tau_fwd, tau_bkwd, opt=o["kind"], lr=o.get("lr", 0.0), beta=o["beta"], beta2=o.get("beta2", 0.98),
                      D=o["D"], K=o["K"], weight_decay=o["weight_decay"], sched=o.get("sched"),
                      tau_recomp=tau_recomp, segment=segment, stochastic=stochastic)
    stream = wl.batch_stream(w)
    pre = 0 if n_steps < 4 else 2
    batches = [stream.batch(k) for k in range(n_steps + pre)]
    for k in range(pre):
        orc.step(batches[k])
    t0 = time.perf_counter()
    for k in range(pre, n_steps + pre):
        orc.step(batches[k])
    dt = time.perf_counter() - t0
    return {"value": round(n_steps / dt, 5), "unit": "steps/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n_steps} whole optimizer step(s) of the same workload (after {pre} untimed), fp64 NumPy, "
                      f"explicit weight histories, {dt:.1f} s of host time"}


if __name__ == "__main__":
    main()
