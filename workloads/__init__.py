"""Seeded synthetic workloads shared by the CPU oracle's tests and the HIP path's tests.

This module only *describes* networks and *draws* numbers: layer lists, initial
weights, input batches and teacher-generated targets.  It contains none of the
method's arithmetic (no delays, no learning-rate rescheduling, no correction, no
optimizer, no forward/backward of the trained network): both the oracle and the
HIP library compute those on their own from the integers and arrays given here.

The paper trains on public image / translation datasets that are not available
here; these generators stand in for them with the same tensor shapes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

__all__ = ["Layer", "Workload", "config", "init_params", "BatchStream", "n_params", "transformer", "TokenStream",
           "batch_stream", "resnet", "ImageStream"]


@dataclass(frozen=True)
class Layer:
    """One weight unit (weight matrix + bias), assigned to pipeline stage `stage` (1-based)."""
    kind: str      # "linear" | "embed" (n_in = vocab, n_out = width, no bias) | "layernorm" (gain + bias of width n_out)
                   # | "conv3x3" (n_in, n_out channels; weight n_out x 3 x 3 x n_in, then per-channel scale and shift)
    n_in: int
    n_out: int
    act: str       # "none" | "relu" | "gelu"
    stage: int


@dataclass(frozen=True)
class Workload:
    name: str
    layers: Tuple[Layer, ...]
    P: int                 # number of pipeline stages
    N: int                 # microbatches per minibatch
    loss: str              # "mse" | "xent"
    dtype: str             # "f32" | "bf16" (bf16 compute, fp32 master)
    microbatch: int
    n_classes: int         # for "xent"; output width for "mse"
    opt: dict = field(default_factory=dict)
    steps: int = 0
    seed_init: int = 2
    seed_data: int = 0
    seed_teacher: int = 1
    init: str = "fan_in"   # "fan_in": W ~ U(+-1/sqrt(fan_in));  "he": W ~ U(+-sqrt(6/fan_in)) behind ReLU/GELU
    arch: dict = field(default_factory=dict)   # {} = plain chain; transformer: n_layers, d_model, n_heads, d_ff, vocab, seq


def n_params(layer: Layer) -> int:
    if layer.kind == "embed":
        return layer.n_in * layer.n_out
    if layer.kind == "layernorm":
        return 2 * layer.n_out
    if layer.kind == "conv3x3":
        return layer.n_out * 9 * layer.n_in + 2 * layer.n_out
    return layer.n_out * layer.n_in + layer.n_out


def _mlp(name, widths, acts, stages, **kw) -> Workload:
    layers = tuple(Layer("linear", widths[j], widths[j + 1], acts[j], stages[j])
                   for j in range(len(acts)))
    return Workload(name=name, layers=layers, P=max(stages), **kw)


def config(idx: int) -> Workload:
    """Workloads by their 1-based position in the task's list of configurations.

    1: tiny fp32 4-stage MLP (64-wide, ReLU, scalar regression head, MSE).
    2: 16-stage MLP, 1024-wide, GELU, 10-class head sharing the last stage,
       bf16 compute with fp32 master weights.
    3: 6-layer fine-grained Transformer (width 512, 8 heads, feed-forward 2048, vocabulary 8192,
       32 sequences of 128 tokens), bf16 compute, AdamW.
    4: ResNet-20-shaped CNN (19 3x3 convolutions with folded per-channel affine + classifier, one stage
       each), 128 images of 3x32x32, bf16 compute, momentum SGD.
    5: 12-layer fine-grained Transformer (width 1024, 16 heads, feed-forward 4096, vocabulary 32000,
       16 sequences of 512 tokens), bf16 compute, AdamW.
    """
    if idx == 1:
        return _mlp("mlp4_f32", [64, 64, 64, 64, 1], ["relu", "relu", "relu", "none"], [1, 2, 3, 4],
                    N=1, loss="mse", dtype="f32", microbatch=16, n_classes=1,
                    opt=dict(kind="sgdm", lr=0.01, beta=0.9, D=0.9, K=20, weight_decay=0.0),
                    steps=50)
    if idx == 2:
        widths = [1024] * 17 + [10]
        acts = ["gelu"] * 16 + ["none"]
        stages = list(range(1, 17)) + [16]
        return _mlp("mlp16_bf16", widths, acts, stages,
                    N=1, loss="xent", dtype="bf16", microbatch=128, n_classes=10,
                    opt=dict(kind="sgdm", lr=0.001, beta=0.9, D=0.9, K=125, weight_decay=0.0),
                    steps=500, init="he")
    if idx == 3:
        # fine-grained 6-layer Transformer, one stage per weight matrix (P = 38, 51 weight units); AdamW with
        # the linear warm-up of the paper's Transformer recipe (App. C: 8000 steps from 1e-7 to 5e-4,
        # betas 0.9 / 0.98, weight decay 1e-4), T1 annealing over 5x the warm-up (Sec. 3.1), D = 0.1 (App. C)
        return transformer(6, 512, 8, 2048, 8192, 128, 32, dtype="bf16", name="tfm6x512_bf16", steps=40,
                           lr=5e-4, D=0.1, K=40000, weight_decay=1e-4,
                           sched=dict(kind="warmup_invsqrt", base=5e-4, init=1e-7, warmup=8000))
    if idx == 4:
        # ResNet-20 shape: 19 convolutions + the classifier, one stage each (P = 20); momentum SGD with a
        # constant base step, T1 annealing over a quarter of the run, D = 0.5 (the paper's CIFAR10 value, App. C)
        return resnet(3, 128, dtype="bf16", name="resnet20_bf16", steps=200, lr=0.01, D=0.5, K=50)
    if idx == 5:
        # 12 layers, width 1024, 16 heads, feed-forward 4096, vocabulary 32000, sequences of 512 tokens:
        # every weight unit a stage of its own: P = 99 (tau_fwd up to 197), ~217 M parameters
        return transformer(12, 1024, 16, 4096, 32000, 512, 16, dtype="bf16", name="tfm12x1024_bf16", steps=6,
                           ln_own_stage=True,
                           lr=7e-4, D=0.1, K=40000, weight_decay=0.0,
                           sched=dict(kind="warmup_invsqrt", base=7e-4, init=1e-7, warmup=8000))
    raise ValueError(f"unknown workload index {idx}")


def small_mlp(width: int, depth: int, n_out: int, act: str, loss: str, dtype: str,
              microbatch: int, layers_per_stage: int = 1, init: str = "fan_in", **opt) -> Workload:
    """A free-form MLP for tests: `depth` hidden Linear+act layers then a head in the last stage."""
    widths = [width] * (depth + 1) + [n_out]
    acts = [act] * depth + ["none"]
    stages = [j // layers_per_stage + 1 for j in range(depth)]
    stages.append(stages[-1])
    o = dict(kind="sgdm", lr=0.01, beta=0.9, D=0.9, K=10, weight_decay=0.0)
    o.update(opt)
    return _mlp(f"mlp{depth}x{width}_{dtype}", widths, acts, stages, N=1, loss=loss, dtype=dtype,
                microbatch=microbatch, n_classes=n_out, opt=o, steps=0, init=init)


def init_params(wl: Workload, seed: int | None = None) -> List[np.ndarray]:
    """Initial parameters, one packed fp32 vector [W (n_out x n_in, row-major) | b (n_out)] per layer.

    init "fan_in": W ~ U(+-1/sqrt(fan_in)) everywhere.
    init "he":     W ~ U(+-sqrt(6/fan_in)) behind ReLU/GELU (keeps activations O(1) through deep
                   stacks), U(+-sqrt(3/fan_in)) for a linear head.
    b ~ U(+-1/sqrt(fan_in)) in both.
    """
    rng = np.random.default_rng(wl.seed_init if seed is None else seed)
    out = []
    for L in wl.layers:
        if L.kind == "embed":          # E ~ N(0, 1/width)
            out.append((rng.standard_normal((L.n_in, L.n_out)) / np.sqrt(L.n_out)).ravel().astype(np.float32))
            continue
        if L.kind == "layernorm":      # gain 1 + U(+-0.1), bias U(+-0.1): off the trivial point so every use of them shows
            g = 1.0 + rng.uniform(-0.1, 0.1, size=L.n_out)
            b = rng.uniform(-0.1, 0.1, size=L.n_out)
            out.append(np.concatenate([g, b]).astype(np.float32))
            continue
        if L.kind == "conv3x3":
            # W ~ U(+-sqrt(6 / fan_in)), fan_in = 9 C_in; scale 0.5 + U(+-0.05), shift U(+-0.1).  The scale stands
            # for a folded normalisation (gamma / sigma): at 0.5 a residual branch adds about a sixteenth of its
            # input's second moment per block, so activations stay O(1) through the 9 blocks and the initial
            # loss is near log(classes)
            bound = np.sqrt(6.0 / (9 * L.n_in))
            W = rng.uniform(-bound, bound, size=(L.n_out, 9 * L.n_in))
            sc = 0.5 + rng.uniform(-0.05, 0.05, size=L.n_out)
            sh = rng.uniform(-0.1, 0.1, size=L.n_out)
            out.append(np.concatenate([W.ravel(), sc, sh]).astype(np.float32))
            continue
        if wl.init == "he":
            bound = np.sqrt((6.0 if L.act in ("relu", "gelu") else 3.0) / L.n_in)
        else:
            bound = 1.0 / np.sqrt(L.n_in)
        W = rng.uniform(-bound, bound, size=(L.n_out, L.n_in))
        b = rng.uniform(-1.0, 1.0, size=(L.n_out,)) / np.sqrt(L.n_in)
        out.append(np.concatenate([W.ravel(), b]).astype(np.float32))
    return out


class BatchStream:
    """Deterministic stream of microbatches: x ~ N(0,1), targets from a fixed random teacher.

    Teacher: 2-layer tanh network n_in -> 64 -> n_classes with N(0, 1/fan_in) weights.
    "mse": y = teacher(x) as fp32 [M, n_classes];  "xent": y = argmax teacher(x) as int32 [M].
    Batch `k` depends only on (seed_data, k), so any step can be regenerated.
    """

    def __init__(self, wl: Workload):
        self.wl = wl
        n_in = wl.layers[0].n_in
        rng = np.random.default_rng(wl.seed_teacher)
        self.T1 = rng.standard_normal((64, n_in)) / np.sqrt(n_in)
        self.T2 = rng.standard_normal((wl.n_classes, 64)) / np.sqrt(64) * 2.0

    def batch(self, k: int):
        wl = self.wl
        rng = np.random.default_rng([wl.seed_data, k])
        x = rng.standard_normal((wl.microbatch, wl.layers[0].n_in)).astype(np.float32)
        t = np.tanh(x.astype(np.float64) @ self.T1.T) @ self.T2.T
        if wl.loss == "mse":
            y = t.astype(np.float32)
        else:
            y = np.argmax(t, axis=1).astype(np.int32)
        return x, y


def transformer(n_layers: int, d_model: int, n_heads: int, d_ff: int, vocab: int, seq: int, microbatch: int,
                dtype: str = "bf16", name: str | None = None, steps: int = 0, ln_own_stage: bool = False, **opt) -> Workload:
    """Fine-grained pre-LN causal Transformer: one pipeline stage per weight unit.  Units in topological
    order: embed | per layer: ln1, Wq, Wk, Wv, Wo, ln2, W1, W2 | final ln, head.
    ln_own_stage False: a LayerNorm rides in the stage of the matrix that consumes it, P = 6 n_layers + 2.
    ln_own_stage True: every unit is a stage of its own, P = 8 n_layers + 3."""
    layers = [Layer("embed", vocab, d_model, "none", 1)]
    st = 1

    def add(kind, n_in, n_out, act, new_stage):
        nonlocal st
        if new_stage:
            st += 1
        layers.append(Layer(kind, n_in, n_out, act, st))

    for _ in range(n_layers):
        add("layernorm", d_model, d_model, "none", True)
        add("linear", d_model, d_model, "none", ln_own_stage)
        add("linear", d_model, d_model, "none", True)
        add("linear", d_model, d_model, "none", True)
        add("linear", d_model, d_model, "none", True)
        add("layernorm", d_model, d_model, "none", True)
        add("linear", d_model, d_ff, "relu", ln_own_stage)
        add("linear", d_ff, d_model, "none", True)
    add("layernorm", d_model, d_model, "none", True)
    add("linear", d_model, vocab, "none", ln_own_stage)
    o = dict(kind="adamw", lr=5e-4, beta=0.9, beta2=0.98, eps=1e-8, D=0.1, K=0, weight_decay=0.0,
             sched=dict(kind="warmup_invsqrt", base=5e-4, init=1e-7, warmup=40))
    o.update(opt)
    return Workload(name=name or f"tfm{n_layers}x{d_model}_{dtype}", layers=tuple(layers), P=st, N=1, loss="xent",
                    dtype=dtype, microbatch=microbatch, n_classes=vocab, opt=o, steps=steps,
                    arch=dict(kind="transformer", n_layers=n_layers, d_model=d_model, n_heads=n_heads, d_ff=d_ff,
                              vocab=vocab, seq=seq))


class TokenStream:
    """Deterministic token microbatches: ids ~ Zipf(1.1) truncated to the vocabulary (inverse CDF of a
    uniform draw), sequences of seq+1 tokens; inputs are the first seq, targets the next token.
    Stands in for tokenised translation corpora (same shapes; rank-frequency law of natural text)."""

    def __init__(self, wl: Workload, exponent: float = 1.1):
        self.wl = wl
        V = wl.arch["vocab"]
        p = 1.0 / np.power(np.arange(1, V + 1, dtype=np.float64), exponent)
        self.cdf = np.cumsum(p / p.sum())

    def batch(self, k: int):
        wl = self.wl
        S, V = wl.arch["seq"], wl.arch["vocab"]
        rng = np.random.default_rng([wl.seed_data, k])
        u = rng.random((wl.microbatch, S + 1))
        ids = np.minimum(np.searchsorted(self.cdf, u), V - 1).astype(np.int32)
        return np.ascontiguousarray(ids[:, :S]), np.ascontiguousarray(ids[:, 1:])


def resnet(n_blocks: int, microbatch: int, dtype: str = "bf16", image: int = 32, n_classes: int = 10,
           name: str | None = None, steps: int = 0, **opt) -> Workload:
    """ResNet-20-shaped CNN (n_blocks = 3): conv 3 -> 16, three groups of n_blocks two-convolution blocks with
    16 / 32 / 64 channels (the first convolution of groups 2 and 3 has stride 2, recognisable by
    n_out = 2 n_in), global average pool, classifier.  One pipeline stage per weight unit."""
    layers = [Layer("conv3x3", 3, 16, "relu", 1)]
    c, st = 16, 1
    for g in range(3):
        for b in range(n_blocks):
            cin = c
            if g > 0 and b == 0:
                c *= 2
            st += 1
            layers.append(Layer("conv3x3", cin, c, "relu", st))
            st += 1
            layers.append(Layer("conv3x3", c, c, "relu", st))
    st += 1
    layers.append(Layer("linear", 64, n_classes, "none", st))
    o = dict(kind="sgdm", lr=0.01, beta=0.9, D=0.5, K=0, weight_decay=0.0)
    o.update(opt)
    return Workload(name=name or f"resnet{6 * n_blocks + 2}_{dtype}", layers=tuple(layers), P=st, N=1, loss="xent",
                    dtype=dtype, microbatch=microbatch, n_classes=n_classes, opt=o, steps=steps,
                    arch=dict(kind="resnet", n_blocks=n_blocks, image=image))


class ImageStream:
    """Deterministic image microbatches: x ~ N(0,1) fp32 [M, 3, H, W] (NCHW), labels uniform over the classes
    (int32 [M]).  Stands in for CIFAR10 / ImageNet batches (same tensor shapes)."""

    def __init__(self, wl: Workload):
        self.wl = wl

    def batch(self, k: int):
        wl = self.wl
        H = wl.arch["image"]
        rng = np.random.default_rng([wl.seed_data, k])
        x = rng.standard_normal((wl.microbatch, 3, H, H)).astype(np.float32)
        y = rng.integers(0, wl.n_classes, size=wl.microbatch).astype(np.int32)
        return x, y


def batch_stream(wl: Workload):
    """The microbatch generator that fits the workload."""
    kind = wl.arch.get("kind")
    return TokenStream(wl) if kind == "transformer" else ImageStream(wl) if kind == "resnet" else BatchStream(wl)
