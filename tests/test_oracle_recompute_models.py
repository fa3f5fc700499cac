"""Pins for recomputation (paper App. "Statistical efficiency and recompute") in the Transformer and CNN
oracle models: the three-weight gradient - forward values from u_fwd, activations inside every segment
rebuilt with u_recomp, data gradients through u_bkwd - is built a second time with torch autograd, segment
by segment, and compared; plus the special cases that reduce to the two-weight gradient."""
import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

import workloads as wl
from oracle import pipemare_oracle as po
from oracle.resnet_oracle import ResNetModel
from oracle.transformer_oracle import TransformerModel, sinusoidal_positions


def staged_gradients(n_units, seg_of, unit_fn, head, dlog):
    """Autograd construction of the recompute gradient.
    unit_fn(u, get, val, leaves) -> {name: tensor}: unit u's tensors computed by torch from get(name), with the
      VALUE given by weight set `val` ("F" or "R"), the derivative w.r.t. its inputs taken through the backward
      weights, and zero-valued parameter-gradient leaves appended to `leaves`.
    head(get, leaves) -> surrogate logits whose input derivative runs through the backward weights.
    Forward: all units with val = "F" under no_grad.  Backward, segments last to first: the segment's units run
    again with val = "R" on (i) leaf copies of the forward tensors produced outside the segment and (ii) their
    own rebuilt tensors; gradients that later segments left on a forward tensor are injected into the rebuilt
    tensor of the same name; gradients arriving at the leaf copies are handed on to earlier segments."""
    with torch.no_grad():
        fwd = {}
        for u in range(n_units - 1):
            fwd.update(unit_fn(u, fwd.__getitem__, "F", []))
    upstream = {}
    grads = {}
    n_seg = max(seg_of) + 1
    for s in range(n_seg - 1, -1, -1):
        ext, mine, leaves = {}, {}, []

        def get(name):
            if name in mine:
                return mine[name]
            if name not in ext:
                ext[name] = fwd[name].clone().requires_grad_(True)
            return ext[name]

        outs, gouts = [], []
        for u in [u for u in range(n_units) if seg_of[u] == s]:
            if u == n_units - 1:
                outs.append(head(get, leaves))
                gouts.append(dlog)
            else:
                mine.update(unit_fn(u, get, "R", leaves))
        for name, t in mine.items():
            if name in upstream and t.requires_grad:
                outs.append(t)
                gouts.append(upstream[name])
        if outs:
            torch.autograd.backward(outs, gouts)
        for name, leaf in ext.items():
            if leaf.grad is not None:
                upstream[name] = upstream.get(name, 0) + leaf.grad
        for u, ls, post in leaves:
            grads[u] = np.concatenate([post(t.grad if t.grad is not None else torch.zeros_like(t)).numpy().ravel() for t in ls])
    return grads


def seg_table(n_units, checkpoints):
    cps = sorted(set([0] + list(checkpoints)))
    return [sum(1 for c in cps if c <= u) - 1 for u in range(n_units)]


# ----------------------------------------------------------------------------------------- Transformer
def _tfm_setup(seed=0, n_layers=2, d=16, h=4, dff=32, V=37, S=6, B=3):
    w = wl.transformer(n_layers, d, h, dff, V, S, B, dtype="f32")
    params = [p.astype(np.float64) for p in wl.init_params(w, seed)]
    model = TransformerModel(n_layers, d, h, dff, V, S)
    toks, tgt = wl.TokenStream(w).batch(0)
    return w, params, model, toks, tgt


def _tfm_units(model, W, tokens):
    """W = {"F": [...], "R": [...], "B": [...]} weight sets.  Returns (unit_fn, head)."""
    d, dff, V, S, H, dh, nl = model.d, model.dff, model.V, model.S, model.h, model.dh, model.nl
    B = tokens.shape[0]
    tok = torch.as_tensor(tokens.reshape(-1), dtype=torch.long)
    pos = torch.tensor(np.tile(sinusoidal_positions(S, d), (B, 1)))
    ident = lambda t: t

    def lin(x, u, n_out, n_in, val, leaves):
        Wv = torch.tensor(W[val][u][:n_out * n_in].reshape(n_out, n_in))
        bv = torch.tensor(W[val][u][n_out * n_in:])
        Wb = torch.tensor(W["B"][u][:n_out * n_in].reshape(n_out, n_in))
        Wg = torch.zeros_like(Wv, requires_grad=True)
        bg = torch.zeros_like(bv, requires_grad=True)
        leaves.append((u, [Wg, bg], ident))
        return x @ Wb.T + x.detach() @ (Wv - Wb).T + x.detach() @ Wg.T + bv + bg

    def ln(x, u, val, leaves):
        gv, bv = torch.tensor(W[val][u][:d]), torch.tensor(W[val][u][d:])
        gb = torch.tensor(W["B"][u][:d])
        gg = torch.zeros_like(gv, requires_grad=True)
        bg = torch.zeros_like(bv, requires_grad=True)
        leaves.append((u, [gg, bg], ident))
        xh = Fn.layer_norm(x, (d,), eps=1e-5)
        return xh * gb + xh.detach() * (gv - gb) + xh.detach() * gg + bv + bg

    def unit_fn(u, get, val, leaves):
        if u == 0:
            E = torch.tensor(W[val][0].reshape(V, d))
            Eg = torch.zeros_like(E, requires_grad=True)
            leaves.append((0, [Eg], ident))
            return {"x0": E[tok] + Eg[tok] + pos}
        if u == 1 + 8 * nl:
            return {"nf": ln(get(f"x{nl}"), u, val, leaves)}
        l, j = divmod(u - 1, 8)
        t = lambda name: f"{name}_{l}"
        if j == 0:
            return {t("n1"): ln(get(f"x{l}"), u, val, leaves)}
        if j in (1, 2, 3):
            return {t("qkv"[j - 1]): lin(get(t("n1")), u, d, d, val, leaves)}
        if j == 4:
            sp = lambda a: a.reshape(B, S, H, dh).transpose(1, 2)
            o = Fn.scaled_dot_product_attention(sp(get(t("q"))), sp(get(t("k"))), sp(get(t("v"))), is_causal=True)
            o = o.transpose(1, 2).reshape(B * S, d)
            return {t("o"): o, t("h"): get(f"x{l}") + lin(o, u, d, d, val, leaves)}
        if j == 5:
            return {t("n2"): ln(get(t("h")), u, val, leaves)}
        if j == 6:
            return {t("f"): torch.relu(lin(get(t("n2")), u, dff, d, val, leaves))}
        return {f"x{l + 1}": get(t("h")) + lin(get(t("f")), u, d, dff, val, leaves)}

    uh = 2 + 8 * nl

    def head(get, leaves):
        # derivative through the backward weights, parameter gradient from the (kept or rebuilt) input; the
        # value is irrelevant here: the loss gradient comes from the forward logits
        return lin(get("nf"), uh, V, d, "F", leaves)

    return unit_fn, head


def _tfm_dlog(model, Fw, tokens, targets):
    """d loss / d logits of the forward pass (weights Fw), by autograd on the logits."""
    unit_fn, _ = _tfm_units(model, {"F": Fw, "R": Fw, "B": Fw}, tokens)
    with torch.no_grad():
        fwd = {}
        for u in range(model.n_units - 1):
            fwd.update(unit_fn(u, fwd.__getitem__, "F", []))
        uh = model.n_units - 1
        Wh = torch.tensor(Fw[uh][:model.V * model.d].reshape(model.V, model.d))
        logits = fwd["nf"] @ Wh.T + torch.tensor(Fw[uh][model.V * model.d:])
    logits = logits.clone().requires_grad_(True)
    loss = Fn.cross_entropy(logits, torch.as_tensor(targets.reshape(-1), dtype=torch.long))
    loss.backward()
    return float(loss), logits.grad


def _three_sets(params, seed):
    rng = np.random.default_rng(seed)
    jit = lambda s: [p + s * rng.standard_normal(p.shape) * (np.abs(p).mean() + 0.01) for p in params]
    return jit(0.2), jit(0.2), jit(0.2)


@pytest.mark.parametrize("checkpoints", [[0], [0, 3], [0, 2, 4, 7, 11, 14, 18], list(range(19)), [0, 5, 9, 17]])
def test_transformer_three_weight_gradient_against_staged_autograd(checkpoints):
    """Segment boundaries in every kind of place: between the query / key / value projections (which share
    their input), between the attention core's producers and the output projection, between the two
    feed-forward matrices (whose ReLU mask belongs to the first), between the final LayerNorm and the head."""
    w, params, model, toks, tgt = _tfm_setup()
    Fw, Bw, Rw = _three_sets(params, 11)
    loss, grads = model.loss_and_grads(Fw, Bw, (toks, tgt), u_recomp=Rw, checkpoints=checkpoints)
    lt, dlog = _tfm_dlog(model, Fw, toks, tgt)
    assert loss == pytest.approx(lt, rel=1e-12)
    unit_fn, head = _tfm_units(model, {"F": Fw, "R": Rw, "B": Bw}, toks)
    want = staged_gradients(model.n_units, seg_table(model.n_units, checkpoints), unit_fn, head, dlog)
    for u in range(model.n_units):
        assert np.allclose(grads[u], want[u], rtol=0, atol=1e-12 * max(1.0, np.max(np.abs(want[u])))), u
    # and the third weight set matters (unless every unit sits alone ... it still rebuilds its own outputs)
    _, g2 = model.loss_and_grads(Fw, Bw, (toks, tgt))
    assert max(np.max(np.abs(a - b)) for a, b in zip(grads, g2)) > 1e-6


def test_transformer_recompute_special_cases():
    w, params, model, toks, tgt = _tfm_setup(seed=3)
    Fw, Bw, Rw = _three_sets(params, 5)
    l0, g0 = model.loss_and_grads(Fw, Bw, (toks, tgt))
    # rebuilding with the forward weights rebuilds the forward tensors: nothing changes, wherever the cuts are
    for cps in ([0], [0, 4, 9], list(range(model.n_units))):
        l1, g1 = model.loss_and_grads(Fw, Bw, (toks, tgt), u_recomp=Fw, checkpoints=cps)
        assert l1 == l0
        for a, b in zip(g0, g1):
            assert np.allclose(a, b, rtol=0, atol=1e-13)
    # the loss never depends on the recompute weights; the embedding's own gradient does (through rebuilt
    # activations downstream in its segment) but not when it sits alone in front of a cut and nothing is shared
    l2, g2 = model.loss_and_grads(Fw, Bw, (toks, tgt), u_recomp=Rw, checkpoints=[0, 1])
    assert l2 == l0
    # a unit that sits alone in its segment rebuilds only its own outputs from kept inputs: its weight gradient
    # input is the kept forward tensor, so e.g. Wq's gradient (unit 2) uses the forward n1 when cut off from ln1
    _, g3 = model.loss_and_grads(Fw, Bw, (toks, tgt), u_recomp=Rw, checkpoints=list(range(model.n_units)))
    _, g4 = model.loss_and_grads(Fw, Bw, (toks, tgt), u_recomp=Rw, checkpoints=[0])
    assert max(np.max(np.abs(a - b)) for a, b in zip(g3, g4)) > 1e-6


def test_transformer_recompute_in_the_recurrence_reads_the_stated_versions():
    """P = 19 stages in segments of 4: tau_recomp,i = 2 (S' - j) (App. "PipeMare Recompute"); the rebuilt activations
    come from version t - tau_recomp,i corrected by (tau_fwd,i - tau_recomp,i) delta_t ("T2 for Recompute")."""
    w, params, model, toks, tgt = _tfm_setup(seed=1)
    P = w.P
    tf, tb = po.pipeline_delays(P, 1)
    tr = po.recompute_delays(P, 4, 1)
    seen = {}

    class Spy:
        def loss_and_grads(self, u_fwd, u_bkwd, batch, u_recomp=None, checkpoints=None):
            seen["r"], seen["c"] = u_recomp, checkpoints
            return model.loss_and_grads(u_fwd, u_bkwd, batch, u_recomp=u_recomp, checkpoints=checkpoints)

    stage = [L.stage for L in w.layers]
    o = po.PipeMareOracle(Spy(), params, stage, tf, tb, dict(kind="sgdm", beta=0.9, D=0.3, K=4, sched=dict(kind="const", base=0.01),
                                                             tau_recomp=tr, segment=4), keep_history=True)
    stream = wl.TokenStream(w)
    for k in range(9):
        delta_before = [d.copy() for d in o.delta]
        o.step(stream.batch(k))
        for u, st in enumerate(stage):
            base = o.hist[u][max(k - tr[st - 1], 0)]
            want = base - (tf[st - 1] - tr[st - 1]) * delta_before[u]
            assert np.array_equal(seen["r"][u], want)
    # a unit opens a segment if it is the first unit of stage 1, 5, 9, 13, 17
    assert seen["c"] == [u for u in range(len(stage)) if stage[u] in (1, 5, 9, 13, 17) and (u == 0 or stage[u - 1] != stage[u])]


# ----------------------------------------------------------------------------------------- CNN
def _cnn_setup(seed=0, n_blocks=1, B=3, image=8):
    w = wl.resnet(n_blocks, B, dtype="f32", image=image)
    params = [p.astype(np.float64) for p in wl.init_params(w, seed)]
    model = ResNetModel(n_blocks, 10, image)
    x, y = wl.ImageStream(w).batch(0)
    return w, params, model, x, y


def _cnn_units(model, W, x):
    specs = model.specs
    nconv = len(specs)
    xt = torch.tensor(np.asarray(x, dtype=np.float64))          # NCHW
    in_name = lambda u: "img" if u == 0 else f"y{u - 1}"
    to_ohwi = lambda t: t.permute(0, 2, 3, 1).contiguous()
    ident = lambda t: t

    def shortcut(a, co, stride):
        if stride == 1 and a.shape[1] == co:
            return a
        a = a[:, :, ::stride, ::stride]
        return Fn.pad(a, (0, 0, 0, 0, 0, co - a.shape[1]))

    def unit_fn(u, get, val, leaves):
        ci, co, stride = specs[u]
        nw = co * 9 * ci
        unpack = lambda p: torch.tensor(p[:nw].reshape(co, 3, 3, ci)).permute(0, 3, 1, 2).contiguous()   # OIHW
        Wv, Wb = unpack(W[val][u]), unpack(W["B"][u])
        sv, tv = torch.tensor(W[val][u][nw:nw + co]), torch.tensor(W[val][u][nw + co:])
        sb = torch.tensor(W["B"][u][nw:nw + co])
        Wg = torch.zeros_like(Wv, requires_grad=True)
        sg = torch.zeros_like(sv, requires_grad=True)
        tg = torch.zeros_like(tv, requires_grad=True)
        leaves.append((u, [Wg], to_ohwi))
        leaves.append((-1 - u, [sg, tg], ident))
        inp = xt if u == 0 else get(in_name(u))
        c = lambda a, K: Fn.conv2d(a, K, stride=stride, padding=1)
        v = lambda s: s.view(1, -1, 1, 1)
        z = c(inp, Wb) + (c(inp.detach(), Wv) - c(inp.detach(), Wb)).detach() + c(inp.detach(), Wg)
        a = z * v(sb) + z.detach() * v(sv - sb) + z.detach() * v(sg) + v(tv) + v(tg)
        if u >= 2 and (u - 1) % 2 == 1:
            blk = xt if u - 1 == 0 else get(in_name(u - 1))
            a = a + shortcut(blk, co, specs[u - 1][2])
        return {f"y{u}": torch.relu(a)}

    nfc = model.ncls * 64

    def head(get, leaves):
        Wb = torch.tensor(W["B"][nconv][:nfc].reshape(model.ncls, 64))
        Wg = torch.zeros_like(Wb, requires_grad=True)
        bg = torch.zeros(model.ncls, dtype=torch.float64, requires_grad=True)
        leaves.append((nconv, [Wg, bg], ident))
        pooled = get(f"y{nconv - 1}").mean(dim=(2, 3))
        return pooled @ Wb.T + pooled.detach() @ Wg.T + bg

    return unit_fn, head


def _cnn_dlog(model, Fw, x, labels):
    unit_fn, _ = _cnn_units(model, {"F": Fw, "R": Fw, "B": Fw}, x)
    nconv = len(model.specs)
    with torch.no_grad():
        fwd = {}
        for u in range(nconv):
            fwd.update(unit_fn(u, fwd.__getitem__, "F", []))
        nfc = model.ncls * 64
        pooled = fwd[f"y{nconv - 1}"].mean(dim=(2, 3))
        logits = pooled @ torch.tensor(Fw[nconv][:nfc].reshape(model.ncls, 64)).T + torch.tensor(Fw[nconv][nfc:])
    logits = logits.clone().requires_grad_(True)
    loss = Fn.cross_entropy(logits, torch.as_tensor(np.asarray(labels), dtype=torch.long))
    loss.backward()
    return float(loss), logits.grad


@pytest.mark.parametrize("checkpoints", [[0], [0, 2], [0, 1, 2, 3, 4, 5, 6, 7], [0, 3, 6], [0, 7]])
def test_cnn_three_weight_gradient_against_staged_autograd(checkpoints):
    """Cuts between the two convolutions of a block (the second then adds a kept block input to a rebuilt branch
    or the other way round), between blocks, in front of the classifier."""
    w, params, model, x, y = _cnn_setup()
    assert model.n_units == 8
    Fw, Bw, Rw = _three_sets(params, 21)
    loss, grads = model.loss_and_grads(Fw, Bw, (x, y), u_recomp=Rw, checkpoints=checkpoints)
    lt, dlog = _cnn_dlog(model, Fw, x, y)
    assert loss == pytest.approx(lt, rel=1e-12)
    unit_fn, head = _cnn_units(model, {"F": Fw, "R": Rw, "B": Bw}, x)
    want = staged_gradients(model.n_units, seg_table(model.n_units, checkpoints), unit_fn, head, dlog)
    nconv = len(model.specs)
    for u in range(nconv):
        ref = np.concatenate([want[u], want[-1 - u]])
        assert np.allclose(grads[u], ref, rtol=0, atol=1e-12 * max(1.0, np.max(np.abs(ref)))), u
    assert np.allclose(grads[nconv], want[nconv], rtol=0, atol=1e-12)
    _, g2 = model.loss_and_grads(Fw, Bw, (x, y))
    assert max(np.max(np.abs(a - b)) for a, b in zip(grads, g2)) > 1e-6


def test_cnn_recompute_with_forward_weights_is_no_recompute():
    w, params, model, x, y = _cnn_setup(seed=2)
    Fw, Bw, _ = _three_sets(params, 4)
    l0, g0 = model.loss_and_grads(Fw, Bw, (x, y))
    for cps in ([0], [0, 2, 5], list(range(model.n_units))):
        l1, g1 = model.loss_and_grads(Fw, Bw, (x, y), u_recomp=Fw, checkpoints=cps)
        assert l1 == l0
        for a, b in zip(g0, g1):
            assert np.allclose(a, b, rtol=0, atol=1e-13)
