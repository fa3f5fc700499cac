"""GPU parity of the fine-grained Transformer stages: LayerNorm and attention primitives against
NumPy fp64, then whole PipeMare training runs against the fp64 oracle (same tolerances as the MLP
tests: slots and step counters bit-exact, master weights within 1e-5 (fp32) / 2e-3 (bf16) max-relative
per unit)."""
import math

import numpy as np
import pytest

import workloads as wl
from oracle import pipemare_oracle as po
from oracle import transformer_oracle as to
from pm_testutil import key_bias_entries, make_gpu, make_oracle, max_rel_err

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3}


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _tdt(torch, dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


# ------------------------------------------------------------------------------- LayerNorm
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,d", [(37, 16), (200, 72), (1000, 512), (4096, 1024)])
def test_layernorm_primitives(torch_cuda, dtype, rows, d):
    import paper_1910_05124_amd as pm
    torch = torch_cuda
    tdt = _tdt(torch, dtype)
    rng = np.random.default_rng(rows + d)
    x = (rng.standard_normal((rows, d)) * 2.0 + 0.5).astype(np.float32)
    gb = torch.from_numpy(np.concatenate([1.0 + 0.2 * rng.standard_normal(d), 0.1 * rng.standard_normal(d)]).astype(np.float32)).cuda().to(tdt)
    gbk = torch.from_numpy((1.0 + 0.2 * rng.standard_normal(d)).astype(np.float32)).cuda().to(tdt)     # backward gain differs
    dy = rng.standard_normal((rows, d)).astype(np.float32)
    dres = rng.standard_normal((rows, d)).astype(np.float32)
    xd, dyd, dresd = (torch.from_numpy(a).cuda() for a in (x, dy, dres))
    y = torch.empty(rows, d, dtype=tdt, device="cuda")
    mean = torch.empty(rows, dtype=torch.float32, device="cuda")
    rstd = torch.empty_like(mean)
    dx = torch.empty(rows, d, dtype=torch.float32, device="cuda")
    dxt = torch.empty(rows, d, dtype=tdt, device="cuda")
    dg = torch.zeros(d, dtype=torch.float32, device="cuda")
    db = torch.zeros(d, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    esz = gb.element_size()
    pm.pm_layernorm_fwd(st, dtype, rows, d, xd.data_ptr(), gb.data_ptr(), gb.data_ptr() + d * esz, y.data_ptr(),
                        mean.data_ptr(), rstd.data_ptr())
    pm.pm_layernorm_bwd(st, dtype, rows, d, dyd.data_ptr(), xd.data_ptr(), mean.data_ptr(), rstd.data_ptr(),
                        gbk.data_ptr(), dresd.data_ptr(), dx.data_ptr(), dxt.data_ptr(), dg.data_ptr(), db.data_ptr())
    torch.cuda.synchronize()
    G = gb.float().cpu().numpy().astype(np.float64)
    Gk = gbk.float().cpu().numpy().astype(np.float64)
    X = x.astype(np.float64)
    y_ref, xhat, rs = to._ln_fwd(X, G[:d], G[d:])
    dx_ref, dg_ref, db_ref = to._ln_bwd(dy.astype(np.float64), xhat, rs, Gk)
    dx_ref = dx_ref + dres
    out_tol = 2.0 ** -8 if dtype == "bf16" else 2e-6
    assert np.max(np.abs(y.float().cpu().numpy() - y_ref)) <= out_tol * np.max(np.abs(y_ref))
    assert np.max(np.abs(mean.cpu().numpy() - X.mean(1))) <= 1e-6 * (1 + np.max(np.abs(X.mean(1))))
    assert np.max(np.abs(rstd.cpu().numpy() - rs[:, 0])) <= 2e-6 * np.max(rs)
    assert np.max(np.abs(dx.cpu().numpy() - dx_ref)) <= 4e-6 * np.max(np.abs(dx_ref))
    assert np.max(np.abs(dxt.float().cpu().numpy() - dx_ref)) <= out_tol * np.max(np.abs(dx_ref))
    assert np.max(np.abs(dg.cpu().numpy() - dg_ref)) <= 1e-5 * np.max(np.abs(dg_ref))
    assert np.max(np.abs(db.cpu().numpy() - db_ref)) <= 1e-5 * np.max(np.abs(db_ref))


# ------------------------------------------------------------------------------- attention core
def _attn_ref(q, k, v, do, B, S, H, dh):
    m = to.TransformerModel(1, H * dh, H, 8, 8, S)
    o, cache = m._attention_fwd(q, k, v, B)
    dq, dk, dv = m._attention_bwd(do, cache, B)
    q4, k4, _, _ = cache
    sc = q4 @ k4.transpose(0, 1, 3, 2) / math.sqrt(dh)
    sc = np.where(np.triu(np.ones((S, S), dtype=bool), k=1), -np.inf, sc)
    mx = sc.max(-1, keepdims=True)
    lse = (np.log(np.exp(sc - mx).sum(-1)) + mx[..., 0])                  # [B, H, S]
    return o, lse, dq, dk, dv


@pytest.mark.parametrize("dtype,B,S,H,dh", [("f32", 2, 6, 4, 4), ("f32", 3, 50, 2, 16), ("f32", 2, 120, 2, 64),
                                            ("bf16", 2, 24, 3, 8), ("bf16", 2, 32, 2, 64), ("bf16", 3, 128, 8, 64),
                                            ("bf16", 2, 512, 4, 64), ("bf16", 1, 96, 2, 64)])
def test_attention_primitives(torch_cuda, dtype, B, S, H, dh):
    import paper_1910_05124_amd as pm
    torch = torch_cuda
    tdt = _tdt(torch, dtype)
    rng = np.random.default_rng(S * 7 + dh)
    d = H * dh

    def dev(a):
        return torch.from_numpy(a.astype(np.float32)).cuda().to(tdt).contiguous()

    def host(t):
        return t.float().cpu().numpy().astype(np.float64)

    q, k, v, do = (dev(rng.standard_normal((B * S, d)) * s) for s in (1.5, 1.5, 1.0, 1.0))
    o = torch.empty_like(q)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    lse = torch.empty(B * H * S, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    pm.pm_attention_fwd(st, dtype, B, S, H, dh, q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr())
    pm.pm_attention_bwd(st, dtype, B, S, H, dh, q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), do.data_ptr(),
                        lse.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr())
    torch.cuda.synchronize()
    o_ref, lse_ref, dq_ref, dk_ref, dv_ref = _attn_ref(host(q), host(k), host(v), host(do), B, S, H, dh)
    # bf16: probabilities and the o / do operands pass through bf16 inside the kernel and the outputs are
    # rounded once more: a few units of 2^-8 of the output scale
    tol = 3 * 2.0 ** -8 if dtype == "bf16" else 1e-5
    assert np.max(np.abs(lse.cpu().numpy().reshape(B, H, S) - lse_ref)) <= (2e-2 if dtype == "bf16" else 1e-5)
    for got, ref, name in ((o, o_ref, "o"), (dq, dq_ref, "dq"), (dk, dk_ref, "dk"), (dv, dv_ref, "dv")):
        err = np.max(np.abs(host(got) - ref)) / np.max(np.abs(ref))
        assert err <= tol, (name, err)


# ------------------------------------------------------------------------------- whole training runs
def run_pair(torch, w, steps, tau=None, N=1, gpu_kw=None, check_tables=True, **kw):
    params = wl.init_params(w)
    tf, tb = tau if tau is not None else po.pipeline_delays(w.P, N)
    stream = wl.TokenStream(w)
    o = make_oracle(w, params, tf, tb, N=N, **kw)
    g = make_gpu(w, params, tf, tb, N=N, **dict(kw, **(gpu_kw or {})))
    losses = []
    for k in range(steps):
        mbs = [stream.batch(k * N + j) for j in range(N)]
        lo = o.step(mbs if N > 1 else mbs[0])
        lg = 0.0
        for x, y in mbs:
            lg += g.step(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda(), want_loss=True) / N
        losses.append((lo, lg))
        if check_tables:
            t_used, fs, bs, ws, lrs = g.step_table()
            assert t_used == k
            for u, L in enumerate(w.layers):
                R = tf[L.stage - 1] + 1
                vf, vb = o.last_versions[u]
                assert (fs[u], bs[u], ws[u]) == (vf % R, vb % R, (k + 1) % R)
                assert lrs[u] == pytest.approx(o.last_lr[u], rel=2e-7)
    return g, o, losses


def _kw(w, **over):
    o = w.opt
    kw = dict(opt=o["kind"], beta=o["beta"], beta2=o["beta2"], eps=o["eps"], D=o["D"], K=o["K"],
              weight_decay=o["weight_decay"], sched=o["sched"])
    kw.update(over)
    return kw


def movement_rel_l2(gpu_w, oracle_w, w0):
    """Per unit ||(w_gpu - w_0) - (w_oracle - w_0)||_2 / ||w_oracle - w_0||_2, max over units: how well the
    TRAINING MOVEMENT agrees (the max-relative weight error is small by construction while the weights
    have moved little)."""
    out = []
    for a, b, c in zip(gpu_w, oracle_w, w0):
        mv = b - c.astype(np.float64)
        out.append(float(np.linalg.norm(a.astype(np.float64) - b) / max(np.linalg.norm(mv), 1e-300)))
    return max(out), out


@pytest.mark.parametrize("case", ["pipemare_f32", "sgdm_bf16", "adamw_bf16", "t2_off", "pipedream", "gpipe", "sgdm_clip",
                                  "microbatches", "sync_warmup", "gelu_ragged_vocab", "wide_vocab", "wide_vocab_bf16"])
def test_tiny_transformer_modes(torch_cuda, case):
    dtype = "bf16" if case.endswith("bf16") else "f32"
    V = 61 if case != "gelu_ragged_vocab" else 45
    if case.startswith("wide_vocab"):
        V = 2501                   # rows wide enough for the row-resident loss kernel, ragged last group of 4
    w = wl.transformer(2, 32, 4, 64, V, 10, 3, dtype=dtype, K=6,
                       sched=dict(kind="warmup_invsqrt", base=2e-3, init=1e-5, warmup=5))
    kw = _kw(w)
    tau, N = None, 1
    if case == "sgdm_bf16":
        # momentum SGD keeps the gradient's magnitude, so bf16 rounding noise stays a small fraction of
        # the movement and the weights may move a lot inside the 2e-3 band
        kw = dict(opt="sgdm", lr=0.004, beta=0.9, D=0.5, K=6)
    elif case == "adamw_bf16":
        # Adam turns every gradient entry into a step of about the step size whatever its magnitude: an
        # entry whose gradient is below the bf16 noise floor moves by +-lr per step at random.  The
        # step size is chosen so that 12 such steps stay inside the band; the movement check below
        # shows the two trajectories still agree in direction and size.
        kw = _kw(w, sched=dict(kind="warmup_invsqrt", base=2e-5, init=1e-7, warmup=5))
    if case == "t2_off":
        kw["t2"] = False
    elif case == "pipedream":
        tau = po.pipeline_delays(w.P, 1, "pipedream")
    elif case == "gpipe":
        tau = po.pipeline_delays(w.P, 1, "gpipe")
        # With all delays zero T1 divides nothing and every unit takes the full step.  One feed-forward
        # entry has a gradient of the order of Adam's eps (1e-8): its update m / (sqrt(v) + eps) passes
        # on the fp32 rounding of that gradient, and it ends 1.2e-5 off at the base step 2e-3 (measured,
        # the same in every run), 6.3e-6 at 1e-3, used here; every other entry is below 3e-7 at both.
        w = wl.transformer(2, 32, 4, 64, V, 10, 3, dtype=dtype, K=6,
                           sched=dict(kind="warmup_invsqrt", base=1e-3, init=1e-5, warmup=5))
        kw = _kw(w)
    elif case == "sgdm_clip":
        kw = dict(opt="sgdm", lr=0.02, beta=0.9, D=0.5, K=6, clip_norm=0.5, weight_decay=0.01)
    elif case == "microbatches":
        N = 2
    elif case == "sync_warmup":
        kw["sync_warmup"] = 4
    elif case == "wide_vocab_bf16":
        kw = dict(opt="sgdm", lr=0.004, beta=0.9, D=0.5, K=6)
    g, o, losses = run_pair(torch_cuda, w, 12, tau=tau, N=N, **kw)
    for lo, lg in losses:
        assert lg == pytest.approx(lo, rel=3e-2 if dtype == "bf16" else 1e-4)
    err, errs = max_rel_err(g.weights(), o.weights(), skip=key_bias_entries(w))
    mv, mvs = movement_rel_l2(g.weights(), o.weights(), wl.init_params(w))
    print(case, "max-rel", err, "movement rel-L2", mv)
    assert err <= TOL[dtype], errs
    if dtype == "bf16":
        # units 3 and 11 (key projections) hold the excluded bias entries
        assert max(m for u, m in enumerate(mvs) if u not in key_bias_entries(w)) <= 0.15, mvs
    g.close()


@pytest.mark.parametrize("opt", ["sgdm", "adamw"])
def test_small_bf16_transformer_mfma_path(torch_cuda, opt):
    """Sizes that take the MFMA GEMMs and the MFMA attention (head size 64, sequence a multiple of 32).
    Step sizes as in test_tiny_transformer_modes: momentum SGD may move far, Adam's step is kept small
    because it amplifies sub-noise-floor gradient entries to full steps."""
    w = wl.transformer(2, 128, 2, 256, 512, 64, 4, dtype="bf16", K=10,
                       sched=dict(kind="warmup_invsqrt", base=2e-5, init=1e-7, warmup=10))
    kw = _kw(w) if opt == "adamw" else dict(opt="sgdm", lr=0.002, beta=0.9, D=0.5, K=10)
    g, o, losses = run_pair(torch_cuda, w, 16, **kw)
    for lo, lg in losses:
        assert lg == pytest.approx(lo, rel=2e-2)
    err, errs = max_rel_err(g.weights(), o.weights(), skip=key_bias_entries(w))
    mv, mvs = movement_rel_l2(g.weights(), o.weights(), wl.init_params(w))
    print("small bf16 transformer", opt, "max-rel", err, "movement rel-L2", mv, np.round(mvs, 3))
    assert err <= TOL["bf16"], errs
    assert max(m for u, m in enumerate(mvs) if u not in key_bias_entries(w)) <= 0.15, mvs
    g.close()


def test_ragged_bf16_transformer_grouped_projections(torch_cuda):
    """3360 tokens of width 320 (five heads of 64): the query / key / value projections go out as one
    three-problem launch and their data gradients as one product over the concatenated contraction,
    both with ragged last tiles (3360 = 52.5 * 64 = 26.25 * 128, 320 = 2.5 * 128)."""
    w = wl.transformer(1, 320, 5, 640, 512, 96, 35, dtype="bf16", K=4,
                       sched=dict(kind="warmup_invsqrt", base=2e-5, init=1e-7, warmup=4))
    kw = dict(opt="sgdm", lr=0.002, beta=0.9, D=0.5, K=4)
    g, o, losses = run_pair(torch_cuda, w, 6, **kw)
    for lo, lg in losses:
        assert lg == pytest.approx(lo, rel=2e-2)
    err, errs = max_rel_err(g.weights(), o.weights(), skip=key_bias_entries(w))
    mv, mvs = movement_rel_l2(g.weights(), o.weights(), wl.init_params(w))
    print("ragged grouped projections", "max-rel", err, "movement rel-L2", mv, np.round(mvs, 3))
    assert err <= TOL["bf16"], errs
    assert max(m for u, m in enumerate(mvs) if u not in key_bias_entries(w)) <= 0.15, mvs
    g.close()


@pytest.mark.parametrize("dtype,steps,lr", [("f32", 420, 2e-5), ("bf16", 210, 5e-5)])
def test_narrow_transformer_with_the_stage_table_of_the_12_layer_workload(torch_cuda, dtype, steps, lr):
    """The delay table and ring depths of the largest workload (12 layers, every unit a stage of its own:
    P = 99, tau_fwd = 197 .. 1) on a narrow model (width 128, 2 heads of 64, feed-forward 256, vocabulary
    512, 4 x 32 tokens) the oracle steps in milliseconds: fp32 for 420 steps (every ring wraps twice),
    bf16 (MFMA products and attention) for 210 steps (past tau_max + 2, so every stage has read a
    genuinely delayed version).  Momentum SGD so that the movement is bounded too."""
    w = wl.transformer(12, 128, 2, 256, 512, 32, 4, dtype=dtype, ln_own_stage=True)
    assert w.P == 99
    tf, tb = po.pipeline_delays(w.P, 1)
    assert tf[0] == 197 and tf[-1] == 1
    params = wl.init_params(w)
    kw = dict(opt="sgdm", lr=lr, beta=0.9, D=0.1, K=50)
    o = make_oracle(w, params, tf, tb, **kw)
    g = make_gpu(w, params, tf, tb, **kw)
    stream = wl.TokenStream(w)
    for k in range(steps):
        x, y = stream.batch(k)
        lo = o.step((x, y))
        chk = k % 30 == 0 or k + 1 == steps
        lg = g.step(torch_cuda.from_numpy(x).cuda(), torch_cuda.from_numpy(y).cuda(), want_loss=chk)
        if not chk:
            continue
        assert lg == pytest.approx(lo, rel=2e-2 if dtype == "bf16" else 1e-4)
        t_used, fs, bs, ws, lrs = g.step_table()
        assert t_used == k
        for u, L in enumerate(w.layers):
            R = tf[L.stage - 1] + 1
            vf, vb = o.last_versions[u]
            assert (fs[u], bs[u], ws[u]) == (vf % R, vb % R, (k + 1) % R)
            assert lrs[u] == pytest.approx(o.last_lr[u], rel=2e-7)
    err, errs = max_rel_err(g.weights(), o.weights(), skip=key_bias_entries(w))
    mv, mvs = movement_rel_l2(g.weights(), o.weights(), params)
    move = [float(np.max(np.abs(a - b.astype(np.float64))) / np.max(np.abs(b))) for a, b in zip(o.weights(), params)]
    print("narrow 12-layer", dtype, "max-rel", err, "movement rel-L2 err", mv, "largest unit movement", max(move))
    print("   per unit max-rel:", np.array2string(np.array(errs), precision=1, max_line_width=400))
    print("   per unit movement:", np.array2string(np.array(move), precision=3, max_line_width=400))
    assert max(move) > 0.02
    # fp32: T1 divides the early step sizes by up to 197, which puts many increments below half an ulp of the
    # fp32 master weight they are added to; each of the N additions w <- w + v rounds by at most 2^-24 |w|, so
    # N 2^-24 (2.5e-5 for 420 steps) is the bound the arithmetic gives where 1e-5 covers the 50- and 100-step runs
    tol = max(TOL[dtype], steps * 2.0 ** -24) if dtype == "f32" else TOL[dtype]
    assert err <= tol, errs
    if dtype == "bf16":
        assert max(m for u, m in enumerate(mvs) if u not in key_bias_entries(w)) <= 0.15, mvs
    g.close()


@pytest.mark.parametrize("opt,tile", [("sgdm", 128), ("adamw", 128), ("adamw", 256)])
def test_update_in_the_weight_gradient_epilogue_matches_the_separate_pass(torch_cuda, opt, tile):
    """Where the update is applied (in the epilogue of the grouped weight-gradient launch for the weight matrices,
    or by the pass over all parameters: pm_opts.update_placement) must not change what is computed: same
    gradients, same recurrences per parameter.  Two contexts step on the same batches; after every step every
    state array of every unit is compared, then the second context is given the first one's state (checkpoint
    image), so that each step starts from identical bits and only the order of the fp32 atomics inside a step
    (loss, LayerNorm and embedding gradients) can differ.  'tile' picks shapes for the launch's 128 x 128 and
    256 x 256 block tiles (the latter needs at least 256 such tiles)."""
    if tile == 128:
        w = wl.transformer(2, 128, 2, 256, 512, 64, 4, dtype="bf16", K=10,
                           sched=dict(kind="warmup_invsqrt", base=2e-3, init=1e-5, warmup=10))
    else:
        w = wl.transformer(4, 512, 8, 2048, 8192, 64, 4, dtype="bf16", K=10,       # 64 + 4 * 48 = 256 tiles of 256 x 256
                           sched=dict(kind="warmup_invsqrt", base=2e-3, init=1e-5, warmup=10))
    kw = _kw(w, weight_decay=0.01) if opt == "adamw" else dict(opt="sgdm", lr=0.002, beta=0.9, D=0.5, K=10, weight_decay=0.01)
    params = wl.init_params(w)
    tf, tb = po.pipeline_delays(w.P, 1)
    ga = make_gpu(w, params, tf, tb, update_placement="launch", **kw)
    gb = make_gpu(w, params, tf, tb, update_placement="pass", **kw)
    ne, npass = ga.update_split()
    n_mat = sum(L.n_in * L.n_out for L in w.layers if L.kind == "linear")
    assert ne == n_mat and npass > 0, (ne, npass, n_mat)
    assert gb.update_split()[0] == 0
    stream = wl.TokenStream(w)
    steps = 7
    worst = {True: 0.0, False: 0.0}
    for k in range(steps):
        x, y = stream.batch(k)
        xa, ya = torch_cuda.from_numpy(x).cuda(), torch_cuda.from_numpy(y).cuda()
        la = ga.step(xa, ya, want_loss=True)
        lb = gb.step(xa, ya, want_loss=True)
        assert la == pytest.approx(lb, rel=1e-5)
        ta, tb_ = ga.step_table(), gb.step_table()
        assert ta[0] == tb_[0] == k and all(np.array_equal(p, q) for p, q in zip(ta[1:], tb_[1:]))
        for u, L in enumerate(w.layers):
            mat = L.kind == "linear"
            for which in (0, 1, 2, 3, 4):          # master weights, delta, momentum, corrected backward weights, gradient
                a, b = ga.state(which, u), gb.state(which, u)
                nm = L.n_in * L.n_out if mat else 0
                for part, tight in ((slice(0, nm), True), (slice(nm, None), False)):
                    if a[part].size == 0:
                        continue
                    if which == 3:
                        # stored in bf16: a last-bit difference of the fp32 value before rounding may flip the
                        # rounding of a few entries by one bf16 step of that entry
                        # (plus the matrices' own bound where an entry is near zero and its terms cancel)
                        diff = np.abs(a[part] - b[part])
                        bound = 2.0 ** -7 * np.abs(b[part]) + 1e-6 * float(np.max(np.abs(b[part])))
                        assert np.all(diff <= bound) and np.mean(diff > 0) <= 1e-3, (k, u, part, float(np.max(diff - bound)), float(np.mean(diff > 0)))
                        continue
                    scale = float(np.max(np.abs(b[part]))) or 1.0
                    dev = float(np.max(np.abs(a[part] - b[part]))) / scale
                    worst[tight] = max(worst[tight], dev)
                    # matrices (same products, same expressions, no atomics): a few times the difference between a
                    # fused and an unfused multiply-add.  The rest goes through the same pass in both contexts, from
                    # gradients summed with atomics; where such a sum cancels, the order of its terms decides the low
                    # bits of an entry whose sign Adam then turns into a full-size step (measured 2.3e-4)
                    assert dev <= (1e-6 if tight else 2e-3), (k, u, which, part, dev)
        gb.restore(ga.checkpoint())
    print("update in the epilogue vs separate pass:", opt, tile, "largest deviation / max: matrices", worst[True],
          "other parameters", worst[False])
    ga.close()
    gb.close()


def test_wide_vocabulary_transformer_large_tile_paths_live_oracle(torch_cuda):
    """One layer of width 1024 (16 heads) over a vocabulary of 16384, 16 x 256 tokens: the smallest shapes that take
    every large-tile path of the 12-layer workload - the grouped weight-gradient launch on 256 x 256 tiles with the
    update of the weight matrices inside it (40 M parameters: the automatic placement chooses it), and the data
    gradient through the vocabulary projection as two halves of the contraction whose fp32 results the final
    LayerNorm backward adds.  Every entry of every unit against the live oracle (the stored-value runs of the large
    workload compare samples and segment sums)."""
    w = wl.transformer(1, 1024, 16, 1024, 16384, 256, 16, dtype="bf16")
    kw = dict(opt="sgdm", lr=0.002, beta=0.9, D=0.5, K=4)
    params = wl.init_params(w)
    tf, tb = po.pipeline_delays(w.P, 1)
    o = make_oracle(w, params, tf, tb, **kw)
    g = make_gpu(w, params, tf, tb, **kw)
    n_mat = sum(L.n_in * L.n_out for L in w.layers if L.kind == "linear")
    assert g.update_split()[0] == n_mat            # the update of the matrices runs inside the weight-gradient launch
    stream = wl.TokenStream(w)
    steps = 3
    for k in range(steps):
        x, y = stream.batch(k)
        lo = o.step((x, y))
        lg = g.step(torch_cuda.from_numpy(x).cuda(), torch_cuda.from_numpy(y).cuda(), want_loss=True)
        assert lg == pytest.approx(lo, rel=2e-2)
        if k == 0:
            # consumed gradients of the first step (same weights on both sides), per unit max |dg| / max |g|
            skip = key_bias_entries(w)
            for u in range(len(w.layers)):
                gg, go = g.state(4, u), o.last_grads[u]
                if u in skip:                      # the matrix part only (the key bias has a zero gradient)
                    gg, go = gg[:skip[u].start], go[:skip[u].start]
                rel = float(np.max(np.abs(gg - go)) / max(float(np.max(np.abs(go))), 1e-300))
                assert rel <= 3e-2, (u, rel)
    err, errs = max_rel_err(g.weights(), o.weights(), skip=key_bias_entries(w))
    mv, mvs = movement_rel_l2(g.weights(), o.weights(), params)
    print("wide vocabulary, large tiles: max-rel", err, "movement rel-L2", mv)
    assert err <= TOL["bf16"], errs
    assert max(m for u, m in enumerate(mvs) if u not in key_bias_entries(w)) <= 0.15, mvs
    g.close()
