"""ctypes binding of libpipemare.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/pipemare.h) and does
nothing but convert arguments; all arithmetic of the training step runs in the HIP kernels.
`PipeMare` is a small convenience holder that lets PyTorch own the device arena and the stream.
There is no CPU fallback: if the shared library is missing, importing fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Sequence

import numpy as np

__all__ = [
    "lib", "PmError", "pm_layer_desc", "pm_lr_sched", "pm_opts",
    "pm_delays", "pm_slots", "pm_t1_lr", "pm_query_bytes", "pm_create", "pm_step", "pm_weights",
    "pm_state", "pm_device_step_table", "pm_stats", "pm_chained_units", "pm_update_split", "pm_recompute_delays", "pm_device_recompute_slots", "pm_delay_thresholds", "pm_stochastic_delays", "pm_set_grads", "pm_apply_update", "pm_destroy",
    "pm_linear_fwd", "pm_linear_bwd_data", "pm_linear_bwd_weight", "pm_profile_begin", "pm_profile_end", "pm_profile_classes", "pm_profile_begin_classes",
    "pm_synchronize", "pm_checkpoint_bytes", "pm_checkpoint_save", "pm_checkpoint_load", "PipeMare", "pm_layernorm_fwd", "pm_layernorm_bwd", "pm_attention_fwd", "pm_attention_bwd",
    "pm_conv3x3_fwd", "pm_conv3x3_bwd_data", "pm_conv3x3_bwd_weight", "pm_conv3x3_bwd_weight_scratch",
    "pm_conv3x3_bwd_weight_static", "pm_static_scratch_bytes",
    "PM_LINEAR", "PM_KIND", "PM_ARCH", "PM_ACT", "PM_METHOD", "PM_LR", "PM_OPT", "PM_DTYPE", "PM_LOSS", "EXPORTS",
]

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpipemare.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python paper_1910_05124_amd/build.py` "
                      "(there is no fallback implementation)")
# The arena and the streams handed to the library belong to PyTorch, so both must talk to ONE HIP
# runtime.  PyTorch ships its own copy of libamdhip64 and loads it by path; loading it first makes
# the library's dependency of the same soname resolve to that copy instead of a second runtime
# (whose calls on PyTorch's pointers fail with "no ROCm-capable device").
import torch  # noqa: E402,F401

lib = C.CDLL(_LIB_PATH)

PM_LINEAR = 0
PM_KIND = {"linear": 0, "embed": 1, "layernorm": 2, "conv3x3": 3}
PM_ARCH = {"chain": 0, "transformer": 1, "resnet": 2}
PM_ACT = {"none": 0, "relu": 1, "gelu": 2}
PM_METHOD = {"pipemare": 0, "pipedream": 1, "gpipe": 2}
PM_LR = {"const": 0, "step": 1, "warmup_invsqrt": 2}
PM_OPT = {"sgdm": 0, "adamw": 1}
PM_DTYPE = {"f32": 0, "bf16": 1}
PM_LOSS = {"mse": 0, "xent": 1}
PM_UPDATE_PLACEMENT = {"auto": 0, "pass": 1, "launch": 2}
_STATUS = {0: "PM_OK", 1: "PM_EINVAL", 2: "PM_ENOMEM", 3: "PM_EHIP", 4: "PM_ESTATE", 5: "PM_EDIVERGED"}

EXPORTS = ["pm_status_str", "pm_last_error", "pm_delays", "pm_slots", "pm_t1_lr", "pm_query_bytes",
           "pm_create", "pm_step", "pm_weights", "pm_state", "pm_device_step_table", "pm_stats", "pm_chained_units", "pm_update_split",
           "pm_recompute_delays", "pm_device_recompute_slots", "pm_delay_thresholds", "pm_stochastic_delays",
           "pm_set_grads", "pm_apply_update", "pm_profile_begin", "pm_profile_end", "pm_profile_classes", "pm_profile_begin_classes", "pm_linear_fwd", "pm_linear_bwd_data",
           "pm_linear_bwd_weight", "pm_layernorm_fwd", "pm_layernorm_bwd", "pm_attention_fwd", "pm_attention_bwd",
           "pm_conv3x3_fwd", "pm_conv3x3_bwd_data", "pm_conv3x3_bwd_weight", "pm_conv3x3_bwd_weight_scratch",
           "pm_conv3x3_bwd_weight_static", "pm_static_scratch_bytes",
           "pm_checkpoint_bytes", "pm_checkpoint_save", "pm_checkpoint_load", "pm_synchronize", "pm_destroy"]


class pm_layer_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_in", C.c_int32), ("n_out", C.c_int32), ("act", C.c_int32),
                ("stage", C.c_int32)]


class pm_lr_sched(C.Structure):
    _fields_ = [("kind", C.c_int32), ("base", C.c_double), ("init", C.c_double), ("factor", C.c_double),
                ("interval", C.c_int64), ("K", C.c_int64)]


class pm_opts(C.Structure):
    _fields_ = [("opt", C.c_int32), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("weight_decay", C.c_double), ("clip_norm", C.c_double), ("D", C.c_double),
                ("gamma_override", C.POINTER(C.c_double)), ("t1_enabled", C.c_int32),
                ("t2_enabled", C.c_int32), ("n_microbatches", C.c_int32), ("dtype", C.c_int32),
                ("loss", C.c_int32), ("microbatch", C.c_int32), ("use_graph", C.c_int32),
                ("sync_warmup_steps", C.c_int64), ("overlap_update", C.c_int32), ("arch", C.c_int32),
                ("n_heads", C.c_int32), ("seq_len", C.c_int32), ("image_size", C.c_int32),
                ("tau_recomp", C.POINTER(C.c_int32)), ("segment_size", C.c_int32),
                ("stochastic_delays", C.c_int32), ("tau_max", C.c_int32), ("delay_seed", C.c_uint64),
                ("chained_launches", C.c_int32), ("update_placement", C.c_int32)]


class PmError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        self.name = _STATUS.get(status, f"PM_{status}")
        super().__init__(f"{self.name}: {lib.pm_last_error().decode()}")


lib.pm_status_str.restype = C.c_char_p
lib.pm_checkpoint_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
lib.pm_checkpoint_save.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
lib.pm_checkpoint_load.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
lib.pm_status_str.argtypes = [C.c_int]
lib.pm_last_error.restype = C.c_char_p
lib.pm_last_error.argtypes = []
_vp, _i32, _i64, _f32p, _i32p = C.c_void_p, C.c_int32, C.c_int64, C.POINTER(C.c_float), C.POINTER(C.c_int32)
lib.pm_delays.argtypes = [_i32, _i32, _i32, _i32p, _i32p]
lib.pm_slots.argtypes = [_i32, _i32, _i64, _i32p, _i32p, _i32p]
lib.pm_t1_lr.argtypes = [C.POINTER(pm_lr_sched), _i32, _i64, _i32, C.POINTER(C.c_double)]
lib.pm_query_bytes.argtypes = [_i32, _i32, C.POINTER(pm_layer_desc), _i32p, C.POINTER(pm_opts), C.POINTER(C.c_size_t)]
lib.pm_create.argtypes = [_i32, _i32, C.POINTER(pm_layer_desc), _i32p, _i32p, C.POINTER(pm_lr_sched),
                          C.POINTER(pm_opts), C.POINTER(_f32p), _vp, C.c_size_t, _vp, C.POINTER(_vp)]
lib.pm_step.argtypes = [_vp, _vp, _vp, _f32p]
lib.pm_weights.argtypes = [_vp, _i32, _f32p, C.c_size_t]
lib.pm_state.argtypes = [_vp, _i32, _i32, _f32p, C.c_size_t]
lib.pm_device_step_table.argtypes = [_vp, C.POINTER(_i64), _i32p, _i32p, _i32p, _f32p]
lib.pm_recompute_delays.argtypes = [_i32, _i32, _i32, _i32p, _i32p]
lib.pm_delay_thresholds.argtypes = [C.c_double, _i32, C.POINTER(C.c_uint32)]
lib.pm_stochastic_delays.argtypes = [_i32, _i32p, _i32, C.c_uint64, _i64, _i32p]
lib.pm_device_recompute_slots.argtypes = [_vp, C.POINTER(_i64), _i32p]
lib.pm_chained_units.argtypes = [_vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
lib.pm_update_split.argtypes = [_vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
lib.pm_stats.argtypes = [_vp, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(_i64)]
lib.pm_set_grads.argtypes = [_vp, _i32, _f32p, C.c_size_t]
lib.pm_apply_update.argtypes = [_vp]
lib.pm_profile_begin.argtypes = [_vp, _i32]
lib.pm_profile_end.argtypes = [_vp, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), _i32p]
lib.pm_profile_begin_classes.argtypes = [_vp, _i32]
lib.pm_profile_classes.argtypes = [_vp, C.POINTER(C.c_double), C.POINTER(C.c_double), _i32p]
lib.pm_linear_fwd.argtypes = [_vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _i32, _vp, _vp]
lib.pm_linear_bwd_data.argtypes = [_vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _i32, _vp]
lib.pm_linear_bwd_weight.argtypes = [_vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _i32]
lib.pm_layernorm_fwd.argtypes = [_vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp]
lib.pm_layernorm_bwd.argtypes = [_vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.pm_attention_fwd.argtypes = [_vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp]
lib.pm_attention_bwd.argtypes = [_vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.pm_conv3x3_fwd.argtypes = [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp]
lib.pm_conv3x3_bwd_data.argtypes = [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp]
lib.pm_conv3x3_bwd_weight.argtypes = [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, C.c_size_t]
lib.pm_conv3x3_bwd_weight_scratch.argtypes = [_i32, _i32, _i32, _i32, _i32, _i32, _i32, C.POINTER(C.c_size_t)]
lib.pm_conv3x3_bwd_weight_static.argtypes = [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp]
lib.pm_static_scratch_bytes.argtypes = [C.POINTER(C.c_size_t)]
lib.pm_synchronize.argtypes = [_vp]
lib.pm_destroy.argtypes = [_vp]
lib.pm_destroy.restype = None
for _n in EXPORTS:
    if _n not in ("pm_status_str", "pm_last_error", "pm_destroy"):
        getattr(lib, _n).restype = C.c_int


def _check(status: int):
    if status != 0:
        raise PmError(status)


def _i32arr(v: Sequence[int]):
    return (C.c_int32 * len(v))(*[int(x) for x in v])


def _f32ptr(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_f32p)


def pm_delays(P: int, N: int = 1, method: str = "pipemare"):
    tf, tb = (C.c_int32 * max(P, 1))(), (C.c_int32 * max(P, 1))()
    _check(lib.pm_delays(P, N, PM_METHOD[method], tf, tb))
    return list(tf), list(tb)


def pm_recompute_delays(P: int, S: int, N: int = 1, tau_bkwd=None):
    tr = (C.c_int32 * max(P, 1))()
    tb = None if tau_bkwd is None else (C.c_int32 * len(tau_bkwd))(*[int(t) for t in tau_bkwd])
    _check(lib.pm_recompute_delays(P, S, N, tb, tr))
    return list(tr)


def pm_delay_thresholds(mean: float, tau_max: int):
    T = (C.c_uint32 * max(tau_max, 1))()
    _check(lib.pm_delay_thresholds(float(mean), tau_max, T))
    return list(T)[:tau_max]


def pm_stochastic_delays(P: int, mean_tau, tau_max: int, seed: int, t: int):
    out = (C.c_int32 * max(P, 1))()
    _check(lib.pm_stochastic_delays(P, _i32arr(mean_tau), tau_max, seed, t, out))
    return list(out)


def pm_slots(tau_fwd: int, tau_bkwd: int, t: int):
    f, b, w = C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib.pm_slots(tau_fwd, tau_bkwd, t, C.byref(f), C.byref(b), C.byref(w)))
    return f.value, b.value, w.value


def pm_t1_lr(sched: pm_lr_sched, tau: int, k: int, t1_enabled: bool = True) -> float:
    out = C.c_double()
    _check(lib.pm_t1_lr(C.byref(sched), tau, k, int(t1_enabled), C.byref(out)))
    return out.value


def _layer_array(layers):
    arr = (pm_layer_desc * len(layers))()
    for i, L in enumerate(layers):
        arr[i] = pm_layer_desc(PM_KIND[getattr(L, "kind", "linear")], L.n_in, L.n_out, PM_ACT[L.act], L.stage)
    return arr


def pm_query_bytes(P: int, layers, tau_fwd, opts: pm_opts) -> int:
    out = C.c_size_t()
    _check(lib.pm_query_bytes(P, len(layers), _layer_array(layers), _i32arr(tau_fwd), C.byref(opts), C.byref(out)))
    return out.value


def pm_create(P, layers, tau_fwd, tau_bkwd, sched: pm_lr_sched, opts: pm_opts, init_weights: List[np.ndarray],
              arena_ptr: int, arena_bytes: int, stream: int) -> int:
    ws = [np.ascontiguousarray(w, dtype=np.float32) for w in init_weights]
    ptrs = (_f32p * len(ws))(*[_f32ptr(w) for w in ws])
    ctx = _vp()
    _check(lib.pm_create(P, len(layers), _layer_array(layers), _i32arr(tau_fwd), _i32arr(tau_bkwd),
                         C.byref(sched), C.byref(opts), ptrs, _vp(arena_ptr), arena_bytes, _vp(stream), C.byref(ctx)))
    return ctx.value


def pm_step(ctx: int, x_ptr: int, y_ptr: int, want_loss: bool = False):
    if want_loss:
        out = C.c_float()
        _check(lib.pm_step(ctx, x_ptr, y_ptr, C.byref(out)))
        return out.value
    _check(lib.pm_step(ctx, x_ptr, y_ptr, None))
    return None


def pm_weights(ctx: int, layer: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.float32)
    _check(lib.pm_weights(ctx, layer, _f32ptr(out), n))
    return out


def pm_state(ctx: int, which: int, layer: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.float32)
    _check(lib.pm_state(ctx, which, layer, _f32ptr(out), n))
    return out


def pm_device_step_table(ctx: int, L: int):
    t = _i64()
    f, b, w = (C.c_int32 * L)(), (C.c_int32 * L)(), (C.c_int32 * L)()
    lr = (C.c_float * L)()
    _check(lib.pm_device_step_table(ctx, C.byref(t), f, b, w, lr))
    return t.value, list(f), list(b), list(w), np.array(lr[:], dtype=np.float32)


def pm_device_recompute_slots(ctx: int, L: int):
    t = _i64()
    r = (C.c_int32 * L)()
    _check(lib.pm_device_recompute_slots(ctx, C.byref(t), r))
    return t.value, list(r)


def pm_checkpoint_bytes(ctx: int) -> int:
    n = C.c_size_t()
    _check(lib.pm_checkpoint_bytes(ctx, C.byref(n)))
    return n.value


def pm_checkpoint_save(ctx: int) -> np.ndarray:
    """The context's training state as one byte image (host)."""
    buf = np.empty(pm_checkpoint_bytes(ctx), dtype=np.uint8)
    _check(lib.pm_checkpoint_save(ctx, buf.ctypes.data_as(C.c_void_p), buf.size))
    return buf


def pm_checkpoint_load(ctx: int, image: np.ndarray):
    image = np.ascontiguousarray(image, dtype=np.uint8)
    _check(lib.pm_checkpoint_load(ctx, image.ctypes.data_as(C.c_void_p), image.size))


def pm_chained_units(ctx: int):
    nf, nb = C.c_int32(0), C.c_int32(0)
    _check(lib.pm_chained_units(ctx, C.byref(nf), C.byref(nb)))
    return nf.value, nb.value


def pm_update_split(ctx: int):
    ne, npass = _i64(), _i64()
    _check(lib.pm_update_split(ctx, C.byref(ne), C.byref(npass)))
    return ne.value, npass.value


def pm_stats(ctx: int, param_norm: bool = False):
    loss, gn, pn, t = C.c_double(), C.c_double(), C.c_double(), _i64()
    _check(lib.pm_stats(ctx, C.byref(loss), C.byref(gn), C.byref(pn) if param_norm else None, C.byref(t)))
    return dict(loss=loss.value, grad_norm=gn.value, param_norm=pn.value if param_norm else None, t=t.value)


def pm_set_grads(ctx: int, layer: int, g: np.ndarray):
    g = np.ascontiguousarray(g, dtype=np.float32)
    _check(lib.pm_set_grads(ctx, layer, _f32ptr(g), g.size))


def pm_apply_update(ctx: int):
    _check(lib.pm_apply_update(ctx))


def pm_profile_begin(ctx: int, max_steps: int):
    _check(lib.pm_profile_begin(ctx, max_steps))


def pm_profile_end(ctx: int):
    f, b, u, n = C.c_double(), C.c_double(), C.c_double(), C.c_int32()
    _check(lib.pm_profile_end(ctx, C.byref(f), C.byref(b), C.byref(u), C.byref(n)))
    return dict(fwd_ms=f.value, bwd_ms=b.value, update_ms=u.value, n=n.value)


def pm_profile_begin_classes(ctx: int, max_steps: int):
    _check(lib.pm_profile_begin_classes(ctx, max_steps))


def pm_profile_classes(ctx: int):
    g, a, n = C.c_double(), C.c_double(), C.c_int32()
    _check(lib.pm_profile_classes(ctx, C.byref(g), C.byref(a), C.byref(n)))
    return dict(product_ms=g.value, attention_ms=a.value, n=n.value)


def pm_synchronize(ctx: int):
    _check(lib.pm_synchronize(ctx))


def pm_destroy(ctx: int):
    lib.pm_destroy(ctx)


def pm_linear_fwd(stream, dtype, M, n_in, n_out, x, W, b, act, z, a):
    _check(lib.pm_linear_fwd(_vp(stream), PM_DTYPE[dtype], M, n_in, n_out, x, W, b, PM_ACT[act], z, a))


def pm_linear_bwd_data(stream, dtype, M, n_in, n_out, dz, W, zprev, act_prev, dzprev):
    _check(lib.pm_linear_bwd_data(_vp(stream), PM_DTYPE[dtype], M, n_in, n_out, dz, W, zprev, PM_ACT[act_prev], dzprev))


def pm_linear_bwd_weight(stream, dtype, M, n_in, n_out, dz, a, dW, db, accumulate=False):
    _check(lib.pm_linear_bwd_weight(_vp(stream), PM_DTYPE[dtype], M, n_in, n_out, dz, a, dW, db, int(accumulate)))


def pm_layernorm_fwd(stream, dtype, rows, d, x, gain, bias, y, mean, rstd):
    _check(lib.pm_layernorm_fwd(_vp(stream), PM_DTYPE[dtype], rows, d, x, gain, bias, y, mean, rstd))


def pm_layernorm_bwd(stream, dtype, rows, d, dy, x, mean, rstd, gain_bkwd, dx_res, dx, dx_t, dgain, dbias):
    _check(lib.pm_layernorm_bwd(_vp(stream), PM_DTYPE[dtype], rows, d, dy, x, mean, rstd, gain_bkwd, dx_res, dx, dx_t,
                                dgain, dbias))


def pm_attention_fwd(stream, dtype, B, S, H, dh, q, k, v, o, lse):
    _check(lib.pm_attention_fwd(_vp(stream), PM_DTYPE[dtype], B, S, H, dh, q, k, v, o, lse))


def pm_attention_bwd(stream, dtype, B, S, H, dh, q, k, v, o, do, lse, dq, dk, dv):
    _check(lib.pm_attention_bwd(_vp(stream), PM_DTYPE[dtype], B, S, H, dh, q, k, v, o, do, lse, dq, dk, dv))


def pm_conv3x3_fwd(stream, dtype, B, H, W, C_in, C_out, stride, x, params, z, y):
    _check(lib.pm_conv3x3_fwd(_vp(stream), PM_DTYPE[dtype], B, H, W, C_in, C_out, stride, x, params, z, y))


def pm_conv3x3_bwd_data(stream, dtype, B, H, W, C_in, C_out, stride, dz, params, dx):
    _check(lib.pm_conv3x3_bwd_data(_vp(stream), PM_DTYPE[dtype], B, H, W, C_in, C_out, stride, dz, params, dx))


def pm_conv3x3_bwd_weight_scratch(dtype, B, H, W, C_in, C_out, stride) -> int:
    out = C.c_size_t()
    _check(lib.pm_conv3x3_bwd_weight_scratch(PM_DTYPE[dtype], B, H, W, C_in, C_out, stride, C.byref(out)))
    return out.value


def pm_conv3x3_bwd_weight(stream, dtype, B, H, W, C_in, C_out, stride, dz, x, dW, scratch=None, scratch_bytes=0):
    _check(lib.pm_conv3x3_bwd_weight(_vp(stream), PM_DTYPE[dtype], B, H, W, C_in, C_out, stride, dz, x, dW, scratch,
                                     scratch_bytes))


def pm_static_scratch_bytes() -> int:
    out = C.c_size_t()
    _check(lib.pm_static_scratch_bytes(C.byref(out)))
    return out.value


def pm_conv3x3_bwd_weight_static(stream, dtype, B, H, W, C_in, C_out, stride, dz, x, dW):
    _check(lib.pm_conv3x3_bwd_weight_static(_vp(stream), PM_DTYPE[dtype], B, H, W, C_in, C_out, stride, dz, x, dW))


def make_sched(kind="const", base=0.01, init=0.0, factor=1.0, interval=1, K=0) -> pm_lr_sched:
    return pm_lr_sched(PM_LR[kind], base, init, factor, interval, K)


def make_opts(opt="sgdm", beta1=0.9, beta2=0.98, eps=1e-8, weight_decay=0.0, clip_norm=0.0, D=1.0,
              gamma_override=None, t1=True, t2=True, N=1, dtype="f32", loss="mse", microbatch=1,
              use_graph=False, sync_warmup=0, overlap_update=False, arch="chain", n_heads=0, seq_len=0,
              image_size=0, tau_recomp=None, segment_size=0, stochastic=None, chained_launches=False,
              update_placement="auto") -> pm_opts:
    o = pm_opts(PM_OPT[opt], beta1, beta2, eps, weight_decay, clip_norm, D, None, int(t1), int(t2), N,
                PM_DTYPE[dtype], PM_LOSS[loss], microbatch, int(use_graph), int(sync_warmup), int(overlap_update),
                PM_ARCH[arch], int(n_heads), int(seq_len), int(image_size), None, int(segment_size),
                0 if stochastic is None else 1, 0 if stochastic is None else int(stochastic["tau_max"]),
                0 if stochastic is None else int(stochastic["seed"]), int(chained_launches), PM_UPDATE_PLACEMENT[update_placement])
    if tau_recomp is not None:
        arr_r = (C.c_int32 * len(tau_recomp))(*[int(t) for t in tau_recomp])
        o._keep_r = arr_r
        o.tau_recomp = C.cast(arr_r, C.POINTER(C.c_int32))
    if gamma_override is not None:
        arr = (C.c_double * len(gamma_override))(*gamma_override)
        o._keep = arr
        o.gamma_override = C.cast(arr, C.POINTER(C.c_double))
    return o


def _unit_size(L) -> int:
    kind = getattr(L, "kind", "linear")
    if kind == "embed":
        return L.n_in * L.n_out
    if kind == "layernorm":
        return 2 * L.n_out
    if kind == "conv3x3":
        return L.n_out * 9 * L.n_in + 2 * L.n_out
    return L.n_out * L.n_in + L.n_out


class PipeMare:
    """Holds a pm_ctx plus the torch-owned arena and stream it runs on (marshalling only)."""

    def __init__(self, layers, P, tau_fwd, tau_bkwd, sched: pm_lr_sched, opts: pm_opts,
                 init_weights: List[np.ndarray], device="cuda:0", stream=None):
        import torch
        self.torch = torch
        self.layers = list(layers)
        self.L = len(self.layers)
        self.sizes = [_unit_size(L) for L in self.layers]
        self.device = torch.device(device)
        nbytes = pm_query_bytes(P, self.layers, tau_fwd, opts)
        with torch.cuda.device(self.device):
            self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
            with torch.cuda.stream(self.stream):
                self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
            ptr = (self.arena.data_ptr() + 255) // 256 * 256
            self.ctx = pm_create(P, self.layers, tau_fwd, tau_bkwd, sched, opts, init_weights, ptr, nbytes,
                                 self.stream.cuda_stream)
        self.arena_bytes = nbytes

    def step(self, x, y, want_loss=False):
        """Chain: x cuda fp32 [M, n_in]; y cuda fp32 [M, n_out] or int32 [M].  Transformer: x, y cuda int32 [M, S].
        ResNet: x cuda fp32 [M, 3, H, H], y cuda int32 [M]."""
        return pm_step(self.ctx, x.data_ptr(), y.data_ptr(), want_loss)

    def weights(self, layer=None):
        if layer is None:
            return [pm_weights(self.ctx, l, self.sizes[l]) for l in range(self.L)]
        return pm_weights(self.ctx, layer, self.sizes[layer])

    def state(self, which, layer):
        return pm_state(self.ctx, which, layer, self.sizes[layer])

    def set_grads(self, grads):
        for l, g in enumerate(grads):
            pm_set_grads(self.ctx, l, g)

    def apply_update(self):
        pm_apply_update(self.ctx)

    def step_table(self):
        return pm_device_step_table(self.ctx, self.L)

    def synchronize(self):
        pm_synchronize(self.ctx)

    def checkpoint(self) -> np.ndarray:
        return pm_checkpoint_save(self.ctx)

    def restore(self, image: np.ndarray):
        pm_checkpoint_load(self.ctx, image)

    def stats(self, param_norm=False):
        return pm_stats(self.ctx, param_norm)

    def chained_units(self):
        return pm_chained_units(self.ctx)

    def update_split(self):
        return pm_update_split(self.ctx)

    def close(self):
        if self.ctx:
            pm_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


__all__ += ["make_sched", "make_opts"]
