"""ctypes binding of libphoton.so -- argument marshalling only.

Every function has the name and argument order of its C declaration in
include/photon.h; tensors are torch tensors whose device pointers are passed
through.  Nothing is computed here, and there is no fallback: if the compiled
library is missing, load() raises.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libphoton.so")
_lib = None

OK, EINVAL, ENOMEM, EHIP, ENONFINITE, ENOTIMPL, ELIMIT = 0, -1, -2, -3, -4, -5, -6
FP32, BF16 = 0, 1
CLIENT_PARAMS, CLIENT_DELTAS = 0, 1
MAX_CLIENTS = 64
STATIC_MAX_CLIENTS = 16


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_ff", C.c_int32), ("vocab", C.c_int32), ("seq_len", C.c_int32),
                ("ln_eps", C.c_float), ("compute_dtype", C.c_int32), ("recompute", C.c_int32),
                ("micro_fuse", C.c_int32)]


class AdamWHP(C.Structure):
    _fields_ = [("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("weight_decay", C.c_float)]


class OptState(C.Structure):
    _fields_ = [("m", C.c_void_p), ("v", C.c_void_p), ("step", C.c_int64)]


class OuterOpt(C.Structure):
    _fields_ = [("eta_s", C.c_float), ("mu", C.c_float), ("nesterov", C.c_int32),
                ("momentum", C.c_void_p), ("round", C.c_int64)]


class AggMetrics(C.Structure):
    _fields_ = [("delta_norm2", C.c_double), ("client_norm2", C.c_double * MAX_CLIENTS)]


class Profile(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("gemm_ms", "gemm_flops", "attn_ms", "attn_flops", "adamw_ms",
                                          "adamw_bytes", "agg_ms", "agg_bytes", "delta_ms", "delta_bytes")] + \
               [(n, C.c_int64) for n in ("gemm_launches", "attn_launches", "adamw_launches", "agg_launches",
                                         "delta_launches", "gemm_launches_total", "attn_launches_total")]


class PhotonError(RuntimeError):
    def __init__(self, status: int, where: str, hip: int = 0):
        self.status = status
        self.hip = hip
        msg = _lib.photon_strerror(status).decode() if _lib is not None else str(status)
        super().__init__(f"{where}: {msg} (status {status}, hip error {hip})")


def load(path: str | None = None):
    """Loads the compiled library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: run `python __graft_entry__.py` (build()) first")
    lib = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.photon_param_count.restype = i64
    lib.photon_param_count.argtypes = [C.POINTER(ModelCfg)]
    lib.photon_create.restype = C.c_int
    lib.photon_create.argtypes = [C.POINTER(ModelCfg), i32, vp, C.POINTER(vp)]
    lib.photon_create_flat.restype = C.c_int
    lib.photon_create_flat.argtypes = [i64, vp, C.POINTER(vp)]
    lib.photon_destroy.restype = None
    lib.photon_destroy.argtypes = [vp]
    lib.photon_strerror.restype = C.c_char_p
    lib.photon_strerror.argtypes = [C.c_int]
    lib.photon_last_hip_error.restype = C.c_int
    lib.photon_last_hip_error.argtypes = [vp]
    lib.photon_workspace_bytes.restype = i64
    lib.photon_workspace_bytes.argtypes = [vp]
    lib.photon_client_local_steps.restype = C.c_int
    lib.photon_client_local_steps.argtypes = [vp, vp, C.POINTER(OptState), vp, i32, i32,
                                              C.POINTER(C.c_float), C.POINTER(AdamWHP), C.POINTER(C.c_float)]
    lib.photon_client_loss_grad.restype = C.c_int
    lib.photon_client_loss_grad.argtypes = [vp, vp, vp, vp, C.POINTER(C.c_float)]
    lib.photon_adamw_step.restype = C.c_int
    lib.photon_adamw_step.argtypes = [vp, vp, C.POINTER(OptState), vp, C.c_float, C.POINTER(AdamWHP), vp]
    lib.photon_export_delta.restype = C.c_int
    lib.photon_export_delta.argtypes = [vp, vp, vp, vp, i32]
    lib.photon_aggregate.restype = C.c_int
    lib.photon_aggregate.argtypes = [vp, vp, C.POINTER(vp), i32, i32, i32, C.POINTER(C.c_double),
                                     C.POINTER(OuterOpt), C.POINTER(AggMetrics)]
    lib.photon_aggregate_static.restype = C.c_int
    lib.photon_aggregate_static.argtypes = [vp, i64, vp, C.POINTER(vp), i32, i32, i32, C.POINTER(C.c_double),
                                            C.POINTER(OuterOpt), vp, C.POINTER(i32)]
    lib.photon_clip_delta.restype = C.c_int
    lib.photon_clip_delta.argtypes = [vp, vp, i32, C.c_double, C.POINTER(C.c_double)]
    lib.photon_client_init.restype = C.c_int
    lib.photon_client_init.argtypes = [vp, vp, vp, C.POINTER(OptState)]
    lib.photon_stream_probe.restype = C.c_int
    lib.photon_stream_probe.argtypes = [vp, i32, i32, vp, vp, i64, i32, C.POINTER(C.c_double)]
    lib.photon_profile_begin.restype = C.c_int
    lib.photon_profile_begin.argtypes = [vp]
    lib.photon_profile_begin_sampled.restype = C.c_int
    lib.photon_profile_begin_sampled.argtypes = [vp, C.c_int32]
    lib.photon_profile_end.restype = C.c_int
    lib.photon_profile_end.argtypes = [vp, C.POINTER(Profile)]
    _lib = lib
    return lib


def missing_symbols(names: Sequence[str], path: str | None = None) -> list[str]:
    lib = C.CDLL(path or LIB_PATH)
    return [n for n in names if not hasattr(lib, n)]


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _check(status: int, where: str, ctx=None, allow=()):
    if status != OK and status not in allow:
        hip = _lib.photon_last_hip_error(ctx) if ctx else 0
        raise PhotonError(status, where, hip)
    return status


def model_cfg(shape, dtype: str, recompute: int = 0, micro_fuse: int = 1) -> ModelCfg:
    return ModelCfg(shape.n_layers, shape.d_model, shape.n_heads, shape.d_ff, shape.vocab, shape.seq_len,
                    shape.ln_eps, BF16 if dtype == "bf16" else FP32, recompute, micro_fuse)


def photon_param_count(cfg: ModelCfg) -> int:
    return int(load().photon_param_count(C.byref(cfg)))


class Ctx:
    """Owner of a photon_ctx handle."""

    def __init__(self, handle: int):
        self.handle = C.c_void_p(handle)

    def close(self):
        if self.handle:
            _lib.photon_destroy(self.handle)
            self.handle = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def workspace_bytes(self) -> int:
        return int(_lib.photon_workspace_bytes(self.handle))


def photon_create(cfg: ModelCfg, micro_batch: int, stream: int = 0) -> Ctx:
    lib = load()
    h = C.c_void_p(0)
    _check(lib.photon_create(C.byref(cfg), micro_batch, C.c_void_p(stream), C.byref(h)), "photon_create")
    return Ctx(h.value)


def photon_create_flat(n: int, stream: int = 0) -> Ctx:
    lib = load()
    h = C.c_void_p(0)
    _check(lib.photon_create_flat(n, C.c_void_p(stream), C.byref(h)), "photon_create_flat")
    return Ctx(h.value)


def photon_client_local_steps(ctx: Ctx, params, opt_state: OptState, token_batches, n_steps: int, n_micro: int,
                              lr_schedule: Sequence[float], hp: AdamWHP, allow_nonfinite: bool = False):
    """Returns the per-step losses (list of float); params / opt_state are updated in place."""
    lrs = (C.c_float * n_steps)(*lr_schedule)
    losses = (C.c_float * max(1, n_steps))()
    rc = _lib.photon_client_local_steps(ctx.handle, _ptr(params), C.byref(opt_state), _ptr(token_batches),
                                        n_steps, n_micro, lrs, C.byref(hp), losses)
    _check(rc, "photon_client_local_steps", ctx.handle, allow=(ENONFINITE,) if allow_nonfinite else ())
    return [float(x) for x in losses[:n_steps]]


def photon_client_loss_grad(ctx: Ctx, params, tokens, grads_out) -> float:
    loss = C.c_float(0)
    _check(_lib.photon_client_loss_grad(ctx.handle, _ptr(params), _ptr(tokens), _ptr(grads_out), C.byref(loss)),
           "photon_client_loss_grad", ctx.handle)
    return float(loss.value)


def photon_adamw_step(ctx: Ctx, params, opt_state: OptState, grads, lr: float, hp: AdamWHP, bf16_out=None):
    _check(_lib.photon_adamw_step(ctx.handle, _ptr(params), C.byref(opt_state), _ptr(grads), lr, C.byref(hp),
                                  _ptr(bf16_out)), "photon_adamw_step", ctx.handle)


def photon_export_delta(ctx: Ctx, global_params, client_params, delta_out, dtype: int):
    _check(_lib.photon_export_delta(ctx.handle, _ptr(global_params), _ptr(client_params), _ptr(delta_out), dtype),
           "photon_export_delta", ctx.handle)


def photon_aggregate(ctx: Ctx, global_params, client_bufs, kind: int, dtype: int, client_weights: Sequence[float],
                     outer_opt: OuterOpt, want_metrics: bool = True):
    k = len(client_bufs)
    ptrs = (C.c_void_p * k)(*[_ptr(t) for t in client_bufs])
    w = (C.c_double * k)(*client_weights)
    met = AggMetrics() if want_metrics else None
    _check(_lib.photon_aggregate(ctx.handle, _ptr(global_params), ptrs, k, kind, dtype, w, C.byref(outer_opt),
                                 C.byref(met) if met is not None else None), "photon_aggregate", ctx.handle)
    if met is None:
        return None
    return {"delta_norm2": met.delta_norm2, "client_norm2": list(met.client_norm2[:k])}


def photon_aggregate_static(stream: int, n: int, global_params, client_bufs, kind: int, dtype: int,
                            client_weights: Sequence[float], outer_opt: OuterOpt, norms_out=None):
    """norms_out: device float64 tensor of K + 1 elements, or None.  Enqueues only."""
    lib = load()
    k = len(client_bufs)
    ptrs = (C.c_void_p * k)(*[_ptr(t) for t in client_bufs])
    w = (C.c_double * k)(*client_weights)
    hip = C.c_int32(0)
    rc = lib.photon_aggregate_static(C.c_void_p(stream), n, _ptr(global_params), ptrs, k, kind, dtype, w,
                                     C.byref(outer_opt), _ptr(norms_out), C.byref(hip))
    if rc != OK:
        raise PhotonError(rc, "photon_aggregate_static", int(hip.value))


def photon_clip_delta(ctx: Ctx, delta, dtype: int, max_norm: float, want_norm: bool = True):
    nrm = C.c_double(0)
    _check(_lib.photon_clip_delta(ctx.handle, _ptr(delta), dtype, max_norm, C.byref(nrm) if want_norm else None),
           "photon_clip_delta", ctx.handle)
    return float(nrm.value) if want_norm else None


def photon_client_init(ctx: Ctx, global_params, client_params, opt_state: OptState):
    _check(_lib.photon_client_init(ctx.handle, _ptr(global_params), _ptr(client_params), C.byref(opt_state)),
           "photon_client_init", ctx.handle)


def photon_stream_probe(ctx: Ctx, reads: int, writes: int, src, dst, n: int, repeats: int = 10) -> float:
    """Average milliseconds per launch of the plain streaming kernel with the given read : write mix."""
    ms = C.c_double(0)
    _check(_lib.photon_stream_probe(ctx.handle, reads, writes, _ptr(src), _ptr(dst), n, repeats, C.byref(ms)),
           "photon_stream_probe", ctx.handle)
    return float(ms.value)


def photon_profile_begin(ctx: Ctx):
    _check(_lib.photon_profile_begin(ctx.handle), "photon_profile_begin", ctx.handle)


def photon_profile_begin_sampled(ctx: Ctx, every: int):
    _check(_lib.photon_profile_begin_sampled(ctx.handle, every), "photon_profile_begin_sampled", ctx.handle)


def photon_profile_end(ctx: Ctx) -> dict:
    p = Profile()
    _check(_lib.photon_profile_end(ctx.handle, C.byref(p)), "photon_profile_end", ctx.handle)
    return {n: getattr(p, n) for n, _ in Profile._fields_}
