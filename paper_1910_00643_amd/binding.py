"""ctypes binding of libslowmo.so: the same entry points as include/slowmo.h,
argument marshalling only.  No arithmetic on tensor elements happens here.

The library must have been built (python -m paper_1910_00643_amd.build or
__graft_entry__.build()); loading fails loudly otherwise -- there is no
fallback implementation.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
# SLOWMO_LIBRARY selects another build of the same library (tuning runs).
LIB_PATH = os.environ.get("SLOWMO_LIBRARY") or os.path.join(_HERE, "libslowmo.so")

SLOWMO_OK, SLOWMO_ERR_ARG, SLOWMO_ERR_STATE = 0, -1, -2
SLOWMO_ERR_ALIGN, SLOWMO_ERR_HIP, SLOWMO_ERR_NOMEM = -3, -4, -5
SLOWMO_SGD_NESTEROV, SLOWMO_ADAM = 0, 1
SLOWMO_BUF_RESET, SLOWMO_BUF_MAINTAIN, SLOWMO_BUF_AVERAGE = 0, 1, 2
SLOWMO_F32, SLOWMO_BF16 = 0, 1
SLOWMO_BUF_X0, SLOWMO_BUF_U, SLOWMO_BUF_H, SLOWMO_BUF_V = 0, 1, 2, 3
SLOWMO_MAX_WORKERS = 1024
SLOWMO_STATIC_MAX_POINTERS = 65536

STATUS_NAMES = {0: "SLOWMO_OK", -1: "SLOWMO_ERR_ARG", -2: "SLOWMO_ERR_STATE",
                -3: "SLOWMO_ERR_ALIGN", -4: "SLOWMO_ERR_HIP", -5: "SLOWMO_ERR_NOMEM"}

# every symbol include/slowmo.h declares
EXPORTS = ["slowmo_state_bytes", "slowmo_create", "slowmo_local_step", "slowmo_outer_step",
           "slowmo_destroy", "slowmo_last_error", "slowmo_get_buffer", "slowmo_get_counters",
           "slowmo_plan_local", "slowmo_plan_outer", "slowmo_version", "slowmo_mix_step",
           "slowmo_expgraph_in_peers", "slowmo_set_tensor_hparams", "slowmo_export_bytes",
           "slowmo_export_state", "slowmo_import_state", "slowmo_local_outer_step",
           "slowmo_get_pushsum_weights", "slowmo_debias", "slowmo_plan_mix",
           "slowmo_local_mix_step", "slowmo_check_device_range", "slowmo_debias_static",
           "slowmo_lr_step_decay", "slowmo_lr_inverse_sqrt"]


(SLOWMO_MIX_OWN_HELD, SLOWMO_MIX_SOURCE_HELD, SLOWMO_MIX_SOURCE_IS_FIRST, SLOWMO_MIX_OPENS_CYCLE,
 SLOWMO_MIX_NO_SOURCE, SLOWMO_MIX_GROUP_START) = 1, 2, 4, 8, 16, 32
SLOWMO_MIX_SAVED_REGISTERS = 4


def SLOWMO_MIX_SAVE(flags: int) -> int:
    return (flags >> 6) & 7


def SLOWMO_MIX_OWN_SAVED(flags: int) -> int:
    return (flags >> 9) & 7


def SLOWMO_MIX_SOURCE_SAVED(flags: int) -> int:
    return (flags >> 12) & 7


class slowmo_mix_entry(C.Structure):
    _fields_ = [("worker", C.c_int32), ("source", C.c_int32), ("keep", C.c_float),
                ("take", C.c_float), ("flags", C.c_int32), ("reserved", C.c_int32)]


class slowmo_config(C.Structure):
    _fields_ = [("m", C.c_int32), ("tau", C.c_int32), ("alpha", C.c_float), ("beta", C.c_float),
                ("base", C.c_int32), ("policy", C.c_int32), ("grad_dtype", C.c_int32),
                ("momentum", C.c_float), ("weight_decay", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("no_average", C.c_int32)]


class slowmo_plan_run(C.Structure):
    _fields_ = [("tile", C.c_int32), ("worker", C.c_int32), ("tensor", C.c_int32),
                ("n", C.c_int32), ("offset", C.c_int64)]


class SlowMoError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status
        self.message = message


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -m paper_1910_00643_amd.build` (needs hipcc); "
                          "there is no fallback path")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    cfgp = C.POINTER(slowmo_config)
    L.slowmo_state_bytes.argtypes = [cfgp, i32, C.POINTER(i64)]
    L.slowmo_state_bytes.restype = C.c_size_t
    L.slowmo_create.argtypes = [C.POINTER(vp), cfgp, i32, C.POINTER(i64), C.POINTER(vp), vp,
                                C.c_size_t, vp]
    L.slowmo_create.restype = C.c_int
    L.slowmo_local_step.argtypes = [vp, C.POINTER(vp), C.c_float, vp]
    L.slowmo_local_step.restype = C.c_int
    L.slowmo_local_outer_step.argtypes = [vp, C.POINTER(vp), C.c_float, C.c_float, vp]
    L.slowmo_local_outer_step.restype = C.c_int
    L.slowmo_outer_step.argtypes = [vp, C.c_float, vp]
    L.slowmo_outer_step.restype = C.c_int
    L.slowmo_destroy.argtypes = [vp]
    L.slowmo_destroy.restype = C.c_int
    L.slowmo_last_error.argtypes = [vp]
    L.slowmo_last_error.restype = C.c_char_p
    L.slowmo_get_buffer.argtypes = [vp, i32, i32, i32, C.POINTER(vp)]
    L.slowmo_get_buffer.restype = C.c_int
    L.slowmo_get_counters.argtypes = [vp, C.POINTER(i64), C.POINTER(i32), C.POINTER(i64)]
    L.slowmo_get_counters.restype = C.c_int
    L.slowmo_plan_local.argtypes = [i32, i32, C.POINTER(i64), C.POINTER(slowmo_plan_run), i64]
    L.slowmo_plan_local.restype = i64
    L.slowmo_plan_outer.argtypes = [i32, i32, C.POINTER(i64), C.POINTER(slowmo_plan_run), i64]
    L.slowmo_plan_outer.restype = i64
    L.slowmo_mix_step.argtypes = [vp, C.POINTER(i32), vp]
    L.slowmo_mix_step.restype = C.c_int
    L.slowmo_local_mix_step.argtypes = [vp, C.POINTER(vp), C.c_float, C.POINTER(i32), vp]
    L.slowmo_local_mix_step.restype = C.c_int
    L.slowmo_check_device_range.argtypes = [vp, C.c_size_t]
    L.slowmo_check_device_range.restype = C.c_int
    L.slowmo_plan_mix.argtypes = [i32, C.POINTER(i32), C.POINTER(slowmo_mix_entry)]
    L.slowmo_plan_mix.restype = C.c_int32
    L.slowmo_get_pushsum_weights.argtypes = [vp, C.POINTER(C.c_float)]
    L.slowmo_get_pushsum_weights.restype = C.c_int
    L.slowmo_debias.argtypes = [vp, C.POINTER(vp), vp]
    L.slowmo_debias.restype = C.c_int
    L.slowmo_debias_static.argtypes = [vp, C.POINTER(vp), vp]
    L.slowmo_debias_static.restype = C.c_int
    L.slowmo_lr_step_decay.argtypes = [C.c_float, C.c_float, i64, C.POINTER(i64), i32, C.c_float, i64,
                                       C.POINTER(C.c_float)]
    L.slowmo_lr_step_decay.restype = C.c_int
    L.slowmo_lr_inverse_sqrt.argtypes = [C.c_float, C.c_float, i64, i64, C.POINTER(C.c_float)]
    L.slowmo_lr_inverse_sqrt.restype = C.c_int
    L.slowmo_expgraph_in_peers.argtypes = [i32, i64, C.POINTER(i32)]
    L.slowmo_expgraph_in_peers.restype = C.c_int
    L.slowmo_set_tensor_hparams.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_float), vp]
    L.slowmo_set_tensor_hparams.restype = C.c_int
    L.slowmo_export_bytes.argtypes = [vp]
    L.slowmo_export_bytes.restype = C.c_size_t
    L.slowmo_export_state.argtypes = [vp, vp, C.c_size_t, vp]
    L.slowmo_export_state.restype = C.c_int
    L.slowmo_import_state.argtypes = [vp, vp, C.c_size_t, vp]
    L.slowmo_import_state.restype = C.c_int
    L.slowmo_version.argtypes = []
    L.slowmo_version.restype = C.c_char_p
    _lib = L
    return L


def _i64_array(values: Sequence[int]):
    return (C.c_int64 * len(values))(*[int(v) for v in values])


def _ptr_array(values: Optional[Sequence[int]]):
    if values is None:
        return None
    return (C.c_void_p * len(values))(*[C.c_void_p(int(v)) if v else None for v in values])


def _check(status: int, ctx) -> None:
    if status != SLOWMO_OK:
        raise SlowMoError(status, slowmo_last_error(ctx))


def slowmo_version() -> str:
    return lib().slowmo_version().decode()


def slowmo_last_error(ctx=None) -> str:
    return lib().slowmo_last_error(ctx).decode()


def slowmo_state_bytes(cfg: slowmo_config, numel: Sequence[int]) -> int:
    """Bytes of device workspace; 0 if the arguments are invalid."""
    arr = _i64_array(numel) if numel is not None else None
    return int(lib().slowmo_state_bytes(C.byref(cfg) if cfg is not None else None,
                                        len(numel) if numel is not None else 0, arr))


def slowmo_create(cfg: slowmo_config, numel: Sequence[int], params: Sequence[int],
                  state: int, state_bytes: int, stream: int = 0) -> C.c_void_p:
    """params: m * n_tensors device addresses (worker-major); state: device
    address of the workspace.  Returns the context handle."""
    ctx = C.c_void_p()
    st = lib().slowmo_create(C.byref(ctx), C.byref(cfg) if cfg is not None else None,
                             len(numel) if numel is not None else 0,
                             _i64_array(numel) if numel is not None else None,
                             _ptr_array(params), C.c_void_p(state) if state else None,
                             state_bytes, C.c_void_p(stream) if stream else None)
    _check(st, None)
    return ctx


def slowmo_local_step(ctx, grads, lr: float, stream: int = 0) -> None:
    """grads: m * n_tensors device addresses, or a prepared ctypes array."""
    arr = grads if (grads is None or isinstance(grads, C.Array)) else _ptr_array(grads)
    _check(lib().slowmo_local_step(ctx, arr, lr, C.c_void_p(stream) if stream else None), ctx)


def slowmo_local_outer_step(ctx, grads, lr: float, outer_lr: float, stream: int = 0) -> None:
    """The last local step of an outer iteration and the outer step in one call."""
    arr = grads if (grads is None or isinstance(grads, C.Array)) else _ptr_array(grads)
    _check(lib().slowmo_local_outer_step(ctx, arr, lr, outer_lr,
                                         C.c_void_p(stream) if stream else None), ctx)


def slowmo_outer_step(ctx, lr: float, stream: int = 0) -> None:
    _check(lib().slowmo_outer_step(ctx, lr, C.c_void_p(stream) if stream else None), ctx)


def slowmo_mix_step(ctx, in_peer: Sequence[int], stream: int = 0) -> None:
    """in_peer: m worker indices; worker i receives from in_peer[i]."""
    arr = (C.c_int32 * len(in_peer))(*[int(v) for v in in_peer]) if in_peer is not None else None
    _check(lib().slowmo_mix_step(ctx, arr, C.c_void_p(stream) if stream else None), ctx)


def slowmo_local_mix_step(ctx, grads, lr: float, in_peer: Sequence[int], stream: int = 0) -> None:
    """A local step and the mixing step after it in one call."""
    arr = grads if (grads is None or isinstance(grads, C.Array)) else _ptr_array(grads)
    peers = (C.c_int32 * len(in_peer))(*[int(v) for v in in_peer]) if in_peer is not None else None
    _check(lib().slowmo_local_mix_step(ctx, arr, lr, peers,
                                       C.c_void_p(stream) if stream else None), ctx)


def slowmo_check_device_range(ptr: int, nbytes: int) -> None:
    """Raises SlowMoError unless [ptr, ptr + nbytes) is device-accessible memory."""
    _check(lib().slowmo_check_device_range(C.c_void_p(ptr) if ptr else None, nbytes), None)


def slowmo_plan_mix(in_peer: Sequence[int]):
    """The in-place update order of a mixing step: a list of
    (worker, source, keep, take, flags); None for bad arguments."""
    m = len(in_peer)
    arr = (C.c_int32 * max(m, 1))(*[int(v) for v in in_peer])
    out = (slowmo_mix_entry * max(m, 1))()
    n = lib().slowmo_plan_mix(m, arr, out)
    if n < 0:
        return None
    return [(out[i].worker, out[i].source, out[i].keep, out[i].take, out[i].flags)
            for i in range(n)]


def slowmo_get_pushsum_weights(ctx, m: int):
    """The m push-sum weights as a list of floats (fp32 values)."""
    arr = (C.c_float * max(m, 1))()
    _check(lib().slowmo_get_pushsum_weights(ctx, arr), ctx)
    return [arr[i] for i in range(m)]


def slowmo_debias(ctx, z, stream: int = 0) -> None:
    """z: m * n_tensors device addresses that receive x^{(i)} / w_i."""
    arr = z if (z is None or isinstance(z, C.Array)) else _ptr_array(z)
    _check(lib().slowmo_debias(ctx, arr, C.c_void_p(stream) if stream else None), ctx)


def slowmo_debias_static(ctx, z, stream: int = 0) -> None:
    """slowmo_debias with its table in the library's static device array
    (no allocation; m * n_tensors <= SLOWMO_STATIC_MAX_POINTERS)."""
    arr = z if (z is None or isinstance(z, C.Array)) else _ptr_array(z)
    _check(lib().slowmo_debias_static(ctx, arr, C.c_void_p(stream) if stream else None), ctx)


def slowmo_lr_step_decay(base_lr: float, start_lr: float, warmup_steps: int, milestones,
                         factor: float, step: int) -> float:
    """Linear warm-up, then one factor per milestone passed (Section 4)."""
    ms = list(milestones or [])
    arr = (C.c_int64 * max(len(ms), 1))(*ms)
    out = C.c_float()
    _check(lib().slowmo_lr_step_decay(base_lr, start_lr, warmup_steps, arr if ms else None, len(ms),
                                      factor, step, C.byref(out)), None)
    return out.value


def slowmo_lr_inverse_sqrt(peak_lr: float, init_lr: float, warmup_steps: int, step: int) -> float:
    """Linear warm-up, then proportional to 1 / sqrt(step) (Appendix A.3)."""
    out = C.c_float()
    _check(lib().slowmo_lr_inverse_sqrt(peak_lr, init_lr, warmup_steps, step, C.byref(out)), None)
    return out.value


def slowmo_expgraph_in_peers(m: int, step: int):
    """The one-peer exponential graph's in-neighbours at iteration `step`."""
    arr = (C.c_int32 * max(m, 1))()
    _check(lib().slowmo_expgraph_in_peers(m, step, arr), None)
    return list(arr[:m])


def _f32_array(values):
    if values is None:
        return None
    return (C.c_float * len(values))(*[float(v) for v in values])


def slowmo_set_tensor_hparams(ctx, weight_decay=None, lr_scale=None, stream: int = 0) -> None:
    """Per-tensor weight decay / learning-rate scale (sequences of n_tensors or None)."""
    _check(lib().slowmo_set_tensor_hparams(ctx, _f32_array(weight_decay), _f32_array(lr_scale),
                                           C.c_void_p(stream) if stream else None), ctx)


def slowmo_export_bytes(ctx) -> int:
    return int(lib().slowmo_export_bytes(ctx))


def slowmo_export_state(ctx, dst: int, nbytes: int, stream: int = 0) -> None:
    """dst: device address of a buffer of at least slowmo_export_bytes(ctx)."""
    _check(lib().slowmo_export_state(ctx, C.c_void_p(dst) if dst else None, nbytes,
                                     C.c_void_p(stream) if stream else None), ctx)


def slowmo_import_state(ctx, src: int, nbytes: int, stream: int = 0) -> None:
    _check(lib().slowmo_import_state(ctx, C.c_void_p(src) if src else None, nbytes,
                                     C.c_void_p(stream) if stream else None), ctx)


def slowmo_destroy(ctx) -> None:
    _check(lib().slowmo_destroy(ctx), None)


def slowmo_get_buffer(ctx, which: int, worker: int, tensor: int) -> int:
    """Device address of the first element of an internal buffer of `tensor`."""
    out = C.c_void_p()
    _check(lib().slowmo_get_buffer(ctx, which, worker, tensor, C.byref(out)), ctx)
    return int(out.value or 0)


def slowmo_get_counters(ctx):
    """(t, k, l): outer iterations done, local steps in this one, Adam steps."""
    t, k, l = C.c_int64(), C.c_int32(), C.c_int64()
    _check(lib().slowmo_get_counters(ctx, C.byref(t), C.byref(k), C.byref(l)), ctx)
    return t.value, k.value, l.value


def _plan(fn, m: int, numel: Sequence[int]):
    arr = _i64_array(numel)
    n = fn(m, len(numel), arr, None, 0)
    if n < 0:
        raise SlowMoError(SLOWMO_ERR_ARG, "invalid arguments to the plan query")
    buf = (slowmo_plan_run * max(n, 1))()
    fn(m, len(numel), arr, buf, n)
    return [(r.tile, r.worker, r.tensor, r.n, r.offset) for r in buf[:n]]


def slowmo_plan_local(m: int, numel: Sequence[int]):
    """[(tile, worker, tensor, n, offset)] of the local-step tiling."""
    return _plan(lib().slowmo_plan_local, m, numel)


def slowmo_plan_outer(m: int, numel: Sequence[int]):
    return _plan(lib().slowmo_plan_outer, m, numel)
