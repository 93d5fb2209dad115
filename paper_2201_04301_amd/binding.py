"""ctypes binding of libgcada.so -- argument marshalling only.

Function names and arguments mirror ``include/gcada.h``; every step of the iteration runs in the
library's HIP kernels.  There is no fallback: if the library is missing, importing fails.
PyTorch appears only as the owner of device buffers and streams (``tensor.data_ptr()``,
``torch.cuda.current_stream().cuda_stream``).
"""
from __future__ import annotations

import ctypes as C
import os

# PyTorch ships its own HIP runtime; it has to be in the process BEFORE this library is loaded so
# that both use the same one (two runtimes in one process do not see the device).
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgcada.so")

GCADA_OK, GCADA_EINVAL, GCADA_ENOMEM, GCADA_EDEVICE, GCADA_ESTATE = range(5)
GCADA_LOGREG, GCADA_MLP, GCADA_LINREG = 0, 1, 2
GCADA_F32, GCADA_BF16 = 0, 1
GCADA_MAX_WIDTHS = 8
GCADA_OPT_SINGLE_PASS_LOGREG = 1
GCADA_OPT_FUSED_FINISH = 2
GCADA_OPT_LAZY_GRADIENT_STORE = 3
GCADA_OPT_GRAM_STATISTIC = 4
GCADA_OPT_EXPIRE_NEXT_WAIT = 5
GCADA_OPT_DEFERRED_FINISH = 6

EXPORTS = ["gcada_create", "gcada_destroy", "gcada_set_shard", "gcada_set_theta", "gcada_step",
           "gcada_state", "gcada_get_state", "gcada_set_state", "gcada_cost_model",
           "gcada_last_error", "gcada_version", "gcada_time_gradient_stage", "gcada_set_option",
           "gcada_timed_stage", "gcada_set_rule", "gcada_estimate_smoothness", "gcada_step_workers",
           "gcada_estimate_smoothness_static", "gcada_hbm_read_calibration", "gcada_gather_read_calibration"]

GCADA_RULE_GRADIENT_DIFFERENCE, GCADA_RULE_SERVER = 0, 1


class gcada_dims(C.Structure):
    _fields_ = [("model", C.c_int32), ("dtype", C.c_int32), ("n_widths", C.c_int32),
                ("widths", C.c_int32 * GCADA_MAX_WIDTHS), ("batch", C.c_int32), ("l2", C.c_float)]


class gcada_state_view(C.Structure):
    _fields_ = [("p", C.c_int64), ("G", C.c_int32), ("D", C.c_int32), ("M_G", C.c_int32),
                ("k", C.c_int64), ("slot_stride", C.c_int64), ("grad_stride", C.c_int64),
                ("cur_slot", C.c_int32),
                ("theta_ring", C.c_void_p), ("h", C.c_void_p), ("vhat", C.c_void_p),
                ("agg", C.c_void_p), ("gbuf", C.c_void_p), ("which", C.c_void_p),
                ("tau", C.c_void_p), ("dtheta_sq", C.c_void_p), ("stat", C.c_void_p),
                ("rhs", C.c_void_p), ("mask", C.c_void_p), ("loss", C.c_void_p)]


class gcada_state_host(C.Structure):
    _fields_ = [("theta", C.c_void_p), ("h", C.c_void_p), ("vhat", C.c_void_p),
                ("agg", C.c_void_p), ("theta_stale", C.c_void_p), ("last", C.c_void_p),
                ("tau", C.c_void_p), ("dtheta_sq", C.c_void_p), ("k", C.c_int64)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is not built; run `python paper_2201_04301_amd/build.py` "
            "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    L.gcada_create.restype = C.c_int
    L.gcada_create.argtypes = [C.POINTER(gcada_dims), C.c_int32, C.c_int32, C.c_int32, C.c_double,
                               C.c_double, C.c_double, C.c_double, C.c_double,
                               C.POINTER(C.c_void_p)]
    L.gcada_destroy.restype = None
    L.gcada_destroy.argtypes = [C.c_void_p]
    L.gcada_set_shard.restype = C.c_int
    L.gcada_set_shard.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64,
                                  C.c_int64]
    L.gcada_set_theta.restype = C.c_int
    L.gcada_set_theta.argtypes = [C.c_void_p, C.c_void_p]
    L.gcada_step.restype = C.c_int
    L.gcada_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.gcada_state.restype = C.c_int
    L.gcada_state.argtypes = [C.c_void_p, C.POINTER(gcada_state_view)]
    L.gcada_get_state.restype = C.c_int
    L.gcada_get_state.argtypes = [C.c_void_p, C.POINTER(gcada_state_host)]
    L.gcada_set_state.restype = C.c_int
    L.gcada_set_state.argtypes = [C.c_void_p, C.POINTER(gcada_state_host)]
    L.gcada_cost_model.restype = C.c_int
    L.gcada_cost_model.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                   C.POINTER(C.c_double),
                                   C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    L.gcada_step_workers.restype = C.c_int
    L.gcada_step_workers.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p]
    L.gcada_set_rule.restype = C.c_int
    L.gcada_set_rule.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    L.gcada_estimate_smoothness.restype = C.c_int
    L.gcada_estimate_smoothness.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    L.gcada_estimate_smoothness_static.restype = C.c_int
    L.gcada_estimate_smoothness_static.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    L.gcada_hbm_read_calibration.restype = C.c_int
    L.gcada_hbm_read_calibration.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.POINTER(C.c_double),
                                             C.POINTER(C.c_double)]
    L.gcada_gather_read_calibration.restype = C.c_int
    L.gcada_gather_read_calibration.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p,
                                                C.POINTER(C.c_double)]
    L.gcada_set_option.restype = C.c_int
    L.gcada_set_option.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    L.gcada_timed_stage.restype = C.c_char_p
    L.gcada_timed_stage.argtypes = [C.c_void_p]
    L.gcada_time_gradient_stage.restype = C.c_int
    L.gcada_time_gradient_stage.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p,
                                            C.POINTER(C.c_double)]
    L.gcada_last_error.restype = C.c_char_p
    L.gcada_last_error.argtypes = [C.c_void_p]
    L.gcada_version.restype = C.c_char_p
    L.gcada_version.argtypes = []
    return L


lib = _load()


class GcadaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"gcada error {code}: {msg}")
        self.code = code


def _check(rc: int, ctx=None):
    if rc != GCADA_OK:
        raise GcadaError(rc, (lib.gcada_last_error(ctx) or b"").decode())


def make_dims(model: int, dtype: int, widths, batch: int, l2: float = 0.0) -> gcada_dims:
    d = gcada_dims()
    d.model, d.dtype, d.n_widths, d.batch, d.l2 = model, dtype, len(widths), batch, l2
    for i, w in enumerate(widths):
        d.widths[i] = int(w)
    return d


def gcada_create(dims: gcada_dims, G, M_G, D, c, alpha, beta1, beta2, eps) -> C.c_void_p:
    out = C.c_void_p()
    _check(lib.gcada_create(C.byref(dims), G, M_G, D, c, alpha, beta1, beta2, eps, C.byref(out)))
    return out


def gcada_destroy(ctx):
    lib.gcada_destroy(ctx)


def gcada_set_shard(ctx, g: int, X_ptr: int, y_ptr: int, rows: int, ld: int):
    _check(lib.gcada_set_shard(ctx, g, X_ptr, y_ptr, rows, ld), ctx)


def gcada_set_theta(ctx, theta0_ptr: int):
    _check(lib.gcada_set_theta(ctx, theta0_ptr), ctx)


def gcada_step(ctx, idx_ptr, mask_out_ptr, loss_out_ptr, stream_ptr=None):
    _check(lib.gcada_step(ctx, idx_ptr, mask_out_ptr, loss_out_ptr, stream_ptr), ctx)


def gcada_state(ctx) -> gcada_state_view:
    v = gcada_state_view()
    _check(lib.gcada_state(ctx, C.byref(v)), ctx)
    return v


def gcada_get_state(ctx, st: gcada_state_host):
    _check(lib.gcada_get_state(ctx, C.byref(st)), ctx)


def gcada_set_state(ctx, st: gcada_state_host):
    _check(lib.gcada_set_state(ctx, C.byref(st)), ctx)


def gcada_cost_model(G: int, M_G: int, mu: int, mask_ptr, T_ptr):
    t, cm, cp = C.c_double(), C.c_int64(), C.c_int64()
    rc = lib.gcada_cost_model(G, M_G, mu, mask_ptr, T_ptr, C.byref(t), C.byref(cm), C.byref(cp))
    if rc != GCADA_OK:
        raise GcadaError(rc, "gcada_cost_model: bad argument")
    return t.value, cm.value, cp.value


def gcada_version() -> str:
    return lib.gcada_version().decode()


def gcada_last_error(ctx=None) -> str:
    return (lib.gcada_last_error(ctx) or b"").decode()


def gcada_time_gradient_stage(ctx, idx_ptr, idx_stride: int, reps: int, stream_ptr=None) -> float:
    ms = C.c_double()
    _check(lib.gcada_time_gradient_stage(ctx, idx_ptr, idx_stride, reps, stream_ptr, C.byref(ms)), ctx)
    return ms.value


def gcada_set_option(ctx, option: int, value: int):
    _check(lib.gcada_set_option(ctx, option, value), ctx)


def gcada_step_workers(ctx, idx_workers, delays, worker_out, mask_out, loss_out, stream):
    _check(lib.gcada_step_workers(ctx, idx_workers, delays, worker_out, mask_out, loss_out, stream), ctx)


def gcada_set_rule(ctx, rule: int, L_ptr):
    _check(lib.gcada_set_rule(ctx, rule, L_ptr), ctx)


def gcada_estimate_smoothness(ctx, iters: int, L_out_ptr, stream):
    _check(lib.gcada_estimate_smoothness(ctx, iters, L_out_ptr, stream), ctx)


def gcada_timed_stage(ctx) -> str:
    return (lib.gcada_timed_stage(ctx) or b"").decode()


def gcada_estimate_smoothness_static(ctx, iters: int, L_out_dev_ptr, stream):
    _check(lib.gcada_estimate_smoothness_static(ctx, iters, L_out_dev_ptr, stream), ctx)


def gcada_gather_read_calibration(ctx, idx_ptr, idx_stride: int, reps: int, stream_ptr=None) -> float:
    g = C.c_double()
    _check(lib.gcada_gather_read_calibration(ctx, idx_ptr, idx_stride, reps, stream_ptr, C.byref(g)), ctx)
    return g.value


def gcada_hbm_read_calibration(buf_ptr, nbytes: int, reps: int, stream=None):
    """(best GB/s over all launch shapes and load kinds, best GB/s with ordinary loads)."""
    g, gp = C.c_double(), C.c_double()
    _check(lib.gcada_hbm_read_calibration(buf_ptr, nbytes, reps, stream, C.byref(g), C.byref(gp)))
    return g.value, gp.value
