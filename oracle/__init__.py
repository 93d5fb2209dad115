"""fp64 CPU oracle for one G-CADA iteration -- TEST INFRASTRUCTURE.

Thin ctypes access to ``gcada_oracle.c`` (the arithmetic lives there, written from the
paper: Sec. II-A minibatch gradient, Eq. (3) / Sec. IV aggregate, Eq. (8a)-(8c) server
update, Eq. (9) threshold, Algorithm 1 age counters).  Only tests, the smoke check and the
benchmark's cpu-baseline leg may import this package; the GPU library never does, and
this package never imports the GPU library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gcada_oracle.c")
_LIB = os.path.join(_HERE, "libgcada_oracle.so")

LOGISTIC, MLP, QUADRATIC = 0, 1, 2

(F_THETA, F_H, F_VHAT, F_AGG, F_THETA_STALE, F_LAST, F_GRAD, F_GRAD_STALE, F_STAT, F_RING,
 F_LOSS_G, F_KINK, F_KINK_UNIT) = range(13)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP over groups only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [("model", C.c_int32), ("n_widths", C.c_int32), ("widths", C.c_int32 * 8),
                ("batch", C.c_int32), ("G", C.c_int32), ("D", C.c_int32),
                ("round_bf16", C.c_int32), ("l2", C.c_double), ("c", C.c_double),
                ("alpha", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_param_count.restype = C.c_int64
        L.orc_param_count.argtypes = [C.POINTER(_Cfg)]
        L.orc_loss_grad_sum.restype = C.c_double
        L.orc_loss_grad_sum.argtypes = [C.POINTER(_Cfg), C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_int64, C.c_void_p]
        L.orc_amsgrad.restype = C.c_double
        L.orc_amsgrad.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                  C.c_double, C.c_double, C.c_double, C.c_double]
        L.orc_create.restype = C.c_void_p
        L.orc_create.argtypes = [C.POINTER(_Cfg)]
        L.orc_destroy.argtypes = [C.c_void_p]
        L.orc_reset.argtypes = [C.c_void_p, C.c_void_p]
        L.orc_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_field.restype = C.POINTER(C.c_double)
        L.orc_field.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int64)]
        L.orc_tau.restype = C.POINTER(C.c_int32)
        L.orc_tau.argtypes = [C.c_void_p]
        L.orc_mask.restype = C.POINTER(C.c_uint8)
        L.orc_mask.argtypes = [C.c_void_p]
        L.orc_rhs.restype = C.c_double
        L.orc_rhs.argtypes = [C.c_void_p]
        L.orc_loss.restype = C.c_double
        L.orc_loss.argtypes = [C.c_void_p]
        L.orc_k.restype = C.c_int64
        L.orc_k.argtypes = [C.c_void_p]
        L.orc_set_k.argtypes = [C.c_void_p, C.c_int64]
        L.orc_set_rule.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        L.orc_bf16_round.restype = C.c_double
        L.orc_bf16_round.argtypes = [C.c_double]
        _lib = L
    return _lib


@dataclass
class Config:
    """Problem statement of one run (Algorithm 1's inputs plus the model)."""
    model: int
    widths: Sequence[int]
    batch: int
    G: int
    D: int = 10
    c: float = 1.0
    alpha: float = 1e-2
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    l2: float = 0.0
    round_bf16: int = 0        # 0 none; 1 X and theta; 2 also the hidden activations (see gcada_oracle.c)
    _c: _Cfg = field(init=False, repr=False, default=None)

    def c_struct(self) -> _Cfg:
        s = _Cfg()
        s.model = self.model
        s.n_widths = len(self.widths)
        for i, w in enumerate(self.widths):
            s.widths[i] = int(w)
        s.batch, s.G, s.D = self.batch, self.G, self.D
        s.round_bf16 = int(self.round_bf16)
        s.l2, s.c, s.alpha = self.l2, self.c, self.alpha
        s.beta1, s.beta2, s.eps = self.beta1, self.beta2, self.eps
        return s


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _labels(cfg: Config, y):
    if cfg.model == MLP:
        return np.ascontiguousarray(y, dtype=np.int32)
    return np.ascontiguousarray(y, dtype=np.float32)


def param_count(cfg: Config) -> int:
    return int(lib().orc_param_count(C.byref(cfg.c_struct())))


def loss_grad_sum(cfg: Config, theta, X, y, want_grad: bool = True):
    """Sum over the rows of X of loss(theta; x, y) [+ (l2/2)||theta||^2 each], and its gradient."""
    theta = np.ascontiguousarray(theta, dtype=np.float64)
    X = _f32(X)
    yv = _labels(cfg, y)
    n = X.shape[0]
    assert X.shape[1] == cfg.widths[0] and yv.shape[0] == n
    assert theta.shape[0] == param_count(cfg)
    g = np.empty_like(theta) if want_grad else None
    loss = lib().orc_loss_grad_sum(C.byref(cfg.c_struct()), theta.ctypes.data, X.ctypes.data,
                                   yv.ctypes.data, n, g.ctypes.data if want_grad else None)
    return float(loss), g


def amsgrad(theta, h, vhat, agg, alpha, beta1, beta2, eps) -> float:
    """In-place Eq. (8a)-(8c) on float64 arrays; returns ||theta_new - theta_old||^2."""
    for a in (theta, h, vhat, agg):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    return float(lib().orc_amsgrad(theta.ctypes.data, h.ctypes.data, vhat.ctypes.data,
                                   agg.ctypes.data, theta.shape[0], alpha, beta1, beta2, eps))


def bf16_round(x: float) -> float:
    return float(lib().orc_bf16_round(float(x)))


def cyclic_window(k: int, mu: int, n_rows: int) -> np.ndarray:
    """Deterministic minibatch of step k when no row ids are supplied: rows (k*mu + i) mod n."""
    return ((k * mu + np.arange(mu, dtype=np.int64)) % n_rows).astype(np.int32)


class Oracle:
    """State of one run: theta, h, v-hat, aggregate, per-group stale iterate / last uploaded
    gradient / age, history ring, iteration counter.  Arrays are live views into the C state."""

    def __init__(self, cfg: Config, theta0=None):
        self.cfg = cfg
        self._h = lib().orc_create(C.byref(cfg.c_struct()))
        if not self._h:
            raise ValueError("invalid oracle configuration")
        self.p = param_count(cfg)
        self.reset(np.zeros(self.p) if theta0 is None else theta0)

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_destroy(self._h)
            self._h = None

    def reset(self, theta0):
        t0 = np.ascontiguousarray(theta0, dtype=np.float64)
        assert t0.shape == (self.p,)
        lib().orc_reset(self._h, t0.ctypes.data)

    def _view(self, fid, shape):
        n = C.c_int64()
        ptr = lib().orc_field(self._h, fid, C.byref(n))
        return np.ctypeslib.as_array(ptr, shape=(n.value,)).reshape(shape)

    theta = property(lambda s: s._view(F_THETA, (s.p,)))
    h = property(lambda s: s._view(F_H, (s.p,)))
    vhat = property(lambda s: s._view(F_VHAT, (s.p,)))
    agg = property(lambda s: s._view(F_AGG, (s.p,)))
    theta_stale = property(lambda s: s._view(F_THETA_STALE, (s.cfg.G, s.p)))
    last = property(lambda s: s._view(F_LAST, (s.cfg.G, s.p)))
    grad = property(lambda s: s._view(F_GRAD, (s.cfg.G, s.p)))
    grad_stale = property(lambda s: s._view(F_GRAD_STALE, (s.cfg.G, s.p)))
    stat = property(lambda s: s._view(F_STAT, (s.cfg.G,)))
    ring = property(lambda s: s._view(F_RING, (s.cfg.D,)))
    loss_g = property(lambda s: s._view(F_LOSS_G, (s.cfg.G,)))
    kink = property(lambda s: s._view(F_KINK, (s.cfg.G,)))
    # the same per hidden unit (layer 1's units first): (G, sum of the hidden widths)
    kink_unit = property(lambda s: s._view(F_KINK_UNIT, (s.cfg.G, sum(s.cfg.widths[1:-1]) if s.cfg.model == MLP else 0)))

    @property
    def tau(self):
        return np.ctypeslib.as_array(lib().orc_tau(self._h), shape=(self.cfg.G,))

    @property
    def mask(self):
        return np.ctypeslib.as_array(lib().orc_mask(self._h), shape=(self.cfg.G,))

    @property
    def rhs(self) -> float:
        return float(lib().orc_rhs(self._h))

    @property
    def loss(self) -> float:
        return float(lib().orc_loss(self._h))

    @property
    def k(self) -> int:
        return int(lib().orc_k(self._h))

    @k.setter
    def k(self, v: int):
        lib().orc_set_k(self._h, int(v))

    def set_rule(self, rule: int, L=None):
        """rule 0: same-minibatch gradient difference (default).  rule 1: the server-side condition
        of Sec. IV, L_g^2 ||theta^k - theta^{k-tau_g}||^2 against the threshold, with the G
        smoothness constants L; only selected groups then evaluate a gradient."""
        Lp = None
        if L is not None:
            La = np.ascontiguousarray(L, dtype=np.float64)
            assert La.shape == (self.cfg.G,)
            Lp = La.ctypes.data
        lib().orc_set_rule(self._h, int(rule), Lp)

    def step(self, X, y):
        """X: (G, mu, d) fp32 minibatch rows, y: (G, mu).  Returns (mask copy, loss)."""
        cfg = self.cfg
        X = _f32(X)
        yv = _labels(cfg, y)
        assert X.shape == (cfg.G, cfg.batch, cfg.widths[0]), X.shape
        assert yv.shape == (cfg.G, cfg.batch), yv.shape
        mask = np.empty(cfg.G, dtype=np.uint8)
        loss = C.c_double()
        lib().orc_step(self._h, X.ctypes.data, yv.ctypes.data, mask.ctypes.data, C.byref(loss))
        return mask, loss.value

    def step_shards(self, shards_X, shards_y, idx=None):
        """Gather each group's minibatch from its shard (row ids idx[g], or the cyclic window
        of the current step) and take one step."""
        cfg = self.cfg
        k = self.k
        Xs, ys = [], []
        for g in range(cfg.G):
            rows = cyclic_window(k, cfg.batch, shards_X[g].shape[0]) if idx is None else idx[g]
            Xs.append(np.asarray(shards_X[g])[rows])
            ys.append(np.asarray(shards_y[g])[rows])
        return self.step(np.stack(Xs), np.stack(ys))
