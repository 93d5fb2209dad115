"""Convenience wrapper around one library context.

It only keeps torch tensors alive (device memory), passes their pointers and the current stream
to the C entry points, and copies state between device and numpy.  No arithmetic of the method
happens here.
"""
from __future__ import annotations

import ctypes as C
from typing import Optional, Sequence

import numpy as np
import torch

from . import binding as B

_hip = None


def _hiprt():
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
        _hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        _hip.hipMemcpy.restype = C.c_int
        _hip.hipDeviceSynchronize.restype = C.c_int
    return _hip


def _d2h(ptr: int, count: int, dtype) -> np.ndarray:
    out = np.empty(count, dtype=dtype)
    rc = _hiprt().hipMemcpy(out.ctypes.data, ptr, out.nbytes, 2)   # hipMemcpyDeviceToHost
    if rc != 0:
        raise RuntimeError(f"hipMemcpy D2H failed with {rc}")
    return out


class Gcada:
    """One G-CADA run on the current HIP device."""

    def __init__(self, model: str, widths: Sequence[int], batch: int, G: int, M_G: int = 1,
                 D: int = 10, c: float = 1.0, alpha: float = 1e-2, beta1: float = 0.9,
                 beta2: float = 0.999, eps: float = 1e-8, l2: float = 0.0, dtype: str = "f32"):
        self.model = {"logreg": B.GCADA_LOGREG, "mlp": B.GCADA_MLP, "linreg": B.GCADA_LINREG}[model]
        self.dtype = {"f32": B.GCADA_F32, "bf16": B.GCADA_BF16}[dtype]
        self.widths, self.batch, self.G, self.M_G, self.D = tuple(widths), batch, G, M_G, D
        dims = B.make_dims(self.model, self.dtype, widths, batch, l2)
        self.ctx = B.gcada_create(dims, G, M_G, D, c, alpha, beta1, beta2, eps)
        self._keep = {}
        self.p = B.gcada_state(self.ctx).p
        self.mask_out = torch.zeros(G, dtype=torch.uint8, device="cuda")
        self.loss_out = torch.zeros(1, dtype=torch.float32, device="cuda")

    @classmethod
    def from_workload(cls, w, **over):
        kw = dict(model=w.model, widths=w.widths, batch=w.mu, G=w.G, M_G=w.M_G, D=w.D, c=w.c,
                  alpha=w.alpha, beta1=w.beta1, beta2=w.beta2, eps=w.eps, l2=w.l2, dtype=w.dtype)
        kw.update(over)
        return cls(**kw)

    def close(self):
        if getattr(self, "ctx", None):
            B.gcada_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        self.close()

    # ---- inputs
    def set_shards(self, Xs, ys):
        for g, (X, y) in enumerate(zip(Xs, ys)):
            assert X.is_cuda and y.is_cuda and X.dim() == 2 and X.stride(1) == 1
            want = torch.bfloat16 if self.dtype == B.GCADA_BF16 else torch.float32
            assert X.dtype == want, (X.dtype, want)
            assert y.dtype == (torch.int32 if self.model == B.GCADA_MLP else torch.float32)
            B.gcada_set_shard(self.ctx, g, X.data_ptr(), y.data_ptr(), X.shape[0], X.stride(0))
            self._keep[("shard", g)] = (X, y)

    def set_theta(self, theta0):
        t = np.ascontiguousarray(np.asarray(theta0, dtype=np.float32))
        assert t.shape == (self.p,)
        B.gcada_set_theta(self.ctx, t.ctypes.data)

    # ---- the iteration
    def step(self, idx: Optional[torch.Tensor] = None, mask_out=None, loss_out=None):
        """Enqueue one iteration on torch's current stream; returns nothing (asynchronous)."""
        if idx is not None:
            assert idx.is_cuda and idx.dtype == torch.int32 and idx.is_contiguous()
            assert idx.numel() == self.G * self.batch
        mo = self.mask_out if mask_out is None else mask_out
        lo = self.loss_out if loss_out is None else loss_out
        B.gcada_step(self.ctx, idx.data_ptr() if idx is not None else None, mo.data_ptr(),
                     lo.data_ptr(), torch.cuda.current_stream().cuda_stream)

    def step_workers(self, idx_workers: torch.Tensor, delays: torch.Tensor, worker_out=None,
                     mask_out=None, loss_out=None):
        """One iteration with per-worker minibatches: idx_workers int32 (G, M_G, mu), delays float64
        (G, M_G), both on the device; the fastest worker's minibatch is used for each group."""
        assert idx_workers.is_cuda and idx_workers.dtype == torch.int32 and idx_workers.is_contiguous()
        assert delays.is_cuda and delays.dtype == torch.float64 and delays.is_contiguous()
        assert idx_workers.numel() == self.G * self.M_G * self.batch and delays.numel() == self.G * self.M_G
        mo = self.mask_out if mask_out is None else mask_out
        lo = self.loss_out if loss_out is None else loss_out
        B.gcada_step_workers(self.ctx, idx_workers.data_ptr(), delays.data_ptr(),
                             worker_out.data_ptr() if worker_out is not None else None, mo.data_ptr(),
                             lo.data_ptr(), torch.cuda.current_stream().cuda_stream)

    # ---- outputs / state
    def outputs(self):
        """Synchronise and copy the last step's mask, loss, stat, rhs and fresh gradients."""
        torch.cuda.synchronize()
        v = B.gcada_state(self.ctx)
        mask = _d2h(v.mask, self.G, np.uint8)
        which = _d2h(v.which, self.G, np.int32)
        # the fresh gradient of the last step: the stored row if the group uploaded, else the other
        half = np.where(mask != 0, which, 1 - which)
        grad = np.empty((self.G, self.p), np.float32)
        for g in range(self.G):
            grad[g] = _d2h(v.gbuf + 4 * (int(half[g]) * self.G + g) * v.grad_stride, self.p, np.float32)
        return dict(mask=mask, loss=float(_d2h(v.loss, 1, np.float64)[0]),
                    stat=_d2h(v.stat, self.G, np.float64), rhs=float(_d2h(v.rhs, 1, np.float64)[0]),
                    grad=grad)

    def get_state(self):
        p, G, D = self.p, self.G, self.D
        bufs = dict(theta=np.empty(p, np.float32), h=np.empty(p, np.float32),
                    vhat=np.empty(p, np.float32), agg=np.empty(p, np.float32),
                    theta_stale=np.empty((G, p), np.float32), last=np.empty((G, p), np.float32),
                    tau=np.empty(G, np.int32), dtheta_sq=np.empty(D, np.float64))
        st = B.gcada_state_host()
        for k, a in bufs.items():
            setattr(st, k, a.ctypes.data)
        B.gcada_get_state(self.ctx, st)
        bufs["k"] = int(st.k)
        return bufs

    def set_state(self, theta, h, vhat, agg, theta_stale, last, tau, dtheta_sq, k):
        p, G, D = self.p, self.G, self.D
        arrs = dict(theta=(theta, np.float32, (p,)), h=(h, np.float32, (p,)),
                    vhat=(vhat, np.float32, (p,)), agg=(agg, np.float32, (p,)),
                    theta_stale=(theta_stale, np.float32, (G, p)), last=(last, np.float32, (G, p)),
                    tau=(tau, np.int32, (G,)), dtheta_sq=(dtheta_sq, np.float64, (D,)))
        st = B.gcada_state_host()
        keep = []
        for name, (a, dt, shape) in arrs.items():
            a = np.ascontiguousarray(np.asarray(a), dtype=dt)
            assert a.shape == shape, (name, a.shape, shape)
            keep.append(a)
            setattr(st, name, a.ctypes.data)
        st.k = int(k)
        B.gcada_set_state(self.ctx, st)

    # ---- selection rule
    def set_rule(self, rule: str, L=None):
        """rule: "gradient_difference" (default) or "server" (the paper's condition with the
        smoothness constants L_g, lazy gradient evaluation).  L: G floats (host)."""
        code = {"gradient_difference": B.GCADA_RULE_GRADIENT_DIFFERENCE, "server": B.GCADA_RULE_SERVER}[rule]
        Lp = None
        if L is not None:
            La = np.ascontiguousarray(np.asarray(L, dtype=np.float64))
            assert La.shape == (self.G,)
            Lp = La.ctypes.data
        B.gcada_set_rule(self.ctx, code, Lp)

    def estimate_smoothness(self, iters: int = 30) -> np.ndarray:
        out = np.empty(self.G, np.float64)
        B.gcada_estimate_smoothness(self.ctx, iters, out.ctypes.data,
                                    torch.cuda.current_stream().cuda_stream)
        return out

    def estimate_smoothness_static(self, out: torch.Tensor, iters: int = 30):
        """The same through the entry point that allocates nothing: `out` is a float64 device tensor
        of G elements, written in stream order (asynchronous)."""
        assert out.is_cuda and out.dtype == torch.float64 and out.numel() == self.G and out.is_contiguous()
        B.gcada_estimate_smoothness_static(self.ctx, iters, out.data_ptr(),
                                           torch.cuda.current_stream().cuda_stream)

    def cost_model(self, mask: np.ndarray, T: np.ndarray):
        mask = np.ascontiguousarray(mask, dtype=np.uint8)
        T = np.ascontiguousarray(T, dtype=np.float64)
        assert mask.shape == (self.G,) and T.shape == (self.G, self.M_G)
        return B.gcada_cost_model(self.G, self.M_G, self.batch, mask.ctypes.data, T.ctypes.data)
