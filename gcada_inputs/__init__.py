"""Seeded synthetic workloads for G-CADA runs: shapes, data, initial iterate, minibatch row ids
and per-worker compute delays.

This module produces INPUTS only -- it contains none of the method's arithmetic (no loss, no
gradient, no selection rule, no optimiser).  Both the GPU library's harness and the CPU oracle's
harness read the values made here; neither of those imports the other.

The paper's experiment (Sec. VI) uses a public image dataset that is not available here; these
synthetic workloads stand in for it.  Logistic-regression data: features N(0, I/d), labels from a
planted weight vector with a fraction of flips.  MLP data: ten Gaussian clusters, label = cluster.
Linear-regression data (the model of the paper's experiment): same features, real targets from a
planted weight vector plus Gaussian noise.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    model: str                 # "logreg" | "mlp" | "linreg"
    widths: Tuple[int, ...]    # logreg, linreg: (d,), mlp: layer widths including the input
    G: int                     # worker groups
    M_G: int                   # workers per group (host cost model only)
    mu: int                    # minibatch per group
    rows: int                  # rows per group shard
    dtype: str = "f32"         # storage type of X and of the compute copy of the weights
    l2: float = 0.0
    flip: float = 0.05         # logreg: fraction of flipped labels
    lo: float = 0.0            # mlp: cluster means ~ U[lo, hi]^d, samples clipped to [lo, hi]
    hi: float = 1.0
    sigma: float = 0.1
    D: int = 10
    c: float = 1.0
    alpha: float = 1e-2
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    iters: int = 200
    seed: int = 2201

    @property
    def p(self) -> int:
        if self.model in ("logreg", "linreg"):
            return self.widths[0]
        return sum(self.widths[l] * self.widths[l - 1] + self.widths[l]
                   for l in range(1, len(self.widths)))

    @property
    def M(self) -> int:
        return self.G * self.M_G


# The five benchmark configurations (hyper-parameters not stated for 2-5 inherit those of 1).
CONFIGS = {
    "lr_small": Workload("lr_small", "logreg", (64,), G=3, M_G=2, mu=32, rows=512, flip=0.10,
                         iters=200),
    "lr_4k": Workload("lr_4k", "logreg", (4096,), G=16, M_G=2, mu=256, rows=65536, l2=1e-4,
                      iters=1000),
    "mlp_784": Workload("mlp_784", "mlp", (784, 200, 10), G=10, M_G=2, mu=512, rows=6000,
                        iters=500),
    "lr_64k": Workload("lr_64k", "logreg", (65536,), G=32, M_G=4, mu=1024, rows=16384, iters=200),
    "mlp_3072_bf16": Workload("mlp_3072_bf16", "mlp", (3072, 1024, 1024, 10), G=64, M_G=4, mu=256,
                              rows=781, dtype="bf16", lo=-1.0, hi=1.0, iters=200),
    # geometry of the paper's experiment (Sec. VI): linear regression with the quadratic error
    # loss, M = 12 workers in G = 3 groups of M_G = 4, input width of that dataset (784), rule
    # constant 0.3 on the SUM over the history, i.e. c = 0.3 D here; D and mu are not stated
    "linreg_784": Workload("linreg_784", "linreg", (784,), G=3, M_G=4, mu=256, rows=20000, c=3.0,
                           sigma=0.1, iters=500),
}


def scaled(w: Workload, **kw) -> Workload:
    """A smaller or altered copy of a workload (same recipe, other sizes)."""
    return replace(w, **kw)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_shards(w: Workload, device="cpu", chunk_rows: int = 4096):
    """Return (X, y): lists with one tensor per group.  X[g]: rows x d (fp32 or bf16, row-major);
    y[g]: fp32 +-1 (logreg), fp32 target (linreg) or int32 class id (mlp).  Generated on ``device`` chunk by chunk so a
    137 GB dataset never needs a host copy."""
    device = torch.device(device)
    d = w.widths[0]
    xdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    gen = _gen(w.seed, device)
    Xs: List[torch.Tensor] = []
    ys: List[torch.Tensor] = []
    if w.model in ("logreg", "linreg"):
        wstar = torch.randn(d, generator=gen, device=device, dtype=torch.float32)
        scale = 1.0 / math.sqrt(d)
        for g in range(w.G):
            X = torch.empty(w.rows, d, device=device, dtype=xdt)
            y = torch.empty(w.rows, device=device, dtype=torch.float32)
            for r0 in range(0, w.rows, chunk_rows):
                r1 = min(w.rows, r0 + chunk_rows)
                xc = torch.randn(r1 - r0, d, generator=gen, device=device, dtype=torch.float32)
                xc.mul_(scale)
                xc = xc.to(xdt)
                if w.model == "linreg":     # real targets: planted weights plus noise
                    yc = xc.float() @ wstar + w.sigma * torch.randn(r1 - r0, generator=gen, device=device)
                else:
                    yc = torch.where(xc.float() @ wstar >= 0, 1.0, -1.0)
                    fl = torch.rand(r1 - r0, generator=gen, device=device) < w.flip
                    yc = torch.where(fl, -yc, yc)
                X[r0:r1] = xc
                y[r0:r1] = yc
            Xs.append(X)
            ys.append(y)
    elif w.model == "mlp":
        ncls = w.widths[-1]
        means = torch.rand(ncls, d, generator=gen, device=device) * (w.hi - w.lo) + w.lo
        for g in range(w.G):
            lab = torch.randint(0, ncls, (w.rows,), generator=gen, device=device)
            X = torch.empty(w.rows, d, device=device, dtype=xdt)
            for r0 in range(0, w.rows, chunk_rows):
                r1 = min(w.rows, r0 + chunk_rows)
                xc = means[lab[r0:r1]] + w.sigma * torch.randn(r1 - r0, d, generator=gen,
                                                              device=device)
                X[r0:r1] = xc.clamp_(w.lo, w.hi).to(xdt)
            Xs.append(X)
            ys.append(lab.to(torch.int32))
    else:
        raise ValueError(w.model)
    return Xs, ys


def make_theta0(w: Workload) -> np.ndarray:
    """Initial iterate (fp32).  logreg: zeros.  mlp: W ~ U(+-1/sqrt(fan_in)), b = 0, laid out per
    layer as W (out x in, row-major) followed by b."""
    if w.model in ("logreg", "linreg"):
        return np.zeros(w.p, dtype=np.float32)
    rng = np.random.default_rng(w.seed + 17)
    parts = []
    for l in range(1, len(w.widths)):
        fan_in, fan_out = w.widths[l - 1], w.widths[l]
        bound = 1.0 / math.sqrt(fan_in)
        parts.append(rng.uniform(-bound, bound, size=fan_out * fan_in).astype(np.float32))
        parts.append(np.zeros(fan_out, dtype=np.float32))
    return np.concatenate(parts)


def make_indices(w: Workload, steps: int, seed: Optional[int] = None) -> np.ndarray:
    """Minibatch row ids, int32 (steps, G, mu): per step and group, uniform without replacement
    within the group's shard."""
    rng = np.random.default_rng((w.seed if seed is None else seed) + 101)
    out = np.empty((steps, w.G, w.mu), dtype=np.int32)
    for k in range(steps):
        for g in range(w.G):
            out[k, g] = rng.choice(w.rows, size=w.mu, replace=False, shuffle=False)
    return out


def make_worker_indices(w: Workload, steps: int, seed: Optional[int] = None) -> np.ndarray:
    """Per-worker minibatch row ids, int32 (steps, G, M_G, mu): every worker of a group draws its own
    minibatch from the group's shard (Sec. IV: the workers of a group hold the same data)."""
    rng = np.random.default_rng((w.seed if seed is None else seed) + 303)
    out = np.empty((steps, w.G, w.M_G, w.mu), dtype=np.int32)
    for k in range(steps):
        for g in range(w.G):
            for m in range(w.M_G):
                out[k, g, m] = rng.choice(w.rows, size=w.mu, replace=False, shuffle=False)
    return out


def make_delays(w: Workload, steps: int, eta: float = 1e-4, seed: Optional[int] = None) -> np.ndarray:
    """Per-worker compute times T_m^k ~ Exp(mean eta), float64 (steps, G, M_G), iid over workers
    and iterations (the compute-time model of Sec. II-B; eta = 1e-4 s is the value of Sec. VI)."""
    rng = np.random.default_rng((w.seed if seed is None else seed) + 202)
    u = rng.random((steps, w.G, w.M_G))
    return -eta * np.log1p(-u)


def gather_rows(Xs: Sequence[torch.Tensor], ys: Sequence[torch.Tensor], idx_step: np.ndarray):
    """Host copies of the rows one step touches: (G, mu, d) fp32 and (G, mu) labels.  Plain
    indexing, used to hand the oracle the same input values the GPU reads in place."""
    Xo, yo = [], []
    for g, (X, y) in enumerate(zip(Xs, ys)):
        rows = torch.as_tensor(np.asarray(idx_step[g], dtype=np.int64), device=X.device)
        Xo.append(X.index_select(0, rows).float().cpu().numpy())
        yo.append(y.index_select(0, rows).cpu().numpy())
    return np.stack(Xo), np.stack(yo)
