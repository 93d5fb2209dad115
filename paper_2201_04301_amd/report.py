"""Baselines as special cases of the same path, with the paper's per-iteration metrics.

Runs three schemes on ONE synthetic data set (the geometry of the paper's experiment, Sec. VI:
linear regression with the quadratic error loss, M = 12 workers) through the library and
reports training loss against the MODELLED wall-clock time, communication load and computation
load of Sec. II-B (compute times T_m^k ~ Exp(eta), seeded; Eq. (4)-(6)):

* G-CADA        G groups of M_G workers, rule constant c (Sec. IV);
* CADA          the same path with M_G = 1: every worker is its own group (Sec. III);
* D-Adam        CADA with c = 0: every worker uploads every iteration (distributed Adam, Sec. V).

The selection statistic is the library's (same-minibatch gradient difference), so CADA here is
"CADA with that statistic".  The modelled metrics come from gcada_cost_model; nothing here is a
measurement of the GPU.  Usage:

    python -m paper_2201_04301_amd.report [--iters 400] [--rows-per-worker 2000] [--json out.json]
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import numpy as np

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if _ROOT not in sys.path:
    sys.path.insert(0, _ROOT)


def harmonic(n: int) -> float:
    return sum(1.0 / i for i in range(1, n + 1))


def run_scheme(name, w, Xs, ys, iters, eta=1e-4):
    """One run of `iters` iterations from theta^0 = 0.  Returns per-iteration arrays: minibatch
    loss, number of selected groups, modelled time, communication and computation load."""
    import torch
    from gcada_inputs import make_delays, make_indices, make_theta0
    from . import Gcada

    gpu = Gcada.from_workload(w)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    idx = torch.as_tensor(make_indices(w, iters), device="cuda")
    masks = torch.zeros(iters, w.G, dtype=torch.uint8, device="cuda")
    losses = torch.zeros(iters, dtype=torch.float32, device="cuda")
    for k in range(iters):
        gpu.step(idx[k].contiguous(), mask_out=masks[k], loss_out=losses[k:k + 1])
    torch.cuda.synchronize()
    m = masks.cpu().numpy()
    T = make_delays(w, iters, eta=eta)
    t = np.zeros(iters)
    comm = np.zeros(iters)
    comp = np.zeros(iters)
    for k in range(iters):
        t[k], comm[k], comp[k] = gpu.cost_model(m[k], T[k])
    gpu.close()
    return dict(name=name, G=w.G, M_G=w.M_G, mu=w.mu, c=w.c, loss=losses.cpu().numpy().astype(np.float64),
                selected=m.sum(1).astype(np.int64), time=t, comm=comm, comp=comp)


def schemes(rows_per_worker: int, mu: int, D: int, c_gcada: float, c_cada: float):
    """The three workloads on M = 12 workers; G-CADA's group shard is the union of its four
    workers' shards (storage redundancy r = M_G, Sec. IV)."""
    from gcada_inputs import CONFIGS, scaled
    base = CONFIGS["linreg_784"]
    per_worker = scaled(base, name="workers", G=12, M_G=1, rows=rows_per_worker, mu=mu, D=D)
    return {
        "G-CADA": scaled(base, name="G-CADA", G=3, M_G=4, rows=4 * rows_per_worker, mu=mu, D=D, c=c_gcada),
        "CADA": scaled(per_worker, name="CADA", c=c_cada),
        "D-Adam": scaled(per_worker, name="D-Adam", c=0.0),
    }, per_worker


def first_reach(loss_smooth, level):
    hit = np.nonzero(loss_smooth <= level)[0]
    return int(hit[0]) if hit.size else None


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--iters", type=int, default=400)
    ap.add_argument("--rows-per-worker", type=int, default=2000)
    ap.add_argument("--mu", type=int, default=64)
    ap.add_argument("--D", type=int, default=10)
    ap.add_argument("--c-gcada", type=float, default=3.0, help="0.3 on the sum over D = 10 history terms")
    ap.add_argument("--c-cada", type=float, default=20.0, help="2 on the sum over D = 10 history terms")
    ap.add_argument("--eta", type=float, default=1e-4)
    ap.add_argument("--json", type=str, default=None)
    a = ap.parse_args(argv)

    import torch
    from gcada_inputs import make_shards
    ws, per_worker = schemes(a.rows_per_worker, a.mu, a.D, a.c_gcada, a.c_cada)
    Xw, yw = make_shards(per_worker, "cuda")                 # 12 worker shards
    Xg = [torch.cat(Xw[4 * g:4 * g + 4]).contiguous() for g in range(3)]
    yg = [torch.cat(yw[4 * g:4 * g + 4]).contiguous() for g in range(3)]

    runs = {}
    for name, w in ws.items():
        Xs, ys = (Xg, yg) if name == "G-CADA" else (Xw, yw)
        runs[name] = run_scheme(name, w, Xs, ys, a.iters, a.eta)

    # smoothed minibatch loss (window of 10 iterations) against the cumulative metrics
    out = {"eta_s": a.eta, "iters": a.iters, "schemes": {}}
    print(f"# loss vs modelled wall-clock / communication / computation, {a.iters} iterations, eta = {a.eta} s")
    print("| scheme | G x M_G | c | mean selected | time/iter (model) | closed form if all selected | comm/iter | comp/iter |")
    print("|---|---|---|---|---|---|---|---|")
    for name, r in runs.items():
        G, M_G = r["G"], r["M_G"]
        closed = a.eta / M_G * harmonic(G)                      # Eq. (10)/(14): max of G minima of M_G
        print(f"| {name} | {G} x {M_G} | {r['c']:g} | {r['selected'].mean():.2f} | {r['time'].mean():.3e} s | "
              f"{closed:.3e} s | {r['comm'].mean():.2f} | {r['comp'].mean():.1f} |")
    levels = None
    ker = np.ones(10) / 10
    for name, r in runs.items():
        sm = np.convolve(r["loss"], ker, mode="valid")
        r["loss_smooth"] = np.concatenate([np.full(9, sm[0]), sm])
    final = max(r["loss_smooth"][-1] for r in runs.values())
    start = min(r["loss_smooth"][0] for r in runs.values())
    levels = [start - f * (start - final) for f in (0.5, 0.9, 0.99)]
    print("\n| loss level | scheme | iterations | modelled time | communication | computation |")
    print("|---|---|---|---|---|---|")
    for lv in levels:
        for name, r in runs.items():
            k = first_reach(r["loss_smooth"], lv)
            if k is None:
                print(f"| {lv:.4f} | {name} | not reached | | | |")
            else:
                print(f"| {lv:.4f} | {name} | {k + 1} | {r['time'][:k + 1].sum():.4f} s | "
                      f"{r['comm'][:k + 1].sum():.0f} | {r['comp'][:k + 1].sum():.0f} |")
    for name, r in runs.items():
        out["schemes"][name] = {k: (v.tolist() if isinstance(v, np.ndarray) else v) for k, v in r.items()}
    if a.json:
        with open(a.json, "w") as f:
            json.dump(out, f)
    return runs


if __name__ == "__main__":
    main()
