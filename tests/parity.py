"""Step-by-step comparison of the GPU library with the fp64 oracle (used by the -m gpu tests).

Teacher forcing: before every step the oracle's state is rounded to fp32 in place and copied to
the GPU, so both sides start the step from identical values and a flipped selection cannot fork
the run.  The shared state always comes from the oracle; nothing the GPU computed enters the
oracle.  Tolerances: vectors are compared norm-wise,
max|a-b| <= tol * max|b|; scalars relatively; masks must agree unless the oracle's statistic is
within `edge` (relative) of the threshold.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle as O
from gcada_inputs import Workload, gather_rows, make_indices, make_shards, make_theta0
from paper_2201_04301_amd import Gcada


def oracle_config(w: Workload) -> O.Config:
    model = O.LOGISTIC if w.model == "logreg" else O.MLP
    return O.Config(model, list(w.widths), batch=w.mu, G=w.G, D=w.D, c=w.c, alpha=w.alpha,
                    beta1=w.beta1, beta2=w.beta2, eps=w.eps, l2=w.l2,
                    round_bf16=(w.dtype == "bf16"))


def vec_err(a, b) -> float:
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.abs(b).max()
    return float(np.abs(a - b).max() / den) if den > 0 else float(np.abs(a).max())


def round_state_to_f32(orc: O.Oracle):
    for name in ("theta", "h", "vhat", "agg", "theta_stale", "last"):
        a = getattr(orc, name)
        a[...] = a.astype(np.float32).astype(np.float64)


def push_state(orc: O.Oracle, gpu: Gcada):
    gpu.set_state(orc.theta, orc.h, orc.vhat, orc.agg, orc.theta_stale, orc.last, orc.tau,
                  orc.ring, orc.k)


def teacher_forced(w: Workload, steps, Xs, ys, idx=None, tol=1e-5, edge=1e-6, check_steps=None,
                   groups=None, verbose=False):
    """Run `steps` iterations; idx: int32 (steps, G, mu) row ids or None for the cyclic window.
    Returns a dict of the worst errors seen.  Raises AssertionError on a violation."""
    orc = O.Oracle(oracle_config(w), make_theta0(w))
    gpu = Gcada.from_workload(w)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    idx_dev = torch.as_tensor(idx, device="cuda") if idx is not None else None
    worst = dict(grad=0.0, stat=0.0, rhs=0.0, loss=0.0, theta=0.0, h=0.0, vhat=0.0, agg=0.0,
                 ring=0.0, edge_flips=0, selected=0)
    rows_all = [X.shape[0] for X in Xs]
    for k in range(steps):
        round_state_to_f32(orc)
        push_state(orc, gpu)
        if idx is not None:
            step_idx = idx[k]
        else:
            step_idx = np.stack([O.cyclic_window(k, w.mu, rows_all[g]) for g in range(w.G)])
        Xmb, ymb = gather_rows(Xs, ys, step_idx)
        mask_o, loss_o = orc.step(Xmb, ymb)
        gpu.step(idx_dev[k].contiguous() if idx_dev is not None else None)
        out = gpu.outputs()
        st = gpu.get_state()
        assert st["k"] == orc.k == k + 1
        # a1: fresh gradients, per group
        for g in range(w.G):
            e = vec_err(out["grad"][g], orc.grad[g])
            worst["grad"] = max(worst["grad"], e)
            assert e <= tol, f"step {k} group {g}: gradient error {e:.3e}"
        # a2: statistic, threshold, mask
        s_o = orc.stat
        for g in range(w.G):
            e = abs(out["stat"][g] - s_o[g]) / s_o[g] if s_o[g] > 0 else abs(out["stat"][g])
            worst["stat"] = max(worst["stat"], e)
            assert e <= tol, f"step {k} group {g}: stat {out['stat'][g]} vs {s_o[g]} ({e:.3e})"
        e = abs(out["rhs"] - orc.rhs) / orc.rhs if orc.rhs > 0 else abs(out["rhs"])
        worst["rhs"] = max(worst["rhs"], e)
        assert e <= tol, f"step {k}: rhs {out['rhs']} vs {orc.rhs}"
        flips = out["mask"] != mask_o
        for g in np.nonzero(flips)[0]:
            assert abs(s_o[g] - orc.rhs) < edge * orc.rhs, \
                f"step {k} group {g}: mask {out['mask'][g]} vs {mask_o[g]}, stat {s_o[g]} rhs {orc.rhs}"
            worst["edge_flips"] += 1
        worst["selected"] += int(mask_o.sum())
        assert np.array_equal(gpu.mask_out.cpu().numpy(), out["mask"])
        e = abs(out["loss"] - loss_o) / abs(loss_o)
        worst["loss"] = max(worst["loss"], e)
        assert e <= tol, f"step {k}: loss {out['loss']} vs {loss_o}"
        assert abs(float(gpu.loss_out.item()) - loss_o) <= 1e-6 * abs(loss_o) + tol * abs(loss_o)
        if flips.any():
            continue   # knife-edge: the states legitimately differ after this step
        # a3 / a4
        for name in ("agg", "h", "vhat"):
            e = vec_err(st[name], getattr(orc, name))
            worst[name] = max(worst[name], e)
            assert e <= tol, f"step {k}: {name} error {e:.3e}"
        # theta: the update divides by sqrt(eps + vhat), so an absolute error da in the aggregate
        # moves theta_j by up to kappa_j * da with kappa_j = alpha (1-beta1) / sqrt(eps + vhat_j)
        # (large while vhat_j ~ 0).  When no group uploaded, the aggregate is the forced state
        # itself and only the update's own rounding remains.
        th_o = orc.theta
        scale = np.abs(th_o).max()
        err = np.abs(st["theta"].astype(np.float64) - th_o)
        if mask_o.any():
            kappa = w.alpha * (1 - w.beta1) / np.sqrt(w.eps + orc.vhat)
            bound = tol * scale + 2 * kappa * tol * np.abs(orc.agg).max()
        else:
            bound = np.full_like(err, 1e-6 * scale)
        worst["theta"] = max(worst["theta"], float(err.max() / scale))
        j = int(np.argmax(err - bound))
        assert err[j] <= bound[j], f"step {k}: theta[{j}] error {err[j]:.3e} > bound {bound[j]:.3e}"
        np.testing.assert_array_equal(st["tau"], orc.tau)
        e = vec_err(st["last"], orc.last)
        assert e <= tol, f"step {k}: stored gradients error {e:.3e}"
        e = vec_err(st["theta_stale"], orc.theta_stale)
        assert e <= tol, f"step {k}: stale iterates error {e:.3e}"
        e = vec_err(st["dtheta_sq"], orc.ring)
        worst["ring"] = max(worst["ring"], e)
        assert e <= tol, f"step {k}: history error {e:.3e}"
        if verbose:
            print(k, mask_o, loss_o, flush=True)
    gpu.close()
    return worst


def free_running(w: Workload, steps, Xs, ys, idx=None):
    """Both sides run `steps` iterations on their own from theta^0.  Returns per-step masks and
    losses of both and the final iterates."""
    orc = O.Oracle(oracle_config(w), make_theta0(w))
    gpu = Gcada.from_workload(w)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    idx_dev = torch.as_tensor(idx, device="cuda") if idx is not None else None
    masks_g = torch.zeros(steps, w.G, dtype=torch.uint8, device="cuda")
    loss_g = torch.zeros(steps, dtype=torch.float32, device="cuda")
    rows_all = [X.shape[0] for X in Xs]
    for k in range(steps):
        gpu.step(idx_dev[k].contiguous() if idx_dev is not None else None,
                 mask_out=masks_g[k], loss_out=loss_g[k:k + 1])
    torch.cuda.synchronize()
    masks_o = np.zeros((steps, w.G), np.uint8)
    loss_o = np.zeros(steps)
    for k in range(steps):
        step_idx = idx[k] if idx is not None else np.stack(
            [O.cyclic_window(k, w.mu, rows_all[g]) for g in range(w.G)])
        Xmb, ymb = gather_rows(Xs, ys, step_idx)
        masks_o[k], loss_o[k] = orc.step(Xmb, ymb)
    theta_g = gpu.get_state()["theta"]
    gpu.close()
    return dict(masks_gpu=masks_g.cpu().numpy(), masks_oracle=masks_o,
                loss_gpu=loss_g.cpu().numpy().astype(np.float64), loss_oracle=loss_o,
                theta_gpu=theta_g, theta_oracle=orc.theta.copy())
