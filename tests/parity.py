"""Step-by-step comparison of the GPU library with the fp64 oracle (used by the -m gpu tests).

Teacher forcing: before every step the oracle's state is rounded to fp32 in place and copied to
the GPU, so both sides start the step from identical values and a flipped selection cannot fork
the run.  The shared state always comes from the oracle; nothing the GPU computed enters the
oracle.  Tolerances: vectors are compared twice -- norm-wise, max|a-b| <= tol * max|b|, and
element by element, |a_j - b_j| <= tol * |b_j| + tol * rms(b) with the rms over the element's
block of the parameter vector (a layer's weight matrix or bias vector: elements of one scale; an
element that is itself a cancelled sum is held to its block's typical size, not to its own);
scalars relatively; masks
must agree unless the oracle's statistic is within `edge` (relative) of the threshold or, where
said, within the measured error of the statistic itself.
"""
from __future__ import annotations

import time

import numpy as np
import torch

import oracle as O
from gcada_inputs import Workload, gather_rows, make_indices, make_shards, make_theta0
from paper_2201_04301_amd import Gcada
from paper_2201_04301_amd import binding as B


def oracle_config(w: Workload) -> O.Config:
    model = {"logreg": O.LOGISTIC, "mlp": O.MLP, "linreg": O.QUADRATIC}[w.model]
    return O.Config(model, list(w.widths), batch=w.mu, G=w.G, D=w.D, c=w.c, alpha=w.alpha,
                    beta1=w.beta1, beta2=w.beta2, eps=w.eps, l2=w.l2,
                    round_bf16=(2 if w.dtype == "bf16" else 0))


ATOL = 1e-12   # quantities below this are numerically zero for these workloads (e.g. the gradient
               # of a network whose loss has underflowed to 0)


def vec_err(a, b) -> float:
    """max|a-b| / max|b|, with an absolute floor so that two vanishing vectors compare equal."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.abs(a - b).max() / max(np.abs(b).max(), ATOL / 1e-5))


def param_blocks(w: Workload):
    """Slices of the parameter vector whose elements share a scale: per layer the weight matrix
    and the bias vector (one block for the linear models)."""
    if w.model != "mlp":
        return [slice(0, w.p)]
    out, off = [], 0
    for l in range(1, len(w.widths)):
        nw = w.widths[l] * w.widths[l - 1]
        out += [slice(off, off + nw), slice(off + nw, off + nw + w.widths[l])]
        off += nw + w.widths[l]
    return out


def block_rms(b, blocks):
    """rms of every block of b, as one value per element."""
    b = np.asarray(b, dtype=np.float64).reshape(-1)
    out = np.empty_like(b)
    for s in blocks:
        out[s] = np.sqrt(np.mean(b[s] * b[s])) if s.stop > s.start else 0.0
    return out


def flip_rows(w: Workload, a, b, tol, near_units, max_rows=4, max_share=2e-3):
    """bf16 MLP: which elements the element-by-element comparison has to leave out because a
    ReLU decision fell differently.  Both sides round the hidden activations to bf16, the GPU from
    its fp32 pre-activation, the oracle from the fp64 one; now and then the two land on either
    side of a bf16 rounding boundary, the activation differs by one bf16 ulp (2^-8 relative), and a
    unit of the NEXT layer whose pre-activation is within that of zero takes the other branch for
    that sample: one of the mu terms of that unit's row of the layer's weight gradient (and of its
    bias gradient) appears or disappears.  Such a row is found by the comparison itself (some
    element beyond `tol`), must belong to a unit the oracle reports close to a kink
    (`near_units`, bool per hidden unit, layer 1's units first), and there may be few of them per
    layer: max(max_rows, max_share * units).  When the layer is narrow and the minibatch short the
    flip also shows in the layers before it (it changes its sample's back-propagated signal by a
    1/sqrt(n_l) share, an earlier gradient element by a 1/sqrt(n_l mu) share): those layers are
    then left out too.  Returns (bool mask of left-out elements, rows left out).  Everything stays
    under the norm-wise check."""
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    b = np.asarray(b, dtype=np.float64).reshape(-1)
    skip = np.zeros(w.p, bool)
    offs, off = [], 0
    for l in range(1, len(w.widths)):
        offs.append(off)
        off += w.widths[l] * w.widths[l - 1] + w.widths[l]
    units0 = np.concatenate([[0], np.cumsum(w.widths[1:-1])])
    n_rows = 0
    for l in range(len(w.widths) - 2, 0, -1):                 # hidden layers, last one first
        nin, nout, o0 = w.widths[l - 1], w.widths[l], offs[l - 1]
        if skip[o0]:
            continue                                          # already left out with a later layer
        W = slice(o0, o0 + nout * nin)
        bb = slice(o0 + nout * nin, o0 + nout * nin + nout)
        rW = np.abs(a[W] - b[W]) / (np.abs(b[W]) + max(np.sqrt(np.mean(b[W] ** 2)), ATOL / 1e-5))
        rb = np.abs(a[bb] - b[bb]) / (np.abs(b[bb]) + max(np.sqrt(np.mean(b[bb] ** 2)), ATOL / 1e-5))
        bad = (rW.reshape(nout, nin).max(axis=1) > tol) | (rb > tol)
        rows = np.nonzero(bad)[0]
        if len(rows) == 0:
            continue
        assert len(rows) <= max(max_rows, max_share * nout), \
            f"layer {l}: {len(rows)} of {nout} rows differ element-wise -- more than flipped ReLU decisions explain"
        not_near = [int(o) for o in rows if not near_units[units0[l - 1] + o]]
        assert not not_near, f"layer {l}: rows {not_near} differ element-wise but their units are not near a kink"
        n_rows += len(rows)
        for o in rows:
            skip[o0 + o * nin: o0 + (o + 1) * nin] = True
            skip[o0 + nout * nin + o] = True
        if 1.0 / np.sqrt(nout * w.mu) > tol / 4:
            skip[:o0] = True
    return skip, n_rows


def elem_err(a, b, blocks=None, where=None, skip=None, extra=None) -> float:
    """max_j |a_j - b_j| / (|b_j| + rms(b) [+ extra_j]): the mixed element-wise error, rms taken
    over the element's block (same absolute floor as vec_err).  where: a list that receives a
    description of the worst element.  skip: elements left out.  extra: a further per-element
    scale the error is held against (where the arithmetic gives one)."""
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    b = np.asarray(b, dtype=np.float64).reshape(-1)
    worst = 0.0
    for s in (blocks if blocks is not None else [slice(0, b.size)]):
        bs, as_ = b[s], a[s]
        rms = max(float(np.sqrt(np.mean(bs * bs))), ATOL / 1e-5)
        den = np.abs(bs) + rms
        if extra is not None:
            den = den + extra[s]
        r = np.abs(as_ - bs) / den
        if skip is not None:
            r = np.where(skip[s], 0.0, r)
        j = int(np.argmax(r))
        if r[j] > worst:
            worst = float(r[j])
            if where is not None:
                where[:] = [f"element {s.start + j} (block {s.start}:{s.stop}, rms {rms:.3e}, max {np.abs(bs).max():.3e}): "
                            f"{as_[j]:.9e} vs {bs[j]:.9e}"]
    return worst


def check_vec(a, b, tol, what, blocks=None, skip=None, extra=None) -> float:
    """Assert both vector criteria; returns the norm-wise error."""
    e = vec_err(a, b)
    assert e <= tol, f"{what}: error {e:.3e} (norm-wise)"
    where = []
    ee = elem_err(a, b, blocks, where, skip, extra)
    assert ee <= tol, f"{what}: error {ee:.3e} (element-wise) at {where}"
    return e


def check_theta(w, theta_gpu, orc, uploaded: bool, tol, what) -> float:
    """theta after the update: the step divides by sqrt(eps + vhat), so an absolute error da in
    the aggregate moves theta_j by up to kappa_j * da, kappa_j = alpha (1-beta1) / sqrt(eps + vhat_j)
    (large while vhat_j ~ 0).  When no group uploaded, the aggregate is the forced state itself and
    only the update's own rounding remains.  Returns max error / max|theta|."""
    th_o = orc.theta
    scale = np.abs(th_o).max()
    err = np.abs(np.asarray(theta_gpu, dtype=np.float64) - th_o)
    if uploaded:
        kappa = w.alpha * (1 - w.beta1) / np.sqrt(w.eps + orc.vhat)
        bound = tol * scale + 2 * kappa * tol * np.abs(orc.agg).max()
    else:
        bound = np.full_like(err, 1e-6 * scale)
    j = int(np.argmax(err - bound))
    assert err[j] <= bound[j], f"{what}: theta[{j}] error {err[j]:.3e} > bound {bound[j]:.3e}"
    return float(err.max() / scale)


def rel_err(a: float, b: float) -> float:
    return abs(a - b) / max(abs(b), ATOL / 1e-5)


def round_state_to_f32(orc: O.Oracle):
    for name in ("theta", "h", "vhat", "agg", "theta_stale", "last"):
        a = getattr(orc, name)
        a[...] = a.astype(np.float32).astype(np.float64)


def push_state(orc: O.Oracle, gpu: Gcada):
    gpu.set_state(orc.theta, orc.h, orc.vhat, orc.agg, orc.theta_stale, orc.last, orc.tau,
                  orc.ring, orc.k)


def teacher_forced(w: Workload, steps, Xs, ys, idx=None, tol=1e-5, edge=1e-6, kink_tol=None,
                   kink_grad_tol=5e-2, stat_vs_threshold=False, verbose=False, server_rule_L=None, lazy_store=None,
                   edge_stat_err=False, options=(), kink_unit_tol=None):
    """Run `steps` iterations; idx: int32 (steps, G, mu) row ids or None for the cyclic window.
    kink_tol (MLP): a group is "near a ReLU kink" in a step when some hidden pre-activation of the
    oracle lies within kink_tol (relative to the sum of the magnitudes of its terms) of zero.
    There both subgradients are valid results and a lower-precision evaluation may take the other
    one, so for such a group only a loose gradient check (kink_grad_tol) is made and its
    statistic / mask are not compared; the state checks of that step are skipped when such a
    group takes part in the aggregate.
    stat_vs_threshold (bf16): the statistic's error is measured against max(stat, rhs) -- the
    statistic only matters through its comparison with the threshold, and once the gradients have
    collapsed below the bf16 noise floor its relative error alone says nothing.
    edge_stat_err (bf16): a mask difference is also accepted where the oracle's statistic lies no
    further from the threshold than the GPU's statistic lies from the oracle's -- that error has
    just been held to `tol`, and a statistic that is off by it may land on the other side.  The
    plain rule (|stat - rhs| < edge * rhs with edge = 1e-6) stays in force otherwise.
    options: (option, value) pairs for gcada_set_option.
    kink_unit_tol (bf16 MLP): the same closeness measure per hidden unit; the element-by-element
    comparison leaves out the few rows in which a ReLU decision fell differently (flip_rows: found
    by the comparison, confirmed by this measure, bounded in number); they stay under the
    norm-wise check.  The number of such rows is returned.
    The element-wise check of the aggregate and the moments holds their error against the sizes
    of what was added: agg_new = agg_old + sum over the uploading groups of (fresh - stored), so
    its error is at most the sum of those gradients' errors, each held to tol (|g_j| + rms(g));
    h inherits (1 - beta1) of it and v-hat 2 (1 - beta2) |agg_j| of it (Eq. (8a), (8b)).
    server_rule_L: G smoothness constants -> both sides run the server-side rule of Sec. IV
    (selection from the iterates before the gradients; only selected groups evaluate one); then
    the gradients of the selected groups only are compared, and `stat` is the rule's left side.
    lazy_store: 0 / 1 sets GCADA_OPT_LAZY_GRADIENT_STORE; with 1 the fresh gradient of a group
    that does not upload is not materialised, so only the uploading groups' gradients are compared
    (the statistic, which is made of the whole gradient difference, is compared for all).
    Returns a dict of the worst errors seen.  Raises AssertionError on a violation."""
    orc = O.Oracle(oracle_config(w), make_theta0(w))
    gpu = Gcada.from_workload(w)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    if lazy_store is not None:
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_LAZY_GRADIENT_STORE, int(lazy_store))
    for opt, val in options:
        B.gcada_set_option(gpu.ctx, opt, val)
    if server_rule_L is not None:
        orc.set_rule(1, server_rule_L)
        gpu.set_rule("server", server_rule_L)
    idx_dev = torch.as_tensor(idx, device="cuda") if idx is not None else None
    worst = dict(grad=0.0, grad_elem=0.0, stat=0.0, rhs=0.0, loss=0.0, theta=0.0, h=0.0, vhat=0.0, agg=0.0,
                 ring=0.0, edge_flips=0, selected=0, kink_groups=0, clean_groups=0, state_steps=0,
                 forced_late=0, by_statistic=0, max_age=0, flip_rows=0)
    rows_all = [X.shape[0] for X in Xs]
    blocks = param_blocks(w)
    t_said = time.time()
    for k in range(steps):
        if time.time() - t_said > 30:        # a long case says where it is
            print(f"  ... step {k} of {steps}", flush=True)
            t_said = time.time()
        round_state_to_f32(orc)
        push_state(orc, gpu)
        tau_before = orc.tau.copy()
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
        near = (orc.kink < kink_tol) if kink_tol is not None else np.zeros(w.G, bool)
        worst["kink_groups"] += int(near.sum())
        worst["clean_groups"] += int((~near).sum())
        skips = [None] * w.G
        if kink_unit_tol is not None and w.model == "mlp" and len(w.widths) > 2:
            near_units = orc.kink_unit < kink_unit_tol                 # (G, hidden units)
            for g in range(w.G):
                if (server_rule_L is not None and not mask_o[g]) or (lazy_store and not out["mask"][g]):
                    continue                                           # no gradient to compare
                skips[g], nr = flip_rows(w, out["grad"][g], orc.grad[g], tol, near_units[g])
                worst["flip_rows"] += nr
        # a1: fresh gradients, per group
        for g in range(w.G):
            if server_rule_L is not None and not mask_o[g]:
                continue                      # evaluated nothing on either side
            if lazy_store and not out["mask"][g]:
                continue                      # not materialised
            e = vec_err(out["grad"][g], orc.grad[g])
            if near[g]:
                assert e <= kink_grad_tol, f"step {k} group {g} (near a kink): gradient error {e:.3e}"
                continue
            worst["grad"] = max(worst["grad"], e)
            assert e <= tol, f"step {k} group {g}: gradient error {e:.3e}"
            where = []
            ee = elem_err(out["grad"][g], orc.grad[g], blocks, where, skips[g])
            worst["grad_elem"] = max(worst["grad_elem"], ee)
            assert ee <= tol, f"step {k} group {g}: gradient error {ee:.3e} (element-wise) at {where}"
        # a2: statistic, threshold, mask
        s_o = orc.stat
        for g in range(w.G):
            if near[g]:
                continue
            # stat_g is the squared norm of a difference of two gradients that are each pinned to
            # a relative `tol`: below (tol * ||g||)^2 it is rounding noise (exactly so when the
            # two iterates coincide, as at step 0), hence that floor under the reference value
            gn2 = float(np.dot(orc.grad[g], orc.grad[g]))
            e = abs(out["stat"][g] - s_o[g]) / max(abs(s_o[g]), tol * gn2, ATOL / 1e-5)
            if stat_vs_threshold:
                e = abs(out["stat"][g] - s_o[g]) / max(s_o[g], orc.rhs, tol * gn2, ATOL)
            worst["stat"] = max(worst["stat"], e)
            assert e <= tol, f"step {k} group {g}: stat {out['stat'][g]} vs {s_o[g]} ({e:.3e})"
        e = rel_err(out["rhs"], orc.rhs)
        worst["rhs"] = max(worst["rhs"], e)
        assert e <= tol, f"step {k}: rhs {out['rhs']} vs {orc.rhs}"
        flips = out["mask"] != mask_o
        for g in np.nonzero(flips)[0]:
            if near[g]:
                continue
            slack = abs(out["stat"][g] - s_o[g]) if edge_stat_err else 0.0
            assert abs(s_o[g] - orc.rhs) < edge * orc.rhs or abs(s_o[g] - orc.rhs) <= slack, \
                f"step {k} group {g}: mask {out['mask'][g]} vs {mask_o[g]}, stat {s_o[g]} rhs {orc.rhs}"
            worst["edge_flips"] += 1
        worst["selected"] += int(mask_o.sum())
        if k > 0:       # uploads forced by the age bound, and uploads the statistic asked for
            worst["forced_late"] += int(((mask_o != 0) & (tau_before >= w.D)).sum())
            worst["by_statistic"] += int(((mask_o != 0) & (tau_before < w.D)).sum())
        worst["max_age"] = max(worst["max_age"], int(tau_before.max()) if k > 0 else 0)
        assert np.array_equal(gpu.mask_out.cpu().numpy(), out["mask"])
        e = rel_err(out["loss"], loss_o)
        worst["loss"] = max(worst["loss"], e)
        assert e <= tol, f"step {k}: loss {out['loss']} vs {loss_o}"
        assert abs(float(gpu.loss_out.item()) - loss_o) <= (1e-6 + tol) * abs(loss_o) + ATOL
        if flips.any() or (near & (mask_o != 0)).any():
            continue   # knife-edge / kink: the states legitimately differ after this step
        worst["state_steps"] += 1
        # a3 / a4
        sel = np.nonzero(mask_o)[0]
        skip_any = None
        if any(skips[g] is not None for g in sel):
            skip_any = np.zeros(w.p, bool)
            for g in sel:
                if skips[g] is not None:
                    skip_any |= skips[g]
        added = np.zeros(w.p)
        for g in sel:
            added += np.abs(orc.grad[g]) + block_rms(orc.grad[g], blocks)
        extra = dict(agg=added, h=(1 - w.beta1) * added,
                     vhat=2 * (1 - w.beta2) * np.abs(orc.agg) * (np.abs(orc.agg) + block_rms(orc.agg, blocks) + added))
        for name in ("agg", "h", "vhat"):
            worst[name] = max(worst[name], check_vec(st[name], getattr(orc, name), tol, f"step {k}: {name}", blocks,
                                                     skip_any, extra[name]))
        worst["theta"] = max(worst["theta"], check_theta(w, st["theta"], orc, bool(mask_o.any()), tol, f"step {k}"))
        np.testing.assert_array_equal(st["tau"], orc.tau)
        for g in range(w.G):
            check_vec(st["last"][g], orc.last[g], tol, f"step {k}: stored gradient of group {g}", blocks,
                      skips[g] if mask_o[g] else None)
        check_vec(st["theta_stale"], orc.theta_stale, tol, f"step {k}: stale iterates")
        e = vec_err(st["dtheta_sq"], orc.ring)
        worst["ring"] = max(worst["ring"], e)
        assert e <= tol, f"step {k}: history error {e:.3e}"
        if verbose:
            print(k, mask_o, loss_o, flush=True)
    gpu.close()
    return worst


def free_running(w: Workload, steps, Xs, ys, idx=None, options=()):
    """Both sides run `steps` iterations on their own from theta^0.  Returns per-step masks and
    losses of both and the final iterates.  options: (option, value) pairs for gcada_set_option."""
    orc = O.Oracle(oracle_config(w), make_theta0(w))
    gpu = Gcada.from_workload(w)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    for opt, val in options:
        B.gcada_set_option(gpu.ctx, opt, val)
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


def synthetic_state(w: Workload, seed=7, tau=None):
    """A valid mid-run state made from seeded random numbers only (no run needed): ages in [1, D]
    (drawn, or the G given ones), groups of equal age share their stale iterate, moments and stored
    gradients of plausible size."""
    rng = np.random.default_rng(seed)
    p, G, D = w.p, w.G, w.D
    theta0 = make_theta0(w).astype(np.float64)
    scale = max(np.abs(theta0).max(), 0.05)
    # hist[t] = iterate t steps ago: further back, further away from the current iterate
    hist = [theta0 + 0.02 * scale * (t + 1) * rng.standard_normal(p) for t in range(D + 1)]
    drawn = rng.integers(1, D + 1, size=G).astype(np.int32)
    tau = drawn if tau is None else np.asarray(tau, dtype=np.int32)
    f32 = lambda a: np.asarray(a, np.float32).astype(np.float64)
    st = dict(theta=f32(hist[0]), h=f32(0.1 * rng.standard_normal(p)), vhat=f32(rng.random(p) * 0.5),
              agg=f32(rng.standard_normal(p)), theta_stale=f32(np.stack([hist[t] for t in tau])),
              last=f32(rng.standard_normal((G, p))), tau=tau,
              dtheta_sq=rng.random(D) * 1e-3 * p * scale ** 2, k=D + 3)
    return st


def sampled_oracle_step(w: Workload, st, Xs, ys, idx_step, groups):
    """The oracle's step for the sampled `groups` only, from the state `st` of the whole workload
    (each group's gradients, statistic and mask depend on its own shard and state only)."""
    ws = replace_groups(w, len(groups))
    orc = O.Oracle(oracle_config(ws), make_theta0(w))
    for name in ("theta", "h", "vhat", "agg"):
        getattr(orc, name)[...] = st[name]
    orc.theta_stale[...] = st["theta_stale"][groups]
    orc.last[...] = st["last"][groups]
    orc.tau[...] = st["tau"][groups]
    orc.ring[...] = st["dtheta_sq"]
    orc.k = st["k"]
    Xmb, ymb = gather_rows([Xs[g] for g in groups], [ys[g] for g in groups], idx_step[groups])
    mask_o, _ = orc.step(Xmb, ymb)
    return orc, mask_o


def sampled_groups_step(w: Workload, Xs, ys, idx_step, groups, tol=1e-5, edge=1e-6, kink_tol=None,
                        seed=7, lazy_store=None, edge_stat_err=False, options=(), reference=None,
                        whole_state=False, kink_unit_tol=None):
    """One iteration of the full-size workload on the GPU from a synthetic state; the oracle
    evaluates only the sampled `groups` and those groups' gradients, statistics and masks are
    compared.  reference: (state, oracle, mask) of an earlier call on the same inputs (the oracle's
    step is the expensive part; it does not depend on the GPU options).
    whole_state: the workload must make the sampled groups the ONLY ones that can be selected
    (their age is D, everybody else is younger, and c is so large that no statistic reaches the
    threshold): then the aggregate, moments, iterate, history entry, ages and stored gradients
    after the step are determined by what the oracle evaluated, and the whole state is compared."""
    groups = list(groups)
    if reference is None:
        tau = None
        if whole_state:
            rng = np.random.default_rng(seed + 1)
            tau = rng.integers(1, w.D, size=w.G)             # 1 .. D-1: cannot be forced
            tau[groups] = w.D
        st = synthetic_state(w, seed, tau)
        orc, mask_o = sampled_oracle_step(w, st, Xs, ys, idx_step, groups)
    else:
        st, orc, mask_o = reference
    gpu = Gcada.from_workload(w)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    gpu.set_state(**st)
    if lazy_store is not None:
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_LAZY_GRADIENT_STORE, int(lazy_store))
    for opt, val in options:
        B.gcada_set_option(gpu.ctx, opt, val)
    gpu.step(torch.as_tensor(idx_step, device="cuda").contiguous())
    out = gpu.outputs()
    blocks = param_blocks(w)
    worst = dict(grad=0.0, grad_elem=0.0, stat=0.0, rhs=rel_err(out["rhs"], orc.rhs), kink_groups=0,
                 selected=int(mask_o.sum()), ages=sorted(set(int(t) for t in st["tau"][groups])))
    assert worst["rhs"] <= 1e-9
    near_any = False
    skips = [None] * len(groups)
    if kink_unit_tol is not None:
        near_units = orc.kink_unit < kink_unit_tol
        worst["flip_rows"] = 0
        for j, g in enumerate(groups):
            if not lazy_store or bool(out["mask"][g]):
                skips[j], nr = flip_rows(w, out["grad"][g], orc.grad[j], tol, near_units[j])
                worst["flip_rows"] += nr
    for j, g in enumerate(groups):
        near = kink_tol is not None and orc.kink[j] < kink_tol
        materialised = not lazy_store or bool(out["mask"][g])
        e = vec_err(out["grad"][g], orc.grad[j]) if materialised else 0.0
        if near:
            worst["kink_groups"] += 1
            near_any = near_any or bool(mask_o[j])
            assert e <= 5e-2, f"group {g} (near a kink): gradient error {e:.3e}"
            continue
        worst["grad"] = max(worst["grad"], e)
        assert e <= tol, f"group {g}: gradient error {e:.3e}"
        if materialised:
            where = []
            ee = elem_err(out["grad"][g], orc.grad[j], blocks, where, skips[j])
            worst["grad_elem"] = max(worst["grad_elem"], ee)
            assert ee <= tol, f"group {g}: gradient error {ee:.3e} (element-wise) at {where}"
        gn2 = float(np.dot(orc.grad[j], orc.grad[j]))
        e = abs(out["stat"][g] - orc.stat[j]) / max(abs(orc.stat[j]), tol * gn2, ATOL / 1e-5)
        worst["stat"] = max(worst["stat"], e)
        assert e <= tol, f"group {g}: stat {out['stat'][g]} vs {orc.stat[j]}"
        if out["mask"][g] != mask_o[j]:
            slack = abs(out["stat"][g] - orc.stat[j]) if edge_stat_err else 0.0
            d = abs(orc.stat[j] - orc.rhs)
            assert d < edge * orc.rhs or d <= slack, f"group {g}: mask differs"
    if whole_state:
        assert mask_o.all()
        others = np.setdiff1d(np.arange(w.G), groups)
        expect = np.zeros(w.G, np.uint8)
        expect[groups] = 1
        np.testing.assert_array_equal(out["mask"], expect)
        after = gpu.get_state()
        assert after["k"] == st["k"] + 1
        tau_expect = st["tau"] + 1
        tau_expect[groups] = 1
        np.testing.assert_array_equal(after["tau"], tau_expect)
        # groups that did not upload keep their stored gradient and their stale iterate, bit for bit
        np.testing.assert_array_equal(after["last"][others], st["last"][others].astype(np.float32))
        np.testing.assert_array_equal(after["theta_stale"][others], st["theta_stale"][others].astype(np.float32))
        if not near_any:
            skip_any = None
            if kink_unit_tol is not None:
                skip_any = np.zeros(w.p, bool)
                for sk in skips:
                    if sk is not None:
                        skip_any |= sk
            added = np.zeros(w.p)
            for j in range(len(groups)):
                added += np.abs(orc.grad[j]) + block_rms(orc.grad[j], blocks)
            extra = dict(agg=added, h=(1 - w.beta1) * added,
                         vhat=2 * (1 - w.beta2) * np.abs(orc.agg) * (np.abs(orc.agg) + block_rms(orc.agg, blocks) + added))
            for name in ("agg", "h", "vhat"):
                worst[name] = check_vec(after[name], getattr(orc, name), tol, name, blocks, skip_any, extra[name])
            worst["theta"] = check_theta(w, after["theta"], orc, True, tol, "after the step")
            for j, g in enumerate(groups):
                check_vec(after["last"][g], orc.last[j], tol, f"stored gradient of group {g}", blocks, skips[j])
                np.testing.assert_array_equal(after["theta_stale"][g], st["theta"].astype(np.float32))
            worst["ring"] = vec_err(after["dtheta_sq"], orc.ring)
            assert worst["ring"] <= tol, f"history error {worst['ring']:.3e}"
    gpu.close()
    return worst, (st, orc, mask_o)


def replace_groups(w: Workload, G: int) -> Workload:
    from dataclasses import replace
    return replace(w, G=G)
