"""GPU parity of the MLP path (MFMA GEMMs, fp32 and bf16) with the fp64 oracle."""
import numpy as np
import pytest
import torch

from gcada_inputs import CONFIGS, make_indices, make_shards, scaled

pytestmark = pytest.mark.gpu

KINK = 5e-8   # fp32: a hidden pre-activation this close to 0 (relative) may flip its ReLU


@pytest.fixture(scope="module")
def par():
    import parity
    return parity


def _say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("widths,mu,G,rows,steps", [
    ((20, 12, 5), 16, 3, 50, 15),             # everything ragged, one hidden layer
    ((30, 6), 24, 2, 60, 12),                 # no hidden layer: softmax regression
    ((100, 70, 50, 7), 40, 3, 90, 12),        # two hidden layers
    ((784, 200, 10), 64, 4, 300, 12),         # layer widths of the fp32 configuration, small batch
    ((130, 260, 129, 3), 130, 2, 200, 8),     # several GEMM tiles with ragged edges
    ((60, 40, 50), 32, 3, 120, 10),           # fifty classes: the wide output-layer tile
    ((48, 64, 32), 70, 2, 150, 8),            # 32 classes: the narrow output-layer tile, full; two row blocks
])
def test_mlp_f32_shapes(par, widths, mu, G, rows, steps):
    w = scaled(CONFIGS["mlp_784"], name="mlp_f32", widths=widths, mu=mu, G=G, rows=rows, D=4)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    idx = make_indices(w, steps)
    worst = par.teacher_forced(w, steps, Xs, ys, idx, kink_tol=KINK)
    _say(worst)
    assert worst["clean_groups"] > 0.6 * G * steps
    assert worst["state_steps"] > 0.4 * steps


def test_mlp_f32_cyclic_window(par):
    w = scaled(CONFIGS["mlp_784"], name="mlp_f32", widths=(50, 33, 4), mu=20, G=3, rows=70, D=3)
    Xs, ys = make_shards(w, "cuda")
    worst = par.teacher_forced(w, 10, Xs, ys, None, kink_tol=KINK)
    _say(worst)


def test_mlp_784_full_size(par):
    # configuration 3: 784-200-10, G=10, mu=512, 6000 rows per shard, fp32
    w = CONFIGS["mlp_784"]
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    steps = 6
    idx = make_indices(w, steps)
    worst = par.teacher_forced(w, steps, Xs, ys, idx, kink_tol=KINK)
    _say(worst)
    assert worst["clean_groups"] >= 0.9 * w.G * steps
    assert worst["state_steps"] >= 4


def test_mlp_784_full_size_free_run_loss_curve(par):
    # configuration 3 at full size, both sides on their own for 60 iterations: the loss curves
    # and the selections are compared
    w = CONFIGS["mlp_784"]
    Xs, ys = make_shards(w, "cuda")
    steps = 60
    idx = make_indices(w, steps)
    r = par.free_running(w, steps, Xs, ys, idx)
    agree = (r["masks_gpu"] == r["masks_oracle"]).mean()
    _say("mask agreement", agree, "loss", r["loss_gpu"][0], "->", r["loss_gpu"][-1], r["loss_oracle"][-1],
         "uploads", int(r["masks_gpu"].sum()), "of", steps * w.G)
    assert agree >= 0.9
    assert r["loss_gpu"][-1] < 0.5 * r["loss_gpu"][0]
    np.testing.assert_allclose(r["loss_gpu"], r["loss_oracle"], rtol=5e-2, atol=1e-4)


# bf16: X, the weights the gradients are evaluated at, the activations and the back-propagated
# signals are bf16 on the GPU with fp32 accumulation.  The oracle evaluates at the bf16-rounded X
# and iterates and rounds the hidden activations to bf16 (every layer's product has bf16 inputs),
# so both sides form each ReLU decision from the same values, up to the rounding of the fp32
# accumulation.  No kink excuse is made here: a unit that such rounding does flip is one term of a
# sum over the minibatch, far inside this tolerance (and at the full widths nearly every group
# has SOME unit within 5e-8 of its kink among its million pre-activations: the per-group excuse
# of the fp32 tests would skip everything).  The back-propagated signals' rounding is what the 2e-2
# tolerance is for.  Masks: the plain 1e-6 edge, or a statistic that is closer to the threshold
# than the GPU's statistic is to the oracle's (that error is held to the tolerance).
# Element by element, the few rows in which a ReLU decision fell differently are left out
# (parity.flip_rows: a one-ulp difference of a bf16 activation moves the next layer's
# pre-activation by up to ~1e-4 of the sum of its terms' magnitudes).
BF16 = dict(tol=2e-2, edge=1e-6, edge_stat_err=True, kink_tol=None, kink_unit_tol=1e-4)


@pytest.mark.parametrize("widths,mu,G,rows,steps", [
    ((128, 96, 64, 10), 48, 4, 100, 7),
    ((200, 150, 10), 256, 3, 300, 6),
    ((3072, 1024, 1024, 10), 64, 2, 150, 3),   # layer widths of the bf16 configuration
    ((256, 128, 100), 128, 3, 400, 5),          # a hundred classes: the wide output-layer tile
    ((256, 128, 24), 96, 3, 300, 5),            # rows a multiple of 256 bytes: the narrow one
])
def test_mlp_bf16_shapes(par, widths, mu, G, rows, steps):
    w = scaled(CONFIGS["mlp_3072_bf16"], name="mlp_bf16", widths=widths, mu=mu, G=G, rows=rows, D=4)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    idx = make_indices(w, steps)
    worst = par.teacher_forced(w, steps, Xs, ys, idx, **BF16)
    _say(worst)
    assert worst["clean_groups"] == G * steps and worst["state_steps"] >= steps - 1


# ---- configuration 5 at full size (G=64, mu=256, 781 rows per shard, p = 4.2 M): iterations from
# seeded synthetic mid-run states; the oracle evaluates sampled groups (seconds per group)

@pytest.fixture(scope="module")
def cfg5():
    w = CONFIGS["mlp_3072_bf16"]
    Xs, ys = make_shards(w, "cuda")
    return w, Xs, ys, make_indices(w, 1)[0]


def test_mlp_3072_bf16_full_size_groups_of_every_age(par, cfg5):
    # ten groups, one of every age 1..D: gradients (of the uploading groups: the lazy store is on
    # at this size), statistics and masks; then the same three groups as before with the lazy
    # store off, where every fresh gradient is written
    w, Xs, ys, idx = cfg5
    st = par.synthetic_state(w, 7)
    groups = [int(np.nonzero(st["tau"] == t)[0][0]) for t in range(1, w.D + 1) if (st["tau"] == t).any()]
    _say("case", w, "groups", groups, "ages", [int(st["tau"][g]) for g in groups])
    assert len(groups) >= 8
    worst, ref = par.sampled_groups_step(w, Xs, ys, idx, groups=groups, lazy_store=1, **BF16)
    _say(worst)
    worst, _ = par.sampled_groups_step(w, Xs, ys, idx, groups=groups, lazy_store=0, reference=ref, **BF16)
    _say(worst)


def test_mlp_3072_bf16_full_size_whole_state(par, cfg5):
    # a state in which only the eight sampled groups can be selected (age D; all others younger,
    # c = 1e30): aggregate, moments, iterate, stored gradients, ages and history after the step
    # are determined by the groups the oracle evaluates and are compared in full at p = 4.2 M --
    # in the default configuration of this size (lazy gradient store, first-layer statistic from
    # the Gram matrices), with the Gram statistic off, and with the lazy store off
    from paper_2201_04301_amd import binding as B
    w, Xs, ys, idx = cfg5
    w = scaled(w, c=1e30)
    groups = [3, 9, 20, 31, 32, 47, 55, 62]
    ref = None
    for name, lazy, opts in (("lazy store + Gram statistic", 1, ()),
                             ("lazy store", 1, ((B.GCADA_OPT_GRAM_STATISTIC, 0),)),
                             ("every gradient stored", 0, ())):
        worst, ref = par.sampled_groups_step(w, Xs, ys, idx, groups=groups, lazy_store=lazy, options=opts,
                                             reference=ref, whole_state=True, seed=11, **BF16)
        _say(name, worst)
        assert "theta" in worst and worst["selected"] == len(groups)


def test_mlp_3072_bf16_full_width_teacher_forced_past_the_age_bound(par):
    # the full layer widths and minibatch with six groups (the lazy gradient store and the Gram
    # statistic are on from 64 MiB of gradients), teacher-forced over steps 0 .. D+1 with the whole
    # state compared after every step; the threshold is out of the statistic's reach, so every
    # group ages to D and the forced uploads run at this size
    from paper_2201_04301_amd import binding as B
    w = scaled(CONFIGS["mlp_3072_bf16"], name="mlp_3072_g6", G=6, rows=400, D=5, sigma=1.5, alpha=2e-3, c=1e30)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    steps = w.D + 2
    idx = make_indices(w, steps)
    worst = par.teacher_forced(w, steps, Xs, ys, idx, lazy_store=1,
                               options=((B.GCADA_OPT_GRAM_STATISTIC, 1),), **BF16)
    _say(worst)
    assert worst["state_steps"] >= steps - 2 and worst["max_age"] == w.D and worst["forced_late"] == w.G


@pytest.mark.parametrize("widths,mu,G,rows,steps,dtype_cfg,tol", [
    ((100, 70, 50, 7), 40, 5, 90, 14, "mlp_784", 1e-5),          # fp32, two k-tiles per pass
    ((20, 12, 5), 16, 3, 50, 15, "mlp_784", 1e-5),               # fp32, one k-tile per pass (two pipelines)
    ((200, 150, 10), 256, 3, 300, 8, "mlp_3072_bf16", 2e-2),     # bf16
])
def test_mlp_lazy_gradient_store_parity(par, widths, mu, G, rows, steps, dtype_cfg, tol):
    # teacher-forced parity with the lazy store switched on: statistic of every group, gradients
    # of the uploading groups, and the whole state after every step
    w = scaled(CONFIGS[dtype_cfg], name="mlp_lazy", widths=widths, mu=mu, G=G, rows=rows, D=4)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    idx = make_indices(w, steps)
    bf = dtype_cfg == "mlp_3072_bf16"
    worst = par.teacher_forced(w, steps, Xs, ys, idx, tol=tol, edge=1e-6, edge_stat_err=bf,
                               kink_tol=None if bf else KINK, kink_unit_tol=1e-4 if bf else None, lazy_store=1)
    _say(worst)
    assert worst["selected"] > 0 and worst["state_steps"] > 0.4 * steps


@pytest.mark.parametrize("widths,mu,G,rows,dtype_cfg", [
    ((100, 70, 50, 7), 40, 6, 90, "mlp_784"),
    ((20, 12, 5), 16, 4, 50, "mlp_784"),
    ((300, 260, 10), 128, 5, 200, "mlp_3072_bf16"),
])
def test_mlp_lazy_gradient_store_changes_nothing(widths, mu, G, rows, dtype_cfg):
    # free run, lazy store off and on: masks, statistics, losses and the complete state are
    # bit-identical (the second launch recomputes a selected group's gradient from the same
    # products in the same order); both kinds of selection occur
    from paper_2201_04301_amd import Gcada, binding as B
    from gcada_inputs import make_theta0
    w = scaled(CONFIGS[dtype_cfg], name="mlp_lazy", widths=widths, mu=mu, G=G, rows=rows, D=4, c=0.6)
    Xs, ys = make_shards(w, "cuda")
    steps = 40
    idx = torch.as_tensor(make_indices(w, steps), device="cuda")
    runs = []
    for lazy in (0, 1):
        gpu = Gcada.from_workload(w)
        gpu.set_shards(Xs, ys)
        gpu.set_theta(make_theta0(w))
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_LAZY_GRADIENT_STORE, lazy)
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_GRAM_STATISTIC, 0)     # another route to the statistic: other rounding
        masks, stats, losses, taus = [], [], [], []
        for k in range(steps):
            taus.append(gpu.get_state()["tau"].copy())
            gpu.step(idx[k].contiguous())
            out = gpu.outputs()
            masks.append(out["mask"].copy()); stats.append(out["stat"].copy()); losses.append(out["loss"])
        runs.append(dict(masks=np.array(masks), stats=np.array(stats), losses=np.array(losses),
                         taus=np.array(taus), state=gpu.get_state()))
        gpu.close()
    a, b = runs
    np.testing.assert_array_equal(a["masks"], b["masks"])
    np.testing.assert_array_equal(a["stats"], b["stats"])
    np.testing.assert_array_equal(a["losses"], b["losses"])
    for name in ("theta", "h", "vhat", "agg", "last", "theta_stale", "tau", "dtheta_sq"):
        np.testing.assert_array_equal(a["state"][name], b["state"][name], err_msg=name)
    sel = a["masks"][1:] != 0
    forced = a["taus"][1:] >= w.D
    _say("selected", int(sel.sum()), "of them by age", int((sel & forced).sum()),
         "by the statistic", int((sel & ~forced).sum()), "skipped", int((~sel).sum()))
    assert (sel & forced).any() and (sel & ~forced).any() and (~sel).any()


def test_mlp_lazy_gradient_store_switched_during_a_run_changes_nothing():
    # the store flags of a step are set by the last launch of the step before; switching the
    # option (or the Gram statistic's, or loading a state) in between must make the next step set
    # them anew.  A run that switches back and forth ends in the bits of one that never does.
    from paper_2201_04301_amd import Gcada, binding as B
    from gcada_inputs import make_theta0
    w = scaled(CONFIGS["mlp_3072_bf16"], name="mlp_lazy", widths=(300, 260, 10), mu=128, G=5, rows=200, D=4, c=0.6)
    Xs, ys = make_shards(w, "cuda")
    steps = 24
    idx = torch.as_tensor(make_indices(w, steps), device="cuda")
    runs = []
    for switching in (False, True):
        gpu = Gcada.from_workload(w)
        gpu.set_shards(Xs, ys)
        gpu.set_theta(make_theta0(w))
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_GRAM_STATISTIC, 0)
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_LAZY_GRADIENT_STORE, 1)
        masks = []
        for k in range(steps):
            if switching and k in (5, 13):
                B.gcada_set_option(gpu.ctx, B.GCADA_OPT_LAZY_GRADIENT_STORE, 0)
            if switching and k in (8, 17):
                B.gcada_set_option(gpu.ctx, B.GCADA_OPT_LAZY_GRADIENT_STORE, 1)
            if switching and k == 20:
                gpu.set_state(**gpu.get_state())          # a reload of the same state
            gpu.step(idx[k].contiguous())
            masks.append(gpu.outputs()["mask"].copy())
        runs.append(dict(masks=np.array(masks), state=gpu.get_state()))
        gpu.close()
    a, b = runs
    np.testing.assert_array_equal(a["masks"], b["masks"])
    for name in ("theta", "h", "vhat", "agg", "last", "theta_stale", "tau", "dtheta_sq"):
        np.testing.assert_array_equal(a["state"][name], b["state"][name], err_msg=name)
    assert a["masks"].any() and not a["masks"].all()


def test_mlp_free_run_loss_decreases_and_tracks_oracle(par):
    w = scaled(CONFIGS["mlp_784"], name="mlp_f32", widths=(64, 48, 10), mu=64, G=4, rows=400, D=5)
    Xs, ys = make_shards(w, "cuda")
    steps = 60
    idx = make_indices(w, steps)
    r = par.free_running(w, steps, Xs, ys, idx)
    agree = (r["masks_gpu"] == r["masks_oracle"]).mean()
    _say("mask agreement", agree, "loss", r["loss_gpu"][0], "->", r["loss_gpu"][-1], r["loss_oracle"][-1])
    assert agree >= 0.9
    assert r["loss_gpu"][-1] < 0.7 * r["loss_gpu"][0]
    np.testing.assert_allclose(r["loss_gpu"], r["loss_oracle"], rtol=5e-2)


# ---- first-layer statistic through Gram matrices (bf16, lazy gradient store, wide first layer)

@pytest.mark.parametrize("widths,mu,G,rows,steps", [
    ((256, 192, 10), 64, 4, 150, 8),            # one Gram tile per group
    ((512, 384, 64, 10), 160, 3, 300, 6),       # 2 x 2 Gram tiles, the last ones partly empty
])
def test_mlp_gram_statistic_parity(par, widths, mu, G, rows, steps):
    # teacher-forced parity with the oracle, statistic of the first layer from the Gram matrices
    w = scaled(CONFIGS["mlp_3072_bf16"], name="mlp_gram", widths=widths, mu=mu, G=G, rows=rows, D=4)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    idx = make_indices(w, steps)
    worst = par.teacher_forced(w, steps, Xs, ys, idx, lazy_store=1, **BF16)
    _say(worst)
    assert worst["selected"] > 0 and worst["state_steps"] > 0.4 * steps


def test_mlp_gram_statistic_matches_weight_gradient_statistic():
    # same run with the statistic from the Gram matrices and from the two weight gradients: the
    # statistics agree to bf16 rounding of the signal difference, the masks wherever the
    # statistic is not within that of the threshold, the uploaded gradients to fp32 rounding
    from paper_2201_04301_amd import Gcada, binding as B
    from gcada_inputs import make_theta0
    w = scaled(CONFIGS["mlp_3072_bf16"], name="mlp_gram", widths=(512, 256, 10), mu=96, G=6, rows=300, D=4, c=0.6)
    Xs, ys = make_shards(w, "cuda")
    steps = 10
    idx = torch.as_tensor(make_indices(w, steps), device="cuda")
    ref = None
    for gram in (0, 1):
        gpu = Gcada.from_workload(w)
        gpu.set_shards(Xs, ys)
        gpu.set_theta(make_theta0(w))
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_LAZY_GRADIENT_STORE, 1)
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_GRAM_STATISTIC, gram)
        outs = []
        for k in range(steps):
            st = gpu.get_state()
            if ref is not None:                  # follow the reference run's states: compare step by step
                gpu.set_state(**ref[k][0])
                B.gcada_set_option(gpu.ctx, B.GCADA_OPT_LAZY_GRADIENT_STORE, 1)
                B.gcada_set_option(gpu.ctx, B.GCADA_OPT_GRAM_STATISTIC, gram)
                st = ref[k][0]
            gpu.step(idx[k].contiguous())
            outs.append((st, gpu.outputs()))
        gpu.close()
        if ref is None:
            ref = outs
            continue
        differing = 0
        # noise floor of a statistic: squared rounding error of a gradient (at step 0 both iterates
        # coincide and every statistic is nothing else); every group uploads at step 0
        gn2 = max(float(np.dot(ref[0][1]["grad"][g].astype(np.float64), ref[0][1]["grad"][g])) for g in range(w.G))
        for (_, a), (_, b) in zip(ref, outs):
            np.testing.assert_allclose(b["stat"], a["stat"], rtol=1e-2, atol=1e-2 * a["rhs"] + 1e-5 * gn2)
            assert b["rhs"] == a["rhs"] and b["loss"] == a["loss"]
            for g in range(w.G):
                if a["mask"][g] != b["mask"][g]:
                    assert abs(a["stat"][g] - a["rhs"]) <= 2e-2 * a["rhs"]
                    differing += 1
                elif a["mask"][g]:
                    # the same weight gradients; the first layer's bias gradient is summed in another
                    # order by the kernel that forms the signal difference (fp32 rounding)
                    np.testing.assert_allclose(b["grad"][g], a["grad"][g], rtol=2e-6,
                                               atol=1e-6 * np.abs(a["grad"][g]).max())
        _say("masks that differ at the threshold:", differing)


def test_mlp_bf16_free_run_with_lazy_store_and_gram_statistic_tracks_oracle(par):
    # both sides on their own for 50 iterations, the GPU in the configuration the big bf16
    # workload runs in (lazy gradient store, first-layer statistic from the Gram matrices)
    from paper_2201_04301_amd import binding as B
    # (overlapping clusters: the loss stays away from zero, where a relative comparison means nothing)
    w = scaled(CONFIGS["mlp_3072_bf16"], name="mlp_gram", widths=(256, 192, 10), mu=64, G=6, rows=400, D=5,
               sigma=1.5, alpha=2e-3)
    Xs, ys = make_shards(w, "cuda")
    steps = 50
    idx = make_indices(w, steps)
    r = par.free_running(w, steps, Xs, ys, idx,
                         options=((B.GCADA_OPT_LAZY_GRADIENT_STORE, 1), (B.GCADA_OPT_GRAM_STATISTIC, 1)))
    agree = (r["masks_gpu"] == r["masks_oracle"]).mean()
    _say("mask agreement", agree, "loss", r["loss_gpu"][0], "->", r["loss_gpu"][-1], r["loss_oracle"][-1],
         "uploads", int(r["masks_gpu"].sum()), "of", steps * w.G)
    assert agree >= 0.85
    assert r["loss_gpu"][-1] < 0.7 * r["loss_gpu"][0]
    # (free-running bf16 against fp64: once the loss is four orders below its start the two
    # trajectories differ by tens of percent of it)
    np.testing.assert_allclose(r["loss_gpu"], r["loss_oracle"], rtol=8e-2, atol=2e-4)
    assert 0 < r["masks_gpu"].sum() < steps * w.G
