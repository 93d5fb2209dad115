"""GPU parity of the logistic-regression path with the fp64 oracle (through the C-ABI)."""
import numpy as np
import pytest
import torch

from gcada_inputs import CONFIGS, make_indices, make_shards, scaled

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def par():
    import parity
    return parity


def _say(*a):
    print(*a, flush=True)


def test_lr_small_full_run_teacher_forced(par):
    # configuration 1: d=64, G=3, mu=32, 512 rows per shard, 200 iterations from theta = 0
    w = CONFIGS["lr_small"]
    _say("case lr_small", w)
    Xs, ys = make_shards(w, "cuda")
    idx = make_indices(w, w.iters)
    worst = par.teacher_forced(w, w.iters, Xs, ys, idx)
    _say(worst)
    # the rule must both fire and hold back during the run
    assert w.G * 20 < worst["selected"] < w.G * w.iters


def test_lr_small_cyclic_window(par):
    w = CONFIGS["lr_small"]
    Xs, ys = make_shards(w, "cuda")
    worst = par.teacher_forced(w, 40, Xs, ys, idx=None)
    _say(worst)


@pytest.mark.parametrize("d,mu,G,rows,l2,c", [
    (67, 33, 3, 100, 0.0, 1.0),      # ragged d (scalar path), ragged mu
    (260, 17, 5, 64, 1e-3, 0.5),     # one column slab plus a 4-column tail, l2 on
    (1028, 130, 2, 300, 1e-4, 2.0),  # several slabs, mu not a multiple of the row tiles
    (4, 1, 1, 3, 0.0, 1.0),          # degenerate: one sample, one group
])
def test_lr_ragged_shapes(par, d, mu, G, rows, l2, c):
    w = scaled(CONFIGS["lr_small"], name="ragged", widths=(d,), mu=mu, G=G, rows=rows, l2=l2, c=c,
               D=4)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    idx = make_indices(w, 25)
    worst = par.teacher_forced(w, 25, Xs, ys, idx)
    _say(worst)


@pytest.mark.parametrize("c", [0.0, 0.5, 2.0])
def test_lr_4k_reduced_rows_c_sweep(par, c):
    # configuration 2's geometry (d=4096, G=16, mu=256, l2=1e-4) on shorter shards
    w = scaled(CONFIGS["lr_4k"], rows=2048, c=c)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    idx = make_indices(w, 30)
    worst = par.teacher_forced(w, 30, Xs, ys, idx)
    _say(worst)
    if c == 0.0:
        assert worst["selected"] == w.G * 30


def test_lr_free_run_tracks_oracle(par):
    w = CONFIGS["lr_small"]
    Xs, ys = make_shards(w, "cuda")
    idx = make_indices(w, w.iters)
    r = par.free_running(w, w.iters, Xs, ys, idx)
    agree = (r["masks_gpu"] == r["masks_oracle"]).mean()
    _say("mask agreement", agree, "final loss", r["loss_gpu"][-1], r["loss_oracle"][-1])
    assert agree >= 0.98
    np.testing.assert_allclose(r["loss_gpu"], r["loss_oracle"], rtol=2e-3)
    assert r["loss_gpu"][-1] < 0.9 * r["loss_gpu"][0]


def test_lr_deterministic(par):
    # same inputs twice => bit-identical iterate (all reductions have a fixed order)
    w = scaled(CONFIGS["lr_4k"], rows=1024)
    Xs, ys = make_shards(w, "cuda")
    idx = make_indices(w, 12)
    a = par.free_running(w, 12, Xs, ys, idx)
    b = par.free_running(w, 12, Xs, ys, idx)
    np.testing.assert_array_equal(a["theta_gpu"], b["theta_gpu"])
    np.testing.assert_array_equal(a["masks_gpu"], b["masks_gpu"])


# ---- single-pass kernel (whole-row register tiles): every wave arrangement, one and several
# tiles per group; wider rows take the team kernel, a width that is not a multiple of 4 the general kernels

@pytest.mark.parametrize("d,mu,G,rows,l2,use_idx", [
    (4096, 256, 16, 1024, 1e-4, True),    # 16 x 4096 tiles, 16 tiles per group
    (4096, 48, 40, 600, 0.0, True),       # three tiles per group
    (2048, 128, 7, 300, 1e-3, True),      # 32 x 2048 tiles
    (1024, 64, 5, 100, 0.0, True),        # 64 x 1024 tiles, one tile per group
    (512, 256, 3, 300, 1e-4, True),       # 128 x 512 tiles
    (256, 512, 2, 600, 0.0, True),        # 256 x 256 tiles
    (4096, 256, 16, 700, 1e-4, False),    # cyclic window
    (784, 256, 3, 500, 1e-4, True),       # rows that do not fill the column waves: 64 x 1024 tiles, 784 used
    (3000, 48, 5, 200, 0.0, True),        # 16 x 4096 tiles, 3000 columns used
    (300, 128, 4, 300, 1e-3, False),      # 128 x 512 tiles, 300 columns used, cyclic window
    (4096, 24, 6, 100, 1e-4, True),       # minibatch that does not fill its last tile (16 + 8 rows)
    (1024, 100, 3, 200, 0.0, False),      # 64-row tiles, 100 rows: the second tile holds 36; cyclic window
    (300, 50, 4, 90, 1e-3, True),         # 128-row tiles, one tile with 50 rows
    (64, 512, 20, 600, 1e-4, True),       # narrow rows, too many rows and groups for the one-launch kernel: 256-row tiles, 16 lanes of a wave used
    (128, 200, 5, 300, 0.0, False),       # narrow rows, one partly empty tile; cyclic window
    (4, 40, 3, 50, 1e-3, True),           # one float4 per row
    (8192, 48, 5, 100, 0.0, True),        # team kernel, two members
    (9192, 32, 4, 64, 1e-4, True),        # team of three, the last member owns 1000 columns
    (5000, 16, 3, 40, 0.0, False),        # team of two, the second member owns 904 columns; cyclic window
    (8192, 30, 4, 64, 1e-4, True),        # team kernel, 30 rows: the eighth tile holds two
    (12288, 9, 2, 20, 0.0, False),        # team of three, 9 rows: the third tile holds one; cyclic window
    (65536, 32, 4, 64, 0.0, True),        # team kernel, d of the largest configuration
    (8190, 32, 3, 64, 0.0, True),         # d not a multiple of 4: general kernels
])
def test_lr_tile_shapes(par, d, mu, G, rows, l2, use_idx):
    w = scaled(CONFIGS["lr_small"], name="tiles", widths=(d,), mu=mu, G=G, rows=rows, l2=l2, c=1.0,
               D=5, flip=0.05)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    steps = 14
    idx = make_indices(w, steps) if use_idx else None
    worst = par.teacher_forced(w, steps, Xs, ys, idx)
    _say(worst)


def test_lr_single_pass_matches_general_kernels(par):
    # the single-pass kernel and the general two-pass kernels compute the same iteration
    from paper_2201_04301_amd import Gcada, binding as B
    from gcada_inputs import make_theta0
    w = scaled(CONFIGS["lr_4k"], rows=1024, c=0.5)
    Xs, ys = make_shards(w, "cuda")
    idx = torch.as_tensor(make_indices(w, 25), device="cuda")
    res = []
    for fused in (1, 0):
        gpu = Gcada.from_workload(w)
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_SINGLE_PASS_LOGREG, fused)
        gpu.set_shards(Xs, ys)
        gpu.set_theta(make_theta0(w))
        masks = torch.zeros(25, w.G, dtype=torch.uint8, device="cuda")
        for k in range(25):
            gpu.step(idx[k].contiguous(), mask_out=masks[k])
        st = gpu.get_state()
        res.append((masks.cpu().numpy(), st["theta"], gpu.outputs()["stat"]))
        gpu.close()
    np.testing.assert_array_equal(res[0][0], res[1][0])
    np.testing.assert_allclose(res[0][1], res[1][1], rtol=0, atol=2e-4 * np.abs(res[1][1]).max())
    np.testing.assert_allclose(res[0][2], res[1][2], rtol=2e-5)


@pytest.mark.parametrize("d,mu,G,l2", [
    (4096, 256, 16, 1e-4),     # the benchmark's step shape: 64 blocks meet inside the kernel
    (2048, 64, 40, 0.0),       # more groups than group lanes: three passes over the groups
    (256, 256, 3, 1e-3),       # four blocks
    (784, 128, 5, 1e-4),       # thirteen blocks, the last one with 16 of its 64 columns
    (512, 128, 70, 0.0),       # too many groups for the fused finish: separate kernels either way
])
def test_lr_fused_finish_matches_separate_kernels(par, d, mu, G, l2):
    # reduce + selection + update in one launch against the three separate kernels: the same
    # additions in the same order, so the state agrees bit for bit (the statistic and the history
    # are partitioned differently over blocks and may differ in the last bits)
    from paper_2201_04301_amd import Gcada, binding as B
    from gcada_inputs import make_theta0
    w = scaled(CONFIGS["lr_small"], name="finish", widths=(d,), mu=mu, G=G, rows=400, l2=l2, c=0.5,
               D=5, flip=0.05)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    steps = 30
    idx = torch.as_tensor(make_indices(w, steps), device="cuda")
    res = []
    for fused in (1, 0):
        gpu = Gcada.from_workload(w)
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_FUSED_FINISH, fused)
        gpu.set_shards(Xs, ys)
        gpu.set_theta(make_theta0(w))
        masks = torch.zeros(steps, w.G, dtype=torch.uint8, device="cuda")
        losses = torch.zeros(steps, dtype=torch.float32, device="cuda")
        for k in range(steps):
            gpu.step(idx[k].contiguous(), mask_out=masks[k], loss_out=losses[k:k + 1])
        out = gpu.outputs()
        st = gpu.get_state()
        res.append((masks.cpu().numpy(), losses.cpu().numpy(), st, out))
        gpu.close()
    (m1, l1, s1, o1), (m0, l0, s0, o0) = res
    assert 0 < m1.sum() < m1.size or G == 70
    np.testing.assert_array_equal(m1, m0)
    np.testing.assert_array_equal(l1, l0)
    for name in ("theta", "h", "vhat", "agg", "theta_stale", "last", "tau"):
        np.testing.assert_array_equal(s1[name], s0[name], err_msg=name)
    assert s1["k"] == s0["k"] == steps
    np.testing.assert_allclose(s1["dtheta_sq"], s0["dtheta_sq"], rtol=1e-12)
    np.testing.assert_allclose(o1["stat"], o0["stat"], rtol=1e-12)
    np.testing.assert_allclose(o1["rhs"], o0["rhs"], rtol=1e-12)
    np.testing.assert_array_equal(o1["grad"], o0["grad"])


@pytest.mark.parametrize("model,d,mu,G,l2", [
    ("logreg", 64, 32, 3, 0.0),       # configuration 1's shape
    ("logreg", 256, 128, 3, 1e-3),    # the widest rows and longest minibatch of the one-launch path
    ("linreg", 100, 17, 9, 1e-4),     # column lanes that do not fill a wave, ragged minibatch
    ("logreg", 4, 1, 1, 0.0),         # one sample, one group
])
def test_lr_one_launch_path_matches_general_kernels(par, model, d, mu, G, l2):
    # small linear models run the whole iteration in one launch (lr_micro_kernel); with the
    # single-pass switch off the same run goes through the general kernels and the server kernel
    from paper_2201_04301_amd import Gcada, binding as B
    from gcada_inputs import make_theta0
    w = scaled(CONFIGS["lr_small"], name="micro", model=model, widths=(d,), mu=mu, G=G, rows=300, l2=l2,
               c=0.5, D=5, flip=0.05)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    steps = 40
    idx = torch.as_tensor(make_indices(w, steps), device="cuda")
    res = []
    for one_launch in (1, 0):
        gpu = Gcada.from_workload(w)
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_SINGLE_PASS_LOGREG, one_launch)
        assert ("lr_micro" in B.gcada_timed_stage(gpu.ctx)) == bool(one_launch)
        gpu.set_shards(Xs, ys)
        gpu.set_theta(make_theta0(w))
        masks = torch.zeros(steps, w.G, dtype=torch.uint8, device="cuda")
        losses = torch.zeros(steps, dtype=torch.float32, device="cuda")
        for k in range(steps):
            gpu.step(idx[k].contiguous(), mask_out=masks[k], loss_out=losses[k:k + 1])
        out = gpu.outputs()
        st = gpu.get_state()
        res.append((masks.cpu().numpy(), losses.cpu().numpy(), st, out))
        gpu.close()
    (m1, l1, s1, o1), (m0, l0, s0, o0) = res
    np.testing.assert_array_equal(m1, m0)
    np.testing.assert_allclose(l1, l0, rtol=1e-5)
    scale = max(np.abs(s0["theta"]).max(), 1e-3)
    np.testing.assert_allclose(s1["theta"], s0["theta"], rtol=0, atol=2e-4 * scale)
    np.testing.assert_array_equal(s1["tau"], s0["tau"])
    np.testing.assert_allclose(s1["dtheta_sq"], s0["dtheta_sq"], rtol=1e-3)
    np.testing.assert_allclose(o1["stat"], o0["stat"], rtol=1e-3, atol=1e-12)
    np.testing.assert_allclose(o1["grad"], o0["grad"], rtol=0, atol=2e-4 * np.abs(o0["grad"]).max())


def test_lr_fused_finish_switched_between_steps(par):
    # the fused finish leaves the newest history entry spread over its blocks until the next
    # launch folds it in; switching to the separate kernels (and back) between steps must first
    # complete it.  Same additions either way: the iterates agree bit for bit.
    from paper_2201_04301_amd import Gcada, binding as B
    from gcada_inputs import make_theta0
    w = scaled(CONFIGS["lr_small"], name="switch", widths=(1024,), mu=128, G=6, rows=300, l2=1e-4, c=0.5,
               D=4, flip=0.05)
    Xs, ys = make_shards(w, "cuda")
    steps = 24
    idx = torch.as_tensor(make_indices(w, steps), device="cuda")
    res = []
    for pattern in ("fused", "alternate", "separate"):
        gpu = Gcada.from_workload(w)
        gpu.set_shards(Xs, ys)
        gpu.set_theta(make_theta0(w))
        masks = torch.zeros(steps, w.G, dtype=torch.uint8, device="cuda")
        for k in range(steps):
            on = {"fused": 1, "separate": 0, "alternate": (k // 3) % 2}[pattern]
            B.gcada_set_option(gpu.ctx, B.GCADA_OPT_FUSED_FINISH, on)
            gpu.step(idx[k].contiguous(), mask_out=masks[k])
        st = gpu.get_state()
        res.append((masks.cpu().numpy(), st))
        gpu.close()
    assert 0 < res[0][0].sum() < res[0][0].size
    for m, st in res[1:]:
        np.testing.assert_array_equal(m, res[0][0])
        for name in ("theta", "h", "vhat", "agg", "last", "tau"):
            np.testing.assert_array_equal(st[name], res[0][1][name], err_msg=name)
        np.testing.assert_allclose(st["dtheta_sq"], res[0][1]["dtheta_sq"], rtol=1e-12)


# ---- full-size configurations

def test_lr_4k_full_size_teacher_forced(par):
    # configuration 2 at full size: 16 shards of 65,536 x 4,096 fp32 (17.2 GB), the launch
    # configuration bench.py times; teacher-forced against the oracle
    w = CONFIGS["lr_4k"]
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    steps = 14
    idx = make_indices(w, steps)
    worst = par.teacher_forced(w, steps, Xs, ys, idx)
    _say(worst)
    assert worst["selected"] >= 2 * w.G


def test_lr_4k_full_size_free_run_loss_curve(par):
    # configuration 2 at full size, both sides on their own for 60 iterations
    w = CONFIGS["lr_4k"]
    Xs, ys = make_shards(w, "cuda")
    steps = 60
    idx = make_indices(w, steps)
    r = par.free_running(w, steps, Xs, ys, idx)
    agree = (r["masks_gpu"] == r["masks_oracle"]).mean()
    _say("mask agreement", agree, "loss", r["loss_gpu"][0], "->", r["loss_gpu"][-1], r["loss_oracle"][-1],
         "uploads", int(r["masks_gpu"].sum()), "of", steps * w.G)
    assert agree >= 0.98
    assert r["loss_gpu"][-1] < r["loss_gpu"][0]
    np.testing.assert_allclose(r["loss_gpu"], r["loss_oracle"], rtol=2e-3)
    np.testing.assert_allclose(r["theta_gpu"], r["theta_oracle"], rtol=0, atol=2e-3 * np.abs(r["theta_oracle"]).max())


@pytest.mark.parametrize("c,D,steps", [(1.0, 10, 13), (1e30, 4, 7)])
def test_lr_64k_full_step_shape(par, c, D, steps):
    # configuration 4's step shape (G=32, mu=1024, d=65,536: 8.6 GB of rows touched per step) on
    # shards of 2,048 rows; every group checked against the oracle, teacher-forced over steps
    # 0 .. D+2 (the configuration's D and c), and with a threshold no statistic reaches, where every
    # group ages to D and is forced to upload at this shape
    w = scaled(CONFIGS["lr_64k"], rows=2048, c=c, D=D)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda", chunk_rows=1024)
    idx = make_indices(w, steps)
    worst = par.teacher_forced(w, steps, Xs, ys, idx)
    _say(worst)
    assert worst["state_steps"] == steps
    if c > 1e20:
        assert worst["forced_late"] == w.G and worst["by_statistic"] == 0 and worst["max_age"] == D


@pytest.mark.parametrize("d,mu,G,l2,applies", [
    (4096, 256, 16, 1e-4, True),    # the benchmark's step shape: 256 workgroups, 64 of them finish the step before
    (2048, 64, 40, 0.0, True),      # 80 workgroups, three passes over the groups in the finish
    (1024, 256, 8, 1e-3, True),     # 32 workgroups, 16 finishing
    (4096, 256, 4, 0.0, True),      # as many workgroups as finishing blocks
    (784, 128, 5, 1e-4, False),     # fewer tiles than finishing blocks: the option changes nothing
])
def test_lr_one_launch_per_step_matches_two_launches(par, d, mu, G, l2, applies):
    # GCADA_OPT_DEFERRED_FINISH: the finish of step k at the head of the launch of step k+1 (the new
    # iterate reaches the tiles through tagged words).  Same additions in the same order: masks,
    # losses and the whole state are bit-identical to the tile kernel + fused finish; a state
    # query in the middle (which runs the finish that is still to come) changes nothing
    from paper_2201_04301_amd import Gcada, binding as B
    from gcada_inputs import make_theta0
    w = scaled(CONFIGS["lr_small"], name="one_launch", widths=(d,), mu=mu, G=G, rows=400, l2=l2, c=0.5,
               D=5, flip=0.05)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    steps = 31
    idx = torch.as_tensor(make_indices(w, steps), device="cuda")
    res = []
    for deferred in (0, 1):
        gpu = Gcada.from_workload(w)
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_DEFERRED_FINISH, deferred)
        gpu.set_shards(Xs, ys)
        gpu.set_theta(make_theta0(w))
        masks = torch.zeros(steps, w.G, dtype=torch.uint8, device="cuda")
        losses = torch.zeros(steps, dtype=torch.float32, device="cuda")
        mid = None
        for k in range(steps):
            gpu.step(idx[k].contiguous(), mask_out=masks[k], loss_out=losses[k:k + 1])
            if k == 12:
                mid = gpu.get_state()          # runs the pending finish; the next step starts afresh
        out = gpu.outputs()
        st = gpu.get_state()
        res.append((masks.cpu().numpy(), losses.cpu().numpy(), st, out, mid))
        gpu.close()
    (m0, l0, s0, o0, mid0), (m1, l1, s1, o1, mid1) = res
    assert 0 < m0.sum() < m0.size
    np.testing.assert_array_equal(m1, m0)
    np.testing.assert_array_equal(l1, l0)
    for name in ("theta", "h", "vhat", "agg", "theta_stale", "last", "tau"):
        np.testing.assert_array_equal(s1[name], s0[name], err_msg=name)
        np.testing.assert_array_equal(mid1[name], mid0[name], err_msg="mid-run " + name)
    assert s1["k"] == s0["k"] == steps and mid1["k"] == mid0["k"] == 13
    np.testing.assert_allclose(s1["dtheta_sq"], s0["dtheta_sq"], rtol=1e-12)
    np.testing.assert_array_equal(o1["stat"], o0["stat"])
    assert o1["rhs"] == o0["rhs"]
    np.testing.assert_array_equal(o1["grad"], o0["grad"])


def test_lr_one_launch_per_step_teacher_forced_against_the_oracle(par):
    # the same path against the oracle, step by step (every step ends with a state query, so each
    # launch here is a plain tile launch followed by the stand-alone finish) and on its own for a
    # run of 40 steps (every launch but the first carries the finish of the step before)
    from paper_2201_04301_amd import binding as B
    w = scaled(CONFIGS["lr_4k"], rows=1024, c=0.5)
    Xs, ys = make_shards(w, "cuda")
    idx = make_indices(w, 40)
    worst = par.teacher_forced(w, 8, Xs, ys, idx, options=((B.GCADA_OPT_DEFERRED_FINISH, 1),))
    _say(worst)
    r = par.free_running(w, 40, Xs, ys, idx, options=((B.GCADA_OPT_DEFERRED_FINISH, 1),))
    agree = (r["masks_gpu"] == r["masks_oracle"]).mean()
    _say("mask agreement", agree, "loss", r["loss_gpu"][0], "->", r["loss_gpu"][-1], r["loss_oracle"][-1])
    assert agree >= 0.98
    np.testing.assert_allclose(r["loss_gpu"], r["loss_oracle"], rtol=2e-3)
    np.testing.assert_allclose(r["theta_gpu"], r["theta_oracle"], rtol=0, atol=2e-3 * np.abs(r["theta_oracle"]).max())
