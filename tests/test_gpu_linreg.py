"""GPU parity of the linear-regression model with the quadratic error loss (the model of the
paper's experiment, Sec. VI) with the fp64 oracle, through the C-ABI.  It runs on the kernels of
the logistic path; only the residual of a row differs."""
import numpy as np
import pytest

from gcada_inputs import CONFIGS, make_indices, make_shards, scaled

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def par():
    import parity
    return parity


def _say(*a):
    print(*a, flush=True)


def test_linreg_784_experiment_geometry(par):
    # M = 12 workers, G = 3 groups of 4, width 784, shorter shards; general two-pass kernels
    w = scaled(CONFIGS["linreg_784"], rows=2000)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    steps = 60
    idx = make_indices(w, steps)
    worst = par.teacher_forced(w, steps, Xs, ys, idx)
    _say(worst)
    assert 0 < worst["selected"] < w.G * steps      # the rule both fires and holds back


@pytest.mark.parametrize("d,mu,G,rows,l2,use_idx", [
    (67, 33, 3, 100, 1e-3, True),        # ragged: scalar general kernels
    (4096, 64, 4, 300, 0.0, True),       # whole-row register tiles
    (1024, 128, 3, 200, 1e-4, False),    # tiles, cyclic window
    (8192, 32, 3, 80, 0.0, True),        # teams of two workgroups
    (65536, 16, 2, 40, 0.0, True),       # teams of sixteen workgroups
])
def test_linreg_shapes(par, d, mu, G, rows, l2, use_idx):
    w = scaled(CONFIGS["linreg_784"], name="linreg", widths=(d,), mu=mu, G=G, rows=rows, l2=l2, D=4,
               c=1.0)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    steps = 12
    idx = make_indices(w, steps) if use_idx else None
    worst = par.teacher_forced(w, steps, Xs, ys, idx)
    _say(worst)


def test_linreg_free_run_tracks_oracle(par):
    w = scaled(CONFIGS["linreg_784"], rows=1000, mu=64)
    Xs, ys = make_shards(w, "cuda")
    steps = 80
    idx = make_indices(w, steps)
    r = par.free_running(w, steps, Xs, ys, idx)
    agree = (r["masks_gpu"] == r["masks_oracle"]).mean()
    _say("mask agreement", agree, "loss", r["loss_gpu"][0], "->", r["loss_gpu"][-1], r["loss_oracle"][-1])
    assert agree >= 0.98
    np.testing.assert_allclose(r["loss_gpu"], r["loss_oracle"], rtol=2e-3)
    assert r["loss_gpu"][-1] < 0.9 * r["loss_gpu"][0]
