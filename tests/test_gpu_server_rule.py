"""GPU parity under the selection rule as the paper states it for the parameter server (Sec. IV:
L_g^2 ||theta^k - theta^{k-tau_g}||^2 against the threshold; Algorithm 1: only the selected
groups evaluate a gradient, once), and the smoothness constants by power iteration."""
import numpy as np
import pytest
import torch

from gcada_inputs import CONFIGS, make_indices, make_shards, make_theta0, scaled

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def par():
    import parity
    return parity


def _say(*a):
    print(*a, flush=True)


def _exact_L(w, Xs):
    # textbook definition: kappa * lambda_max(X^T X) / rows + lambda, by a dense eigen-solver
    kappa = 1.0 if w.model == "linreg" else 0.25
    out = []
    for X in Xs:
        A = X.double().cpu().numpy()
        out.append(kappa * np.linalg.eigvalsh(A.T @ A).max() / A.shape[0] + w.l2)
    return np.array(out)


@pytest.mark.parametrize("model,d,rows,l2", [("logreg", 48, 300, 1e-3), ("linreg", 130, 500, 0.0)])
def test_power_iteration_matches_eigensolver(model, d, rows, l2):
    from paper_2201_04301_amd import Gcada
    w = scaled(CONFIGS["lr_small" if model == "logreg" else "linreg_784"], name="pi", widths=(d,),
               G=3, rows=rows, mu=16, l2=l2)
    Xs, ys = make_shards(w, "cuda")
    gpu = Gcada.from_workload(w)
    gpu.set_shards(Xs, ys)
    est = gpu.estimate_smoothness(iters=300)
    exact = _exact_L(w, Xs)
    _say("estimated", est, "exact", exact)
    # power iteration approaches the largest eigenvalue from below
    assert (est <= exact * (1 + 1e-6)).all() and (est >= 0.98 * exact).all()
    gpu.close()


@pytest.mark.parametrize("model,d,mu,G,rows,l2,c,use_idx", [
    ("logreg", 67, 33, 4, 100, 1e-3, 0.3, True),      # general scalar kernels
    ("logreg", 4096, 64, 5, 300, 1e-4, 0.5, True),    # whole-row register tiles
    ("linreg", 1024, 128, 4, 200, 0.0, 0.5, False),   # tiles, cyclic window, quadratic loss
    ("logreg", 8192, 32, 6, 80, 0.0, 0.3, True),      # teams of two workgroups
    ("linreg", 65536, 16, 3, 40, 0.0, 0.5, True),     # teams of sixteen workgroups
])
def test_server_rule_linear_models(par, model, d, mu, G, rows, l2, c, use_idx):
    base = CONFIGS["lr_small" if model == "logreg" else "linreg_784"]
    w = scaled(base, name="server_rule", widths=(d,), mu=mu, G=G, rows=rows, l2=l2, c=c, D=4, alpha=0.02)
    _say("case", w)
    Xs, ys = make_shards(w, "cuda")
    # the exact constants scaled per group, so that the groups fire at different times
    L = _exact_L(w, Xs) * np.linspace(0.4, 2.5, G) if d <= 4096 else np.linspace(0.05, 0.6, G)
    steps = 30
    idx = make_indices(w, steps) if use_idx else None
    worst = par.teacher_forced(w, steps, Xs, ys, idx, server_rule_L=L)
    _say(worst)
    assert 0 < worst["selected"] < G * steps


def test_server_rule_mlp(par):
    w = scaled(CONFIGS["mlp_784"], name="server_rule_mlp", widths=(64, 48, 10), mu=64, G=4, rows=300, D=4,
               c=0.5)
    Xs, ys = make_shards(w, "cuda")
    steps = 16
    idx = make_indices(w, steps)
    L = np.array([0.5, 2.0, 6.0, 12.0])
    worst = par.teacher_forced(w, steps, Xs, ys, idx, kink_tol=5e-8, server_rule_L=L)
    _say(worst)
    assert 0 < worst["selected"] < w.G * steps


def test_server_rule_bf16_mlp(par):
    w = scaled(CONFIGS["mlp_3072_bf16"], name="server_rule_bf16", widths=(256, 128, 10), mu=64, G=3,
               rows=200, D=4, c=0.5)
    Xs, ys = make_shards(w, "cuda")
    steps = 10
    idx = make_indices(w, steps)
    # (under this rule the left side is made of iterates, not of bf16 gradients: plain 1e-6 edge)
    worst = par.teacher_forced(w, steps, Xs, ys, idx, tol=2e-2, edge=1e-6, kink_unit_tol=1e-4,
                               server_rule_L=np.array([1.0, 5.0, 20.0]))
    _say(worst)


def test_switching_rules_on_the_tile_path(par):
    # whole-row tile path: both rules end in the same fused finish kernel (the server-side rule with
    # the mask as an input), so with c = 0 a run that alternates the rules equals one that never
    # switches, bit for bit; the history entry left per block by a default-rule step is completed
    # before the selection kernel of the next server-rule step reads it
    from paper_2201_04301_amd import Gcada
    w = scaled(CONFIGS["lr_small"], name="switch_tiles", widths=(1024,), mu=128, G=5, rows=300, c=0.0, D=4,
               l2=1e-4)
    Xs, ys = make_shards(w, "cuda")
    steps = 14
    idx = torch.as_tensor(make_indices(w, steps), device="cuda")
    res = []
    for alternate in (False, True):
        gpu = Gcada.from_workload(w)
        gpu.set_shards(Xs, ys)
        gpu.set_theta(make_theta0(w))
        for k in range(steps):
            if alternate:
                gpu.set_rule("server" if (k // 2) % 2 else "gradient_difference", np.ones(w.G))
            gpu.step(idx[k].contiguous())
        res.append(gpu.get_state())
        gpu.close()
    for name in ("theta", "h", "vhat", "agg", "last", "tau"):
        np.testing.assert_array_equal(res[0][name], res[1][name], err_msg=name)
    np.testing.assert_allclose(res[0]["dtheta_sq"], res[1]["dtheta_sq"], rtol=1e-12)


def test_switching_rules_between_steps(par):
    # c = 0 selects everybody under either rule: the iterates of a run that alternates the rules
    # equal those of a run that never switches -- bit for bit when both rules go through the same
    # kernels (general kernels forced), to rounding when the default rule takes the one-launch
    # kernel of small models and the server-side rule the general ones (other summation order)
    from paper_2201_04301_amd import Gcada, binding as B
    w = scaled(CONFIGS["lr_small"], c=0.0)
    Xs, ys = make_shards(w, "cuda")
    idx = torch.as_tensor(make_indices(w, 12), device="cuda")
    for single_pass in (0, 1):
        thetas = []
        for alternate in (False, True):
            gpu = Gcada.from_workload(w)
            B.gcada_set_option(gpu.ctx, B.GCADA_OPT_SINGLE_PASS_LOGREG, single_pass)
            gpu.set_shards(Xs, ys)
            gpu.set_theta(make_theta0(w))
            for k in range(12):
                if alternate:
                    gpu.set_rule("server" if k % 2 else "gradient_difference", np.ones(w.G))
                gpu.step(idx[k].contiguous())
            thetas.append(gpu.get_state()["theta"])
            gpu.close()
        if single_pass == 0:
            np.testing.assert_array_equal(thetas[0], thetas[1])
        else:
            np.testing.assert_allclose(thetas[0], thetas[1], rtol=0, atol=1e-5 * np.abs(thetas[1]).max())
