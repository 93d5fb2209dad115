"""Pins for the fp64 oracle: each test ties a part of it to something the paper or the
mathematics fixes (closed forms, finite differences, library autograd, special cases)."""
import math
import os

import numpy as np
import pytest
import torch

import oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed=0):
    return np.random.default_rng(seed)


def _lr_data(rng, n, d, flip=0.1):
    X = (rng.normal(size=(n, d)) / math.sqrt(d)).astype(np.float32)
    w = rng.normal(size=d)
    y = np.where(X @ w >= 0, 1.0, -1.0)
    fl = rng.random(n) < flip
    y = np.where(fl, -y, y).astype(np.float32)
    return X, y


def _mlp_data(rng, n, d, ncls):
    X = rng.random(size=(n, d)).astype(np.float32)
    y = rng.integers(0, ncls, size=n).astype(np.int32)
    return X, y


def _mlp_theta(rng, widths, scale=1.0):
    parts = []
    for l in range(1, len(widths)):
        b = scale / math.sqrt(widths[l - 1])
        parts.append(rng.uniform(-b, b, size=widths[l] * widths[l - 1]))
        parts.append(rng.uniform(-0.1, 0.1, size=widths[l]))
    return np.concatenate(parts)


# ---------------------------------------------------------------- gradients (step a1)

def test_logistic_at_zero_closed_form():
    # theta = 0: every sample's loss is ln 2 and sigmoid(0) = 1/2, so grad = -1/2 sum y_i x_i.
    rng = _rng(1)
    X, y = _lr_data(rng, 37, 11)
    cfg = O.Config(O.LOGISTIC, [11], batch=37, G=1)
    loss, g = O.loss_grad_sum(cfg, np.zeros(11), X, y)
    assert loss == pytest.approx(37 * math.log(2.0), rel=1e-14)
    np.testing.assert_allclose(g, -0.5 * (y[:, None].astype(np.float64) * X).sum(0), rtol=1e-13)


@pytest.mark.parametrize("model,widths,l2", [
    (O.LOGISTIC, [13], 0.0), (O.LOGISTIC, [13], 1e-2), (O.QUADRATIC, [9], 0.0),
    (O.MLP, [7, 5, 3], 0.0), (O.MLP, [6, 8, 5, 4], 1e-3), (O.MLP, [5, 4], 0.0)])
def test_gradient_matches_central_differences(model, widths, l2):
    rng = _rng(2)
    n = 9
    if model == O.MLP:
        X, y = _mlp_data(rng, n, widths[0], widths[-1])
        cfg = O.Config(model, widths, batch=n, G=1, l2=l2)
        theta = _mlp_theta(rng, widths)
    else:
        X, y = _lr_data(rng, n, widths[0])
        if model == O.QUADRATIC:
            y = rng.normal(size=n).astype(np.float32)
        cfg = O.Config(model, widths, batch=n, G=1, l2=l2)
        theta = rng.normal(size=widths[0])
    _, g = O.loss_grad_sum(cfg, theta, X, y)
    eps = 1e-6
    fd = np.empty_like(theta)
    for j in range(theta.size):
        tp, tm = theta.copy(), theta.copy()
        tp[j] += eps
        tm[j] -= eps
        lp, _ = O.loss_grad_sum(cfg, tp, X, y, want_grad=False)
        lm, _ = O.loss_grad_sum(cfg, tm, X, y, want_grad=False)
        fd[j] = (lp - lm) / (2 * eps)
    np.testing.assert_allclose(g, fd, rtol=2e-6, atol=2e-8 * np.abs(g).max())


def test_logistic_matches_library_autograd():
    rng = _rng(3)
    X, y = _lr_data(rng, 50, 17)
    lam = 3e-3
    cfg = O.Config(O.LOGISTIC, [17], batch=50, G=1, l2=lam)
    theta = rng.normal(size=17)
    loss, g = O.loss_grad_sum(cfg, theta, X, y)
    t = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    Xt = torch.tensor(X, dtype=torch.float64)
    y01 = torch.tensor((y + 1) / 2, dtype=torch.float64)
    # binary cross-entropy with logits on labels in {0,1} is the logistic loss on +-1 labels
    ref = torch.nn.functional.binary_cross_entropy_with_logits(Xt @ t, y01, reduction="sum")
    ref = ref + 50 * 0.5 * lam * (t * t).sum()
    ref.backward()
    assert loss == pytest.approx(ref.item(), rel=1e-12)
    np.testing.assert_allclose(g, t.grad.numpy(), rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("widths", [[12, 4], [10, 16, 5], [9, 7, 6, 3]])
def test_mlp_matches_library_autograd(widths):
    rng = _rng(4)
    n = 21
    X, y = _mlp_data(rng, n, widths[0], widths[-1])
    theta = _mlp_theta(rng, widths, scale=2.0)
    cfg = O.Config(O.MLP, widths, batch=n, G=1)
    loss, g = O.loss_grad_sum(cfg, theta, X, y)
    t = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    a = torch.tensor(X, dtype=torch.float64)
    off = 0
    L = len(widths) - 1
    for l in range(1, L + 1):
        nw = widths[l] * widths[l - 1]
        W = t[off:off + nw].view(widths[l], widths[l - 1])
        b = t[off + nw:off + nw + widths[l]]
        off += nw + widths[l]
        a = torch.nn.functional.linear(a, W, b)
        if l < L:
            a = torch.relu(a)
    ref = torch.nn.functional.cross_entropy(a, torch.tensor(y, dtype=torch.int64), reduction="sum")
    ref.backward()
    assert loss == pytest.approx(ref.item(), rel=1e-12)
    np.testing.assert_allclose(g, t.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_mlp_zero_weights_uniform_softmax():
    # all-zero parameters: logits 0, loss = ln(classes) per sample; only the last bias has gradient
    widths = [6, 5, 4]
    rng = _rng(5)
    X, y = _mlp_data(rng, 10, 6, 4)
    cfg = O.Config(O.MLP, widths, batch=10, G=1)
    p = O.param_count(cfg)
    assert p == 6 * 5 + 5 + 5 * 4 + 4
    loss, g = O.loss_grad_sum(cfg, np.zeros(p), X, y)
    assert loss == pytest.approx(10 * math.log(4.0), rel=1e-14)
    expect_b = 10 * 0.25 - np.bincount(y, minlength=4)
    np.testing.assert_allclose(g[-4:], expect_b, atol=1e-13)
    assert np.all(g[:-4] == 0)


def test_two_class_softmax_layer_is_logistic():
    # one affine layer with two classes and no bias: CE(softmax) == logistic loss with
    # theta = w_1 - w_0 on labels +-1; d/dw_1 = -d/dw_0 = logistic gradient.
    rng = _rng(6)
    d, n = 8, 15
    X, ypm = _lr_data(rng, n, d)
    W = rng.normal(size=(2, d))
    theta_mlp = np.concatenate([W.ravel(), np.zeros(2)])
    ycls = ((ypm + 1) / 2).astype(np.int32)
    lm, gm = O.loss_grad_sum(O.Config(O.MLP, [d, 2], batch=n, G=1), theta_mlp, X, ycls)
    ll, gl = O.loss_grad_sum(O.Config(O.LOGISTIC, [d], batch=n, G=1), W[1] - W[0], X, ypm)
    assert lm == pytest.approx(ll, rel=1e-12)
    np.testing.assert_allclose(gm[d:2 * d], gl, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(gm[:d], -gl, rtol=1e-10, atol=1e-13)


def test_bf16_rounding_matches_library():
    rng = _rng(7)
    v = np.concatenate([rng.normal(size=2000), rng.normal(size=500) * 1e-3, [0.0, 1.0, -1.0,
                        1.00390625, 1.01171875, 3.0e38, 1e-40]])
    ref = torch.tensor(v, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64)
    got = np.array([O.bf16_round(x) for x in v])
    np.testing.assert_array_equal(got, ref.numpy())


# ---------------------------------------------------------------- server update (step a4)

def test_amsgrad_constant_gradient_closed_forms():
    # Eq. (8a)-(8c) with a constant aggregate g:  h^k = (1-b1^k) g,  vhat^k = (1-b2^k) g^2,
    # theta^k = theta^0 - alpha sum_{j<=k} (1-b1^j) g / sqrt(eps + (1-b2^j) g^2)
    rng = _rng(8)
    p, K = 7, 25
    g = rng.normal(size=p) * np.array([1e-3, 1, 10, 1e-6, 3, 0.5, 100])
    a, b1, b2, eps = 0.02, 0.9, 0.99, 1e-8
    theta0 = rng.normal(size=p)
    theta, h, vh = theta0.copy(), np.zeros(p), np.zeros(p)
    acc = np.zeros(p)
    for k in range(1, K + 1):
        prev = theta.copy()
        sq = O.amsgrad(theta, h, vh, g.copy(), a, b1, b2, eps)
        acc += (1 - b1 ** k) * g / np.sqrt(eps + (1 - b2 ** k) * g * g)
        np.testing.assert_allclose(h, (1 - b1 ** k) * g, rtol=1e-12)
        np.testing.assert_allclose(vh, (1 - b2 ** k) * g * g, rtol=1e-12)
        np.testing.assert_allclose(theta, theta0 - a * acc, rtol=1e-11, atol=1e-13)
        assert sq == pytest.approx(((theta - prev) ** 2).sum(), rel=1e-12)


def test_amsgrad_first_step_sign_limit():
    # from zero state: dtheta_i = -alpha (1-b1) g_i / sqrt(eps + (1-b2) g_i^2)
    #                 -> -alpha (0.1/sqrt(0.001)) sign(g_i) for |g_i| >> sqrt(eps/(1-b2))
    g = np.array([5.0, -2.0, 0.3, -40.0])
    theta, h, vh = np.zeros(4), np.zeros(4), np.zeros(4)
    sq = O.amsgrad(theta, h, vh, g, 1e-2, 0.9, 0.999, 1e-8)
    np.testing.assert_allclose(theta, -1e-2 * 0.1 * g / np.sqrt(1e-8 + 0.001 * g * g), rtol=1e-13)
    np.testing.assert_allclose(theta, -1e-2 * 0.1 / math.sqrt(0.001) * np.sign(g), rtol=1e-4)
    assert sq == pytest.approx(4 * 10.0 * 1e-4, rel=1e-4)


def test_amsgrad_worked_example_from_golden():
    # hand-worked sequence (tests/golden/amsgrad_worked.txt) that separates Eq. (8b)'s
    # "v from the previous v-hat" from the stock "v from the previous v", and eps inside the
    # root from eps outside it.
    rows = [l.split() for l in open(os.path.join(GOLD, "amsgrad_worked.txt"))
            if l.strip() and not l.startswith("#")]
    hdr = {k: float(v) for k, v in (kv.split("=") for kv in rows[0])}
    theta, h, vh = np.zeros(1), np.zeros(1), np.zeros(1)
    for r in rows[1:]:
        g, h_e, vh_e, th_e = map(float, r)
        O.amsgrad(theta, h, vh, np.array([g]), hdr["alpha"], hdr["beta1"], hdr["beta2"], hdr["eps"])
        assert h[0] == pytest.approx(h_e, rel=1e-9, abs=1e-12)
        assert vh[0] == pytest.approx(vh_e, rel=1e-9)
        assert theta[0] == pytest.approx(th_e, rel=1e-9)


# ---------------------------------------------------------------- whole iteration (a2, a3)

def _make_run(model, widths, G, mu, rows, seed, **kw):
    rng = _rng(seed)
    Xs, ys = [], []
    for g in range(G):
        if model == O.MLP:
            X, y = _mlp_data(rng, rows, widths[0], widths[-1])
        else:
            X, y = _lr_data(rng, rows, widths[0])
            if model == O.QUADRATIC:
                y = rng.normal(size=rows).astype(np.float32)
        Xs.append(X)
        ys.append(y)
    cfg = O.Config(model, widths, batch=mu, G=G, **kw)
    theta0 = _mlp_theta(rng, widths) if model == O.MLP else np.zeros(widths[0])
    return cfg, Xs, ys, theta0


@pytest.mark.parametrize("model,widths", [(O.LOGISTIC, [12]), (O.MLP, [6, 5, 3])])
def test_c_zero_is_distributed_amsgrad(model, widths):
    # c = 0: every group uploads every step (Sec. V, distributed Adam), so the aggregate is the
    # plain sum of fresh group gradients and theta follows Eq. (8a)-(8c) on that sum.
    cfg, Xs, ys, theta0 = _make_run(model, widths, G=4, mu=8, rows=40, seed=11, c=0.0, D=5)
    orc = O.Oracle(cfg, theta0)
    theta, h, vh = theta0.astype(np.float64).copy(), np.zeros(orc.p), np.zeros(orc.p)
    for k in range(23):
        rows = O.cyclic_window(k, 8, 40)
        agg = np.zeros(orc.p)
        one = O.Config(model, widths, batch=8, G=1)
        for g in range(4):
            agg += O.loss_grad_sum(one, theta, Xs[g][rows], ys[g][rows])[1]
        O.amsgrad(theta, h, vh, agg, cfg.alpha, cfg.beta1, cfg.beta2, cfg.eps)
        mask, _ = orc.step_shards(Xs, ys)
        assert mask.all()
        np.testing.assert_allclose(orc.agg, agg, rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(orc.theta, theta, rtol=1e-10, atol=1e-13)
        assert (orc.tau == 1).all()


def test_huge_c_gives_periodic_forced_uploads():
    # c -> infinity: the rule never fires, uploads happen only when the age reaches D
    # (Algorithm 1): all groups at k = 0, D, 2D, ...; the aggregate is frozen in between.
    D = 4
    cfg, Xs, ys, theta0 = _make_run(O.LOGISTIC, [10], G=3, mu=6, rows=30, seed=12, c=1e30, D=D)
    orc = O.Oracle(cfg, theta0)
    prev_agg = None
    for k in range(3 * D + 2):
        mask, _ = orc.step_shards(Xs, ys)
        if k % D == 0:
            assert mask.all(), k
        else:
            assert not mask.any(), k
            np.testing.assert_array_equal(orc.agg, prev_agg)
        prev_agg = orc.agg.copy()
        assert ((orc.tau >= 1) & (orc.tau <= D)).all()


def test_quadratic_statistic_is_gram_product():
    # squared loss: grad(theta) - grad(theta_stale) on the same rows = X^T X (theta - theta_stale)
    cfg, Xs, ys, _ = _make_run(O.QUADRATIC, [9], G=3, mu=7, rows=21, seed=13, c=1e30, D=6)
    rng = _rng(14)
    orc = O.Oracle(cfg, rng.normal(size=9))
    for k in range(9):
        theta = orc.theta.copy()
        stale = orc.theta_stale.copy()
        rows = O.cyclic_window(k, 7, 21)
        orc.step_shards(Xs, ys)
        for g in range(3):
            Xm = Xs[g][rows].astype(np.float64)
            s = Xm.T @ Xm @ (theta - stale[g])
            assert orc.stat[g] == pytest.approx(s @ s, rel=1e-9, abs=1e-18)
            np.testing.assert_allclose(orc.grad[g] - orc.grad_stale[g], s, rtol=1e-8, atol=1e-12)


def test_statistic_bounded_by_smoothness():
    # what Eq. (9)'s left side estimates: stat_g <= L^2 ||theta - theta_stale||^2 with
    # L = lambda_max(X^T X)/4 + mu*lambda for the logistic minibatch-sum loss.
    lam = 1e-2
    cfg, Xs, ys, theta0 = _make_run(O.LOGISTIC, [10], G=3, mu=8, rows=32, seed=15, c=50.0, D=5,
                                    l2=lam, alpha=0.05)
    orc = O.Oracle(cfg, theta0)
    seen_positive = False
    for k in range(30):
        theta, stale = orc.theta.copy(), orc.theta_stale.copy()
        rows = O.cyclic_window(k, 8, 32)
        orc.step_shards(Xs, ys)
        for g in range(3):
            Xm = Xs[g][rows].astype(np.float64)
            Lg = np.linalg.eigvalsh(Xm.T @ Xm).max() / 4 + 8 * lam
            bound = Lg ** 2 * ((theta - stale[g]) ** 2).sum()
            assert orc.stat[g] <= bound * (1 + 1e-9)
            seen_positive |= orc.stat[g] > 0
    assert seen_positive


@pytest.mark.parametrize("model,widths", [(O.LOGISTIC, [12]), (O.MLP, [5, 6, 3])])
def test_aggregate_identity_and_logged_gradients(model, widths):
    # Sec. IV aggregate: after every step agg = sum over groups of the gradient each group
    # uploaded last, evaluated at the iterate and on the minibatch of that upload.
    G, mu, nrows, D = 4, 6, 36, 5
    cfg, Xs, ys, theta0 = _make_run(model, widths, G=G, mu=mu, rows=nrows, seed=16, c=3.0, D=D,
                                    alpha=0.03)
    orc = O.Oracle(cfg, theta0)
    one = O.Config(model, widths, batch=mu, G=1)
    log = [None] * G
    theta_hist = [orc.theta.copy()]
    n_sel = 0
    for k in range(40):
        theta_k = orc.theta.copy()
        tau_before = orc.tau.copy()
        rhs_ring = orc.ring.copy()
        rows = O.cyclic_window(k, mu, nrows)
        mask, loss = orc.step_shards(Xs, ys)
        # threshold recomputed from the stored iterate history (Eq. (9) right side, c_d = c/D)
        diffs = [((theta_hist[j + 1] - theta_hist[j]) ** 2).sum()
                 for j in range(max(0, len(theta_hist) - 1 - D), len(theta_hist) - 1)]
        assert orc.rhs == pytest.approx(cfg.c / D * sum(diffs), rel=1e-12, abs=0)
        assert sum(rhs_ring) == pytest.approx(sum(diffs), rel=1e-12)
        for g in range(G):
            want = (orc.stat[g] > orc.rhs) or tau_before[g] >= D or orc.rhs == 0
            assert bool(mask[g]) == bool(want)
            if mask[g]:
                log[g] = (theta_k, rows)
                assert orc.tau[g] == 1
                np.testing.assert_array_equal(orc.theta_stale[g], theta_k)
            else:
                assert orc.tau[g] == tau_before[g] + 1
        n_sel += int(mask.sum())
        total = np.zeros(orc.p)
        for g in range(G):
            th, rw = log[g]
            gl = O.loss_grad_sum(one, th, Xs[g][rw], ys[g][rw])[1]
            np.testing.assert_allclose(orc.last[g], gl, rtol=1e-12, atol=1e-15)
            total += gl
        np.testing.assert_allclose(orc.agg, total, rtol=1e-9, atol=1e-12)
        # mean minibatch loss at theta^k
        ls = sum(O.loss_grad_sum(one, theta_k, Xs[g][rows], ys[g][rows], False)[0] for g in range(G))
        assert loss == pytest.approx(ls / (G * mu), rel=1e-12)
        theta_hist.append(orc.theta.copy())
        assert ((orc.tau >= 1) & (orc.tau <= D)).all()
    # the run must exercise both branches of the rule
    assert G * 4 < n_sel < G * 40


def test_identical_groups_and_permutation():
    G, mu, nrows = 4, 5, 20
    cfg, Xs, ys, theta0 = _make_run(O.LOGISTIC, [8], G=G, mu=mu, rows=nrows, seed=17, c=2.0, D=4,
                                    alpha=0.05)
    Xs[2], ys[2] = Xs[0].copy(), ys[0].copy()          # groups 0 and 2 hold the same shard
    perm = [3, 0, 2, 1]
    a = O.Oracle(cfg, theta0)
    b = O.Oracle(cfg, theta0)
    for k in range(25):
        ma, _ = a.step_shards(Xs, ys)
        mb, _ = b.step_shards([Xs[i] for i in perm], [ys[i] for i in perm])
        assert a.stat[0] == a.stat[2] and ma[0] == ma[2]
        np.testing.assert_array_equal(a.grad[0], a.grad[2])
        np.testing.assert_array_equal(mb, ma[perm])
        np.testing.assert_allclose(b.theta, a.theta, rtol=1e-11, atol=1e-14)


def test_bf16_mode_evaluates_at_rounded_iterate():
    widths = [6, 5, 3]
    cfg, Xs, ys, theta0 = _make_run(O.MLP, widths, G=2, mu=4, rows=8, seed=18, c=1.0, D=3)
    cfgb = O.Config(O.MLP, widths, batch=4, G=2, D=3, round_bf16=True)
    orc = O.Oracle(cfgb, theta0)
    one = O.Config(O.MLP, widths, batch=4, G=1)
    for k in range(4):
        th = orc.theta.copy()
        rows = O.cyclic_window(k, 4, 8)
        orc.step_shards(Xs, ys)
        thr = torch.tensor(th).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
        np.testing.assert_allclose(orc.grad[1], O.loss_grad_sum(one, thr, Xs[1][rows], ys[1][rows])[1],
                                   rtol=1e-13, atol=0)
    assert not np.array_equal(orc.theta, torch.tensor(orc.theta).to(torch.bfloat16).to(torch.float64).numpy())


def test_zero_threshold_selects_even_when_nothing_moves():
    # degenerate case: all-zero features give a zero gradient, the iterate never moves, so both
    # sides of the rule are 0; the reading taken is "threshold 0 => upload", which keeps
    # "c = 0 <=> distributed AMSGrad" exact.
    cfg = O.Config(O.LOGISTIC, [5], batch=3, G=2, D=4, c=0.0)
    orc = O.Oracle(cfg, np.ones(5))
    X = np.zeros((2, 3, 5), dtype=np.float32)
    y = np.ones((2, 3), dtype=np.float32)
    for k in range(6):
        mask, loss = orc.step(X, y)
        assert mask.all() and orc.rhs == 0.0 and (orc.stat == 0).all()
        assert loss == pytest.approx(math.log(2.0))
        np.testing.assert_array_equal(orc.theta, np.ones(5))


# ---------------------------------------------------------------- the server-side rule (Sec. IV)

def test_server_rule_c_zero_equals_statistic_rule_c_zero():
    # c = 0 selects every group every step under either rule, so the two runs are the same
    # distributed AMSGrad, bit for bit (the gradients at theta^k are the same arithmetic).
    cfg, Xs, ys, theta0 = _make_run(O.QUADRATIC, [9], G=3, mu=6, rows=30, seed=21, c=0.0, D=4)
    a, b = O.Oracle(cfg, theta0), O.Oracle(cfg, theta0)
    b.set_rule(1, np.array([3.0, 0.5, 7.0]))
    for k in range(17):
        ma, la = a.step_shards(Xs, ys)
        mb, lb = b.step_shards(Xs, ys)
        assert ma.all() and mb.all()
        np.testing.assert_array_equal(a.theta, b.theta)
        assert la == lb


def test_server_rule_left_side_mask_and_lazy_evaluation():
    # left side = L_g^2 ||theta^k - theta^{k-tau_g}||^2 recomputed here; mask from it, the age
    # and the threshold; an unselected group's stored gradient, stale iterate and gradient
    # buffer are untouched (it evaluates nothing); aggregate == sum of stored gradients.
    D = 5
    cfg, Xs, ys, theta0 = _make_run(O.LOGISTIC, [11], G=4, mu=7, rows=35, seed=22, c=0.6, D=D,
                                    alpha=0.05)
    L = np.array([0.8, 1.7, 0.3, 2.5])
    orc = O.Oracle(cfg, theta0)
    orc.set_rule(1, L)
    held_back = fired_early = 0
    for k in range(40):
        theta, stale, tau = orc.theta.copy(), orc.theta_stale.copy(), orc.tau.copy()
        last, grad, ring = orc.last.copy(), orc.grad.copy(), orc.ring.copy()
        mask, loss = orc.step_shards(Xs, ys)
        rhs = cfg.c / D * ring.sum()
        lhs = L ** 2 * ((theta[None, :] - stale) ** 2).sum(1)
        np.testing.assert_allclose(orc.stat, lhs, rtol=1e-12)
        assert orc.rhs == pytest.approx(rhs, rel=1e-12)
        np.testing.assert_array_equal(mask, ((lhs > rhs) | (tau >= D) | (rhs == 0)).astype(np.uint8))
        rows = O.cyclic_window(k, 7, 35)
        one = O.Config(O.LOGISTIC, [11], batch=7, G=1)
        tot = 0.0
        for g in range(4):
            if mask[g]:
                l, gr = O.loss_grad_sum(one, theta, Xs[g][rows], ys[g][rows])
                np.testing.assert_allclose(orc.last[g], gr, rtol=1e-12)
                np.testing.assert_array_equal(orc.theta_stale[g], theta)
                tot += l
                fired_early += int(tau[g] < D)
            else:
                np.testing.assert_array_equal(orc.last[g], last[g])
                np.testing.assert_array_equal(orc.theta_stale[g], stale[g])
                np.testing.assert_array_equal(orc.grad[g], grad[g])
                held_back += 1
        if mask.any():
            assert loss == pytest.approx(tot / (mask.sum() * 7), rel=1e-12)
        else:
            assert loss == 0.0
        np.testing.assert_allclose(orc.agg, orc.last.sum(0), rtol=1e-9, atol=1e-12)
        assert ((orc.tau >= 1) & (orc.tau <= D)).all()
    assert held_back > 0 and fired_early > 0


def test_server_rule_huge_c_periodic():
    D = 3
    cfg, Xs, ys, theta0 = _make_run(O.QUADRATIC, [8], G=2, mu=5, rows=20, seed=23, c=1e30, D=D)
    orc = O.Oracle(cfg, theta0)
    orc.set_rule(1, np.array([1.0, 1.0]))
    for k in range(3 * D + 1):
        mask, _ = orc.step_shards(Xs, ys)
        assert mask.all() if k % D == 0 else not mask.any()


def test_server_rule_left_side_bounds_the_statistic():
    # the bridge between the two rules (L-smoothness): with L_g >= the largest eigenvalue of the
    # minibatch Gram matrix, the same-minibatch gradient difference of the quadratic loss never
    # exceeds the server-side left side, so the server-side rule selects whenever the other does.
    cfg, Xs, ys, theta0 = _make_run(O.QUADRATIC, [9], G=3, mu=6, rows=30, seed=24, c=0.4, D=4,
                                    alpha=0.05)
    a = O.Oracle(cfg, theta0)
    for k in range(25):
        theta, stale = a.theta.copy(), a.theta_stale.copy()
        rows = O.cyclic_window(k, 6, 30)
        a.step_shards(Xs, ys)
        for g in range(3):
            Xm = Xs[g][rows].astype(np.float64)
            Lg = np.linalg.eigvalsh(Xm.T @ Xm).max()
            assert a.stat[g] <= Lg ** 2 * ((theta - stale[g]) ** 2).sum() * (1 + 1e-9)
