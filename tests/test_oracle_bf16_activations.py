"""Pins for the oracle's bf16 configuration with rounded hidden activations (round_bf16 = 2).

The bf16 workload is stated as "bf16 inputs and weights, fp32 accumulation".  The reading taken is
that EVERY layer's matrix product has bf16 inputs, i.e. the hidden activations are stored in
bf16.  That matters beyond a tolerance: the sign of the next layer's pre-activation chooses the
ReLU branch, a discrete decision, and both sides of a comparison have to take it from the same
values.  These tests tie the mode to (a) library autograd with the library's own bf16 conversion
applied to the hidden activations (identity in the backward pass), (b) a hand-built network in
which the rounding moves a unit of the next layer across its kink, (c) the unrounded mode when
every activation is representable in bf16 anyway.
"""
import math

import numpy as np
import pytest
import torch

import oracle as O


def _bf16(t):
    return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def _torch_loss_grad(widths, theta, X, y):
    """Sum of softmax cross-entropies and its gradient by library autograd; hidden activations
    pass through the library's bf16 conversion with a straight-through backward."""
    t = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    a = torch.tensor(np.asarray(X, dtype=np.float64))
    off, L = 0, len(widths) - 1
    for l in range(1, L + 1):
        nw = widths[l] * widths[l - 1]
        W = t[off:off + nw].view(widths[l], widths[l - 1])
        b = t[off + nw:off + nw + widths[l]]
        off += nw + widths[l]
        a = torch.nn.functional.linear(a, W, b)
        if l < L:
            a = torch.relu(a)
            a = a + (_bf16(a) - a).detach()
    loss = torch.nn.functional.cross_entropy(a, torch.tensor(np.asarray(y), dtype=torch.long), reduction="sum")
    loss.backward()
    return loss.item(), t.grad.numpy()


@pytest.mark.parametrize("widths", [[10, 16, 5], [9, 7, 6, 3], [12, 4]])
def test_rounded_activations_match_library_autograd(widths):
    rng = np.random.default_rng(41)
    n = 23
    X = _bf16(torch.tensor(rng.random(size=(n, widths[0])) * 2 - 1)).numpy().astype(np.float32)
    y = rng.integers(0, widths[-1], size=n).astype(np.int32)
    parts = []
    for l in range(1, len(widths)):
        b = 2.0 / math.sqrt(widths[l - 1])
        parts.append(rng.uniform(-b, b, size=widths[l] * widths[l - 1]))
        parts.append(rng.uniform(-0.1, 0.1, size=widths[l]))
    theta = _bf16(torch.tensor(np.concatenate(parts))).numpy()
    cfg = O.Config(O.MLP, widths, batch=n, G=1, round_bf16=2)
    loss, g = O.loss_grad_sum(cfg, theta, X, y)
    ref_loss, ref_g = _torch_loss_grad(widths, theta, X, y)
    assert loss == pytest.approx(ref_loss, rel=1e-12)
    np.testing.assert_allclose(g, ref_g, rtol=1e-10, atol=1e-13)
    if len(widths) > 2:
        # and the rounding is really there: the unrounded mode gives another gradient
        _, g1 = O.loss_grad_sum(O.Config(O.MLP, widths, batch=n, G=1, round_bf16=1), theta, X, y)
        assert np.abs(g1 - g).max() > 1e-5 * np.abs(g).max()


def _theta(layers):
    parts = []
    for W, b in layers:
        parts.append(np.asarray(W, dtype=np.float64).reshape(-1))
        parts.append(np.asarray(b, dtype=np.float64))
    return np.concatenate(parts)


def test_rounding_moves_the_next_layer_across_its_kink():
    # a_1 = (x0, x1) = (1 + 2^-9, 1).  In bf16 (8 significant bits) 1 + 2^-9 becomes 1.
    # second hidden layer, unit 0: z = a_1[0] - a_1[1] = 2^-9 unrounded (active), 0 rounded
    # (inactive: ReLU'(0) = 0); unit 1 = a_1[0] + a_1[1], always active.  Output: logits
    # (a_2[0], 0), label 0 -- so unit 0's weights get a gradient only when it is active.
    W1 = [[1, 0], [0, 1]]
    W2 = [[1, -1], [1, 1]]
    W3 = [[1, 0], [0, 0]]
    th = _theta([(W1, [0, 0]), (W2, [0, 0]), (W3, [0, 0])])
    X = np.array([[1 + 2.0 ** -9, 1.0]], dtype=np.float32)
    y = np.array([0], dtype=np.int32)
    g = {}
    for mode in (1, 2):
        cfg = O.Config(O.MLP, [2, 2, 2, 2], batch=1, G=1, round_bf16=mode)
        _, g[mode] = O.loss_grad_sum(cfg, th, X, y)
    gW2 = lambda v: v[6:10].reshape(2, 2)           # layout: W1 (4), b1 (2), W2 (4), b2 (2), W3, b3
    # unrounded: logits (2^-9, 0), dlogit_0 = softmax_0 - 1; unit 0 active: dW2[0] = dlogit_0 * a_1
    p0 = 1.0 / (1.0 + math.exp(-2.0 ** -9))
    np.testing.assert_allclose(gW2(g[1])[0], (p0 - 1.0) * np.array([1 + 2.0 ** -9, 1.0]), rtol=1e-14)
    # rounded: unit 0 sits exactly on the kink: no gradient through it
    np.testing.assert_array_equal(gW2(g[2])[0], [0.0, 0.0])
    # the weight gradient of the FIRST layer's successor multiplies the ROUNDED activation:
    # unit 1 is active in both; it feeds no logit (W3 column 1 is zero), so use W3's own gradient:
    # dW3[0] = dlogit_0 * a_2 with a_2 = (0, 2) rounded, (2^-9, 2 + 2^-9) unrounded
    gW3 = lambda v: v[12:16].reshape(2, 2)
    np.testing.assert_allclose(gW3(g[2])[0], (0.5 - 1.0) * np.array([0.0, 2.0]), rtol=1e-14)
    np.testing.assert_allclose(gW3(g[1])[0], (p0 - 1.0) * np.array([2.0 ** -9, 2 + 2.0 ** -9]), rtol=1e-14)


def test_representable_activations_make_both_modes_equal():
    # small integers times powers of two: every activation is exact in bf16, so rounding the
    # activations changes nothing, bit for bit
    rng = np.random.default_rng(5)
    widths = [4, 3, 3, 2]
    X = rng.integers(-2, 3, size=(6, 4)).astype(np.float32)
    y = rng.integers(0, 2, size=6).astype(np.int32)
    th = _theta([(rng.integers(-1, 2, size=(3, 4)), rng.integers(-1, 2, size=3) * 0.5),
                 (rng.integers(-1, 2, size=(3, 3)), [0.5, 0, -0.5]),
                 (rng.integers(-1, 2, size=(2, 3)) * 0.25, [0, 0])])
    out = [O.loss_grad_sum(O.Config(O.MLP, widths, batch=6, G=1, round_bf16=m), th, X, y) for m in (1, 2)]
    assert out[0][0] == out[1][0]
    np.testing.assert_array_equal(out[0][1], out[1][1])
    assert np.abs(out[0][1]).max() > 0


def test_step_in_mode_2_rounds_iterates_and_activations():
    # the iteration evaluates both gradients at the bf16-rounded iterates with rounded activations
    rng = np.random.default_rng(9)
    widths = [6, 5, 4, 3]
    G, mu = 2, 5
    X = rng.random(size=(G, mu, 6)).astype(np.float32)
    y = rng.integers(0, 3, size=(G, mu)).astype(np.int32)
    p = O.param_count(O.Config(O.MLP, widths, batch=mu, G=G))
    theta = rng.normal(size=p) * 0.4
    stale = theta + 0.01 * rng.normal(size=(G, p))
    orc = O.Oracle(O.Config(O.MLP, widths, batch=mu, G=G, D=3, round_bf16=2), theta)
    orc.theta_stale[...] = stale
    orc.step(X, y)
    one = O.Config(O.MLP, widths, batch=mu, G=1, round_bf16=2)
    for g in range(G):
        tr = _bf16(torch.tensor(theta)).numpy()
        sr = _bf16(torch.tensor(stale[g])).numpy()
        np.testing.assert_allclose(orc.grad[g], O.loss_grad_sum(one, tr, X[g], y[g])[1], rtol=1e-13)
        np.testing.assert_allclose(orc.grad_stale[g], O.loss_grad_sum(one, sr, X[g], y[g])[1], rtol=1e-13)
        ref = _torch_loss_grad(widths, tr, X[g], y[g])[1]
        np.testing.assert_allclose(orc.grad[g], ref, rtol=1e-10, atol=1e-13)
