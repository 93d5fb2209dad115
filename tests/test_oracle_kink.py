"""Pin for the oracle's ReLU-kink diagnostic.

The MLP parity tests use `Oracle.kink` to decide which groups' statistic / mask they may skip (a
hidden pre-activation within rounding of zero has two valid subgradients), so a wrong value there
would silently excuse failures.  Here small networks are built by hand, in powers of two so that
every pre-activation and every sum of magnitudes is exact in binary floating point, and the value
the oracle reports is compared with the number worked out by hand:

    kink_g = min over the group's samples, over BOTH iterates the group evaluates, over the hidden
             layers (not the output layer) and their units with a non-empty sum, of
             |z| / (|b| + sum_i |w_i a_i|),        1 when there is no such unit.
"""
import numpy as np

import oracle as O


def _theta(layers):
    """layers: [(W out x in, b out), ...] -> flat parameter vector (W row-major, then b, per layer)."""
    parts = []
    for W, b in layers:
        parts.append(np.asarray(W, dtype=np.float64).reshape(-1))
        parts.append(np.asarray(b, dtype=np.float64))
    return np.concatenate(parts)


def _step(widths, theta, theta_stale, X, y):
    G, mu = X.shape[0], X.shape[1]
    cfg = O.Config(O.MLP, widths, batch=mu, G=G, D=3)
    orc = O.Oracle(cfg, theta)
    orc.theta_stale[...] = theta_stale
    orc.step(X.astype(np.float32), y.astype(np.int32))
    if orc.kink_unit.shape[1]:
        np.testing.assert_array_equal(orc.kink, orc.kink_unit.min(axis=1))
    _step.units = orc.kink_unit.copy()           # the same per hidden unit, layer 1's units first
    return orc.kink.copy()


def test_kink_value_hidden_layer_only_and_empty_units_ignored():
    # 3 -> 3 -> 2.  hidden unit 0: z = (1 + 2^-20) - 1 = 2^-20, magnitudes 2 + 2^-20
    #               hidden unit 1: z = 0.5 + 0.5 + 0.25 = 1.25 (far from the kink: ratio 1)
    #               hidden unit 2: no weights, no bias: z = 0 with an EMPTY sum -> ignored
    # output unit 0: z = 1.25 - 1.25 = 0 exactly with magnitudes 2.5 -> would read 0 if the
    #               output layer were included; output unit 1: empty.
    W1 = [[1, -1, 0], [0.5, 0.5, 0], [0, 0, 0]]
    b1 = [0, 0.25, 0]
    W2 = [[0, 1, 0], [0, 0, 0]]
    b2 = [-1.25, 0]
    th = _theta([(W1, b1), (W2, b2)])
    x = np.array([[[1 + 2.0 ** -20, 1, 0.5]]])            # one group, one sample
    kink = _step([3, 3, 2], th, th, x, np.array([[0]]))
    expected = 2.0 ** -20 / (2 + 2.0 ** -20)
    assert kink[0] == expected                              # exact: every term is a power-of-two sum
    # per unit: unit 0 as above, unit 1 at distance 1 (all its terms have one sign), unit 2 never counted
    np.testing.assert_array_equal(_step.units, [[expected, 1.0, 1.0]])
    # negative side of the kink counts the same (|z|)
    x = np.array([[[1, 1 + 2.0 ** -20, 0.5]]])
    kink = _step([3, 3, 2], th, th, x, np.array([[1]]))
    assert kink[0] == expected


def test_kink_includes_the_bias_in_the_magnitudes():
    # unit 0: z = 1 - 1 + 2^-10 (bias) -> magnitudes 1 + 1 + 2^-10
    W1 = [[1, -1], [1, 1]]
    b1 = [2.0 ** -10, 0]
    th = _theta([(W1, b1), ([[1, 1], [0, 1]], [0, 0])])
    kink = _step([2, 2, 2], th, th, np.array([[[1.0, 1.0]]]), np.array([[0]]))
    assert kink[0] == 2.0 ** -10 / (2 + 2.0 ** -10)


def test_kink_is_the_minimum_over_samples_and_over_both_iterates_per_group():
    # one hidden unit reading x0 - x1; three samples at distances 2^-4, 2^-12, 2^-8 from the kink
    W1 = [[1, -1], [1, 1]]
    th = _theta([(W1, [0, 0]), ([[1, 0], [0, 1]], [0, 0])])
    xs = [[1 + 2.0 ** -4, 1], [1 + 2.0 ** -12, 1], [1 + 2.0 ** -8, 1]]
    r = lambda e: 2.0 ** -e / (2 + 2.0 ** -e)
    # the stale iterate of group 1 reads x0 - (1 + 2^-12) x1 instead: sample 1 sits EXACTLY on its
    # kink (z = 0 with magnitudes > 0): the minimum over both iterates is 0 there
    th_stale1 = _theta([([[1, -(1 + 2.0 ** -12)], [1, 1]], [0, 0]), ([[1, 0], [0, 1]], [0, 0])])
    X = np.array([xs, xs], dtype=np.float64)
    kink = _step([2, 2, 2], th, np.stack([th, th_stale1]), X, np.zeros((2, 3)))
    assert kink[0] == r(12)           # group 0: the closest of its three samples
    assert kink[1] == 0.0             # group 1: its stale iterate is closer still
    np.testing.assert_array_equal(_step.units, [[r(12), 1.0], [0.0, 1.0]])     # per group and unit
    # and with the current iterate as the close one, the stale far away
    th_far = _theta([([[1, 1], [1, 1]], [0, 0]), ([[1, 0], [0, 1]], [0, 0])])
    kink = _step([2, 2, 2], th, np.stack([th_far, th_far]), X, np.zeros((2, 3)))
    assert kink[0] == r(12) and kink[1] == r(12)
    # a group whose samples are all far from every kink reports its own, larger, minimum
    X2 = X.copy()
    X2[1] = [[2, 1], [3, 1], [1.5, 1]]
    kink = _step([2, 2, 2], th, np.stack([th, th]), X2, np.zeros((2, 3)))
    assert kink[0] == r(12) and kink[1] == 0.5 / 2.5


def test_kink_covers_every_hidden_layer():
    # 2 -> 2 -> 2 -> 2: the first hidden layer is far from its kinks, the second one is close:
    # a1 = (x0 + x1, x0) = (2 + 2^-6, 1 + 2^-6); unit 0 of layer 2 reads a1_0 - 2 a1_1 = -2^-6,
    # magnitudes (2 + 2^-6) + (2 + 2^-5) = 4 + 3 * 2^-6
    W1 = [[1, 1], [1, 0]]
    W2 = [[1, -2], [1, 1]]
    W3 = [[1, 0], [0, 1]]
    th = _theta([(W1, [0, 0]), (W2, [0, 0]), (W3, [0, 0])])
    x = np.array([[[1 + 2.0 ** -6, 1.0]]])
    kink = _step([2, 2, 2, 2], th, th, x, np.array([[1]]))
    assert kink[0] == 2.0 ** -6 / (4 + 3 * 2.0 ** -6)
    # units in layer order: layer 1 (both far: one-signed sums), then layer 2 (unit 0 close, unit 1 far)
    np.testing.assert_array_equal(_step.units, [[1.0, 1.0, 2.0 ** -6 / (4 + 3 * 2.0 ** -6), 1.0]])


def test_kink_is_one_without_hidden_layers():
    th = _theta([([[1, -1], [0, 0]], [0, 0])])              # softmax regression: logits only
    kink = _step([2, 2], th, th, np.array([[[1.0, 1.0]]]), np.array([[0]]))
    assert kink[0] == 1.0
