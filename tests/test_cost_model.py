"""Host cost model of the paper's Sec. II-B / Sec. V against its closed forms."""
import math

import numpy as np
import pytest

from gcada_inputs import CONFIGS, make_delays, scaled


def H(n):
    return sum(1.0 / i for i in range(1, n + 1))


def _cm(G, M_G, mu, mask, T):
    from paper_2201_04301_amd import binding as B
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    T = np.ascontiguousarray(T, dtype=np.float64)
    return B.gcada_cost_model(G, M_G, mu, mask.ctypes.data, T.ctypes.data)


def test_order_statistics_of_delays_match_eq10():
    # Eq. (10): E[a-th smallest of b iid Exp(mean eta)] = eta (H_b - H_{b-a})
    w = scaled(CONFIGS["lr_small"], G=1, M_G=7)
    eta = 1e-4
    T = make_delays(w, 200000, eta=eta)[:, 0, :]
    T.sort(axis=1)
    for a in range(1, 8):
        assert T[:, a - 1].mean() == pytest.approx(eta * (H(7) - H(7 - a)), rel=2e-2)


def test_counts_and_time_small_cases():
    T = np.array([[3.0, 1.0], [5.0, 4.0], [0.5, 9.0]])
    t, comm, comp = _cm(3, 2, 32, [1, 0, 1], T)
    assert t == 1.0 and comm == 2 * 3 and comp == 2 * 2 * 32       # max(min(3,1), min(.5,9))
    t, comm, comp = _cm(3, 2, 32, [1, 1, 1], T)
    assert t == 4.0 and comm == 3 * 3 and comp == 3 * 2 * 32       # Eq. (19), (22) with all groups
    t, comm, comp = _cm(3, 2, 32, [0, 0, 0], T)
    assert t == 0.0 and comm == 0 and comp == 0
    # a straggler that never finishes does not delay its group
    T2 = T.copy()
    T2[1, 0] = np.inf
    assert _cm(3, 2, 32, [0, 1, 0], T2)[0] == 4.0
    # M_G = 1: the server waits for every selected worker (Sec. III)
    assert _cm(3, 1, 8, [1, 1, 0], T[:, :1])[0] == 5.0


def test_mean_time_all_groups_selected_closed_form():
    # every group's time is the min of M_G iid Exp(eta) = Exp(eta/M_G); the max of G of them has
    # mean (eta/M_G) H_G  (Eq. (14) with the minimum's CDF, Eq. (10) with b = a = G)
    w = scaled(CONFIGS["lr_small"], G=5, M_G=4)
    eta = 1e-4
    T = make_delays(w, 40000, eta=eta)
    ones = np.ones(5, np.uint8)
    ts = [_cm(5, 4, w.mu, ones, T[k])[0] for k in range(T.shape[0])]
    assert np.mean(ts) == pytest.approx(eta / 4 * H(5), rel=2e-2)
    # distributed Adam on the same workers (M_G = 1 grouping of all 20): mean eta H_20, Eq. (11)
    ts1 = [_cm(20, 1, w.mu, np.ones(20, np.uint8), T[k].reshape(20, 1))[0] for k in range(4000)]
    assert np.mean(ts1) == pytest.approx(eta * H(20), rel=5e-2)


def test_bad_arguments():
    from paper_2201_04301_amd import binding as B
    with pytest.raises(B.GcadaError):
        B.gcada_cost_model(0, 1, 1, None, None)
