"""The baselines report: distributed Adam (c = 0) and CADA (M_G = 1) as special cases of the same
path, with the per-iteration metrics of Sec. II-B and their closed forms of Sec. V."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def H(n):
    return sum(1.0 / i for i in range(1, n + 1))


def test_report_special_cases_and_load_formulas(capsys):
    from paper_2201_04301_amd import report
    iters, mu, eta = 200, 32, 1e-4
    runs = report.main(["--iters", str(iters), "--rows-per-worker", "300", "--mu", str(mu),
                        "--eta", str(eta)])
    print(capsys.readouterr().out, flush=True)
    da, ca, gc = runs["D-Adam"], runs["CADA"], runs["G-CADA"]
    # distributed Adam: everybody, every iteration -- Eq. (17), (20), and Eq. (10)-(11) for the time
    assert (da["selected"] == 12).all()
    assert (da["comm"] == 2 * 12).all() and (da["comp"] == mu * 12).all()
    assert da["time"].mean() == pytest.approx(eta * H(12), rel=0.1)
    # CADA: the selected workers download and upload -- Eq. (18), (21)
    np.testing.assert_array_equal(ca["comm"], 2 * ca["selected"])
    np.testing.assert_array_equal(ca["comp"], mu * ca["selected"])
    assert 0 < ca["selected"].mean() < 12
    # G-CADA: all workers of a selected group download, the fastest uploads -- Eq. (19), (22)
    np.testing.assert_array_equal(gc["comm"], gc["selected"] * (4 + 1))
    np.testing.assert_array_equal(gc["comp"], mu * gc["selected"] * 4)
    full = gc["selected"] == 3
    assert full.any() and not full.all()
    # time per iteration: never above the all-selected closed form on average, and below D-Adam's
    assert gc["time"][full].mean() == pytest.approx(eta / 4 * H(3), rel=0.25)
    assert gc["time"].mean() < ca["time"].mean() < da["time"].mean() * 1.05
    for r in (da, ca, gc):
        assert r["loss"][-10:].mean() < 0.7 * r["loss"][:10].mean()
