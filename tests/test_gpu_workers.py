"""Per-worker minibatches with the fastest worker's gradient (Sec. IV, Algorithm 1 taken
literally), and checkpoint / resume through gcada_get_state / gcada_set_state."""
import numpy as np
import pytest
import torch

import oracle as O
from gcada_inputs import (CONFIGS, gather_rows, make_delays, make_indices, make_shards, make_theta0,
                          make_worker_indices, scaled)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def par():
    import parity
    return parity


@pytest.mark.parametrize("name,kw", [
    ("lr_small", dict(M_G=4)),
    ("linreg_784", dict(rows=600, mu=64)),
])
def test_fastest_worker_minibatches_match_oracle(par, name, kw):
    # the oracle knows no workers: it is fed the rows of argmin_m T_m^k, chosen here with numpy
    from paper_2201_04301_amd import Gcada
    w = scaled(CONFIGS[name], **kw)
    steps = 40
    Xs, ys = make_shards(w, "cuda")
    idx_w = make_worker_indices(w, steps)                 # (steps, G, M_G, mu)
    T = make_delays(w, steps)                             # (steps, G, M_G)
    fastest = T.argmin(axis=2)
    idx_dev = torch.as_tensor(idx_w, device="cuda")
    T_dev = torch.as_tensor(T, device="cuda")
    picked = torch.zeros(steps, w.G, dtype=torch.int32, device="cuda")
    masks = torch.zeros(steps, w.G, dtype=torch.uint8, device="cuda")
    losses = torch.zeros(steps, dtype=torch.float32, device="cuda")
    gpu = Gcada.from_workload(w)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    for k in range(steps):
        gpu.step_workers(idx_dev[k].contiguous(), T_dev[k].contiguous(), worker_out=picked[k],
                         mask_out=masks[k], loss_out=losses[k:k + 1])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(picked.cpu().numpy(), fastest)
    orc = O.Oracle(par.oracle_config(w), make_theta0(w))
    masks_o = np.zeros((steps, w.G), np.uint8)
    loss_o = np.zeros(steps)
    for k in range(steps):
        used = np.stack([idx_w[k, g, fastest[k, g]] for g in range(w.G)])
        Xmb, ymb = gather_rows(Xs, ys, used)
        masks_o[k], loss_o[k] = orc.step(Xmb, ymb)
    assert (masks.cpu().numpy() == masks_o).mean() >= 0.98
    np.testing.assert_allclose(losses.cpu().numpy(), loss_o, rtol=2e-3)
    np.testing.assert_allclose(gpu.get_state()["theta"], orc.theta, rtol=0, atol=2e-4 * np.abs(orc.theta).max())
    # the modelled time of a selected group is its fastest worker's time (Sec. V)
    t, comm, comp = gpu.cost_model(masks_o[-1], T[-1])
    sel = masks_o[-1].astype(bool)
    assert t == (T[-1].min(axis=1)[sel].max() if sel.any() else 0.0)
    gpu.close()


def test_checkpoint_resume_is_bit_identical():
    from paper_2201_04301_amd import Gcada
    w = scaled(CONFIGS["lr_4k"], rows=1024)
    Xs, ys = make_shards(w, "cuda")
    idx = torch.as_tensor(make_indices(w, 30), device="cuda")
    a = Gcada.from_workload(w)
    a.set_shards(Xs, ys)
    a.set_theta(make_theta0(w))
    for k in range(17):
        a.step(idx[k].contiguous())
    ck = a.get_state()
    for k in range(17, 30):
        a.step(idx[k].contiguous())
    ref = a.get_state()
    a.close()
    b = Gcada.from_workload(w)                 # a new context, restored from the checkpoint
    b.set_shards(Xs, ys)
    b.set_state(ck["theta"], ck["h"], ck["vhat"], ck["agg"], ck["theta_stale"], ck["last"], ck["tau"],
                ck["dtheta_sq"], ck["k"])
    for k in range(17, 30):
        b.step(idx[k].contiguous())
    got = b.get_state()
    b.close()
    for key in ("theta", "h", "vhat", "agg", "last", "tau", "dtheta_sq", "theta_stale"):
        np.testing.assert_array_equal(got[key], ref[key], err_msg=key)
    assert got["k"] == ref["k"] == 30
