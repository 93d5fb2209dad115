"""The C-ABI's error behaviour and stream handling on a device: calls out of order, bad arguments,
unknown options; a run on a side stream gives the bits of a run on the default stream."""
import ctypes as C

import numpy as np
import pytest
import torch

from gcada_inputs import CONFIGS, make_indices, make_shards, make_theta0, scaled

pytestmark = pytest.mark.gpu


def _mk(w):
    from paper_2201_04301_amd import Gcada
    return Gcada.from_workload(w)


def test_calls_out_of_order_and_bad_arguments_are_refused():
    from paper_2201_04301_amd import binding as B
    w = scaled(CONFIGS["lr_small"], name="api", widths=(32,), mu=16, G=3, rows=64, D=4)
    Xs, ys = make_shards(w, "cuda")
    gpu = _mk(w)
    mask = torch.zeros(w.G, dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    # no theta yet
    rc = B.lib.gcada_step(gpu.ctx, None, mask.data_ptr(), loss.data_ptr(), None)
    assert rc == B.GCADA_ESTATE and "set_theta" in B.gcada_last_error(gpu.ctx)
    gpu.set_theta(make_theta0(w))
    # theta, but a group without a shard
    for g in range(w.G - 1):
        B.gcada_set_shard(gpu.ctx, g, Xs[g].data_ptr(), ys[g].data_ptr(), Xs[g].shape[0], Xs[g].stride(0))
    rc = B.lib.gcada_step(gpu.ctx, None, mask.data_ptr(), loss.data_ptr(), None)
    assert rc == B.GCADA_ESTATE and "shard" in B.gcada_last_error(gpu.ctx)
    # shard arguments
    X, y = Xs[-1], ys[-1]
    assert B.lib.gcada_set_shard(gpu.ctx, w.G, X.data_ptr(), y.data_ptr(), X.shape[0], X.stride(0)) == B.GCADA_EINVAL
    assert B.lib.gcada_set_shard(gpu.ctx, 0, None, y.data_ptr(), X.shape[0], X.stride(0)) == B.GCADA_EINVAL
    assert B.lib.gcada_set_shard(gpu.ctx, 0, X.data_ptr(), y.data_ptr(), 0, X.stride(0)) == B.GCADA_EINVAL
    assert B.lib.gcada_set_shard(gpu.ctx, 0, X.data_ptr(), y.data_ptr(), X.shape[0], w.widths[0] - 1) == B.GCADA_EINVAL
    B.gcada_set_shard(gpu.ctx, w.G - 1, X.data_ptr(), y.data_ptr(), X.shape[0], X.stride(0))
    # options and rules
    assert B.lib.gcada_set_option(gpu.ctx, 99, 1) == B.GCADA_EINVAL
    assert B.lib.gcada_set_rule(gpu.ctx, 7, None) == B.GCADA_EINVAL
    assert B.lib.gcada_set_rule(gpu.ctx, B.GCADA_RULE_SERVER, None) == B.GCADA_EINVAL      # no constants yet
    bad_L = (C.c_double * w.G)(*([1.0] * (w.G - 1) + [-1.0]))
    assert B.lib.gcada_set_rule(gpu.ctx, B.GCADA_RULE_SERVER, bad_L) == B.GCADA_EINVAL
    # state with an age outside [1, D]
    st = gpu.get_state()
    st["tau"][0] = w.D + 1
    with pytest.raises(B.GcadaError) as ei:
        gpu.set_state(**st)
    assert ei.value.code == B.GCADA_EINVAL
    # and the context still works
    gpu.step(None)
    out = gpu.outputs()
    assert out["mask"].all() and np.isfinite(out["loss"])
    gpu.close()


@pytest.mark.parametrize("cfg,kw", [
    ("lr_small", dict(widths=(64,), mu=32, G=3, rows=512, D=5)),                 # one-launch kernel
    ("lr_4k", dict(widths=(2048,), mu=64, G=4, rows=256, D=5)),                  # tile kernel + fused finish
    ("mlp_784", dict(widths=(64, 48, 10), mu=64, G=4, rows=300, D=5)),           # MLP
])
def test_side_stream_run_matches_default_stream(cfg, kw):
    w = scaled(CONFIGS[cfg], name="stream", **kw)
    Xs, ys = make_shards(w, "cuda")
    steps = 12
    idx = torch.as_tensor(make_indices(w, steps), device="cuda")
    torch.cuda.synchronize()
    states = []
    for side in (False, True):
        gpu = _mk(w)
        gpu.set_shards(Xs, ys)
        gpu.set_theta(make_theta0(w))
        stream = torch.cuda.Stream() if side else torch.cuda.current_stream()
        with torch.cuda.stream(stream):
            for k in range(steps):
                gpu.step(idx[k].contiguous())
        stream.synchronize()
        states.append(gpu.get_state())
        gpu.close()
    for name in ("theta", "h", "vhat", "agg", "last", "tau", "dtheta_sq"):
        np.testing.assert_array_equal(states[0][name], states[1][name], err_msg=name)


@pytest.mark.parametrize("cfg,kw,kernel", [
    ("lr_small", dict(widths=(64,), mu=32, G=3, rows=512, D=5), "lr_micro"),        # one-launch kernel: workgroup 0 collects
    ("lr_4k", dict(widths=(2048,), mu=64, G=4, rows=256, D=5), "lr_tile"),          # fused finish: its blocks meet once
    ("lr_64k", dict(widths=(8192,), mu=48, G=5, rows=100, D=5), "lr_team"),         # team kernel: members exchange partial dots
    ("lr_4k", dict(widths=(2048,), mu=64, G=20, rows=256, D=5), "one launch per step"),   # tiles wait for the finish of the step before
])
def test_a_wait_that_gives_up_is_reported_by_the_next_step(cfg, kw, kernel):
    # the kernels whose workgroups wait for each other bound that wait.  Here the host makes the
    # next step's waits look for words nobody publishes, with a limit of a few polls: every kernel
    # still runs to its end, the step is reported as failed by the NEXT gcada_step (and by
    # gcada_state / gcada_get_state), the context stays refused until its state is replaced, and
    # works again afterwards -- as does a fresh context
    from paper_2201_04301_amd import binding as B
    w = scaled(CONFIGS[cfg], name="giveup", **kw)
    Xs, ys = make_shards(w, "cuda")
    idx = torch.as_tensor(make_indices(w, 6), device="cuda")
    mask = torch.zeros(w.G, dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")

    def raw_step(gpu, k):
        return B.lib.gcada_step(gpu.ctx, idx[k].contiguous().data_ptr(), mask.data_ptr(), loss.data_ptr(), None)

    gpu = _mk(w)
    if kernel == "one launch per step":
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_DEFERRED_FINISH, 1)
    else:
        assert kernel in B.gcada_timed_stage(gpu.ctx)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    assert raw_step(gpu, 0) == B.GCADA_OK and raw_step(gpu, 1) == B.GCADA_OK
    torch.cuda.synchronize()
    good = gpu.get_state()
    if kernel == "one launch per step":
        assert raw_step(gpu, 5) == B.GCADA_OK        # (leaves a finish to come: the next launch carries it and waits for it)
    B.gcada_set_option(gpu.ctx, B.GCADA_OPT_EXPIRE_NEXT_WAIT, 1)
    assert raw_step(gpu, 2) == B.GCADA_OK            # launched; its waits give up on the device
    torch.cuda.synchronize()                          # the step has finished (normally: nothing hangs)
    rc = raw_step(gpu, 3)
    assert rc == B.GCADA_EDEVICE and "wait" in B.gcada_last_error(gpu.ctx)
    assert raw_step(gpu, 3) == B.GCADA_EDEVICE       # and stays refused
    v = B.gcada_state_view()
    assert B.lib.gcada_state(gpu.ctx, C.byref(v)) == B.GCADA_EDEVICE
    with pytest.raises(B.GcadaError) as ei:
        gpu.get_state()
    assert ei.value.code == B.GCADA_EDEVICE
    # replacing the state clears it; the run continues from the good state exactly as a fresh
    # context does from the same state
    gpu.set_state(**good)
    assert raw_step(gpu, 2) == B.GCADA_OK
    torch.cuda.synchronize()
    a = gpu.get_state()
    gpu.close()
    fresh = _mk(w)
    if kernel == "one launch per step":
        B.gcada_set_option(fresh.ctx, B.GCADA_OPT_DEFERRED_FINISH, 1)
    fresh.set_shards(Xs, ys)
    fresh.set_theta(make_theta0(w))
    fresh.set_state(**good)
    assert raw_step(fresh, 2) == B.GCADA_OK
    torch.cuda.synchronize()
    b = fresh.get_state()
    fresh.close()
    for name in ("theta", "h", "vhat", "agg", "last", "tau", "dtheta_sq"):
        np.testing.assert_array_equal(a[name], b[name], err_msg=name)


def test_history_depth_above_64_runs_with_the_default_rule_only():
    # the server-side rule keeps one bit per age (D <= 64); every other path takes any D
    from paper_2201_04301_amd import binding as B
    w = scaled(CONFIGS["lr_small"], name="deep_history", widths=(32,), mu=16, G=3, rows=64, D=65)
    Xs, ys = make_shards(w, "cuda")
    gpu = _mk(w)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    L = (C.c_double * w.G)(*([1.0] * w.G))
    assert B.lib.gcada_set_rule(gpu.ctx, B.GCADA_RULE_SERVER, L) == B.GCADA_EINVAL
    assert "D <= 64" in B.gcada_last_error(gpu.ctx)
    for k in range(3):
        gpu.step(None)
    out = gpu.outputs()
    assert np.isfinite(out["loss"]) and gpu.get_state()["k"] == 3
    gpu.close()


def test_gather_read_calibration_reads_the_minibatch_rows_and_refuses_other_shapes():
    # the diagnostic reads the rows the ids select, in the wide-row kernel's pattern, and reports
    # a rate; shapes that the pattern does not cover are refused with a message
    from paper_2201_04301_amd import binding as B
    w = scaled(CONFIGS["lr_64k"], name="gather_cal", widths=(8192,), mu=128, G=4, rows=256)
    Xs, ys = make_shards(w, "cuda")
    gpu = _mk(w)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    idx = torch.as_tensor(make_indices(w, 4), device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    rate = B.gcada_gather_read_calibration(gpu.ctx, idx.data_ptr(), w.G * w.mu, 3, stream)
    assert rate > 0
    g = C.c_double()
    assert B.lib.gcada_gather_read_calibration(gpu.ctx, None, w.G * w.mu, 3, stream, C.byref(g)) == B.GCADA_EINVAL
    gpu.close()
    # 96 rows per group and step: 96 tiles of four rows in all do not divide among the 128 teams of two
    w2 = scaled(CONFIGS["lr_64k"], name="gather_cal", widths=(8192,), mu=96, G=4, rows=256)
    Xs, ys = make_shards(w2, "cuda")
    gpu = _mk(w2)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w2))
    idx = torch.as_tensor(make_indices(w2, 4), device="cuda")
    assert B.lib.gcada_gather_read_calibration(gpu.ctx, idx.data_ptr(), w2.G * w2.mu, 3, stream,
                                               C.byref(g)) == B.GCADA_EINVAL
    assert "divide" in B.gcada_last_error(gpu.ctx)
    gpu.close()
    # a narrow model
    w3 = scaled(CONFIGS["lr_4k"], name="gather_cal", widths=(4096,), mu=64, G=4, rows=128)
    Xs, ys = make_shards(w3, "cuda")
    gpu = _mk(w3)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w3))
    idx = torch.as_tensor(make_indices(w3, 4), device="cuda")
    assert B.lib.gcada_gather_read_calibration(gpu.ctx, idx.data_ptr(), w3.G * w3.mu, 3, stream,
                                               C.byref(g)) == B.GCADA_EINVAL
    gpu.close()
