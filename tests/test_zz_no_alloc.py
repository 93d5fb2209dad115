"""The entry point that allocates nothing (gcada_estimate_smoothness_static: scratch in a static
device array, result on the device, no synchronisation) against gcada_estimate_smoothness, through
the C-ABI: two calls in a row, the second on a smaller problem, so that what the first call left
in the shared array must not leak into the second."""
import numpy as np
import pytest
import torch

from gcada_inputs import CONFIGS, make_shards, make_theta0, scaled

pytestmark = pytest.mark.gpu


def _both(w, iters):
    from paper_2201_04301_amd import Gcada
    Xs, ys = make_shards(w, "cuda")
    gpu = Gcada.from_workload(w)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    ref = gpu.estimate_smoothness(iters=iters)                 # allocates, copies, synchronises
    out = torch.full((w.G,), float("nan"), dtype=torch.float64, device="cuda")
    gpu.estimate_smoothness_static(out, iters=iters)           # asynchronous
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    gpu.close()
    return ref, got


def test_static_scratch_entry_point_matches_the_allocating_one_twice():
    # first a shard shape that fills much of the array (d = 2048, 4096 rows: 64 chunks of partial
    # sums), then a smaller one with another width, group count and loss
    big = scaled(CONFIGS["lr_4k"], name="pi_big", widths=(2048,), mu=64, G=3, rows=4096, l2=1e-4)
    small = scaled(CONFIGS["linreg_784"], name="pi_small", widths=(300,), mu=32, G=5, rows=333)
    for w, iters in ((big, 12), (small, 9)):
        ref, got = _both(w, iters)
        print(w.name, "allocating", ref, "static", got, "bit-equal", np.array_equal(ref, got), flush=True)
        assert np.all(np.isfinite(got)) and np.all(got > 0)
        # same kernels on the same data from the same start vector: the same numbers (1e-12
        # leaves room for one differently rounded operation in the start vector's setup)
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=0)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    from paper_2201_04301_amd import Gcada, binding as B
    # 16,384 rows of width 20,000 need 256 x 20,000 partial sums: beyond the 2 Mi doubles of the array
    w = scaled(CONFIGS["lr_64k"], name="pi_wide", widths=(20000,), G=1, mu=16, rows=16384)
    Xs, ys = make_shards(w, "cuda")
    gpu = Gcada.from_workload(w)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    out = torch.zeros(w.G, dtype=torch.float64, device="cuda")
    rc = B.lib.gcada_estimate_smoothness_static(gpu.ctx, 3, out.data_ptr(), None)
    assert rc == B.GCADA_EINVAL and "static array" in B.gcada_last_error(gpu.ctx)
    assert B.lib.gcada_estimate_smoothness_static(gpu.ctx, 0, out.data_ptr(), None) == B.GCADA_EINVAL
    assert B.lib.gcada_estimate_smoothness_static(gpu.ctx, 3, None, None) == B.GCADA_EINVAL
    torch.cuda.synchronize()
    assert float(out.abs().sum()) == 0.0                      # nothing was written
    gpu.close()
