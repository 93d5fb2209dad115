#!/usr/bin/env python3
"""Throughput of the G-CADA hot path on one MI355X.

A step is one whole iteration (dual-iterate gradients of all groups, selection, masked innovation
sum, server update) on one minibatch per group of the synthetic workload.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published

# HBM bytes per launch of the timed kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by
# the copy calibration (profiles/lr_4k_hbm_traffic.md, profiles/lr_64k_hbm_traffic.md).  Valid for
# the kernel named; set to None when that kernel changes.
MEASURED_TRAFFIC = {"lr_4k": ("lr_tile_kernel", 68.1e6 + 8.4e6),
                    "lr_64k": ("lr_team_kernel", 8.612e9 + 16.8e6)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="lr_4k")
    ap.add_argument("--cpu-steps", type=int, default=-1, help="oracle steps to time (-1 = auto)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--rule", choices=["gradient_difference", "server"], default="gradient_difference",
                    help="selection rule: the same-minibatch gradient difference (default, the metric's "
                         "configuration) or the paper's server-side condition with L_g from power "
                         "iteration (linear models): only selected groups evaluate a gradient")
    ap.add_argument("--separate-finish", action="store_true",
                    help="whole-row logistic path: use the separate reduce and server kernels instead "
                         "of the fused finish kernel (for comparison)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="instead of the benchmark: copy a buffer of this many MiB five times with a "
                         "plain device copy kernel (to calibrate rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from gcada_inputs import CONFIGS, gather_rows, make_delays, make_indices, make_shards, make_theta0
    from paper_2201_04301_amd import Gcada, binding as B

    torch.cuda.set_device(0)
    if args.copy_calibration > 0:
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n * 4, "bytes_written": n * 4, "copies": 5}))
        return
    w = CONFIGS[args.workload]
    K, W = args.steps, args.warmup
    t0 = time.time()
    Xs, ys = make_shards(w, "cuda")
    idx = make_indices(w, K + W)
    idx_dev = torch.as_tensor(idx, device="cuda")
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    gpu = Gcada.from_workload(w)
    if args.separate_finish:
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_FUSED_FINISH, 0)
    gpu.set_shards(Xs, ys)
    gpu.set_theta(make_theta0(w))
    if args.rule == "server":
        gpu.set_rule("server", gpu.estimate_smoothness(iters=20))
    masks = torch.zeros(K + W, w.G, dtype=torch.uint8, device="cuda")
    losses = torch.zeros(K + W, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    base_idx, base_m, base_l = idx_dev.data_ptr(), masks.data_ptr(), losses.data_ptr()
    stride_idx = w.G * w.mu * 4

    def run_fast(k0, k1):
        ctx, step = gpu.ctx, B.lib.gcada_step
        for k in range(k0, k1):
            rc = step(ctx, base_idx + k * stride_idx, base_m + k * w.G, base_l + 4 * k, stream)
            if rc != 0:
                raise RuntimeError(B.gcada_last_error(ctx))

    # pass 1: W warm-up steps, then exactly K timed steps, nothing else in the stream
    run_fast(0, W)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_fast(W, W + K)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    m_host = masks[W:].cpu().numpy()
    l_host = losses[W:].cpu().numpy()
    # the dominant kernel(s) of the gradient stage alone, live: many launches back to back between
    # two HIP events on the same stream (per-step event records would open gaps of a few
    # microseconds in the stream, so the throughput above is taken without any)
    reps = min(K, 400)           # a different minibatch per repetition (those of the timed steps)
    grad_ms_avg = B.gcada_time_gradient_stage(gpu.ctx, base_idx + W * stride_idx, w.G * w.mu, reps, stream)

    ms_per_step = dt / K * 1e3
    iters_s = K / dt
    if w.model in ("logreg", "linreg"):
        # algorithmic bytes per launch of the timed kernel(s): one read of the touched minibatch rows
        alg_bytes = w.G * w.mu * w.widths[0] * 4
        achieved = alg_bytes / (grad_ms_avg * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": (MEASURED_TRAFFIC[w.name][1]
                                if w.name in MEASURED_TRAFFIC and
                                MEASURED_TRAFFIC[w.name][0] == B.gcada_timed_stage(gpu.ctx) else None),
                    "kernel": B.gcada_timed_stage(gpu.ctx),
                    "avg_ms": round(grad_ms_avg, 5), "algorithmic_bytes": alg_bytes}
    else:
        # algorithmic flops of the gradient stage per step: forward + weight-gradient GEMMs of
        # every layer and the back-propagation GEMMs of layers 2..L, for two iterates and G groups
        n = w.widths
        per = sum(2 * w.mu * n[l] * n[l - 1] for l in range(1, len(n))) * 2 \
            + sum(2 * w.mu * n[l] * n[l - 1] for l in range(2, len(n)))
        flops = per * 2 * w.G
        peak = 2500.0 if w.dtype == "bf16" else 157.3
        achieved = flops / (grad_ms_avg * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                    "frac": round(achieved / peak, 4), "traffic": None,
                    "kernel": B.gcada_timed_stage(gpu.ctx),
                    "avg_ms": round(grad_ms_avg, 5), "algorithmic_flops": flops}

    # modelled wall-clock / communication / computation of the paper's cost model (reported only)
    T = make_delays(w, K)
    tm = cm = pm = 0.0
    for k in range(K):
        t, c_, p_ = gpu.cost_model(m_host[k], T[k])
        tm += t; cm += c_; pm += p_
    model = {"eta_s": 1e-4, "modelled_time_s": tm, "comm_load": cm, "comp_load": pm,
             "mean_selected": float(m_host.sum(1).mean())}

    cpu = None
    if not args.no_cpu and args.rule == "gradient_difference":
        import oracle as O
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from parity import oracle_config
        orc = O.Oracle(oracle_config(w), make_theta0(w))
        n_cpu = args.cpu_steps
        budget_s = 15.0
        done, spent = 0, 0.0
        kk = 0
        while True:
            Xmb, ymb = gather_rows(Xs, ys, idx[kk])
            t1 = time.perf_counter()
            orc.step(Xmb, ymb)
            spent += time.perf_counter() - t1
            done += 1
            kk += 1
            if (n_cpu > 0 and done >= n_cpu) or (n_cpu <= 0 and (spent > budget_s or kk >= K + W)):
                break
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu_model = ""
        try:
            with open("/proc/cpuinfo") as f:
                cpu_model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
        except OSError:
            pass
        cpu = {"value": round(done / spent, 3), "unit": "iters/s", "cores": cores, "kind": "oracle",
               "cpu_model": cpu_model,
               "sample": f"first {done} iterations of the same workload, same shards and row ids "
                         f"(oracle time only; row gather excluded)"}

    out = {"metric": "G-CADA iterations/s", "value": round(iters_s, 2), "unit": "iters/s",
           "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms_per_step, 5),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32" if w.dtype == "f32" else "bf16",
           "data": "synthetic",
           "config": {"workload": w.name, "rule": args.rule, "model": None, "G": w.G, "M_G": w.M_G, "mu": w.mu,
                      "widths": list(w.widths), "rows_per_shard": w.rows, "D": w.D, "c": w.c,
                      "l2": w.l2, "parallelism": "1 GPU, all groups simulated"},
           "grad_evals_per_s": round(2 * w.G * iters_s, 1),
           "sample_grad_evals_per_s": round(2 * w.G * w.mu * iters_s, 1),
           "final_loss": float(l_host[-1]), "roofline": roofline, "cpu_baseline": cpu,
           "cost_model": model, "setup_s": round(gen_s, 2)}
    out["config"].pop("model")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
