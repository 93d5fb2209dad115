#!/usr/bin/env python3
"""Throughput of the G-CADA hot path on one MI355X.

A step is one whole iteration (dual-iterate gradients of all groups, selection, masked innovation
sum, server update) on one minibatch per group of the synthetic workload.  The headline is the
largest single-GPU configuration (`lr_64k`); the other four configurations are measured in the
same run and reported in `per_config`.  Prints ONE JSON line on stdout (the details of every
configuration go to stderr and, with --details FILE, to that file).

Timing: W untimed warm-up steps, then `repeats` (3) passes of exactly K steps each, every pass
bracketed by a device synchronisation and on minibatches of its own; the median pass is reported.
"""
from __future__ import annotations

import argparse
import ctypes
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}

# steps per timed pass of the configurations that are not the headline (the headline takes --steps)
SIDE_STEPS = {"lr_small": 200, "lr_4k": 200, "mlp_784": 100, "lr_64k": 20, "mlp_3072_bf16": 40}
ORDER = ["lr_small", "lr_4k", "mlp_784", "lr_64k", "mlp_3072_bf16"]


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` from the rocprofv3 counter runs recorded in
    profiles/hbm_traffic.json -- only while the kernel's source file is the one the counters were
    taken on (sha256 recorded there); otherwise None."""
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json")))[workload]
        if rec["kernel"] != kernel:
            return None
        src = os.path.join(ROOT, "paper_2201_04301_amd", "csrc", rec["source"])
        if hashlib.sha256(open(src, "rb").read()).hexdigest() != rec["source_sha256"]:
            return None
        return float(rec["bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def host_cpu():
    """(model name, physical cores seen in /proc/cpuinfo, threads the oracle's OpenMP loops use)."""
    model, cores = "", set()
    try:
        phys = core = None
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name") and not model:
                model = ln.split(":", 1)[1].strip()
            elif ln.startswith("physical id"):
                phys = ln.split(":", 1)[1].strip()
            elif ln.startswith("core id"):
                core = ln.split(":", 1)[1].strip()
            elif not ln.strip():
                if phys is not None and core is not None:
                    cores.add((phys, core))
                phys = core = None
    except OSError:
        pass
    omp = int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1)
    return model, len(cores) or (os.cpu_count() or 1), omp


_gomp = None


def omp_set_threads(n: int):
    """Thread count of the oracle's OpenMP loops (the runtime the oracle library links)."""
    global _gomp
    if _gomp is None:
        _gomp = ctypes.CDLL("libgomp.so.1")
    _gomp.omp_set_num_threads(int(n))


def oracle_rate(w, Xs, ys, idx, budget_s, min_steps, max_steps, threads, sample_groups=None):
    """Time the fp64 oracle, as it stands, on the first steps of the workload: at least min_steps,
    then until budget_s of oracle time is spent or max_steps are done.  sample_groups: time only
    that many groups (one per thread) and scale to all G -- the oracle runs its groups in
    parallel, threads at a time.  Returns (iterations/s of the whole workload, steps timed, note)."""
    import oracle as O
    from dataclasses import replace
    from gcada_inputs import gather_rows, make_theta0
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from parity import oracle_config
    omp_set_threads(threads)
    G_run = w.G if sample_groups is None else min(sample_groups, w.G)
    ws = replace(w, G=G_run)
    orc = O.Oracle(oracle_config(ws), make_theta0(w))
    done, spent = 0, 0.0
    max_steps = min(max_steps, len(idx))
    while done < max_steps and (done < min_steps or spent < budget_s):
        Xmb, ymb = gather_rows(Xs[:G_run], ys[:G_run], idx[done][:G_run])
        t1 = time.perf_counter()
        orc.step(Xmb, ymb)
        spent += time.perf_counter() - t1
        done += 1
    per_step = spent / done
    scale = 1.0
    note = f"first {done} iterations, same shards and row ids, {threads} thread(s), oracle time only (row gather excluded)"
    if G_run < w.G:
        rounds_full = -(-w.G // threads)
        rounds_run = -(-G_run // threads)
        scale = rounds_full / rounds_run
        note += f"; {G_run} of the {w.G} groups timed, scaled by {scale:g} (the oracle runs {threads} groups at a time)"
    return 1.0 / (per_step * scale), done, note


def mlp_flops(w, gram: bool):
    """(algorithmic, executed) flops of the gradient stage per step: forward and weight-gradient
    products of every layer and the back-propagation products of layers 2..L, for two iterates and
    G groups.  With the Gram statistic the stage forms no first-layer weight gradient but two
    mu x mu Gram matrices per group."""
    n = w.widths
    per = sum(2 * w.mu * n[l] * n[l - 1] for l in range(1, len(n))) * 2 \
        + sum(2 * w.mu * n[l] * n[l - 1] for l in range(2, len(n)))
    alg = per * 2 * w.G
    ex = alg
    if gram:
        ex = alg - 2 * w.G * 2 * w.mu * n[1] * n[0] + w.G * 2 * w.mu * w.mu * (n[0] + n[1])
    return alg, ex


def run_config(w, K, W, repeats, args, cpu_info, headline: bool):
    import numpy as np
    import torch
    from gcada_inputs import make_delays, make_indices, make_shards, make_theta0
    from paper_2201_04301_amd import Gcada, binding as B

    print(f"[bench] {w.name}: generating data", file=sys.stderr, flush=True)
    t0 = time.time()
    Xs, ys = make_shards(w, "cuda")
    n_steps = W + repeats * K
    idx = make_indices(w, n_steps)
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
    masks = torch.zeros(n_steps, w.G, dtype=torch.uint8, device="cuda")
    losses = torch.zeros(n_steps, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    base_idx, base_m, base_l = idx_dev.data_ptr(), masks.data_ptr(), losses.data_ptr()
    stride_idx = w.G * w.mu * 4

    def run_fast(k0, k1):
        ctx, step = gpu.ctx, B.lib.gcada_step
        for k in range(k0, k1):
            rc = step(ctx, base_idx + k * stride_idx, base_m + k * w.G, base_l + 4 * k, stream)
            if rc != 0:
                raise RuntimeError(B.gcada_last_error(ctx))

    def check_flag():
        # a wait between workgroups that gave up inside a kernel invalidates the run
        torch.cuda.synchronize()
        B.gcada_state(gpu.ctx)

    run_fast(0, W)
    check_flag()
    passes = []
    for r in range(repeats):
        k0 = W + r * K
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        run_fast(k0, k0 + K)
        torch.cuda.synchronize()
        passes.append(time.perf_counter() - t1)
    check_flag()
    dt = statistics.median(passes)
    r_med = passes.index(dt)
    m_host = masks[W + r_med * K: W + (r_med + 1) * K].cpu().numpy()
    l_host = losses[W:].cpu().numpy()

    # the dominant kernel(s) of the gradient stage alone, live: many launches back to back between
    # two HIP events on the stream they are launched on (per-step event records would open gaps of
    # a few microseconds in the stream, so the throughput above is taken without any)
    reps = min(K, 400)
    grad_ms = statistics.median(
        B.gcada_time_gradient_stage(gpu.ctx, base_idx + (W + r * K) * stride_idx, w.G * w.mu, reps, stream)
        for r in range(repeats))
    check_flag()
    stage = B.gcada_timed_stage(gpu.ctx)

    ms_per_step = dt / K * 1e3
    iters_s = K / dt
    if w.model in ("logreg", "linreg"):
        alg_bytes = w.G * w.mu * w.widths[0] * 4      # one read of the touched minibatch rows
        ach = alg_bytes / (grad_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": measured_traffic(w.name, stage),
                    "kernel": stage, "avg_ms": round(grad_ms, 5), "algorithmic_bytes": alg_bytes,
                    "whole_step_frac": round(alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        if stage == "lr_team_kernel" and w.widths[0] % 4096 == 0 and w.mu % 4 == 0:
            # what the same gathered rows, read in the same pattern without arithmetic or
            # exchange, reach on this machine (the ceiling of this kernel's access pattern)
            try:
                roofline["hbm_gather_read_achievable_gbs"] = round(B.gcada_gather_read_calibration(
                    gpu.ctx, base_idx + W * stride_idx, w.G * w.mu, min(K, 20), stream), 1)
            except RuntimeError as exc:
                print(f"[bench] gather calibration skipped: {exc}", file=sys.stderr, flush=True)
    else:
        gram = "Gram" in stage
        alg, ex = mlp_flops(w, gram)
        peak = MFMA_PEAK_TFLOPS[w.dtype]
        ach = ex / (grad_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(ach, 2), "peak": peak, "unit": "TFLOP/s",
                    "frac": round(ach / peak, 4), "traffic": None,
                    "kernel": stage.split(" (")[0] + (" [first-layer statistic from Gram matrices]" if gram else ""),
                    "avg_ms": round(grad_ms, 5), "executed_flops": ex, "algorithmic_flops": alg,
                    "frac_algorithmic": round(alg / (grad_ms * 1e-3) / 1e12 / peak, 4),
                    "whole_step_frac": round(alg / (ms_per_step * 1e-3) / 1e12 / peak, 4)}

    # modelled wall-clock / communication / computation of the paper's cost model (reported only)
    T = make_delays(w, K)
    tm = cm = pm = 0.0
    for k in range(K):
        t, c_, p_ = gpu.cost_model(m_host[k], T[k])
        tm += t; cm += c_; pm += p_
    model = {"eta_s": 1e-4, "modelled_time_s": tm, "comm_load": cm, "comp_load": pm,
             "mean_selected": round(float(m_host.sum(1).mean()), 3)}

    extra = {}
    if w.name == "mlp_3072_bf16" and args.rule == "gradient_difference":
        extra = mlp_step_kinds(w, gpu, Xs, ys, args)
    if w.name == "lr_4k" and args.rule == "gradient_difference" and not args.separate_finish:
        # the same steps with one launch per step (GCADA_OPT_DEFERRED_FINISH: the finish of step k at
        # the head of the launch of step k+1; mask and loss of a step arrive with the next call)
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_DEFERRED_FINISH, 1)
        gpu.set_theta(make_theta0(w))
        run_fast(0, W)
        torch.cuda.synchronize()
        p2 = []
        for r in range(repeats):
            k0 = W + r * K
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            run_fast(k0, k0 + K)
            torch.cuda.synchronize()
            p2.append(time.perf_counter() - t1)
        check_flag()
        B.gcada_set_option(gpu.ctx, B.GCADA_OPT_DEFERRED_FINISH, 0)
        d2 = statistics.median(p2)
        extra = {"one_launch_per_step": {"iters_per_s": round(K / d2, 2), "ms_per_step": round(d2 / K * 1e3, 5),
                                         "final_loss": float(losses[W + repeats * K - 1].item())}}

    print(f"[bench] {w.name}: {iters_s:.1f} it/s, stage {grad_ms:.4f} ms; timing the oracle", file=sys.stderr, flush=True)
    cpu = None
    if not args.no_cpu and args.rule == "gradient_difference":
        cpu_model, phys, omp = cpu_info
        threads = omp
        big = w.name in ("lr_64k", "mlp_3072_bf16")
        sample = threads if w.name == "mlp_3072_bf16" and w.G > threads else None
        budget = args.cpu_budget if headline else args.cpu_budget / 2
        v, done, note = oracle_rate(w, Xs, ys, idx, budget, 3 if big else 5,
                                    w.iters if args.cpu_steps < 0 else args.cpu_steps, threads, sample)
        cpu = {"value": round(v, 4), "unit": "iters/s", "cores": threads, "kind": "oracle", "sample": note,
               "cpu_model": cpu_model, "physical_cores": phys, "omp_num_threads": omp}
        if not big:
            v1, d1, _ = oracle_rate(w, Xs, ys, idx, 2.0, 2, 50, 1)
            cpu["one_thread_iters_per_s"] = round(v1, 4)
        omp_set_threads(omp)

    gpu.close()
    del Xs, ys, idx_dev
    torch.cuda.empty_cache()
    return {"workload": w.name, "iters_per_s": round(iters_s, 2), "ms_per_step": round(ms_per_step, 5),
            "passes_ms_per_step": [round(p / K * 1e3, 5) for p in passes], "steps": K,
            "grad_evals_per_s": round(2 * w.G * iters_s, 1),
            "sample_grad_evals_per_s": round(2 * w.G * w.mu * iters_s, 1),
            "final_loss": float(l_host[-1]), "roofline": roofline, "cpu_baseline": cpu,
            "cost_model": model, "setup_s": round(gen_s, 2), **extra}


def mlp_step_kinds(w, gpu, Xs, ys, args):
    """The large bf16 MLP as specified drives its loss to zero within a few steps, after which no
    statistic reaches the threshold and all groups upload together every D steps.  So: the time of
    a step without an upload, of a step in which every group uploads, and their mix -- each step
    between two events -- and the same network on a workload that stays alive (overlapping
    clusters, smaller step), where the statistic does select."""
    import numpy as np
    import torch
    from dataclasses import replace
    from gcada_inputs import make_indices, make_shards, make_theta0
    from paper_2201_04301_amd import Gcada

    def timed_steps(g, wl, idx_dev, n):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        masks = torch.zeros(n, wl.G, dtype=torch.uint8, device="cuda")
        ev[0].record()
        for k in range(n):
            g.step(idx_dev[k], mask_out=masks[k])
            ev[k + 1].record()
        torch.cuda.synchronize()
        ms = np.array([ev[k].elapsed_time(ev[k + 1]) for k in range(n)])
        return ms, masks.cpu().numpy().sum(1)

    n = 3 * w.D + 2
    idx_dev = torch.as_tensor(make_indices(w, n, seed=7), device="cuda")
    gpu.set_theta(make_theta0(w))
    ms, ups = timed_steps(gpu, w, idx_dev, n)
    late = np.arange(n) > w.D                          # past the first, upload-heavy steps
    out = {"step_kinds": {
        "no_upload_ms": round(float(np.median(ms[late & (ups == 0)])), 4) if (late & (ups == 0)).any() else None,
        "all_upload_ms": round(float(np.median(ms[late & (ups == w.G)])), 4) if (late & (ups == w.G)).any() else None,
        "mean_ms": round(float(ms[late].mean()), 4), "mean_uploads_per_step": round(float(ups[late].mean()), 2),
        "note": "steps after the first D, each between two events (a few microseconds of gap each)"}}
    # a workload on which the loss does not collapse
    wl = replace(w, name="mlp_3072_bf16_live", sigma=1.5, alpha=2e-3)
    Xl, yl = make_shards(wl, "cuda")
    g2 = Gcada.from_workload(wl)
    g2.set_shards(Xl, yl)
    g2.set_theta(make_theta0(wl))
    idx_l = torch.as_tensor(make_indices(wl, n, seed=9), device="cuda")
    ms2, ups2 = timed_steps(g2, wl, idx_l, n)
    torch.cuda.synchronize()
    out["live_variant"] = {"workload": "same network, sigma = 1.5, alpha = 2e-3", "mean_ms": round(float(ms2[late].mean()), 4),
                           "iters_per_s": round(1e3 / float(ms2[late].mean()), 1),
                           "mean_uploads_per_step": round(float(ups2[late].mean()), 2),
                           "uploads_by_statistic": int(ups2[late].sum() - w.G * ((np.arange(n)[late] % w.D) == 0).sum())}
    g2.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--repeats", type=int, default=3)
    ap.add_argument("--workload", default="lr_64k", help="the headline configuration")
    ap.add_argument("--only", action="store_true", help="measure the headline configuration only")
    ap.add_argument("--cpu-steps", type=int, default=-1, help="oracle steps to time at most (-1 = the run's length)")
    ap.add_argument("--cpu-budget", type=float, default=12.0, help="seconds of oracle time for the headline's baseline")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--library-gemm-reference", action="store_true",
                    help="time the vendor GEMM on the shapes of the MLP configurations' forward products and exit")
    ap.add_argument("--details", default="", metavar="FILE", help="also write the per-configuration details there")
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

    import torch
    from gcada_inputs import CONFIGS
    from paper_2201_04301_amd import binding as B

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

    if args.library_gemm_reference:
        # Context for the MLP rooflines, not part of any measurement of this library: the rate the
        # vendor's GEMM (through torch.matmul) reaches on this machine for the plain products
        # C = A B^T with the shapes of the gradient stage's large GEMMs -- no bias, activation,
        # second output orientation or per-group weights, which the library's kernels carry.
        out = {}
        for name in ("mlp_3072_bf16", "mlp_784"):
            w = CONFIGS[name]
            dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
            rows = 2 * w.G * w.mu                         # both iterates of every group
            shapes = {}
            for l in range(1, len(w.widths) - 1):        # forward and signal products of the hidden layers
                shapes[f"forward layer {l}: {rows} x {w.widths[l]} x {w.widths[l - 1]}"] = (rows, w.widths[l], w.widths[l - 1])
            for label, (M, N, Kd) in shapes.items():
                a = torch.randn(M, Kd, device="cuda", dtype=dt)
                b = torch.randn(N, Kd, device="cuda", dtype=dt)
                for _ in range(5):
                    a @ b.t()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(50):
                    a @ b.t()
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / 50
                out[f"{name}, {label}"] = {"us": round(ms * 1e3, 1), "tflops": round(2 * M * N * Kd / ms / 1e9, 1),
                                           "frac_of_peak": round(2 * M * N * Kd / ms / 1e9 / MFMA_PEAK_TFLOPS[w.dtype], 3)}
        print(json.dumps({"library_gemm_reference": out}))
        return

    cpu_info = host_cpu()
    K, W = args.steps, args.warmup
    stream = torch.cuda.current_stream().cuda_stream
    # what a plain contiguous read reaches on this machine (the library's own streaming kernel,
    # 8 GiB, best of its launch shapes): the ceiling the HBM-bound kernels are held against
    buf = torch.empty(8 << 30, dtype=torch.uint8, device="cuda")
    buf.zero_()
    hbm_read, hbm_read_plain = B.gcada_hbm_read_calibration(buf.data_ptr(), buf.numel(), 3, stream)
    del buf
    torch.cuda.empty_cache()

    head = run_config(CONFIGS[args.workload], K, W, args.repeats, args, cpu_info, True)
    details = {args.workload: head}
    if not args.only:
        for name in ORDER:
            if name != args.workload:
                details[name] = run_config(CONFIGS[name], SIDE_STEPS[name], W, args.repeats, args, cpu_info, False)

    w = CONFIGS[args.workload]
    head["roofline"]["hbm_read_achievable_gbs"] = round(hbm_read, 1)            # non-temporal loads (as the kernel's)
    head["roofline"]["hbm_read_achievable_plain_loads_gbs"] = round(hbm_read_plain, 1)
    # per configuration (short keys keep the line small): iterations/s, gradient evaluations/s
    # (2 G per iteration), ms per step, the dominant stage and its ms, its fraction of the peak
    # (executed flops for the MLPs; "frac_alg": by the algorithmic flop count), the whole step's
    # fraction (algorithmic work / step time / peak), the oracle's iterations/s on all threads and
    # on one, and the oracle steps timed
    per_config = {}
    for name in ORDER:
        if name in details:
            d = details[name]
            r = d["roofline"]
            cb = d["cpu_baseline"] or {}
            e = {"it_s": d["iters_per_s"], "ge_s": d["grad_evals_per_s"], "ms": d["ms_per_step"],
                 "stage": r["kernel"].split(" [")[0].split(" (")[0], "stage_ms": r["avg_ms"], "bound": r["bound"],
                 "frac": r["frac"], "step_frac": r["whole_step_frac"], "cpu_it_s": cb.get("value"),
                 "cpu_1t": cb.get("one_thread_iters_per_s"),
                 "cpu_steps": int(cb["sample"].split(" ")[1]) if cb else None}
            if "frac_algorithmic" in r:
                e["frac_alg"] = r["frac_algorithmic"]
            for k_ in ("step_kinds", "live_variant", "one_launch_per_step"):
                if k_ in d:
                    e[k_] = {a_: b_ for a_, b_ in d[k_].items() if a_ not in ("note", "workload")}
            per_config[name] = e
    out = {"metric": "G-CADA iterations/s", "value": head["iters_per_s"], "unit": "iters/s",
           "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": head["ms_per_step"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32" if w.dtype == "f32" else "bf16", "data": "synthetic",
           "config": {"workload": w.name, "rule": args.rule, "G": w.G, "M_G": w.M_G, "mu": w.mu,
                      "widths": list(w.widths), "rows_per_shard": w.rows, "D": w.D, "c": w.c,
                      "l2": w.l2, "parallelism": "1 GPU, all groups simulated", "repeats": args.repeats,
                      "timing": "median of the passes"},
           "grad_evals_per_s": head["grad_evals_per_s"], "sample_grad_evals_per_s": head["sample_grad_evals_per_s"],
           "final_loss": head["final_loss"], "roofline": head["roofline"], "cpu_baseline": head["cpu_baseline"],
           "cost_model": head["cost_model"], "setup_s": head["setup_s"], "per_config": per_config}
    print(json.dumps({"bench_details": details, "hbm_read_achievable_gbs": hbm_read}), file=sys.stderr, flush=True)
    if args.details:
        with open(args.details, "w") as f:
            json.dump(details, f, indent=1)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
