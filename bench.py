#!/usr/bin/env python3
"""Benchmark of the QSR hot path on one MI355X.

One "step" = one global iteration of Local OPT for all K workers: local gradients, the fused
optimizer update, the device-side scheduler, and -- when the round's H-th step has run -- the
K-axis replica averaging and the next H from the quadratic rule.  The default workload is the
largest one that fits one GPU: the optimizer-only 350 M-parameter, 32-replica Local AdamW run
(179 GB of state, T = 2000, 4 averaging rounds).  Without --steps the timed region is exactly one
complete run; with fewer steps than a run has, the timed window is placed around the run's first
averaging round (the scheduler state is set to the window's first iteration), so that all four
parts of the path are inside it.

After the headline run, the five other workloads are run briefly and reported under
"per_workload" (--headline-only skips them).  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0 # MI355X dense bf16 matrix cores, vendor figure
BYTES_PER_UPDATE = {"adamw": 28, "sgdm": 20}   # algorithmic HBM bytes per replica-parameter
BYTES_PER_AVERAGE = 8

# HBM bytes per launch of the update kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE (scaled by a
# kernel of known size; profiles/*_hbm_traffic_pmc.md).  Valid only for the kernel source the
# counters were taken on: keyed by the first 16 hex digits of its SHA-256; null otherwise.
PMC_SOURCES = ["update.hip", "opt_elem.h", "philox.h"]
PMC_TRAFFIC = {
    # FETCH_SIZE x 2.000 (calibrated on the averaging kernel, which reads exactly 4 B x K x P) + WRITE_SIZE x 1.000
    # (calibrated on broadcast_rows_kernel / fill_zero_kernel), median over the launches of a run
    "flat350m+fuse_gradient": {"sha256_16": "0f04130a3671da8b", "bytes": 268.8004e9},   # algorithmic 268.8e9
    "flat60m+fuse_gradient": {"sha256_16": "0f04130a3671da8b", "bytes": 23.0402e9},     # algorithmic 23.04e9
    "flat60m": {"sha256_16": "0f04130a3671da8b", "bytes": 26.8801e9},                   # gradient read from its buffer: 26.88e9
}


def measured_traffic(workload, fused_gradient):
    import hashlib
    ent = PMC_TRAFFIC.get(workload + ("+fuse_gradient" if fused_gradient else ""))
    if not ent:
        return None
    h = hashlib.sha256()
    try:
        for name in PMC_SOURCES:
            h.update(open(os.path.join(ROOT, "paper_2310_14423_amd", "csrc", name), "rb").read())
    except OSError:
        return None
    return ent["bytes"] if h.hexdigest()[:16] == ent["sha256_16"] else None


# ------------------------------------------------------------------------------------------------
# the CPU oracle beside it
# ------------------------------------------------------------------------------------------------
def _oracle_eta(oracle, w):
    if w["lr"] == "step":
        return oracle.lr_step(w["T"], w.get("T_warm", 0), w["eta_max"], list(w["milestones"]), w["factor"])
    return oracle.lr_cosine(w["T"], w.get("T_warm", 0), w["eta_max"], w.get("eta_min", 0.0))


def cpu_baseline(w, cpu_seconds_target=20.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: gradient, update and
    averaging after every step (H = 1), all K workers, in double precision.  The optimizer-only
    workloads are sampled in P; the block models in depth and tokens (one block, one sequence of
    197 tokens per worker at the full layer width), with the figure extrapolated to the full shape
    given beside the measured one; the two small models run at their full shape."""
    import numpy as np
    import oracle
    import workloads
    oracle.build()
    K = w["K"]
    threads = max(1, min(K, os.cpu_count() or 1, 16))
    ws = dict(w)
    scale_to_full = 1.0
    if w["model"] == "noise":
        ws["P"] = min(w["P"], 1 << 20 if K > 16 else 1 << 18)
        what = "K=%d, P=%d (of %d), noise gradient + %s" % (K, ws["P"], w["P"], w["opt"])
    elif w["model"] == "resmlp":
        tokens = 197
        ws = workloads.get("vit" if w.get("n_heads", 0) else "resmlp", n_blocks=1, B_loc=tokens)
        # time is proportional to blocks x tokens, the parameter count to blocks
        scale_to_full = tokens / w["B_loc"]
        what = ("K=%d, one block of %d/%d%s on %d tokens per worker (of %d blocks on %d tokens), "
                "gradient by plain loops + AdamW" % (K, w["d_in"], w["d_hidden"],
                                                   " with its attention sub-block" if w.get("n_heads", 0) else "",
                                                   tokens, w["n_blocks"], w["B_loc"]))
    else:
        what = "K=%d, P=%d, B_loc=%d (the full shape), gradient by plain loops + %s" % (K, w["P"], w["B_loc"], w["opt"])
    P = ws["P"]
    eta = _oracle_eta(oracle, ws)
    const = workloads.model_const(ws)
    th0 = workloads.theta0(ws)

    def run(steps, n_threads, Kr=K):
        r = oracle.Run(K=Kr, n=P, eta=eta, T_warm=ws.get("T_warm", 0), opt=ws["opt"], mu=ws.get("mu", 0.0),
                       beta1=ws.get("beta1", 0.9), beta2=ws.get("beta2", 0.999), eps=ws.get("eps", 1e-8),
                       lam=ws.get("lam", 0.0), H_base=1, alpha=0.0, model=ws["model"], seed=ws["seed"],
                       grad_sigma=ws.get("grad_sigma", 0.0), data_sigma=ws.get("data_sigma", 0.0),
                       B_loc=ws.get("B_loc", 0), d_in=ws.get("d_in", 0), d_hidden=ws.get("d_hidden", 0),
                       d_out=ws.get("d_out", 0), n_blocks=ws.get("n_blocks", 0), n_heads=ws.get("n_heads", 0),
                       seq_len=ws.get("seq_len", 0), model_const=const, theta0=th0, n_threads=n_threads)
        steps = min(steps, ws["T"])
        t0 = time.perf_counter()
        r.step(steps)                 # H = 1: every step also averages, like the GPU's worst case
        return time.perf_counter() - t0, steps

    t1, _ = run(1, threads)
    # about cpu_seconds_target of CPU work in total: wall time per step times the threads it keeps busy
    steps = int(max(1, min(200, cpu_seconds_target / max(t1 * threads, 1e-3))))
    dt, steps = run(steps, threads)
    # and a few seconds on one core (the block models: one worker only, their gradient takes seconds)
    K1 = 1 if w["model"] == "resmlp" else K
    dt1, steps1 = run(max(1, steps // 8), 1, K1)
    out = {"value": K * P * steps / dt, "unit": "replica-param updates/s", "cores": threads, "kind": "oracle",
           "sample": "%s + averaging every step, double precision, %d iteration%s, %.1f s wall"
                     % (what, steps, "s" if steps > 1 else "", dt),
           "value_one_core": K1 * P * steps1 / dt1,
           "sample_one_core": "the same%s, %d iteration%s on one thread, %.1f s wall"
                              % ("" if K1 == K else " with one worker", steps1, "s" if steps1 > 1 else "", dt1)}
    if w["model"] == "noise":
        # the same 28 + 8 algorithmic bytes per replica-parameter as the GPU's two-kernel step with
        # averaging (the oracle's arrays are double precision: what it really moves is about twice that)
        out["GBs_at_gpu_byte_count"] = out["value"] * (BYTES_PER_UPDATE[w["opt"]] + BYTES_PER_AVERAGE) / 1e9
    if scale_to_full != 1.0:
        out["value_extrapolated_to_full_shape"] = out["value"] * scale_to_full
        out["extrapolation"] = "linear in blocks x tokens: measured value x %d / %d" % (197, w["B_loc"])
    return out


# ------------------------------------------------------------------------------------------------
# the GPU runs
# ------------------------------------------------------------------------------------------------
DEVICE_SCHEDULE_RUN = True      # --no-schedule-run: take the schedule from the library's host routine instead


def schedule_of_full_run(w):
    """Averaging points and periods of one complete run of the workload's schedule, taken from the
    device-side scheduler on a tiny optimizer-only problem: the schedule depends on the learning
    rates, alpha and H_base only (Eq. (2)), not on P or the model.  (Thousands of tiny launches: a
    profiling run asks for the host-side routine instead, which the tests hold equal to it.)"""
    import torch
    import numpy as np
    import paper_2310_14423_amd as qsr
    from paper_2310_14423_amd.binding import make_config
    keep = ("opt", "T", "T_warm", "lr", "eta_max", "eta_min", "milestones", "factor", "H_base", "alpha", "mu", "lam",
            "beta1", "beta2", "eps", "power", "t_local_start", "t_swap_start", "seed")
    w2 = {k: w[k] for k in keep if k in w}
    w2.update(model="noise", K=2, P=8, grad_sigma=1e-3)
    if not DEVICE_SCHEDULE_RUN:
        cfg, keepalive = make_config(w2)
        t_log, H_log = qsr.host_schedule(cfg)
        return [int(x) for x in t_log], [int(x) for x in H_log]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx = qsr.Context(w2, theta0=np.zeros(8, np.float32))
        ctx.run(w2["T"])
        t_log, H_log = ctx.read_sync_log()
        ctx.close()
    return [int(x) for x in t_log], [int(x) for x in H_log]


def run_workload(name, steps, warmup, kernel_timing=True, fuse_gradient=True, placement="plain", **overrides):
    """Runs `steps` iterations of one workload (after `warmup` untimed ones) and returns the fields
    of the JSON line that depend on the workload.  steps = None: one complete run from t = 0.
    Fewer steps than a run: the window [t0, t0 + steps) around the first averaging round.  The
    optimizer-only workloads run with the gradient drawn inside the update kernel unless
    fuse_gradient is False (then a fill kernel writes it first, as a model's backward pass would)."""
    import torch
    import workloads
    import paper_2310_14423_amd as qsr

    w = workloads.get(name, **overrides)
    if w["model"] == "noise" and fuse_gradient and w["P"] % 4 == 0:
        w["fuse_gradient"] = 2                 # drawn in registers, never written: 24 B per update
    K, P, T = w["K"], w["P"], w["T"]
    sched_t, sched_H = schedule_of_full_run(w)
    if steps is None:
        steps = T
    t_start = 0
    if steps < T and sched_t[0] >= steps:
        t_start = max(0, sched_t[0] - (steps + 1) // 2)
    ctx = qsr.Context(w, theta0=workloads.theta0(w), model_const=workloads.model_const(w), placement=placement)

    def begin_run():
        if t_start > 0:
            ctx.set_state((t_start, 0, t_start, sched_H[0]))
        else:
            ctx.restart()

    ctx.step(min(warmup, T))
    begin_run()
    ctx.timing(kernel_timing)
    ms = [0.0] * 4
    cnt = [0] * 4
    rounds = 0

    best = [None] * 4                       # shortest bracket of each kind over the timed region
    median = [None] * 4                     # median of each kind, from the read with the most brackets
    median_n = [0] * 4

    def collect():
        nonlocal ms, cnt, rounds
        if kernel_timing:
            m, c, lo, med = ctx.read_timing_stats()
            ms = [a + b for a, b in zip(ms, m)]; cnt = [a + b for a, b in zip(cnt, c)]
            for i in range(4):
                if c[i] > 0:
                    best[i] = lo[i] if best[i] is None else min(best[i], lo[i])
                    if c[i] > median_n[i]:
                        median[i], median_n[i] = med[i], c[i]
        rounds += ctx.get_H()[1]

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    left = steps
    while left > 0:
        n = min(left, T - t_start)
        ctx.step(n)
        left -= n
        if left > 0 or n == T:                 # a run is complete: collect, start the next one
            collect()
            if left > 0:
                begin_run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if steps % T != 0:
        collect()
    ctx.timing(False)

    # the update that draws its own gradient neither reads nor writes the gradient buffer
    upd_bytes = (BYTES_PER_UPDATE[w["opt"]] - (4 if w.get("fuse_gradient") == 2 else 0)) * K * P
    roofline = None
    kernels = {}
    if cnt[0] > 0:
        kernels["gradient_ms_avg"] = ms[0] / cnt[0]
    if cnt[1] > 0:
        kernels["update_ms_avg"] = ms[1] / cnt[1]
        kernels["update_GBs"] = upd_bytes / (ms[1] / cnt[1] * 1e-3) / 1e9
    if cnt[2] > 0:
        avg_ms = ms[2] / cnt[2]
        kernels["average_in_run_ms_avg"] = avg_ms
        kernels["average_in_run_GBs"] = BYTES_PER_AVERAGE * K * P / (avg_ms * 1e-3) / 1e9
        kernels["average_in_run_launches"] = cnt[2]
    if cnt[3] > 0:
        kernels["average_skipped_ms_avg"] = ms[3] / cnt[3]
    # share of the iteration time spent in the averaging that stands in for the All-Reduce (the
    # quantity the paper's App. F estimates from wall-clock differences), skipped launches included
    kernels["averaging_share_of_time"] = (ms[2] + ms[3]) * 1e-3 / dt if kernel_timing else None
    if w["model"] == "resmlp" and cnt[0] > 0:
        # the dense contraction dominates: 6 GEMMs of 2*M*d*dh flop per block and worker; the
        # duration is that of the whole gradient stage (GEMMs and their HBM-bound helpers)
        flops = 6 * w["n_blocks"] * K * 2.0 * w["B_loc"] * w["d_in"] * w["d_hidden"]
        if w.get("n_heads", 0):
            # attention sub-block: q|k|v and output projections (4 d^2 weights, forward + data
            # gradient + weight gradient) and the core's six products of M x seq_len x d each
            # (q k^T, p v forward; dV, dP, dQ, dK backward; recomputed scores not counted)
            flops += w["n_blocks"] * K * w["B_loc"] * (3 * 2.0 * 4 * w["d_in"] ** 2 + 6 * 2.0 * w["seq_len"] * w["d_in"])
        g_ms = ms[0] / cnt[0]
        ach = flops / (g_ms * 1e-3) / 1e12
        roofline = {"kernel": "gradient stage: gemm_nt_bf16_kernel / gemm_pp_tn_kernel%s + helpers" % (" / attn_*_kernel" if w.get("n_heads", 0) else ""),
                    "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "avg_ms": g_ms,
                    "median_ms": median[0], "min_ms": best[0],
                    "launches": cnt[0], "flops_per_launch": flops}
    elif cnt[1] > 0:
        ach = kernels["update_GBs"]
        roofline = {"kernel": "update_%s_kernel%s" % (w["opt"], " (gradient drawn inside, never in memory: 12 B read + 12 B written)" if w.get("fuse_gradient") else ""),
                    "bound": "hbm", "achieved": ach,
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                    "traffic": measured_traffic(name, bool(w.get("fuse_gradient"))),
                    "avg_ms": kernels["update_ms_avg"], "median_ms": median[1], "min_ms": best[1],
                    "launches": cnt[1], "bytes_per_launch": upd_bytes}

    # the averaging kernel runs only a handful of times per run: time it in a loop of its own
    reps = 20
    qsr.average_rows(ctx.params)
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        qsr.average_rows(ctx.params)
    e1.record(); torch.cuda.synchronize()
    a_ms = e0.elapsed_time(e1) / reps
    kernels["average_standalone_ms_avg"] = a_ms
    kernels["average_standalone_GBs"] = BYTES_PER_AVERAGE * K * P / (a_ms * 1e-3) / 1e9

    out = {
        "value": K * P * steps / dt, "steps": steps, "ms_per_step": dt * 1e3 / steps,
        "dtype": "bf16" if w["model"] == "resmlp" else "f32",
        "config": {"workload": name, "K": K, "P": P, "T": T, "optimizer": w["opt"],
                   "gradient": w["model"] + (" (drawn inside the update kernel, not stored)" if w.get("fuse_gradient") else ""),
                   "H_base": w["H_base"], "alpha": w["alpha"],
                   "lr": w["lr"], "eta_max": w["eta_max"],
                   "placement": ctx.placement,
                   "timed_window": [t_start, t_start + steps] if steps < T else [0, T]},
        "sync_rounds": rounds,                       # averaging rounds inside the timed window
        "sync_rounds_per_run": len(sched_t),         # of one complete run of T iterations
        "sync_schedule": {"source": "device scheduler, complete run at P = 8" if DEVICE_SCHEDULE_RUN else "host routine",
                          "rounds": len(sched_t), "T": T, "communication_volume": len(sched_t) / T,
                          "H": sched_H if len(sched_H) <= 32 else sched_H[:4] + ["..."] + sched_H[-4:],
                          "averaging_after_iteration": sched_t if len(sched_t) <= 32 else sched_t[:4] + ["..."] + sched_t[-4:]},
        "hbm_GBs_update": kernels.get("update_GBs"),
        "kernels": kernels,
        "roofline": roofline,
    }
    ctx.close()
    del ctx
    torch.cuda.empty_cache()
    if kernel_timing and dt / steps < 1e-3:
        # an iteration this short is launch cost, and the event brackets around its kernels add to
        # it: the same run once more without them, through qsr_run on a stream of its own (the
        # launches of several iterations replayed from a captured HIP graph)
        out["ms_per_step_no_event_brackets"] = replayed_run_ms(w)
    return out, w


def replayed_run_ms(w):
    import torch
    import workloads
    import paper_2310_14423_amd as qsr
    T = w["T"]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx = qsr.Context(w, theta0=workloads.theta0(w), model_const=workloads.model_const(w))
        ctx.run(T); ctx.restart()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.run(T)
        rounds = ctx.get_H()[1]                # synchronizes the stream
        dt = time.perf_counter() - t0
        ctx.close()
    return dt * 1e3 / T if rounds > 0 else None


def fused_sync_probe(name, **overrides):
    """The optional fused form (update + averaging of a round's last step in one pass) on the same
    buffers: a short run with a constant period of 4, so that every fourth step synchronizes.
    Bytes per replica-parameter on such a step: AdamW 16 read + 8 (m, v) + 4 (mean) written = 28
    instead of 28 (update) + 8 (averaging); SGD 20 instead of 20 + 8."""
    import torch
    import workloads
    import paper_2310_14423_amd as qsr
    w = workloads.get(name, fuse_sync=True, power=0, H_base=4, alpha=0.0, **overrides)
    K, P = w["K"], w["P"]
    ctx = qsr.Context(w, theta0=workloads.theta0(w), model_const=workloads.model_const(w))
    ctx.step(8)
    ctx.timing(True)
    ctx.read_timing()
    ctx.step(40)
    ms, cnt = ctx.read_timing()
    ctx.timing(False)
    ctx.close()
    del ctx
    torch.cuda.empty_cache()
    if cnt[2] == 0:
        return None
    f_ms = ms[2] / cnt[2]
    nbytes = BYTES_PER_UPDATE[w["opt"]] * K * P
    return {"update_and_average_fused_ms_avg": f_ms, "launches": cnt[2], "bytes_per_launch": nbytes,
            "GBs": nbytes / (f_ms * 1e-3) / 1e9, "skipped_launch_ms_avg": ms[3] / cnt[3] if cnt[3] else None}


def clip_probe(name, **overrides):
    """The optional gradient clipping on the same buffers: the norm pass reads the gradients once
    more (4 B per replica-parameter), the factors are applied inside the update kernel; the update
    bracket then covers 28 + 4 = 32 B (AdamW) per replica-parameter."""
    import torch
    import workloads
    import paper_2310_14423_amd as qsr
    w = workloads.get(name, clip_norm=1.0, **overrides)
    K, P = w["K"], w["P"]
    ctx = qsr.Context(w, theta0=workloads.theta0(w), model_const=workloads.model_const(w))
    ctx.step(5)
    ctx.timing(True)
    ctx.read_timing()
    ctx.step(30)
    ms, cnt = ctx.read_timing()
    ctx.timing(False)
    ctx.close()
    del ctx
    torch.cuda.empty_cache()
    u_ms = ms[1] / cnt[1]
    nbytes = (BYTES_PER_UPDATE[w["opt"]] + 4) * K * P
    return {"norm_and_update_ms_avg": u_ms, "launches": cnt[1], "bytes_per_launch": nbytes,
            "GBs": nbytes / (u_ms * 1e-3) / 1e9}


# short runs of the other workloads, reported next to the headline one
OTHER_WORKLOADS = {"lsq": dict(steps=None, warmup=5), "mlp": dict(steps=None, warmup=5),
                   "resmlp": dict(steps=20, warmup=5), "vit": dict(steps=20, warmup=5),
                   "flat60m": dict(steps=400, warmup=5),
                   "flat350m": dict(steps=40, warmup=5)}
PER_WORKLOAD_KEYS = ("value", "steps", "ms_per_step", "ms_per_step_no_event_brackets", "dtype", "sync_rounds",
                     "sync_rounds_per_run", "sync_schedule", "hbm_GBs_update", "kernels", "roofline")


def flat350m_overrides(torch):
    """The largest workload fills 179 of 288 GB: if another process holds part of the HBM, the
    largest number of workers that fits is run, and named as such."""
    free, _ = torch.cuda.mem_get_info()
    need = lambda K: 4 * K * 350_000_000 * 4 + (6 << 30)
    return [{} if K == 32 else {"K": K} for K in (32, 24, 16) if free >= need(K)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="flat350m", choices=["flat60m", "flat350m", "lsq", "mlp", "resmlp", "vit"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fuse-gradient", action="store_true",
                    help="optimizer-only workloads: fill the gradient buffer with a kernel of its own "
                         "instead of drawing the gradient inside the update kernel")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="skip the per-kernel HIP events (the roofline object is then null)")
    ap.add_argument("--no-schedule-run", action="store_true",
                    help="take the averaging schedule from the library's host-side routine instead of a "
                         "complete run of the device scheduler on a tiny problem (for profiling runs)")
    ap.add_argument("--headline-only", action="store_true",
                    help="do not add the short runs of the other workloads (per_workload)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the K workers are simulated on ONE GPU; "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    global DEVICE_SCHEDULE_RUN
    DEVICE_SCHEDULE_RUN = not args.no_schedule_run

    head_over = {}
    if args.workload == "flat350m":
        tries = flat350m_overrides(torch)
        if not tries:
            print("bench.py: not enough free HBM for flat350m even with 16 workers", file=sys.stderr)
            sys.exit(1)
        head_over = tries[0]
    res, w = run_workload(args.workload, args.steps, args.warmup, not args.no_kernel_timing,
                          not args.no_fuse_gradient, **head_over)
    out = {"metric": "replica-param updates/s", "value": res["value"], "unit": "updates/s",
           "n_gpus": 1, "steps": res["steps"], "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": res["dtype"], "data": "synthetic", "config": res["config"],
           "sync_rounds": res["sync_rounds"], "sync_rounds_per_run": res["sync_rounds_per_run"],
           "sync_schedule": res["sync_schedule"], "hbm_GBs_update": res["hbm_GBs_update"],
           "kernels": res["kernels"], "roofline": res["roofline"]}
    if head_over:
        out["config"]["reduced_to"] = head_over
    if "ms_per_step_no_event_brackets" in res:
        out["ms_per_step_no_event_brackets"] = res["ms_per_step_no_event_brackets"]
    out["cpu_baseline"] = None if args.no_cpu_baseline else cpu_baseline(w)
    if not args.headline_only:
        per = {}
        for name, kw in OTHER_WORKLOADS.items():
            if name == args.workload:
                continue
            tries = flat350m_overrides(torch) if name == "flat350m" else [{}]
            for over in tries:
                try:
                    r, wn = run_workload(name, kw["steps"], kw["warmup"], **over)
                    per[name] = {k: r[k] for k in PER_WORKLOAD_KEYS if k in r}
                    per[name]["placement"] = r["config"]["placement"]
                    per[name]["timed_window"] = r["config"]["timed_window"]
                    if over:
                        per[name]["reduced_to"] = over
                    if not args.no_cpu_baseline:
                        per[name]["cpu_baseline"] = cpu_baseline(wn, 10.0)
                    break
                except Exception as e:
                    per[name] = {"error": "%s: %s" % (type(e).__name__, e)}
                    torch.cuda.empty_cache()
        out["per_workload"] = per
        # the update as it looks behind a real model's backward pass: the gradient written by a
        # kernel of its own first, 28 B per replica-parameter (at the 60 M x 16 size)
        flat = "flat60m"
        r, _ = run_workload(flat, 100, 5, True, False)
        out["separate_gradient_fill"] = dict({k: r[k] for k in ("value", "steps", "ms_per_step", "kernels", "roofline")},
                                             workload=flat)
        # the experiment with the state arrays spread over the HBM's three physical ranges (the
        # binding's opt-in placement): the same kernels, 20 launches, beside the plain figures above
        try:
            r, _ = run_workload(flat, 20, 5, True, True, placement="spread")
            out["placement_spread"] = {"workload": flat, "placement": r["config"]["placement"],
                                       "timed_window": r["config"]["timed_window"], "ms_per_step": r["ms_per_step"],
                                       "kernels": r["kernels"], "roofline": r["roofline"]}
        except Exception as e:
            out["placement_spread"] = {"error": "%s: %s" % (type(e).__name__, e)}
            torch.cuda.empty_cache()
        out["fused_sync"] = dict(fused_sync_probe(flat) or {}, workload=flat)
        out["gradient_clipping"] = dict(clip_probe(flat), workload=flat)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
