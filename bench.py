#!/usr/bin/env python3
"""Benchmark of the CoCoD-SGD round on one MI355X.

A "step" is one round of Algorithm 1 for all W workers: store the models, start the cross-worker
mean on the averaging stream, take k local momentum-SGD steps on the compute stream, join, apply
line 6.  Workload: the ResNet18-sized flat vector (W=16, d=11.2M fp32, momentum 0.9, weight decay
5e-4, lr 0.05, noise 0.01), all state resident in HBM before timing starts; synthetic data.

Prints ONE JSON line.  `value` = worker-param-updates/s = W*d*k / round time at k=2; the k sweep,
the other schedules, the roofline of the dominant kernel (the fused local step) and the CPU oracle
timed on the host cores ride along in the same line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E bandwidth
STEP_BYTES = 24                 # local step: read x, v, h, c; write x, v (fp32)
# HBM bytes per launch of the step kernel at this workload from two rocprofv3 --pmc runs
# (FETCH_SIZE x 2.000 + WRITE_SIZE x 0.999, factors from the known-size copy kernel):
# profiles/kernels_C2_W16_d11.2M_hbm_counters.md
STEP_TRAFFIC_BYTES = 4.3038e9


def round_bytes(W, d, k):
    """Algorithmic HBM bytes of one round: k steps, mean (read W rows, write 1), line 6 (read x, snap, mean once; write x)."""
    return W * d * (STEP_BYTES * k + 4 * (1 + 1 / W) + 12 + 4 / W)


def time_rounds(ctx, torch, k, rounds, warmup, want_step_times):
    """Seconds per round over `rounds` timed rounds, and the average step-kernel duration in seconds
    measured over the same rounds (the kernel's own start/stop timestamps on the compute stream)."""
    for _ in range(warmup):
        ctx.round(k)
    ctx.sync()
    ctx.step_timing(rounds * k if want_step_times else 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(rounds):
        ctx.average_begin()
        ctx.local_steps(k)
        ctx.average_end_apply()
    ctx.sync()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    step_s = None
    if want_step_times:
        total_ms, n = ctx.step_timing_read()
        step_s = total_ms / max(n, 1) / 1e3
        ctx.step_timing(0)
    return elapsed / rounds, step_s


def cpu_baseline(cfg, k):
    """The oracle as it stands, timed on the host cores at the full workload shape for a few rounds."""
    from oracle import cocod_oracle as orc
    W, d = cfg["W"], cfg["d"]
    h, c = orc.fill_quadratic(cfg["seed"], W, d)
    o = orc.QuadraticOracle(h, c, lr=cfg["lr"], momentum=cfg["momentum"], weight_decay=cfg["weight_decay"],
                            noise_sigma=cfg["noise_sigma"], seed=cfg["seed"])
    t0 = time.perf_counter()
    o.round(k)
    first = time.perf_counter() - t0
    rounds = int(max(2, min(20, round(12.0 / max(first, 1e-3)))))
    t0 = time.perf_counter()
    for _ in range(rounds):
        o.round(k)
    per_round = (time.perf_counter() - t0) / rounds
    return {"value": W * d * k / per_round, "unit": "worker-param-updates/s", "cores": orc.num_threads(),
            "kind": "oracle", "ms_per_round": per_round * 1e3,
            "algorithmic_GBps_fp32_equiv": round_bytes(W, d, k) / per_round / 1e9,
            "sample": "full shape W=%d d=%d k=%d, %d rounds after 1 untimed, fp64 C oracle with OpenMP" % (W, d, k, rounds)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50, help="timed rounds")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--k", type=int, default=2, help="local steps per round for the headline value")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true", help="skip the k sweep and the other schedules")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the W workers are replicas in one MI355X's HBM); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import torch
    import paper_1906_12043_amd as P
    import synth_inputs
    if not os.path.exists(P.lib_path()):
        from paper_1906_12043_amd import build as hip_build
        hip_build.build()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1

    cfg = synth_inputs.CONFIGS["C2_resnet18"]
    W, d = cfg["W"], cfg["d"]
    dev = torch.device("cuda:0")
    stride, _, _ = P.plan_layout(d)
    xA = torch.zeros((W, stride), device=dev)
    xB = torch.zeros((W, stride), device=dev)
    v = torch.zeros((W, stride), device=dev)
    mean = torch.zeros(stride, device=dev)
    h = torch.empty((W, stride), device=dev)
    c = torch.empty((W, stride), device=dev)
    s_compute, s_avg = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)
    torch.cuda.synchronize()
    ctx = P.Context(W=W, d=d, stride=stride, xA=xA, xB=xB, v=v, mean=mean, h=h, c=c, lr=cfg["lr"],
                    momentum=cfg["momentum"], weight_decay=cfg["weight_decay"], noise_sigma=cfg["noise_sigma"],
                    seed=cfg["seed"], compute_stream=s_compute, avg_stream=s_avg)
    ctx.fill_quadratic()
    ctx.sync()

    k = args.k
    per_round, avg_step_s = time_rounds(ctx, torch, k, args.steps, args.warmup, True)
    achieved = STEP_BYTES * W * d / avg_step_s / 1e9
    out = {
        "metric": "worker-param-updates/s per CoCoD round (W=16, d=11.2M)",
        "value": W * d * k / per_round,
        "unit": "worker-param-updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": per_round * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "C2 ResNet18-sized flat vector: W=16 workers x d=11.2M fp32, quadratic+Philox-noise "
                               "gradient, momentum 0.9, wd 5e-4, lr 0.05", "k": k, "schedule": "overlap (2 streams)",
                   "W": W, "d": d},
        "round_algorithmic_GBps": round_bytes(W, d, k) / per_round / 1e9,
        "round_frac_of_hbm_peak": round_bytes(W, d, k) / per_round / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": "quad_step_kernel<momentum, noise>", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": STEP_TRAFFIC_BYTES, "avg_launch_ms": avg_step_s * 1e3,
                     "launches_timed": args.steps * k, "algorithmic_bytes_per_launch": STEP_BYTES * W * d},
    }
    if not args.headline_only:
        sweep = {}
        for kk in cfg["k"]:
            pr, sm = time_rounds(ctx, torch, kk, args.steps, 2, True)
            sweep["k=%d" % kk] = {"ms_per_round": pr * 1e3, "updates_per_s": W * d * kk / pr,
                                  "round_GBps": round_bytes(W, d, kk) / pr / 1e9,
                                  "step_kernel_ms": sm * 1e3}
        out["k_sweep"] = sweep
        sched = {}
        for name, code in (("serial", P.SCHED_SERIAL), ("fused", P.SCHED_FUSED), ("overlap", P.SCHED_OVERLAP)):
            ctx.set_schedule(code)
            pr, _ = time_rounds(ctx, torch, k, args.steps, 2, False)
            sched[name] = pr * 1e3
        out["schedule_ms_per_round"] = sched
    ctx.close()
    del xA, xB, v, mean, h, c
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, k)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
