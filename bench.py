#!/usr/bin/env python3
"""Benchmark of the CoCoD-SGD round on one MI355X.

A "step" is one round of Algorithm 1 for all W workers: store the models, start the cross-worker
mean on the averaging stream, take k local momentum-SGD steps on the compute stream, join, apply
line 6.  Headline workload: the ResNet18-sized flat vector (C2: W=16, d=11.2M fp32, momentum 0.9,
weight decay 5e-4, lr 0.05, noise 0.01), k = 2, all state resident in HBM before timing starts;
synthetic data.

Two ways of running the same round are timed:
  separate    cocod_average_begin; cocod_local_steps(k); cocod_average_end_apply
  fused_tail  cocod_average_begin; cocod_local_steps_end_apply(k)   (line 6 inside the last step)
Prints ONE JSON line.  `value` = worker-param-updates/s = W*d*k / round time for the variant named in
config.variant under the overlapped two-stream schedule.  The same line carries: the k sweep (both
variants, each also replayed from a HIP graph, and under the schedule that forms the mean inside the
round's first step), the serial schedules, what the overlap hides by interval and by cost, the roofline
of the step kernels, the CPU oracle timed on the host cores, and under "workloads" a compact
measurement of the other configurations (C3 VGG16-sized, C5 bucketed tensor list with W=64, C4
MLP-gradient workers).  `--workload X` measures one configuration alone; `--kernels-alone` launches
every kernel of the round by itself (the program to put under rocprofv3 for per-dispatch counters).
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
MFMA_F32_PEAK_TFLOPS = 157.3    # MI355X published dense fp32 matrix rate
STEP_BYTES = 24                 # plain local step: read x, v, h, c; write x, v (fp32); 16 without momentum
# HBM bytes per launch at C2 from two rocprofv3 --pmc runs (FETCH_SIZE x 2.000 + WRITE_SIZE x 0.999,
# factors from the known-size copy kernel): profiles/kernels_C2_W16_d11.2M_hbm_counters.md, checked
# against that file by tests/test_bench_contract.py
STEP_TRAFFIC_BYTES = 4.3034e9                        # plain step
TAIL_TRAFFIC_BYTES = {1: 5.0620e9, 2: 5.7788e9}      # step that carries line 6: k = 1 / k >= 2

NAMES = {"C1": "C1_tiny", "C2": "C2_resnet18", "C3": "C3_vgg16", "C4": "C4_mlp", "C5": "C5_bucketed"}
LABELS = {"C1": "C1 tiny flat vector", "C2": "C2 ResNet18-sized flat vector", "C3": "C3 ImageNet-VGG16-sized flat vector",
          "C5": "C5 ResNet18-like list of 62 tensors in 25 MiB buckets"}


def step_bytes(momentum):
    return STEP_BYTES if momentum else 16


def model_round_bytes(W, d, k, per_step=STEP_BYTES):
    """Bytes of one round in the accounting where line 6 is a pass of its own:
    k steps (24) + mean (4(1+1/W)) + line 6 with the mean read once per column (12+4/W)."""
    return W * d * (per_step * k + 16 + 8 / W)


def tail_step_bytes(W, d, k, per_step=STEP_BYTES):
    """Step that carries line 6: the plain step's 24 B plus the stored model (not at k=1, where the
    step reads it anyway) plus the mean, shared by the W workers of a column."""
    return W * d * (per_step + (4 if k > 1 else 0) + 4 / W)


def moved_round_bytes(W, d, k, variant, per_step=STEP_BYTES):
    if variant.startswith("head_"):              # no pass for the mean: only its store, and its read by line 6
        if k == 1 and variant.endswith("fused_tail"):
            return W * d * (per_step + 4 / W)    # one pass: mean, step and line 6 together; the mean is only written
        return moved_round_bytes(W, d, k, variant[len("head_"):], per_step) - W * d * 4
    if variant in ("separate", "graph_separate"):
        return model_round_bytes(W, d, k, per_step)
    return W * d * (per_step * (k - 1) + 4 * (1 + 1 / W)) + tail_step_bytes(W, d, k, per_step)


def time_rounds(ctx, torch, k, rounds, warmup, variant, want_step_times=True):
    """Seconds per round over `rounds` timed rounds and, measured over the same rounds from the
    kernels' own start/stop timestamps on the compute stream, the average duration in seconds of the
    plain step kernel, of the step kernel that carries line 6 and of the first step that also forms the
    mean (None where there was no launch)."""
    import paper_1906_12043_amd as P
    head = variant.startswith("head_")           # Step I inside the round's first step (one stream)
    if head:
        variant = variant[len("head_"):]
        ctx.set_schedule(P.SCHED_HEAD)

    def one_round():
        if variant.startswith("graph"):          # the whole round as one graph launch
            ctx.graph_round(k, variant == "graph_fused_tail")
            return
        ctx.average_begin()
        if variant == "separate":
            ctx.local_steps(k)
            ctx.average_end_apply()
        else:
            ctx.local_steps_end_apply(k)
    for _ in range(warmup):
        one_round()
    ctx.sync()
    want_step_times = want_step_times and not variant.startswith("graph")   # launches in a graph are not timed
    ctx.step_timing(rounds * k if want_step_times else 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(rounds):
        one_round()
    ctx.sync()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    avg = [None, None, None]
    if want_step_times:
        for i, (total_ms, n) in enumerate(ctx.step_timing_read()):
            if n:
                avg[i] = total_ms / n / 1e3
        ctx.step_timing(0)
    if head:
        ctx.set_schedule(P.SCHED_OVERLAP)
    return elapsed / rounds, avg[0], avg[1], avg[2]


def timelines(ctx, torch, P, k, rounds):
    """The four timelines that the paper's time-speedup analysis compares, built from the same
    kernels on one GPU, as average milliseconds per local step (the paper's T_N^av up to the factor N):
      s_sgd      one step, then blocking average of the models          (communicate every step, sequential)
      local_sgd  k steps, then blocking average                         (communicate every k steps, sequential)
      cocod      the round with the mean overlapped and line 6 separate (every k steps, in parallel)
      cocod_fused_tail  the same with line 6 inside the last step
    Blocking average = cocod_average_apply_fused while idle: every worker lands on the mean of the current models."""
    def timed(body, steps_per_iter):
        for _ in range(2):
            body()
        ctx.sync()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(rounds):
            body()
        ctx.sync()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / rounds / steps_per_iter * 1e3

    out = {}
    out["s_sgd"] = timed(lambda: (ctx.local_steps(1), ctx.average_apply_fused()), 1)
    out["local_sgd"] = timed(lambda: (ctx.local_steps(k), ctx.average_apply_fused()), k)
    ctx.set_schedule(P.SCHED_OVERLAP)
    out["cocod"] = timed(lambda: ctx.round(k), k)
    out["cocod_fused_tail"] = timed(lambda: ctx.round_fused_tail(k), k)
    out["k"] = k
    return out


def external_gradient_rounds(ctx, torch, W, d, stride, k, rounds, g32, scratch):
    """The round with the caller's gradient (a real model's backward pass would write it): k steps of
    cocod_external_step, the last one closing the round with line 6 inside, for fp32 gradients (20 B per
    worker-parameter and step) and 16-bit ones (18 B).  The gradient buffers are whatever the workload's
    h array holds (fp32) and a 16-bit view of its c array: the arithmetic does not matter here, the bytes do."""
    g16 = scratch.view(torch.bfloat16).reshape(-1)[:W * stride].view(W, stride)   # a dense [W][stride] block of 16-bit elements
    out = {}
    for name, call, g, gbytes in (("fp32", ctx.external_step, g32, 4), ("bf16", ctx.external_step_bf16, g16, 2)):
        def one_round():
            ctx.average_begin()
            for s in range(k):
                call(g, close_round=(s == k - 1))
        for _ in range(2):
            one_round()
        ctx.sync()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(rounds):
            one_round()
        ctx.sync()
        per_round = (time.perf_counter() - t0) / rounds
        per_step = STEP_BYTES - 8 + gbytes                    # r x, v, g; w x, v
        # + the mean's pass, + the mean read by the last step, + the stored model there (at k = 1 the step reads it anyway)
        moved = W * d * (per_step * k + 4 * (1 + 1 / W) + 4 / W + (4 if k > 1 else 0))
        out[name] = {"ms_per_round": per_round * 1e3, "updates_per_s": W * d * k / per_round,
                     "moved_GBps": moved / per_round / 1e9, "bytes_per_worker_param_step": per_step}
    out["k"] = k
    return out


def round_event_times(ctx, torch, stream, k, rounds, variant):
    """Median and minimum round time from events recorded on the compute stream around every round
    (every variant ends its round on that stream)."""
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(rounds + 1)]
    ctx.sync()
    marks[0].record(stream)
    for r in range(rounds):
        ctx.average_begin()
        if variant == "separate":
            ctx.local_steps(k)
            ctx.average_end_apply()
        else:
            ctx.local_steps_end_apply(k)
        marks[r + 1].record(stream)
    ctx.sync()
    ms = sorted(marks[r].elapsed_time(marks[r + 1]) for r in range(rounds))
    return {"round_ms_median": ms[len(ms) // 2], "round_ms_min": ms[0]}


def overlap_figures(ctx, torch, P, s_avg, k, rounds, step_beside_mean_s):
    """What running Step I beside Step II buys on one GPU, by cost (the interval figure comes from the
    kernel trace under profiles/): the plain step alone, the same step while the mean runs on the other
    stream, and the mean alone.  mean_cost_hidden_frac = 1 - (step beside the mean - step alone) / mean alone:
    the share of the mean's own duration that does NOT reappear as a slower step."""
    ctx.set_schedule(P.SCHED_OVERLAP)
    ctx.local_steps(2)
    ctx.sync()
    ctx.step_timing(8)
    ctx.local_steps(8)                                   # outside a round: nothing runs beside them
    alone_ms, n = ctx.step_timing_read()[0]
    ctx.step_timing(0)
    step_alone_s = alone_ms / n / 1e3
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    mean_ms = []
    for _ in range(min(rounds, 20) + 2):
        ctx.sync()
        a.record(s_avg)
        ctx.average_begin()                              # the mean starts on the averaging stream at once: compute is idle
        b.record(s_avg)
        ctx.average_end_apply()
        ctx.sync()
        mean_ms.append(a.elapsed_time(b))
    mean_alone_s = sorted(mean_ms[2:])[len(mean_ms[2:]) // 2] / 1e3
    out = {"plain_step_alone_ms": step_alone_s * 1e3, "mean_alone_ms": mean_alone_s * 1e3}
    if step_beside_mean_s:
        out["plain_step_beside_mean_ms"] = step_beside_mean_s * 1e3
        out["mean_cost_hidden_frac"] = 1.0 - (step_beside_mean_s - step_alone_s) / mean_alone_s
    return out


def diagnostics_figures(ctx, torch, stream, W, d, quadratic):
    """The two scalar diagnostics at this workload: consensus distance sum_i p_i ||x^ - x_i||^2 (read: the W
    models, 4 B per worker-parameter; timed through the entry point that only enqueues, events around 10
    calls) and objective + squared gradient norm at the mean (read: models, h, c: 12 B; the call copies
    its two scalars back, so it is timed by the host clock)."""
    out = {}
    result = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    try:
        ctx.consensus_distance_noalloc(result)
        ctx.sync()
        a.record(stream)
        for _ in range(10):
            ctx.consensus_distance_noalloc(result)
        b.record(stream)
        ctx.sync()
        ms = a.elapsed_time(b) / 10
        out["consensus_distance"] = {"ms": ms, "GBps": 4.0 * W * d / ms / 1e6, "value": float(result.item())}
    except Exception as e:                       # more chunks than the static scratch holds
        out["consensus_distance"] = {"ms": None, "note": str(e)[:120]}
    if quadratic:
        ctx.quadratic_objective()
        t0 = time.perf_counter()
        for _ in range(5):
            f, g2 = ctx.quadratic_objective()
        ms = (time.perf_counter() - t0) / 5 * 1e3
        out["quadratic_objective"] = {"ms": ms, "GBps": 12.0 * W * d / ms / 1e6, "f_at_mean": f, "grad_norm_sq_at_mean": g2}
    return out


SINGLE_THREAD_SAMPLE = """
import json, sys, time
sys.path.insert(0, %r)
import synth_inputs
from oracle import cocod_oracle as orc
cfg = synth_inputs.CONFIGS["C2_resnet18"]
W, n, k = cfg["W"], cfg["d"] // 16, %d
h, c = orc.fill_quadratic(cfg["seed"], W, n)
o = orc.QuadraticOracle(h, c, lr=cfg["lr"], momentum=cfg["momentum"], weight_decay=cfg["weight_decay"],
                        noise_sigma=cfg["noise_sigma"], seed=cfg["seed"])
o.round(k)
t0 = time.perf_counter()
for _ in range(3):
    o.round(k)
print(json.dumps({"per_round": (time.perf_counter() - t0) / 3, "threads": orc.num_threads(), "W": W, "n": n}))
"""


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
    out = {"value": W * d * k / per_round, "unit": "worker-param-updates/s", "cores": orc.num_threads(),
           "kind": "oracle", "ms_per_round": per_round * 1e3,
           "model_GBps": model_round_bytes(W, d, k) / per_round / 1e9,     # the round's fp32 byte model, for comparison only
           "sample": "full shape W=%d d=%d k=%d, %d rounds after 1 untimed, fp64 C oracle with OpenMP" % (W, d, k, rounds)}
    # the same oracle on ONE thread (child process with OMP_NUM_THREADS=1), on the first d/16 columns
    import subprocess
    try:
        r = subprocess.run([sys.executable, "-c", SINGLE_THREAD_SAMPLE % (ROOT, k)], capture_output=True, text=True,
                           timeout=240, env=dict(os.environ, OMP_NUM_THREADS="1"))
        one = json.loads(r.stdout.strip().splitlines()[-1])
        out["single_thread"] = {"value": one["W"] * one["n"] * k / one["per_round"], "threads": one["threads"],
                                "sample": "W=%d, first %d columns, k=%d, 3 rounds after 1 untimed" % (one["W"], one["n"], k)}
    except Exception as e:                  # the baseline is a report, never a reason to fail the benchmark
        out["single_thread"] = {"value": None, "error": str(e)[:200]}
    return out


def roofline(name, algorithmic_bytes, seconds, launches, traffic):
    achieved = algorithmic_bytes / seconds / 1e9
    return {"bound": "hbm", "kernel": name, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "avg_launch_ms": seconds * 1e3,
            "launches_timed": launches, "algorithmic_bytes_per_launch": algorithmic_bytes}


class QuadraticWorkload:
    """Device buffers and context of one of the quadratic-gradient configurations, state resident in HBM."""

    def __init__(self, workload):
        import torch
        import paper_1906_12043_amd as P
        import synth_inputs
        self.torch, self.P = torch, P
        self.workload = workload
        self.cfg = cfg = synth_inputs.CONFIGS[NAMES[workload]]
        self.W, self.d = cfg["W"], cfg["d"]
        self.sizes = (synth_inputs.tensor_sizes(cfg["seed"], cfg["n_tensors"], self.d, cfg["tensor_lo"], cfg["tensor_hi"])
                      if "n_tensors" in cfg else None)
        dev = torch.device("cuda:0")
        stride, _, _ = P.plan_layout(self.d, self.sizes, cfg.get("bucket_bytes", 0))
        self.stride = (stride + 1023) // 1024 * 1024     # worker rows start on 4 KiB boundaries (measured: faster streaming)
        W = self.W
        self.xA = torch.zeros((W, self.stride), device=dev)
        self.xB = torch.zeros((W, self.stride), device=dev)
        self.v = torch.zeros((W, self.stride), device=dev) if cfg["momentum"] else None
        self.mean = torch.zeros(self.stride, device=dev)
        self.h = torch.empty((W, self.stride), device=dev)
        self.c = torch.empty((W, self.stride), device=dev)
        self.s_compute, self.s_avg = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)
        torch.cuda.synchronize()
        self.ctx = P.Context(W=W, d=self.d, stride=self.stride, xA=self.xA, xB=self.xB, v=self.v, mean=self.mean, h=self.h,
                             c=self.c, lr=cfg["lr"], momentum=cfg["momentum"], weight_decay=cfg["weight_decay"],
                             noise_sigma=cfg["noise_sigma"], seed=cfg["seed"], tensor_numel=self.sizes,
                             bucket_bytes=cfg.get("bucket_bytes", 0), compute_stream=self.s_compute, avg_stream=self.s_avg)
        self.per_step = step_bytes(cfg["momentum"])

    def copy_rate(self):
        """What a plain copy of one [W][stride] array reaches on this machine, same launch path (h -> c, before they are filled)."""
        for timed in (False, True):
            self.torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20 if timed else 3):
                self.P.debug_copy(self.s_compute, self.h, self.c, self.W * self.stride)
            self.ctx.sync()
            copy_s = (time.perf_counter() - t0) / 20
        return 8.0 * self.W * self.stride / copy_s / 1e9

    def fill(self):
        self.ctx.fill_quadratic()
        self.ctx.sync()

    def close(self):
        self.ctx.close()
        del self.xA, self.xB, self.v, self.mean, self.h, self.c
        self.torch.cuda.empty_cache()


def bench_quadratic(workload, k, variant, steps, warmup, full):
    """One of C1, C2, C3, C5.  full: also the k sweep, the schedules, the timelines and the caller's-gradient rounds."""
    import torch
    import paper_1906_12043_amd as P
    wl = QuadraticWorkload(workload)
    cfg, W, d, ctx, per_step = wl.cfg, wl.W, wl.d, wl.ctx, wl.per_step
    if k not in cfg["k"] and workload != "C2":
        k = cfg["k"][0]
    copy_gbps = wl.copy_rate()
    wl.fill()
    per_round, plain_s, tail_s, _ = time_rounds(ctx, torch, k, steps, warmup, variant)
    moved = moved_round_bytes(W, d, k, variant, per_step)
    out = {
        "metric": "worker-param-updates/s per CoCoD round (W=%d, d=%.4gM)" % (W, d / 1e6),
        "value": W * d * k / per_round,
        "unit": "worker-param-updates/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": per_round * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: W=%d workers x d=%d fp32, quadratic+Philox-noise gradient, momentum %g, wd %g, lr %g"
                               % (LABELS[workload], W, d, cfg["momentum"], cfg["weight_decay"], cfg["lr"]),
                   "k": k, "variant": variant,
                   "schedule": "overlap (2 streams)", "W": W, "d": d},
        "round_model_GBps": model_round_bytes(W, d, k, per_step) / per_round / 1e9,
        "round_moved_GBps": moved / per_round / 1e9,
        "round_moved_frac_of_hbm_peak": moved / per_round / 1e9 / HBM_PEAK_GBS,
        "copy_kernel_GBps": copy_gbps,          # plain copy of a [W][stride] array on this machine, read + write
        "round_moved_frac_of_copy_kernel": moved / per_round / 1e9 / copy_gbps,
    }
    if workload == "C2" and variant == "fused_tail" and k >= 1:
        # the same round by the hardware counters (bytes across the L2 boundary per launch, from the counter
        # runs under profiles/): k-1 plain steps, the mean (4(1+1/W) B, ratio 1.000), the step with line 6
        counted = (k - 1) * STEP_TRAFFIC_BYTES + 4 * (1 + 1 / W) * W * d + TAIL_TRAFFIC_BYTES[min(k, 2)]
        out["round_counter_GBps"] = counted / per_round / 1e9
    out.update(round_event_times(ctx, torch, wl.s_compute, k, steps, variant))
    # "roofline" is the step that carries line 6 when the round has one: it moves the most bytes per launch
    # and has the memory system to itself.  The plain step rides along; as the FIRST step of a round it shares
    # HBM with the mean on the other stream and runs about as long, so its own bytes over its duration
    # understate what the memory system moves then: "roofline_first_step_and_mean" counts both kernels' bytes
    # over the step's duration (the mean lies inside it: profiles/round_C2_...md).
    plain = tail = None
    if plain_s:
        n_plain = steps * (k if variant == "separate" else k - 1)
        traffic = STEP_TRAFFIC_BYTES if workload == "C2" else None
        plain = roofline("local_step_kernel<momentum, noise, plain>", per_step * W * d, plain_s, n_plain, traffic)
        if k <= 2:
            plain["shares_hbm_with"] = "wmean_kernel on the averaging stream (every timed launch is a round's first step)"
    if tail_s:
        tail_traffic = TAIL_TRAFFIC_BYTES[min(k, 2)] if workload == "C2" else None
        tail = roofline("local_step_kernel<momentum, noise, line 6>", tail_step_bytes(W, d, k, per_step), tail_s, steps, tail_traffic)
    if tail:
        out["roofline"] = tail
        if plain:
            out["roofline_plain_step"] = plain
            if k == 2:
                both = per_step * W * d + 4 * (1 + 1 / W) * W * d
                out["roofline_first_step_and_mean"] = roofline("local_step_kernel<plain> + wmean_kernel running beside it", both,
                                                               plain_s, steps, None)
    else:
        out["roofline"] = plain
    if full:
        prop = torch.cuda.get_device_properties(0)
        out["device"] = {"name": prop.name, "arch": getattr(prop, "gcnArchName", ""), "compute_units": prop.multi_processor_count,
                         "hbm_GiB": prop.total_memory / 2**30, "hip": torch.version.hip}
        out["overlap"] = overlap_figures(ctx, torch, P, wl.s_avg, k, steps, plain_s if variant == "fused_tail" and k == 2 else None)
        sweep_rounds = min(steps, 50)
        variants = {}
        for name in ("separate", "fused_tail", "graph_separate", "graph_fused_tail", "head_separate", "head_fused_tail",
                     "head_graph_fused_tail"):
            sweep = {}
            for kk in cfg["k"]:
                pr, ps, ts, hs = time_rounds(ctx, torch, kk, sweep_rounds, 2, name)
                sweep["k=%d" % kk] = {"ms_per_round": pr * 1e3, "updates_per_s": W * d * kk / pr,
                                      "model_GBps": model_round_bytes(W, d, kk, per_step) / pr / 1e9,
                                      "moved_GBps": moved_round_bytes(W, d, kk, name, per_step) / pr / 1e9,
                                      "plain_step_ms": ps * 1e3 if ps else None,
                                      "tail_step_ms": ts * 1e3 if ts else None,
                                      "head_step_ms": hs * 1e3 if hs else None}
            variants[name] = sweep
        out["k_sweep"] = variants
        sched = {}
        for name, code in (("serial", P.SCHED_SERIAL), ("serial_fused_mean_line6", P.SCHED_FUSED), ("overlap", P.SCHED_OVERLAP)):
            ctx.set_schedule(code)
            sched[name] = time_rounds(ctx, torch, k, sweep_rounds, 2, "separate", False)[0] * 1e3
        out["separate_schedule_ms_per_round"] = sched
        # line 6 inside the last step, with the mean (a) beside the first k-1 steps on its own stream,
        # (b) on the compute stream right before the last step, (c) inside the first step
        sched = {}
        for name, code in (("overlap", P.SCHED_OVERLAP), ("serial", P.SCHED_SERIAL), ("head", P.SCHED_HEAD)):
            ctx.set_schedule(code)
            sched[name] = time_rounds(ctx, torch, k, sweep_rounds, 2, "fused_tail", False)[0] * 1e3
        ctx.set_schedule(P.SCHED_OVERLAP)
        out["fused_tail_schedule_ms_per_round"] = sched
        out["timelines_ms_per_local_step"] = timelines(ctx, torch, P, k, sweep_rounds)
        out["diagnostics"] = diagnostics_figures(ctx, torch, wl.s_compute, W, d, True)
        out["external_gradient"] = external_gradient_rounds(ctx, torch, W, d, wl.stride, k, sweep_rounds, wl.h, wl.c)
    wl.close()
    return out


def bench_mlp(k, variant, steps, warmup, full):
    """C4: W=16 perceptron workers 3072-1024-10, batch 128: rounds/s, and the MFMA roofline of a
    local step (the two big contractions are 2 * 2*B*in*hid flops per worker-step)."""
    import torch
    import paper_1906_12043_amd as P
    import synth_inputs
    cfg = synth_inputs.CONFIGS["C4_mlp"]
    W, shape, batch = cfg["W"], cfg["mlp"], cfg["batch"]
    d = synth_inputs.mlp_param_count(*shape)
    dev = torch.device("cuda:0")
    stride, _, _ = P.plan_layout(d)
    xA = torch.zeros((W, stride), device=dev)
    xA[:, :d] = torch.from_numpy(synth_inputs.mlp_he_init(cfg["seed"], *shape)).to(dev)
    xB, v = torch.zeros((W, stride), device=dev), torch.zeros((W, stride), device=dev)
    mean = torch.zeros(stride, device=dev)
    s_compute, s_avg = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)
    torch.cuda.synchronize()
    ctx = P.Context(W=W, d=d, stride=stride, xA=xA, xB=xB, v=v, mean=mean, grad=P.GRAD_MLP, mlp=(*shape, batch),
                    lr=cfg["lr"], momentum=cfg["momentum"], weight_decay=cfg["weight_decay"], seed=cfg["seed"],
                    compute_stream=s_compute, avg_stream=s_avg)
    fused = variant == "fused_tail"
    per_round, plain_s, tail_s, _ = time_rounds(ctx, torch, k, steps, warmup, variant)
    # average local step over the round: k-1 plain steps and one that also applies line 6, or k plain ones
    step_s = ((plain_s or 0.0) * (k - 1) + tail_s) / k if fused else plain_s
    n_in, n_hid, n_out = shape
    gemm_flops = W * 2 * (2 * batch * n_in * n_hid)
    all_flops = gemm_flops + W * 3 * (2 * batch * n_hid * n_out)
    achieved = gemm_flops / step_s / 1e12
    # HBM bytes a local step must move: the parameters and their momentum in and out (the update of every
    # parameter), the mini-batch written once and read by both contractions' first touch, H and dA once each way
    step_hbm_bytes = W * (16 * d + 4 * batch * (2 * n_in + 4 * n_hid))
    out = {
        "metric": "worker-param-updates/s per CoCoD round, MLP-gradient workers (W=16, d=3.16M)",
        "value": W * d * k / per_round, "unit": "worker-param-updates/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": per_round * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "C4 MLP workers 3072-1024-10, batch 128 fresh N(0,1) inputs per worker-step, momentum 0.9, "
                               "lr 0.05", "k": k, "W": W, "d": d, "variant": variant, "schedule": "overlap (2 streams)"},
        "local_step_ms": step_s * 1e3,
        "plain_step_ms": plain_s * 1e3 if plain_s else None,
        "line6_step_ms": tail_s * 1e3 if tail_s else None,
        "local_step_TFLOPs_all": all_flops / step_s / 1e12,
        "local_step_hbm_GBps": step_hbm_bytes / step_s / 1e9,
        "roofline": {"bound": "mfma", "kernel": "one local step (4 launches; mlp_gemm_kernel<fwd>, <bwd> carry the flops)",
                     "achieved": achieved, "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_F32_PEAK_TFLOPS, "traffic": None, "avg_launch_ms": step_s * 1e3,
                     "launches_timed": steps * k, "algorithmic_flops_per_launch": gemm_flops},
    }
    if full:
        other = "separate" if fused else "fused_tail"
        out[other + "_ms_per_round"] = time_rounds(ctx, torch, k, steps, warmup, other, False)[0] * 1e3
        out["graph_ms_per_round"] = time_rounds(ctx, torch, k, steps, warmup, "graph_" + variant)[0] * 1e3
    ctx.close()
    del xA, xB, v, mean
    torch.cuda.empty_cache()
    return out


def compact(line):
    """The part of a workload's line that rides along in the default run."""
    keep = ("metric", "value", "unit", "ms_per_step", "steps", "warmup", "dtype", "config", "roofline", "roofline_plain_step",
            "round_moved_GBps", "round_moved_frac_of_hbm_peak", "local_step_ms", "local_step_hbm_GBps")
    return {key: line[key] for key in keep if key in line}


def kernels_alone(reps=5):
    """Launch each kernel of the round a few times, alone, at the benchmark shape (C2: W=16, d=11.2M), plus a
    plain copy of known size -- the program to put under rocprofv3 for per-dispatch hardware counters:

        rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT -- python3 bench.py --kernels-alone
        rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT -- python3 bench.py --kernels-alone

    The copy moves exactly 4*W*stride bytes in and 4*W*stride bytes out per launch; the ratio of its counter
    reading to that figure is the scale factor applied to the other kernels' readings."""
    import paper_1906_12043_amd as P
    wl = QuadraticWorkload("C2")
    ctx = wl.ctx
    ctx.set_schedule(P.SCHED_SERIAL)            # one stream: every kernel runs by itself
    for _ in range(reps):                       # copy: 4*W*stride bytes each way
        P.debug_copy(wl.s_compute, wl.h, wl.xB, wl.W * wl.stride)
    ctx.sync()
    wl.fill()
    ctx.local_steps(reps)                       # plain step, in place
    ctx.sync()
    for _ in range(reps):                       # mean, plain step (out of place), line 6 back to back
        ctx.round(1)
    ctx.sync()
    for _ in range(reps):                       # mean + line 6 in one kernel
        ctx.local_steps(1)
        ctx.average_apply_fused()
    ctx.sync()
    for _ in range(reps):                       # line 6 inside the last step: mean, plain step, step with line 6
        ctx.round_fused_tail(2)
    ctx.sync()
    for _ in range(reps):                       # k = 1: the step with line 6 reads the stored models as its input
        ctx.round_fused_tail(1)
    ctx.sync()
    ctx.set_schedule(P.SCHED_HEAD)              # the mean formed inside the round's first step
    for _ in range(reps):
        ctx.round_fused_tail(2)
    ctx.sync()
    for _ in range(reps):                       # k = 1: mean, step and line 6 in one kernel
        ctx.round_fused_tail(1)
    ctx.sync()
    print("kernels alone: done, W=%d d=%d stride=%d reps=%d" % (wl.W, wl.d, wl.stride, reps))
    wl.close()
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", choices=("C1", "C2", "C3", "C4", "C5"), default=None,
                    help="measure one configuration alone.  Default: the headline workload C2 (ResNet18-sized, W=16) in "
                         "full, with compact measurements of C3 (VGG16-sized), C5 (bucketed tensor list, W=64) and C4 "
                         "(MLP-gradient workers) under \"workloads\"")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200, help="timed rounds")
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--k", type=int, default=2, help="local steps per round for the headline value")
    ap.add_argument("--variant", choices=("separate", "fused_tail"), default="fused_tail")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true", help="skip the k sweep, the schedules and the other workloads")
    ap.add_argument("--kernels-alone", action="store_true", help="launch every kernel of the C2 round by itself (for counter runs)")
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
    if args.kernels_alone:
        return kernels_alone()
    full = not args.headline_only
    if args.workload == "C4":
        print(json.dumps(bench_mlp(args.k, args.variant, args.steps, args.warmup, full)))
        return 0
    if args.workload is not None:
        out = bench_quadratic(args.workload, args.k, args.variant, args.steps, args.warmup, full)
        if not args.no_cpu_baseline and args.workload == "C2":
            out["cpu_baseline"] = cpu_baseline(synth_inputs.CONFIGS[NAMES["C2"]], args.k)
        print(json.dumps(out))
        return 0

    out = bench_quadratic("C2", args.k, args.variant, args.steps, args.warmup, full)
    if full:                                    # the other configurations, a few timed rounds each
        others = {}
        others["C3"] = compact(bench_quadratic("C3", 2, args.variant, 10, 3, False))
        others["C5"] = compact(bench_quadratic("C5", 2, args.variant, 20, 3, False))
        others["C4"] = compact(bench_mlp(2, args.variant, 30, 5, False))
        out["workloads"] = others
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(synth_inputs.CONFIGS[NAMES["C2"]], args.k)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
