"""Launch each kernel of the round a few times, alone, at the benchmark shape (W=16, d=11.2M), plus
a plain copy of known size -- the program to put under rocprofv3 for per-dispatch hardware counters:

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT -- python3 paper_1906_12043_amd/profile_kernels.py
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT -- python3 paper_1906_12043_amd/profile_kernels.py

The copy moves exactly 4*W*d bytes in and 4*W*d bytes out per launch; the ratio of its counter
reading to that figure is the scale factor applied to the other kernels' readings.
"""
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_1906_12043_amd as P  # noqa: E402
import synth_inputs  # noqa: E402


def main(reps=5):
    cfg = synth_inputs.CONFIGS["C2_resnet18"]
    W, d = cfg["W"], cfg["d"]
    dev = torch.device("cuda:0")
    stride, _, _ = P.plan_layout(d)
    bufs = {name: torch.zeros((W, stride), device=dev) for name in ("xA", "xB", "v", "h", "c")}
    mean = torch.zeros(stride, device=dev)
    stream = torch.cuda.Stream(device=dev)
    torch.cuda.synchronize()
    ctx = P.Context(W=W, d=d, stride=stride, mean=mean, lr=cfg["lr"], momentum=cfg["momentum"],
                    weight_decay=cfg["weight_decay"], noise_sigma=cfg["noise_sigma"], seed=cfg["seed"],
                    compute_stream=stream, avg_stream=stream, **bufs)
    ctx.fill_quadratic()
    ctx.sync()
    for _ in range(reps):                       # copy: 4*W*stride bytes each way
        P.debug_copy(stream, bufs["h"], bufs["xB"], W * stride)
    ctx.sync()
    ctx.local_steps(reps)                       # step kernel alone, in place
    ctx.sync()
    ctx.set_schedule(P.SCHED_SERIAL)            # one stream: step (out of place), mean, line 6 back to back
    for _ in range(reps):
        ctx.round(1)
    ctx.sync()
    ctx.set_schedule(P.SCHED_FUSED)
    for _ in range(reps):
        ctx.round(1)
    ctx.sync()
    ctx.set_schedule(P.SCHED_SERIAL)            # line 6 inside the last step: mean, plain step, step with line 6
    for _ in range(reps):
        ctx.round_fused_tail(2)
    ctx.sync()
    for _ in range(reps):                       # k = 1: the step with line 6 reads the stored models as its input
        ctx.round_fused_tail(1)
    ctx.sync()
    ctx.set_schedule(P.SCHED_HEAD)              # the mean formed inside the round's first step (column-wise step kernel)
    for _ in range(reps):
        ctx.round_fused_tail(2)
    ctx.sync()
    ctx.close()
    print("profile_kernels: done, W=%d d=%d stride=%d reps=%d" % (W, d, stride, reps))


if __name__ == "__main__":
    main()
