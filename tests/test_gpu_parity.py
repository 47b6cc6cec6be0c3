"""GPU parity: the HIP library behind the C-ABI against the CPU oracle, element by element, on the
same seeded inputs.  Bar (fp32 device arithmetic against the fp64 oracle): max |dx| <= 1e-5 (1 + |x|)."""
import numpy as np
import pytest
import torch

import paper_1906_12043_amd as P
import synth_inputs
from oracle import cocod_oracle as orc
from tests.gpu_harness import GpuWorkers, rel_err

pytestmark = pytest.mark.gpu
TOL = 1e-5


def hyper_of(cfg):
    return dict(lr=cfg["lr"], momentum=cfg["momentum"], weight_decay=cfg["weight_decay"],
                noise_sigma=cfg["noise_sigma"], seed=cfg["seed"])


def check_state(gpu, o, cols=None, tol=TOL, what=""):
    ex = rel_err(gpu.x(cols), o.x)
    assert ex <= tol, "%s x: %.3g" % (what, ex)
    if o.v is not None:
        ev = rel_err(gpu.vel(cols), o.v)
        assert ev <= 10 * tol, "%s v: %.3g" % (what, ev)      # v is ~1/lr times more sensitive than x
    return ex


# ---- the generator ---------------------------------------------------------------------------

@pytest.mark.parametrize("fast,bound", [(1, 2e-5), (0, 2e-6)])
def test_device_normals_match_oracle(fast, bound):
    seed, n, j0 = 0xABCDEF0123456789, 1 << 18, 12345
    out = torch.empty(n, device="cuda:0")
    P.debug_normals(None, seed, orc.TAG_NOISE, 3, 17, j0, n, fast, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    want = orc.normals(seed, orc.TAG_NOISE, 3, 17, j0, n)
    err = np.max(np.abs(got - want))
    print("max |z_gpu - z_oracle| fast=%d: %.3g" % (fast, err))
    assert err < bound


def test_device_fill_matches_oracle():
    W, d = 3, 10007
    g = GpuWorkers(W, d, device_fill=True, lr=0.1, seed=0x1234567887654321)
    h, c = g.data()
    ho, co = orc.fill_quadratic(0x1234567887654321, W, d)
    assert np.array_equal(h, ho)
    assert np.max(np.abs(c.astype(np.float64) - co)) < 2e-6
    assert float(g.h[:, d:g.padded].abs().max()) == 0.0      # alignment pads are zeroed
    g.close()


# ---- full-vector parity ------------------------------------------------------------------------

def test_tiny_config_every_round():
    cfg = synth_inputs.CONFIGS["C1_tiny"]
    W, d, k = cfg["W"], cfg["d"], cfg["k"][0]
    h, c = synth_inputs.quadratic_data(cfg["seed"], W, d)
    g = GpuWorkers(W, d, h=h, c=c, **hyper_of(cfg))
    o = orc.QuadraticOracle(h, c, **hyper_of(cfg))
    worst = 0.0
    for r in range(cfg["rounds"]):
        g.ctx.round(k); o.round(k)
        worst = max(worst, check_state(g, o, what="round %d" % r))
        assert rel_err(g.avg(), o.mean) <= TOL
    assert g.ctx.get_step() == o.step == cfg["rounds"] * k
    print("C1 worst rel err %.3g" % worst)
    g.close()


@pytest.mark.parametrize("W,d,mu,wd,sigma,k", [
    (1, 1, 0.0, 0.0, 0.01, 2), (1, 5, 0.9, 5e-4, 0.01, 3), (3, 3, 0.9, 0.0, 0.0, 1), (2, 4, 0.5, 0.01, 0.1, 4),
    (4, 4097, 0.9, 5e-4, 0.01, 2), (16, 10007, 0.9, 5e-4, 0.01, 2), (5, 12289, 0.0, 0.0, 0.01, 3),
    (64, 4100, 0.9, 5e-4, 0.01, 1), (7, 8192, 0.9, 0.0, 0.0, 8),
    (65535, 3, 0.9, 5e-4, 0.01, 2), (1000, 5, 0.9, 5e-4, 0.01, 2), (3, 1023, 0.9, 5e-4, 0.01, 2), (3, 1025, 0.0, 5e-4, 0.01, 2), (17, 2047, 0.9, 0.0, 0.01, 3),
])
def test_small_shapes_ragged_tails(W, d, mu, wd, sigma, k):
    hyper = dict(lr=0.05, momentum=mu, weight_decay=wd, noise_sigma=sigma, seed=1000 + d)
    h, c = synth_inputs.quadratic_data(d, W, d)
    x0 = np.random.default_rng(d).standard_normal(d).astype(np.float32)
    g = GpuWorkers(W, d, h=h, c=c, x0=x0, extra_stride=8, **hyper)
    o = orc.QuadraticOracle(h, c, x0, **hyper)
    for r in range(4):
        g.ctx.round(k); o.round(k)
        check_state(g, o, what="round %d" % r)
    g.close()


def test_steps_outside_a_round_and_zero_step_round():
    W, d = 4, 5000
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=5)
    h, c = synth_inputs.quadratic_data(9, W, d)
    g = GpuWorkers(W, d, h=h, c=c, **hyper)
    o = orc.QuadraticOracle(h, c, **hyper)
    g.ctx.local_steps(3); o.local_steps(3)                 # plain local SGD
    check_state(g, o, what="local only")
    g.ctx.average_begin(); g.ctx.average_end_apply()       # pure averaging: every worker lands on the mean
    o.average_begin(); o.average_end_apply()
    check_state(g, o, what="zero-step round")
    x = g.x()
    assert np.array_equal(x[0], x[1]) and np.array_equal(x[0], x[3])
    g.ctx.average_begin(); g.ctx.local_steps(1); g.ctx.local_steps(2); g.ctx.average_end_apply()
    o.average_begin(); o.local_steps(3); o.average_end_apply()
    check_state(g, o, what="split calls")
    g.close()


@pytest.mark.parametrize("graph", [False, True])
def test_step_counter_at_the_top_of_its_range(graph):
    """t is a 32-bit word of the generator's counter: the last representable steps must key the noise
    as the oracle does, also when a graph replay reads t from its device word."""
    W, d, k = 3, 4100, 3
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=0xFFFFFFFF12345678)
    h, c = synth_inputs.quadratic_data(41, W, d)
    g = GpuWorkers(W, d, h=h, c=c, **hyper)
    o = orc.QuadraticOracle(h, c, **hyper)
    for start in (2**31 - 2, 2**32 - 1 - 2 * k):
        g.ctx.set_step(start); o.step = start
        for _ in range(2):
            if graph:
                g.ctx.graph_round(k, True)
            else:
                g.ctx.round(k)
            o.round(k)
            check_state(g, o, what="t = %d" % o.step)
        assert g.ctx.get_step() == o.step
    with pytest.raises(P.CocodError):
        g.ctx.local_steps(1)                      # the counter itself must stay below 2^32
    g.close()


def test_single_worker_first_round_is_exactly_plain_sgd():
    """N = 1 from x0 = 0: snapshot and mean are 0, so line 6 returns the local model bit for bit."""
    d = 9000
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=3)
    h, c = synth_inputs.quadratic_data(4, 1, d)
    a = GpuWorkers(1, d, h=h, c=c, **hyper)
    b = GpuWorkers(1, d, h=h, c=c, **hyper)
    a.ctx.round(3)
    b.ctx.local_steps(3)
    assert torch.equal(a.x_raw()[:, :d], b.x_raw()[:, :d])
    a.close(); b.close()


@pytest.mark.parametrize("W", [4, 16, 64])
def test_identical_workers_without_noise_follow_one_worker_bit_for_bit(W):
    """Same h, c on every worker and no noise: the mean of W equal values is exact for a power of two,
    so every worker retraces the single-worker rounds bit for bit."""
    d, k = 5001, 2
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.0, seed=1)
    h1, c1 = synth_inputs.quadratic_data(33, 1, d)
    one = GpuWorkers(1, d, h=h1, c=c1, **hyper)
    many = GpuWorkers(W, d, h=np.repeat(h1, W, 0), c=np.repeat(c1, W, 0), **hyper)
    o = orc.QuadraticOracle(h1, c1, **hyper)
    for r in range(4):
        for g in (one, many):
            g.ctx.round(k) if r % 2 else g.ctx.round_fused_tail(k)
        o.round(k)
    x1, xm = one.x_raw()[:, :d], many.x_raw()[:, :d]
    assert all(torch.equal(xm[i], x1[0]) for i in range(W))
    check_state(one, o, what="single worker")
    one.close(); many.close()


@pytest.mark.parametrize("weights", [None, [0.4, 0.3, 0.2, 0.1]])
def test_line6_invariants_on_device_data(weights):
    """The two representations in the proof of Lemma 2, checked on what the device itself holds (no
    oracle): after line 6 the weighted mean of the models is the old mean plus the weighted mean of the
    local progress, and each worker's deviation from it is its own progress minus the mean progress."""
    W, d, k = 4, 20_003, 3
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=19, weights=weights)
    h, c = synth_inputs.quadratic_data(23, W, d)
    g = GpuWorkers(W, d, h=h, c=c, **hyper)
    p = np.full(W, 1.0 / W) if weights is None else np.asarray(weights, dtype=np.float64)
    g.ctx.round(k); g.ctx.round(k)                              # a state where the workers differ
    snap = g.x()
    g.ctx.average_begin(); g.ctx.local_steps(k)
    pre = g.x()
    g.ctx.average_end_apply()
    post, mean = g.x(), g.avg()
    delta = pre - snap
    tol = 4e-7 * (1 + np.abs(post).max())
    assert np.max(np.abs(mean - p @ snap)) <= tol
    assert np.max(np.abs(p @ post - (mean + p @ delta))) <= tol
    assert np.max(np.abs((post - p @ post) - (delta - p @ delta))) <= tol
    g.close()


def test_weighted_mean():
    W, d, k = 4, 6001, 2
    p = [0.125, 0.25, 0.25, 0.375]
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=0.0, noise_sigma=0.01, seed=8)
    h, c = synth_inputs.quadratic_data(2, W, d)
    g = GpuWorkers(W, d, h=h, c=c, weights=p, **hyper)
    o = orc.QuadraticOracle(h, c, weights=p, **hyper)
    for r in range(3):
        g.ctx.round(k); o.round(k)
        check_state(g, o, what="round %d" % r)
    g.close()


def test_heterogeneous_workers_weighted_mean_and_per_worker_noise():
    """Workers with mini-batch sizes M_i: mean weights M_i / sum M and noise sigma / sqrt(M_i)."""
    W, k = 5, 3
    sizes = [1030, 7, 4099, 2]
    d = sum(sizes)
    M = np.array([32, 64, 64, 128, 256], dtype=np.float64)
    p = (M / M.sum()).tolist()
    sigma_w = (0.08 / np.sqrt(M)).astype(np.float32).tolist()
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=123.0, seed=31)   # noise_sigma is overridden
    h, c = synth_inputs.quadratic_data(3, W, d)
    g = GpuWorkers(W, d, h=h, c=c, tensor_numel=sizes, weights=p, noise_sigma_w=sigma_w, **hyper)
    o = orc.QuadraticOracle(h, c, weights=p, noise_sigma_w=sigma_w, **hyper)
    for r in range(4):
        if r % 2:
            g.ctx.round_fused_tail(k)
        else:
            g.ctx.round(k)
        o.round(k)
        check_state(g, o, what="round %d" % r)
    assert abs(g.ctx.consensus_distance() - o.consensus_distance()) <= 1e-5 * o.consensus_distance()
    g.close()


# ---- schedules and layouts give the same bits ----------------------------------------------------

def run_bits(W, d, rounds, k, schedule, two_streams, tensor_numel=None, bucket_bytes=0):
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=77)
    h, c = synth_inputs.quadratic_data(6, W, d)
    g = GpuWorkers(W, d, h=h, c=c, two_streams=two_streams, tensor_numel=tensor_numel,
                   bucket_bytes=bucket_bytes, **hyper)
    g.ctx.set_schedule(schedule)
    for _ in range(rounds):
        g.ctx.round(k)
    g.ctx.sync()
    out = (g.live()[:, :d] if g.pos is None else g.live()[:, g.pos]).clone()
    vel = (g.v[:, :d] if g.pos is None else g.v[:, g.pos]).clone()
    g.close()
    return out, vel


def test_overlapped_round_is_bit_identical_to_serialised_rounds():
    W, d, rounds, k = 8, 300_001, 6, 2
    ref = run_bits(W, d, rounds, k, P.SCHED_OVERLAP, two_streams=False)
    for schedule, two in [(P.SCHED_OVERLAP, True), (P.SCHED_SERIAL, True), (P.SCHED_FUSED, True), (P.SCHED_FUSED, False),
                          (P.SCHED_HEAD, True), (P.SCHED_HEAD, False), (P.SCHED_OVERLAP, "null"), (P.SCHED_FUSED, "null")]:
        got = run_bits(W, d, rounds, k, schedule, two_streams=two)
        assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1]), (schedule, two)


@pytest.mark.parametrize("weights,mu,sigma", [(None, 0.9, 0.01), ([0.1, 0.2, 0.3, 0.15, 0.25], 0.9, 0.01), (None, 0.0, 0.01),
                                              ([0.1, 0.2, 0.3, 0.15, 0.25], 0.0, 0.0), (None, 0.9, 0.0)])
def test_mean_formed_inside_the_first_step_gives_the_same_bits(weights, mu, sigma):
    """COCOD_SCHED_HEAD against the two-stream schedule: packed list with every start alignment, k = 0
    (no step to ride on), 1 (first step is the last), 2, 3, both ways of applying line 6, mean included."""
    W = 5
    sizes = [5, 4096, 1, 3, 8191, 64, 4097, 2, 3000, 7]
    d = sum(sizes)
    hyper = dict(lr=0.05, momentum=mu, weight_decay=5e-4, noise_sigma=sigma, seed=78, weights=weights)
    h, c = synth_inputs.quadratic_data(16, W, d)
    a = GpuWorkers(W, d, h=h, c=c, tensor_numel=sizes, **hyper)
    b = GpuWorkers(W, d, h=h, c=c, tensor_numel=sizes, **hyper)
    b.ctx.set_schedule(P.SCHED_HEAD)
    o = orc.QuadraticOracle(h, c, **hyper)
    for k in (2, 3, 1, 0, 2, 1):
        for fused_tail in (False, True):
            for w in (a, b):
                if fused_tail:
                    w.ctx.round_fused_tail(k)
                else:
                    w.ctx.round(k)
                w.ctx.sync()
            o.round(k)
            for name in ("live", "v", "mean") if mu else ("live", "mean"):
                ta, tb = (getattr(w, name)() if name == "live" else getattr(w, name) for w in (a, b))
                assert torch.equal(ta[..., a.pos], tb[..., b.pos]), (k, fused_tail, name)
    check_state(b, o, what="head schedule")
    a.close(); b.close()


@pytest.mark.parametrize("W,d", [(16, 20_011), (17, 9_001), (40, 6_003), (65, 3_001), (70, 2_500), (131, 1_100), (140, 1_030), (1, 5_000)])
def test_head_schedule_for_every_worker_count_class(W, d):
    """The mean-forming first step keeps the tile of all W workers in LDS: one column quad per lane up
    to 16 workers, two up to 65, one again up to 131 (the LDS budget), and beyond that the mean is
    formed by a pass of its own.  Every class, k = 1 (mean, step and line 6 in one pass) and k = 2,
    against the two-stream schedule bit for bit, mean included, and against the oracle."""
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=79)
    h, c = synth_inputs.quadratic_data(17, W, d)
    a = GpuWorkers(W, d, h=h, c=c, **hyper)
    b = GpuWorkers(W, d, h=h, c=c, **hyper)
    b.ctx.set_schedule(P.SCHED_HEAD)
    o = orc.QuadraticOracle(h, c, **hyper)
    for k, fused_tail in ((1, True), (2, True), (1, False), (2, False), (1, True)):
        for w in (a, b):
            w.ctx.round_fused_tail(k) if fused_tail else w.ctx.round(k)
        o.round(k)
        assert np.array_equal(a.x(), b.x()) and np.array_equal(a.vel(), b.vel()) and np.array_equal(a.avg(), b.avg()), (k, fused_tail)
    check_state(b, o, what="head schedule W=%d" % W)
    a.close(); b.close()


def test_packed_tensor_list_is_bit_identical_to_flat_and_matches_oracle():
    W, rounds, k = 4, 3, 2
    sizes = [5, 4096, 1, 3, 8191, 64, 4097, 2, 10000, 7]      # every start alignment, tails of 1..3
    d = sum(sizes)
    flat = run_bits(W, d, rounds, k, P.SCHED_OVERLAP, True)
    packed = run_bits(W, d, rounds, k, P.SCHED_OVERLAP, True, tensor_numel=sizes, bucket_bytes=40000)
    assert torch.equal(flat[0], packed[0]) and torch.equal(flat[1], packed[1])
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=77)
    h, c = synth_inputs.quadratic_data(6, W, d)
    o = orc.QuadraticOracle(h, c, **hyper)
    for _ in range(rounds):
        o.round(k)
    assert rel_err(packed[0].cpu().numpy().astype(np.float64), o.x) <= TOL


def test_checkpoint_resume_is_bit_identical():
    """State = models, momentum, step counter: restoring them continues the same trajectory."""
    W, d, k = 4, 20_000, 2
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=21)
    h, c = synth_inputs.quadratic_data(3, W, d)
    a = GpuWorkers(W, d, h=h, c=c, **hyper)
    for _ in range(4):
        a.ctx.round(k)
    want = a.x_raw()[:, :d].clone()
    b = GpuWorkers(W, d, h=h, c=c, **hyper)
    b.ctx.round(k); b.ctx.round(k)
    x_mid, v_mid, step_mid = b.x_raw()[:, :d].cpu().numpy(), b.v[:, :d].cpu().numpy(), b.ctx.get_step()
    b.close()
    r = GpuWorkers(W, d, h=h, c=c, x0=x_mid, **hyper)
    r.v[:, :d] = torch.from_numpy(v_mid).to(r.dev)
    torch.cuda.synchronize()
    r.ctx.set_step(step_mid)
    r.ctx.round(k); r.ctx.round(k)
    assert torch.equal(r.x_raw()[:, :d], want)
    a.close(); r.close()


@pytest.mark.parametrize("k", [1, 2, 3])
@pytest.mark.parametrize("packed", [False, True])
def test_line6_inside_last_step_is_bit_identical_to_separate_kernels(k, packed):
    W, rounds = 5, 4
    sizes = [5, 4096, 1, 3, 8191, 64, 4097, 2, 10000, 7] if packed else None
    d = sum(sizes) if packed else 50_003
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=31)
    h, c = synth_inputs.quadratic_data(12, W, d)
    a = GpuWorkers(W, d, h=h, c=c, tensor_numel=sizes, **hyper)
    b = GpuWorkers(W, d, h=h, c=c, tensor_numel=sizes, **hyper)
    o = orc.QuadraticOracle(h, c, **hyper)
    for r in range(rounds):
        a.ctx.round(k)
        b.ctx.round_fused_tail(k)
        o.round(k)
        assert not b.ctx.is_averaging() and b.ctx.get_step() == a.ctx.get_step()
    assert np.array_equal(a.x(), b.x()) and np.array_equal(a.vel(), b.vel())
    check_state(b, o, what="fused tail k=%d" % k)
    for sched in (P.SCHED_SERIAL, P.SCHED_FUSED):           # mean taken on the compute stream just before the last step
        b.ctx.set_schedule(sched)
        a.ctx.round(k); b.ctx.round_fused_tail(k)
        assert np.array_equal(a.x(), b.x())
    b.ctx.average_begin(); b.ctx.local_steps_end_apply(0)    # k = 0: plain line 6
    a.ctx.average_begin(); a.ctx.average_end_apply()
    assert np.array_equal(a.x(), b.x())
    a.close(); b.close()


@pytest.mark.parametrize("packed,weights", [(False, None), (True, None), (False, [0.1, 0.2, 0.3, 0.15, 0.25])])
def test_consensus_distance_and_local_sgd_schedule(packed, weights):
    """The diagnostic of Lemma 2's quantity, and Local-SGD built from the same calls: k local steps,
    then a round with zero local steps (every worker lands on the mean of the CURRENT models)."""
    W, k = 5, 3
    sizes = [7, 1024, 2050, 3, 1021] if packed else None
    d = sum(sizes) if packed else 30_011
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=23, weights=weights)
    h, c = synth_inputs.quadratic_data(14, W, d)
    g = GpuWorkers(W, d, h=h, c=c, tensor_numel=sizes, **hyper)
    o = orc.QuadraticOracle(h, c, **hyper)
    assert g.ctx.consensus_distance() == 0.0
    f0, g0 = g.ctx.quadratic_objective()                                 # at x = 0
    want_f0, want_g0 = o.objective_at_mean()
    assert abs(f0 - want_f0) <= 1e-5 * want_f0 and abs(g0 - want_g0) <= 1e-5 * want_g0
    for r in range(3):
        g.ctx.round(k); o.round(k)
        got, want = g.ctx.consensus_distance(), o.consensus_distance()
        assert want > 0 and abs(got - want) <= 1e-5 * want, (got, want)
        assert g.ctx.consensus_distance() == got                         # deterministic reduction
        (f, g2), (want_f, want_g2) = g.ctx.quadratic_objective(), o.objective_at_mean()
        assert abs(f - want_f) <= 1e-5 * want_f and abs(g2 - want_g2) <= 1e-5 * want_g2, (f, want_f, g2, want_g2)
        assert g.ctx.quadratic_objective() == (f, g2) and g.ctx.consensus_distance() == got
        assert f < f0 and g2 < g0                                        # the workers are descending
    for schedule in (P.SCHED_OVERLAP, P.SCHED_FUSED):                    # Local-SGD rounds
        g.ctx.set_schedule(schedule)
        g.ctx.local_steps(k); g.ctx.average_begin(); g.ctx.average_end_apply()
        o.local_steps(k); o.average_begin(); o.average_end_apply()
        check_state(g, o, what="local-sgd")
        assert g.ctx.consensus_distance() <= 1e-9                        # fp32 mean of equal rows: last-bit noise only
        x = g.x()
        assert all(np.array_equal(x[0], x[i]) for i in range(1, W))
    g.close()


@pytest.mark.parametrize("packed,mu", [(False, 0.9), (True, 0.9), (False, 0.0)])
def test_external_gradient_steps(packed, mu):
    """The caller supplies G: here the oracle's own logged gradients (oracle -> device), so the device
    must reproduce the oracle's trajectory through cocod_external_step."""
    W, k, rounds = 3, 3, 3
    sizes = [7, 1024, 2050, 3, 1021] if packed else None
    d = sum(sizes) if packed else 5003
    hyper = dict(lr=0.05, momentum=mu, weight_decay=5e-4, seed=17)
    h, c = synth_inputs.quadratic_data(13, W, d)
    o = orc.QuadraticOracle(h, c, noise_sigma=0.01, **hyper)
    g = GpuWorkers(W, d, tensor_numel=sizes, grad=P.GRAD_EXTERNAL, **hyper)
    with pytest.raises(P.CocodError) as e:
        g.ctx.local_steps(1)                                  # no built-in gradient in this context
    assert e.value.status == P.ERR_INVALID
    with pytest.raises(P.CocodError) as e:
        g.ctx.external_step(g.h, close_round=True)            # no round open
    assert e.value.status == P.ERR_STATE
    for r in range(rounds):
        g.ctx.average_begin(); o.average_begin()
        for s in range(k):
            G = o.local_steps(1, log_gradients=True)[0]
            g.ctx.sync()                                      # the previous step has consumed the buffer
            gbuf = g._upload(G.astype(np.float32))
            torch.cuda.synchronize()
            last = s == k - 1 and r % 2 == 0                  # alternate: line 6 inside the step / separate
            g.ctx.external_step(gbuf, close_round=last)
        if r % 2 == 1:
            g.ctx.average_end_apply()
        o.average_end_apply()
        assert not g.ctx.is_averaging()
        check_state(g, o, what="external round %d" % r)
    assert g.ctx.get_step() == o.step
    g.close()


@pytest.mark.parametrize("packed,mu", [(False, 0.9), (True, 0.9), (True, 0.0)])
def test_external_bf16_gradient_steps(packed, mu):
    """16-bit gradients: a noisy quadratic gradient rounded to brain floats on the host goes to the
    oracle (widened exactly to fp64) and to the device (16-bit buffer); both apply the same update."""
    W, k, rounds = 4, 3, 3
    sizes = [5, 1024, 2051, 2, 1023, 4100] if packed else None
    d = sum(sizes) if packed else 6007
    hyper = dict(lr=0.05, momentum=mu, weight_decay=5e-4, seed=23)
    h, c = synth_inputs.quadratic_data(29, W, d)
    src = orc.QuadraticOracle(h, c, noise_sigma=0.01, **hyper)           # only supplies gradients
    o = orc.QuadraticOracle(h, c, noise_sigma=0.0, **hyper)
    g = GpuWorkers(W, d, tensor_numel=sizes, grad=P.GRAD_EXTERNAL, **hyper)
    for r in range(rounds):
        g.ctx.average_begin(); o.average_begin()
        for s in range(k):
            src.x[...] = o.x                                             # gradient at the tracked model
            G = src.local_steps(1, log_gradients=True)[0]
            G16 = torch.from_numpy(G.astype(np.float32)).to(torch.bfloat16)
            assert not torch.equal(G16.float(), torch.from_numpy(G.astype(np.float32)))   # rounding really happens
            g.ctx.sync()
            gbuf = g._upload(G16.float().numpy()).to(torch.bfloat16)     # exact: values are 16-bit already
            assert gbuf.is_contiguous() and gbuf.shape == (W, g.stride)
            torch.cuda.synchronize()
            last = s == k - 1 and r != 1
            g.ctx.external_step_bf16(gbuf, close_round=last)
            o.external_step(G16.double().numpy())
        if r == 1:
            g.ctx.average_end_apply()
        o.average_end_apply()
        check_state(g, o, what="bf16 external round %d" % r)
    assert g.ctx.get_step() == o.step
    g.close()


@pytest.mark.parametrize("packed,weights", [(False, None), (True, None), (False, [0.1, 0.2, 0.3, 0.15, 0.25])])
def test_average_apply_fused_matches_every_schedule_bit_for_bit(packed, weights):
    """cocod_average_apply_fused (mean + line 6 in one pass, whatever schedule is set) against
    cocod_average_end_apply under the fused schedule and under the overlapped one, and, while idle,
    against a zero-step round (the blocking average of Local SGD); then against the oracle."""
    W, k = 5, 2
    sizes = [5, 4096, 1, 3, 8191, 64, 4097, 2] if packed else None
    d = sum(sizes) if packed else 40_007
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=41, weights=weights)
    h, c = synth_inputs.quadratic_data(15, W, d)
    a = GpuWorkers(W, d, h=h, c=c, tensor_numel=sizes, **hyper)          # reference calls
    b = GpuWorkers(W, d, h=h, c=c, tensor_numel=sizes, **hyper)          # the new call
    o = orc.QuadraticOracle(h, c, **hyper)
    for r, sched in enumerate((P.SCHED_FUSED, P.SCHED_OVERLAP, P.SCHED_SERIAL, P.SCHED_HEAD, P.SCHED_OVERLAP)):
        a.ctx.set_schedule(P.SCHED_FUSED if r % 2 == 0 else P.SCHED_OVERLAP)
        b.ctx.set_schedule(sched)
        a.ctx.round(k)
        b.ctx.average_begin(); b.ctx.local_steps(k); b.ctx.average_apply_fused()
        o.round(k)
        assert not b.ctx.is_averaging()
        assert np.array_equal(a.x(), b.x()) and np.array_equal(a.vel(), b.vel()) and np.array_equal(a.avg(), b.avg()), sched
    check_state(b, o, what="average_apply_fused")
    a.ctx.local_steps(k); a.ctx.average_begin(); a.ctx.average_end_apply()      # Local SGD: steps, then blocking average
    b.ctx.local_steps(k); b.ctx.average_apply_fused()
    o.local_steps(k); o.average_begin(); o.average_end_apply()
    assert np.array_equal(a.x(), b.x()) and np.array_equal(a.avg(), b.avg())
    check_state(b, o, what="blocking average")
    x = b.x()
    assert all(np.array_equal(x[0], x[i]) for i in range(1, W))
    a.close(); b.close()


def test_graph_round_on_the_null_stream_is_refused_before_any_gpu_call():
    W, d = 3, 5000
    h, c = synth_inputs.quadratic_data(16, W, d)
    g = GpuWorkers(W, d, h=h, c=c, two_streams="null", lr=0.05, momentum=0.9)
    with pytest.raises(P.CocodError) as e:
        g.ctx.graph_round(2)
    assert e.value.status == P.ERR_INVALID
    g.ctx.round(2)                                    # the context is still usable, and untouched by the refusal
    assert g.ctx.get_step() == 2
    g.close()
