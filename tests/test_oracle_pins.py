"""Pins for the oracle's round of Algorithm 1 (CoCoD-SGD), CPU only.

The paper prints no worked example, so every pin is derived from its equations:
special cases of Algorithm 1, the two model representations used in the proof of
Lemma 2, a closed form for the noiseless quadratic, and a hand-computed case.
"""
import os

import numpy as np
import pytest

import synth_inputs
from oracle import cocod_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
HYPER = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=77)


def make(W, n, kind="f64", data_seed=3, **kw):
    h, c = synth_inputs.quadratic_data(data_seed, W, n)
    return orc.QuadraticOracle(h, c, kind=kind, **kw)


def plain_sgd(h, c, steps, *, lr, momentum=0.0, weight_decay=0.0, noise_sigma=0.0, seed=0, worker=0):
    """Textbook momentum SGD on one worker in numpy fp64 (not the oracle's step loop)."""
    lr, mu, wd, sg = (orc.f32(t) for t in (lr, momentum, weight_decay, noise_sigma))
    h = h.astype(np.float64)
    c = c.astype(np.float64)
    x = np.zeros_like(h)
    v = np.zeros_like(h)
    for s in range(steps):
        z = orc.normals(seed, orc.TAG_NOISE, worker, s, 0, h.size) if sg else 0.0
        g = h * (x - c) + sg * z + wd * x
        v = mu * v + g
        x = x - lr * v
    return x


# ---- hand-computed case (tests/golden/hand_case_W2_d1.txt) -------------------------------

def test_hand_case():
    h = np.array([[1.0], [2.0]], np.float32)
    c = np.array([[1.0], [-1.0]], np.float32)
    rows = []
    with open(os.path.join(GOLDEN, "hand_case_W2_d1.txt")) as fh:
        for line in fh:
            if not line.startswith("#") and line.strip():
                rows.append(line.split())
    assert len(rows) == 5
    for mu in (0.0, 0.5):
        # lr 0.1 is not an fp32 number; the hand arithmetic is in exact decimals
        o = orc.QuadraticOracle(h, c, lr=0.1, momentum=mu)
        o.lr = 0.1
        for row in [r for r in rows if float(r[0]) == mu]:
            o.round(2)
            assert o.step == 2 * int(row[1])
            assert np.allclose(o.x[:, 0], [float(row[2]), float(row[3])], rtol=0, atol=1e-14)
            if mu:
                assert np.allclose(o.v[:, 0], [float(row[4]), float(row[5])], rtol=0, atol=1e-13)


# ---- special cases of Algorithm 1 --------------------------------------------------------

def test_single_worker_is_plain_sgd():
    """N = 1: the mean is the stored model, so line 6 returns the local model."""
    n, R, k = 257, 6, 3
    o = make(1, n, **HYPER)
    for r in range(R):
        o.round(k)
        if r == 0:                       # x0 = 0: snapshot and mean are 0, line 6 is exact
            first = plain_sgd(o.h[0], o.c[0], k, **HYPER)
            assert np.array_equal(o.x[0], first)
    want = plain_sgd(o.h[0], o.c[0], R * k, **HYPER)
    assert np.max(np.abs(o.x[0] - want)) < 1e-14


def test_single_worker_with_nonzero_start_and_split_calls():
    n = 64
    h, c = synth_inputs.quadratic_data(5, 1, n)
    x0 = np.linspace(-1, 1, n)
    a = orc.QuadraticOracle(h, c, x0, **HYPER)
    b = orc.QuadraticOracle(h, c, x0, **HYPER)
    a.round(4)
    b.average_begin(); b.local_steps(1); b.local_steps(3); b.average_end_apply()
    assert np.array_equal(a.x, b.x) and np.array_equal(a.v, b.v) and a.step == b.step == 4


@pytest.mark.parametrize("W", [4, 16, 64])
def test_identical_workers_without_noise_follow_one_worker(W):
    n, R, k = 100, 5, 2
    h1, c1 = synth_inputs.quadratic_data(8, 1, n)
    hyper = dict(HYPER, noise_sigma=0.0)
    o = orc.QuadraticOracle(np.repeat(h1, W, 0), np.repeat(c1, W, 0), **hyper)
    for _ in range(R):
        o.round(k)
    for i in range(1, W):
        assert np.array_equal(o.x[i], o.x[0])
    want = plain_sgd(h1[0], c1[0], R * k, **hyper)
    assert np.max(np.abs(o.x[0] - want)) < 1e-14


def test_zero_local_steps_gives_pure_averaging():
    o = make(4, 33, **HYPER)
    o.local_steps(3)                      # make the workers disagree first
    mean_before = o.x.mean(axis=0)
    o.average_begin(); o.average_end_apply()
    for i in range(4):
        assert np.allclose(o.x[i], mean_before, rtol=0, atol=1e-15)


def test_first_round_correction_is_identity():
    """All workers start from the same point, so the first mean equals it (initialisation of Algorithm 1)."""
    W, n, k = 4, 50, 3
    o = make(W, n, **HYPER)
    ref = make(W, n, **HYPER)
    o.round(k)
    ref.local_steps(k)
    assert np.array_equal(o.x, ref.x)


# ---- representations from the proof of Lemma 2 -------------------------------------------

def test_correction_preserves_worker_mean_and_resets_deviation():
    """After line 6: mean_i x_i = mean + mean_i delta_i, and x_i - mean_i x_i = delta_i - mean delta."""
    W, n, k = 8, 40, 3
    o = make(W, n, **HYPER)
    o.round(2); o.round(2)                 # get a state where workers differ
    o.average_begin()
    snap, mean = o.snap.copy(), o.mean.copy()
    assert np.allclose(mean, snap.mean(axis=0), rtol=0, atol=1e-15)
    o.local_steps(k)
    pre = o.x.copy()
    o.average_end_apply()
    delta = pre - snap
    assert np.allclose(o.x.mean(axis=0), mean + delta.mean(axis=0), rtol=0, atol=1e-14)
    assert np.allclose(o.x.mean(axis=0), pre.mean(axis=0), rtol=0, atol=1e-14)
    assert np.allclose(o.x - o.x.mean(axis=0), delta - delta.mean(axis=0), rtol=0, atol=1e-14)


def test_local_model_is_mean_minus_summed_gradients():
    """Plain SGD (no momentum, no weight decay): x_i after line 6 = mean_t - lr * sum of G over the round."""
    W, n, k = 4, 30, 4
    hyper = dict(lr=0.1, noise_sigma=0.01, seed=9)
    o = make(W, n, **hyper)
    o.round(k)
    o.average_begin()
    mean = o.mean.copy()
    grads = o.local_steps(k, log_gradients=True)
    o.average_end_apply()
    want = mean[None, :] - o.lr * np.sum(grads, axis=0)
    assert np.max(np.abs(o.x - want)) < 1e-14
    # and the averaged model moves by the averaged gradients
    assert np.allclose(o.x.mean(axis=0), mean - o.lr * np.sum(grads, axis=0).mean(axis=0), rtol=0, atol=1e-14)


def test_weighted_mean_invariant():
    W, n, k = 4, 20, 2
    p = np.array([1, 2, 2, 3], np.float64) / 8
    h, c = synth_inputs.quadratic_data(21, W, n)
    o = orc.QuadraticOracle(h, c, weights=p, **HYPER)
    o.round(k)
    o.average_begin()
    assert np.allclose(o.mean, p @ o.snap, rtol=0, atol=1e-15)
    o.local_steps(k)
    pre = o.x.copy()
    o.average_end_apply()
    assert np.allclose(p @ o.x, p @ pre, rtol=0, atol=1e-14)
    # equal weights are the uniform mean
    a = orc.QuadraticOracle(h, c, weights=np.full(W, 0.25), **HYPER)
    b = orc.QuadraticOracle(h, c, **HYPER)
    a.round(k); a.round(k); b.round(k); b.round(k)
    assert np.array_equal(a.x, b.x)


def test_shared_curvature_mean_follows_mean_objective():
    """Same h on every worker, no noise: the averaged model is single-worker SGD on the averaged centre."""
    W, n, R, k = 4, 60, 5, 3
    h1, _ = synth_inputs.quadratic_data(1, 1, n)
    _, c = synth_inputs.quadratic_data(2, W, n)
    hyper = dict(HYPER, noise_sigma=0.0)
    o = orc.QuadraticOracle(np.repeat(h1, W, 0), c, **hyper)
    for _ in range(R):
        o.round(k)
    lr, mu, wd = (orc.f32(hyper[t]) for t in ("lr", "momentum", "weight_decay"))
    hh = h1[0].astype(np.float64)
    cbar = c.astype(np.float64).mean(axis=0)
    x = np.zeros(n); v = np.zeros(n)
    for _ in range(R * k):
        v = mu * v + hh * (x - cbar) + wd * x
        x = x - lr * v
    assert np.max(np.abs(o.x.mean(axis=0) - x)) < 1e-13


# ---- closed form: the round is an affine map per coordinate -------------------------------

def round_matrix(h, c, lr, mu, wd, k):
    """(2W+1)x(2W+1) homogeneous matrix of one round acting on (x_1..x_W, v_1..v_W, 1)."""
    W = h.size
    L = np.eye(2 * W + 1)
    for i in range(W):
        a, b = h[i] + wd, h[i] * c[i]
        # v' = mu v + a x - b ;  x' = x - lr v'
        L[W + i, W + i] = mu; L[W + i, i] = a; L[W + i, -1] = -b
        L[i, i] = 1 - lr * a; L[i, W + i] = -lr * mu; L[i, -1] = lr * b
    M = np.linalg.matrix_power(L, k)
    M[:W, :W] += np.full((W, W), 1.0 / W) - np.eye(W)      # + (mean - own) of the stored models
    return M


@pytest.mark.parametrize("mu,wd,k", [(0.0, 0.0, 4), (0.9, 5e-4, 2), (0.5, 0.01, 1)])
def test_noiseless_trajectory_matches_affine_closed_form(mu, wd, k):
    W, n, R = 4, 12, 10
    h, c = synth_inputs.quadratic_data(31, W, n)
    o = orc.QuadraticOracle(h, c, lr=0.1, momentum=mu, weight_decay=wd)
    for _ in range(R):
        o.round(k)
    for j in range(n):
        M = round_matrix(h[:, j].astype(np.float64), c[:, j].astype(np.float64),
                         orc.f32(0.1), orc.f32(mu), orc.f32(wd), k)
        state = np.zeros(2 * W + 1); state[-1] = 1.0
        state = np.linalg.matrix_power(M, R) @ state
        assert np.max(np.abs(o.x[:, j] - state[:W])) < 1e-12
        if mu:
            assert np.max(np.abs(o.v[:, j] - state[W:2 * W])) < 1e-11


def test_plain_sgd_closed_form_scalar():
    """mu = 0: x after a round is (J + D) x - D c with D = diag((1 - lr h)^k - 1), J = averaging."""
    W, k, R, lr = 3, 4, 7, orc.f32(0.1)
    h = np.array([[0.5], [1.0], [2.0]], np.float32)
    c = np.array([[1.0], [-2.0], [0.25]], np.float32)
    o = orc.QuadraticOracle(h, c, lr=0.1)
    x = np.zeros(W)
    D = np.diag((1 - lr * h[:, 0].astype(np.float64)) ** k - 1)
    J = np.full((W, W), 1 / W)
    for _ in range(R):
        o.round(k)
        x = (J + D) @ x - D @ c[:, 0].astype(np.float64)
        assert np.max(np.abs(o.x[:, 0] - x)) < 1e-13


# ---- structure -----------------------------------------------------------------------------

def test_subset_equals_full_run():
    """The synthetic objective is separable: any column subset reproduces the full run bit for bit."""
    W, n, R, k = 4, 1000, 3, 2
    h, c = synth_inputs.quadratic_data(17, W, n)
    full = orc.QuadraticOracle(h, c, **HYPER)
    idx = np.array([0, 1, 2, 3, 4, 7, 8, 250, 251, 997, 998, 999], np.uint64)
    ii = idx.astype(np.int64)
    sub = orc.QuadraticOracle(h[:, ii], c[:, ii], idx=idx, **HYPER)
    for _ in range(R):
        full.round(k); sub.round(k)
    assert np.array_equal(sub.x, full.x[:, ii]) and np.array_equal(sub.v, full.v[:, ii])


def test_f32_mirror_stays_close_to_reference():
    """The fp32 mirror drifts from fp64 far less than the 1e-5 parity budget on the tiny config."""
    cfg = synth_inputs.CONFIGS["C1_tiny"]
    W, n = cfg["W"], 4096
    h, c = synth_inputs.quadratic_data(cfg["seed"], W, n)
    kw = dict(lr=cfg["lr"], momentum=cfg["momentum"], weight_decay=cfg["weight_decay"],
              noise_sigma=cfg["noise_sigma"], seed=cfg["seed"])
    a = orc.QuadraticOracle(h, c, kind="f64", **kw)
    b = orc.QuadraticOracle(h, c, kind="f32", **kw)
    for _ in range(cfg["rounds"]):
        a.round(cfg["k"][0]); b.round(cfg["k"][0])
    assert np.max(np.abs(a.x - b.x) / (1 + np.abs(a.x))) < 2e-6


def test_step_counter_is_global_across_rounds():
    """Noise is keyed by the global step t, which continues across rounds (tau = t .. t+k-1)."""
    W, n = 2, 16
    h = np.zeros((W, n), np.float32); c = np.zeros((W, n), np.float32)
    o = orc.QuadraticOracle(h, c, lr=1.0, noise_sigma=1.0, seed=4)
    o.round(2)
    assert o.step == 2
    before = o.x.copy()
    o.average_begin(); o.local_steps(1)
    z = np.stack([orc.normals(4, orc.TAG_NOISE, i, 2, 0, n) for i in range(W)])
    assert np.allclose(o.x, before - z, rtol=0, atol=1e-15)


def test_consensus_distance():
    """The left-hand quantity of Lemma 2 for one t: hand value, the variance identity
    sum p ||x - xbar||^2 = sum p ||x||^2 - ||xbar||^2, zero at consensus, reset by averaging."""
    h = np.ones((2, 1), np.float32); c = np.zeros((2, 1), np.float32)
    o = orc.QuadraticOracle(h, c, np.array([[0.0], [2.0]]), lr=0.1)
    assert o.consensus_distance() == 1.0                       # mean 1, both workers at distance 1
    ow = orc.QuadraticOracle(h, c, np.array([[0.0], [2.0]]), lr=0.1, weights=[0.25, 0.75])
    assert abs(ow.consensus_distance() - (0.25 * 1.5**2 + 0.75 * 0.5**2)) < 1e-15
    big = make(8, 200, **HYPER)
    assert big.consensus_distance() == 0.0                     # all workers start equal
    big.round(3); big.round(3)
    x = big.x
    want = np.mean(np.sum(x * x, axis=1)) - np.sum(x.mean(axis=0) ** 2)
    assert abs(big.consensus_distance() - want) < 1e-12 and big.consensus_distance() > 0
    # Local-SGD style averaging (a round with zero local steps) brings every worker to the mean
    big.average_begin(); big.average_end_apply()
    assert big.consensus_distance() < 1e-28


def test_objective_and_gradient_norm():
    """f = sum_i p_i f_i and its gradient: hand values, the minimiser's closed form, and the analytic
    gradient against central differences of f itself."""
    # one worker, unit curvature: f = 1/2 ||x - c||^2, ||grad f||^2 = 2 f
    c1 = np.array([[1.0, -2.0, 0.5]], np.float32)
    o = orc.QuadraticOracle(np.ones((1, 3), np.float32), c1, x0=[2.0, 0.0, 0.5], lr=0.1)
    f, g2 = o.objective_at_mean()
    assert f == 0.5 * (1.0 + 4.0) and g2 == 5.0
    # two weighted workers, one coordinate: f(x) = 0.25*1/2*2*(x-1)^2 + 0.75*1/2*4*(x+1)^2
    h = np.array([[2.0], [4.0]], np.float32); c = np.array([[1.0], [-1.0]], np.float32)
    o = orc.QuadraticOracle(h, c, lr=0.1, weights=[0.25, 0.75])
    o.x[...] = [[3.0], [1.0]]                                 # xbar = 0.75 + 0.75 = 1.5
    f, g2 = o.objective_at_mean()
    assert abs(f - (0.25 * 0.25 + 1.5 * 6.25)) < 1e-15       # 0.25*(0.5)^2 + 1.5*(2.5)^2
    assert abs(g2 - (0.25 * 2 * 0.5 + 0.75 * 4 * 2.5) ** 2) < 1e-12
    # minimiser x*_j = sum_i p_i h_ij c_ij / sum_i p_i h_ij: gradient vanishes there, f is larger nearby
    W, d = 4, 9
    h, c = synth_inputs.quadratic_data(21, W, d)
    p = np.array([0.1, 0.2, 0.3, 0.4])
    o = orc.QuadraticOracle(h, c, lr=0.1, weights=p)
    hp = p[:, None] * h.astype(np.float64)
    xstar = np.sum(hp * c, axis=0) / np.sum(hp, axis=0)
    fstar, grad = o.objective(xstar)
    assert np.max(np.abs(grad)) < 1e-14
    rng = np.random.default_rng(0)
    for _ in range(5):
        assert o.objective(xstar + 0.1 * rng.standard_normal(d))[0] > fstar
    # analytic gradient vs central differences (f is quadratic: central differences are exact up to rounding)
    x = rng.standard_normal(d)
    _, grad = o.objective(x)
    for j in range(d):
        e = np.zeros(d); e[j] = 1e-3
        num = (o.objective(x + e)[0] - o.objective(x - e)[0]) / 2e-3
        assert abs(num - grad[j]) < 1e-9
    # all workers at the same point: objective_at_mean is objective(that point)
    o.x[...] = x
    f, g2 = o.objective_at_mean()
    assert abs(f - o.objective(x)[0]) < 1e-14 and abs(g2 - grad @ grad) < 1e-12


def test_per_worker_noise_scale():
    """sigma_i per worker: (a) equal entries are the scalar sigma; (b) with zero curvature, step size 1
    and a start at 0 the first step lands on -sigma_i z_i, the generator's own normals; (c) a worker
    with sigma_i = 0 follows the noiseless trajectory whatever the others do."""
    W, d = 3, 515
    h, c = synth_inputs.quadratic_data(9, W, d)
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, seed=77)
    a = orc.QuadraticOracle(h, c, noise_sigma=0.02, **hyper)
    b = orc.QuadraticOracle(h, c, noise_sigma=9.0, noise_sigma_w=[0.02] * W, **hyper)
    a.round(3); b.round(3)
    assert np.array_equal(a.x, b.x) and np.array_equal(a.v, b.v)
    sig = np.array([0.5, 0.0, 2.0], dtype=np.float32)
    z = orc.QuadraticOracle(np.zeros((W, d)), np.zeros((W, d)), lr=1.0, seed=77, noise_sigma_w=sig)
    z.local_steps(1)
    for i in range(W):
        assert np.array_equal(z.x[i], -float(sig[i]) * orc.normals(77, orc.TAG_NOISE, i, 0, 0, d))
    assert np.all(z.x[1] == 0) and np.std(z.x[2]) > 3 * np.std(z.x[0]) > 0
    quiet = orc.QuadraticOracle(h, c, noise_sigma=0.0, **hyper)
    mixed = orc.QuadraticOracle(h, c, noise_sigma_w=[0.1, 0.0, 0.3], **hyper)
    quiet.local_steps(4); mixed.local_steps(4)
    assert np.array_equal(quiet.x[1], mixed.x[1]) and not np.array_equal(quiet.x[0], mixed.x[0])


def test_external_step_hand_values_and_replay_of_logged_gradients():
    """The step with a given gradient: one hand-computed update (values exact in binary), and a
    replay of another oracle's logged gradients, which must retrace that oracle bit for bit."""
    one = np.ones((1, 1), np.float32)
    o = orc.QuadraticOracle(one, one, x0=1.0, lr=0.125, momentum=0.5, weight_decay=0.5)
    o.v[...] = 4.0
    o.external_step(np.array([[2.0]]))              # g = 2 + 0.5*1 = 2.5; v = 0.5*4 + 2.5 = 4.5; x = 1 - 0.125*4.5
    assert o.v[0, 0] == 4.5 and o.x[0, 0] == 0.4375 and o.step == 1
    W, d, k = 3, 257, 4
    h, c = synth_inputs.quadratic_data(5, W, d)
    for mu in (0.0, 0.9):
        hyper = dict(lr=0.05, momentum=mu, weight_decay=5e-4, seed=3)
        a = orc.QuadraticOracle(h, c, noise_sigma=0.01, **hyper)
        b = orc.QuadraticOracle(h, c, noise_sigma=0.0, **hyper)
        for r in range(3):
            a.average_begin(); b.average_begin()
            for G in a.local_steps(k, log_gradients=True):
                b.external_step(G)
            a.average_end_apply(); b.average_end_apply()
        assert np.array_equal(a.x, b.x) and a.step == b.step
        assert mu == 0.0 or np.array_equal(a.v, b.v)


def _theorem1_sides(o, k, rounds, L, sigma2, zeta2):
    """Runs `rounds` rounds of Algorithm 1 on oracle o (plain SGD) and returns both sides of the bound of
    Theorem 1: (1/T) sum_t D1 ||grad f(xhat_t)||^2 over ALL iterations t (xhat_t = weighted mean of the
    local models at iteration t), and 2 (f(xhat_0) - f*) / (T gamma) + D2 (N sigma^2 / sum M + 2 k zeta^2)
    + gamma L sigma^2 / sum M, here with M_i = 1."""
    gamma, T = o.lr, k * rounds
    D2 = 8 * gamma**2 * L**2 * k / (1 - 16 * gamma**2 * k**2 * L**2)
    D1 = 1 - 2 * k * D2
    assert gamma <= 1 / L and D1 > 0
    p = np.full(o.W, 1.0 / o.W)
    hp = p[:, None] * o.h.astype(np.float64)
    fstar = o.objective(np.sum(hp * o.c, axis=0) / np.sum(hp, axis=0))[0]
    f0 = o.objective(p @ o.x)[0]
    total = 0.0
    for _ in range(rounds):
        o.average_begin()
        for _ in range(k):
            grad = o.objective(p @ o.x)[1]
            total += D1 * float(grad @ grad)
            o.local_steps(1)
        o.average_end_apply()
    lhs = total / T
    rhs = 2 * (f0 - fstar) / (T * gamma) + D2 * (o.W * sigma2 / o.W + 2 * k * zeta2) + gamma * L * sigma2 / o.W
    return lhs, rhs


def test_convergence_bound_of_theorem_1_holds_and_catches_a_wrong_correction():
    """Theorem 1 on workers that satisfy its assumptions exactly: shared curvature h (so that the
    between-worker gradient variance zeta^2 = E_i ||h (c_i - cbar)||^2 is a constant), L = max h, noise
    of variance sigma_noise^2 per coordinate (sigma^2 = d sigma_noise^2), plain SGD, M_i = 1.  The
    measured left-hand side must respect the bound; with line 6 applied with the wrong sign (planted in
    a copy of the oracle's step, on the CPU) it must not."""
    W, d, k, rounds = 4, 512, 2, 300
    rng = np.random.default_rng(12)
    h = np.tile(rng.uniform(0.5, 2.0, d).astype(np.float32), (W, 1))
    c = rng.standard_normal((W, d)).astype(np.float32)
    sn = 0.05
    L = float(h.max())
    dev = h[0].astype(np.float64) * (c - c.mean(axis=0))
    zeta2 = float(np.mean(np.sum(dev * dev, axis=1)))
    hyper = dict(lr=0.02, noise_sigma=sn, seed=99)
    x0 = 3.0 * rng.standard_normal(d)
    lhs, rhs = _theorem1_sides(orc.QuadraticOracle(h, c, x0, **hyper), k, rounds, L, d * sn * sn, zeta2)
    assert 0 < lhs <= rhs, (lhs, rhs)
    assert lhs > 0.02 * rhs                       # the bound is not vacuous at this horizon

    class WrongSign(orc.QuadraticOracle):
        def average_end_apply(self):
            self.x[...] = self.mean[None, :] - (self.x - self.snap)
            self.averaging = False
    bad_lhs, bad_rhs = _theorem1_sides(WrongSign(h, c, x0, **hyper), k, rounds, L, d * sn * sn, zeta2)
    assert bad_lhs > bad_rhs, (bad_lhs, bad_rhs)


def test_mid_round_representation_of_the_local_model():
    """Proof of Lemma 2: at ANY iteration t the local model is the averaged model of the last complete
    communication, xhat at step (floor(t/k) - 1) k, minus gamma times the worker's own gradients since
    that step -- a statement across two rounds (plain SGD)."""
    W, n, k = 3, 25, 3
    o = make(W, n, lr=0.1, noise_sigma=0.02, seed=4)
    o.round(k)                                              # iterations 0 .. k-1
    boundary_mean, since = None, []
    for r in range(1, 4):                                   # rounds starting at t = r k
        o.average_begin()
        prev_mean, prev_grads = boundary_mean, since        # xhat_{(r-1)k} and the gradients of round r-1
        boundary_mean, since = o.mean.copy(), []
        for j in range(k):
            if prev_mean is not None:                       # t = r k + j: floor(t/k) - 1 = r - 1
                want = prev_mean[None, :] - o.lr * (np.sum(prev_grads, axis=0) + (np.sum(since, axis=0) if since else 0.0))
                assert np.max(np.abs(o.x - want)) < 1e-13, (r, j)
            since.append(o.local_steps(1, log_gradients=True)[0])
        o.average_end_apply()


def test_consensus_bound_of_lemma_2():
    """Lemma 2 on the same kind of workers as the Theorem 1 pin: sum_i p_i sum_t ||xhat_t - x_t^i||^2 <=
    8 gamma^2 k / (1 - 16 gamma^2 k^2 L^2) * (T N sigma^2 / sum M + 2 k T zeta^2 + 2 k sum_t ||grad f(xhat_t)||^2)."""
    W, d, k, rounds = 4, 256, 3, 100
    rng = np.random.default_rng(5)
    h = np.tile(rng.uniform(0.5, 2.0, d).astype(np.float32), (W, 1))
    c = rng.standard_normal((W, d)).astype(np.float32)
    sn, gamma = 0.05, 0.02
    L = float(h.max())
    dev = h[0].astype(np.float64) * (c - c.mean(axis=0))
    zeta2 = float(np.mean(np.sum(dev * dev, axis=1)))
    o = orc.QuadraticOracle(h, c, rng.standard_normal(d), lr=gamma, noise_sigma=sn, seed=6)
    gamma = o.lr
    p = np.full(W, 1.0 / W)
    lhs = grads = 0.0
    for _ in range(rounds):
        o.average_begin()
        for _ in range(k):
            lhs += o.consensus_distance()
            g = o.objective(p @ o.x)[1]
            grads += float(g @ g)
            o.local_steps(1)
        o.average_end_apply()
    T = k * rounds
    rhs = 8 * gamma**2 * k / (1 - 16 * gamma**2 * k**2 * L**2) * (T * d * sn * sn + 2 * k * T * zeta2 + 2 * k * grads)
    assert 0 < lhs <= rhs and lhs > 0.01 * rhs, (lhs, rhs)
