"""GPU parity of the MLP-gradient workers (fp32 MFMA contractions) against the numpy fp64 oracle.
Bar: max |dx| <= 1e-4 (1 + |x|).  The pieces of one step (mini-batch, hidden layer, logit gradient,
hidden gradient) are checked on their own first, so that a wrong operand layout names itself."""
import numpy as np
import pytest
import torch

import paper_1906_12043_amd as P
import synth_inputs
from oracle import mlp_oracle as mlp
from tests.gpu_harness import GpuMlp, rel_err

pytestmark = pytest.mark.gpu
TOL = 1e-4


HYPER = dict(lr=0.05, momentum=0.9, weight_decay=1e-3, seed=0x5EED0004)


# the last shape has more hidden units (1152) than the output-layer kernel keeps of a sample's row in registers (1024)
@pytest.mark.parametrize("W,shape,batch", [(2, (128, 64, 10), 128), (3, (256, 192, 3), 256), (1, (384, 128, 16), 128),
                                           (2, (128, 1152, 10), 128)])
def test_pieces_of_one_step(W, shape, batch):
    n_in, n_hidden, n_out = shape
    theta0 = synth_inputs.mlp_he_init(7, *shape).astype(np.float64)
    theta0 += 0.05 * np.random.default_rng(1).standard_normal(theta0.size)      # biases away from zero
    theta0 = theta0.astype(np.float32)
    g = GpuMlp(W, shape, batch, theta0, **HYPER)
    g.ctx.set_step(5)
    g.ctx.local_steps(1)
    ws = g.workspace()
    th = theta0.astype(np.float64)
    W1, b1, W2, b2 = mlp.split(th, *shape)
    for i in range(W):
        X, y = mlp.minibatch(HYPER["seed"], i, 5, batch, n_in, n_out)
        assert np.array_equal(ws["y"][i], y)
        assert np.max(np.abs(ws["X"][i] - X)) < 2e-6
        A = X @ W1 + b1
        H = np.maximum(A, 0)
        scale = 1 + np.abs(A).max()
        assert np.max(np.abs(ws["H"][i] - H)) < 2e-5 * scale
        Z = H @ W2 + b2
        E = np.exp(Z - Z.max(axis=1, keepdims=True))
        dZ = E / E.sum(axis=1, keepdims=True)
        dZ[np.arange(batch), y] -= 1
        dZ /= batch
        assert np.max(np.abs(ws["dZ"][i] - dZ)) < 1e-6
        dA = (dZ @ W2.T) * (A > 0)
        sure = np.abs(A) > 1e-4                         # the relu decision is taken in fp32 on the device
        assert np.max(np.abs(ws["dA"][i] - dA)[sure]) < 1e-6
    g.close()


def test_every_step_trains_on_its_own_minibatch():
    """A local step draws the NEXT step's mini-batch beside its output layer, into the other of two buffers.
    Whatever precedes a step - another step, a jump of the step counter, a round boundary - the batch it
    used (read back from the work space) is the one keyed by its own step index."""
    W, shape, batch = 2, (128, 64, 10), 128
    g = GpuMlp(W, shape, batch, synth_inputs.mlp_he_init(3, *shape), **HYPER)

    def check(step):
        ws = g.workspace()
        for i in range(W):
            X, y = mlp.minibatch(HYPER["seed"], i, step, batch, shape[0], shape[2])
            assert np.array_equal(ws["y"][i], y), (step, i)
            assert np.max(np.abs(ws["X"][i] - X)) < 2e-6, (step, i)

    g.ctx.local_steps(1); check(0)
    g.ctx.local_steps(3); check(3)
    g.ctx.set_step(40)                               # the batch drawn ahead (for step 4) must not be used
    g.ctx.local_steps(2); check(41)
    g.ctx.round(3); check(44)
    g.ctx.set_step(45)                               # same value as the counter already has: the batch drawn ahead is right
    g.ctx.round_fused_tail(1); check(45)
    g.ctx.set_step(3)
    g.ctx.local_steps(1); check(3)
    g.close()


# the last shape has 16 x 2 x 32 = 1024 tiles of 64 x 128 in W1: several per compute unit, 4 M relu decisions per round
@pytest.mark.parametrize("W,shape,batch,k", [(3, (128, 64, 10), 128, 2), (2, (256, 192, 3), 256, 1), (4, (384, 128, 16), 128, 3),
                                             (32, (1024, 256, 10), 128, 2)])
def test_small_networks_rounds(W, shape, batch, k):
    theta0 = synth_inputs.mlp_he_init(11, *shape)
    g = GpuMlp(W, shape, batch, theta0, **HYPER)
    o = mlp.MlpOracle(theta0, W, *shape, batch, **HYPER)
    # Columns of W1 fed by a hidden unit whose pre-activation came within 2e-5 of zero for some sample are
    # held to a loose bound only: there the relu decision depends on rounding (the largest shape takes
    # 4 M such decisions per round and loses one: worker 27, unit 164, in the second averaging round).
    for r in range(4):
        g.ctx.round(k); o.round(k)
        sure = o.certain_mask()
        gx, gv = g.x(), g.vel()
        ex, ev = rel_err(gx[sure], o.x[sure]), rel_err(gv[sure], o.v[sure])
        # once a decision has gone the other way, the next forward pass carries its column's difference into
        # every gradient: the momentum is then held to ten times the bar, as in the full-size test
        assert ex <= TOL and ev <= (TOL if sure.all() else 10 * TOL), (r, ex, ev)
        assert (~sure).mean() < 0.05 and rel_err(gx, o.x) <= 5e-3 and rel_err(gv, o.v) <= 5e-2, (r, (~sure).mean())
    assert g.ctx.get_step() == o.step
    g.ctx.average_begin(); g.ctx.local_steps_end_apply(k)         # same round through the other entry point
    o.round(k)
    sure = o.certain_mask()
    assert rel_err(g.x()[sure], o.x[sure]) <= TOL
    g.close()


@pytest.mark.parametrize("W,shape,batch", [(3, (128, 64, 10), 128), (2, (256, 192, 3), 256), (2, (128, 128, 16), 128)])
def test_line6_inside_the_last_step_gives_the_same_bits(W, shape, batch):
    """cocod_local_steps_end_apply applies line 6 in the update epilogues of the round's last step; the
    result must equal cocod_local_steps + cocod_average_end_apply bit for bit, for k = 1 (the step reads
    the stored models), 2, 3 and 0, under each schedule, and follow the oracle."""
    theta0 = synth_inputs.mlp_he_init(5, *shape)
    a, b = GpuMlp(W, shape, batch, theta0, **HYPER), GpuMlp(W, shape, batch, theta0, **HYPER)
    o = mlp.MlpOracle(theta0, W, *shape, batch, **HYPER)
    for k, sched in [(2, P.SCHED_OVERLAP), (1, P.SCHED_OVERLAP), (3, P.SCHED_SERIAL), (0, P.SCHED_OVERLAP), (2, P.SCHED_FUSED),
                     (1, P.SCHED_HEAD)]:
        for w in (a, b):
            w.ctx.set_schedule(sched)
        a.ctx.round(k)
        b.ctx.average_begin(); b.ctx.local_steps_end_apply(k)
        o.round(k)
        assert np.array_equal(a.x(), b.x()) and np.array_equal(a.vel(), b.vel()), (k, sched)
        assert not b.ctx.is_averaging() and a.ctx.get_step() == b.ctx.get_step() == o.step
    assert rel_err(b.x(), o.x) <= TOL and rel_err(b.vel(), o.v) <= TOL
    a.close(); b.close()


def test_mlp_shape_validation():
    dev = torch.device("cuda:0")
    for shape, batch in [((100, 64, 10), 128), ((128, 60, 10), 128), ((128, 64, 17), 128), ((128, 64, 10), 100)]:
        d = synth_inputs.mlp_param_count(*shape)
        stride = (d + 3) // 4 * 4
        bufs = [torch.zeros((2, stride), device=dev) for _ in range(3)]
        mean = torch.zeros(stride, device=dev)
        with pytest.raises(P.CocodError) as e:
            P.Context(W=2, d=d, stride=stride, xA=bufs[0], xB=bufs[1], v=bufs[2], mean=mean, grad=P.GRAD_MLP,
                      mlp=(*shape, batch), lr=0.1)
        assert e.value.status == P.ERR_UNSUPPORTED


def test_full_size_config_thirty_rounds_free_running():
    """C4 as specified, all 30 rounds free-running (the device never sees the oracle's state).

    Two facts about this workload shape the comparison (neither is about the kernels):
    1. relu decides A > 0 in the device's fp32.  With 2.1 M pre-activations per step a few land within
       rounding of zero, and there the fp64 oracle may take the other branch.  Such a unit changes
       column n of dW1 and db1[n] of that worker in that step (pinned on the CPU); those columns are
       held to a loose bound, everything else to the bar.  The mask accumulates over the run and its
       size is reported per round.
    2. The iteration amplifies rounding differences geometrically (CPU evidence:
       test_fp32_evaluations_of_the_benchmark_mlp_drift_apart), and a relu decision taken the other
       way seeds a difference of ~1e-5 that then grows at the same rate, so NO fp32 evaluation
       follows fp64 to 1e-4 for 30 rounds.  In every round the device must stay within
       max(bar, 4 x the deviation of the oracle's own fp32 mirror from fp64): the mirror is the same
       numpy code run in fp32 on the same inputs, its deviation taken as the running maximum over the
       same (certain) parameters.  While the mirror is still far below the bar this IS the bar
       1e-4 (1 + |x|); and whatever the mirror does (its own rounding depends on the host's BLAS),
       the device is held to the plain bar outright for the first eight rounds."""
    cfg = synth_inputs.CONFIGS["C4_mlp"]
    W, shape, batch, k = cfg["W"], cfg["mlp"], cfg["batch"], cfg["k"][0]
    hyper = dict(lr=cfg["lr"], momentum=cfg["momentum"], weight_decay=cfg["weight_decay"], seed=cfg["seed"])
    theta0 = synth_inputs.mlp_he_init(cfg["seed"], *shape)
    g = GpuMlp(W, shape, batch, theta0, **hyper)
    o = mlp.MlpOracle(theta0, W, *shape, batch, **hyper)
    mirror = mlp.MlpOracle(theta0, W, *shape, batch, compute_dtype=np.float32, **hyper)
    mx = mv = ml = 0.0                              # running envelope of the mirror's deviation
    strict = 0                                      # rounds in which the plain bar was in force
    for r in range(cfg["rounds"]):
        g.ctx.round_fused_tail(k) if r % 2 else g.ctx.round(k)      # both ways of closing the round
        o.round(k); mirror.round(k)
        sure = o.certain_mask()
        gx, gv = g.x(), g.vel()
        ex, ev = rel_err(gx[sure], o.x[sure]), rel_err(gv[sure], o.v[sure])
        loose = rel_err(gx[~sure], o.x[~sure]) if (~sure).any() else 0.0
        mirror_x, mirror_v = mirror.x.astype(np.float64), mirror.v.astype(np.float64)
        mx = max(mx, rel_err(mirror_x[sure], o.x[sure]))
        mv = max(mv, rel_err(mirror_v[sure], o.v[sure]))
        ml = max(ml, rel_err(mirror_x, o.x))
        bound_x, bound_v = max(TOL, 4 * mx), max(10 * TOL, 4 * mv)
        if bound_x == TOL and strict == r:
            strict = r + 1
        print("C4 round %2d free-running: rel err x %.3g (bound %.3g) v %.3g (bound %.3g) | fp32 mirror x %.3g v %.3g | "
              "borderline-relu columns: %d params (%.2f %%), x err %.3g | oracle loss %.4f"
              % (r + 1, ex, bound_x, ev, bound_v, mx, mv, int((~sure).sum()), 100.0 * (~sure).mean(), loose, o.last_loss.mean()),
              flush=True)
        assert ex <= bound_x and ev <= bound_v, (r, ex, ev, mx, mv)
        assert loose <= max(5e-3, 4 * ml), (r, loose, ml)
        if r < 8:
            assert ex <= TOL and ev <= 10 * TOL, (r, ex, ev)
    print("C4: by the mirror's evidence the plain bar was in force for the first %d rounds" % strict, flush=True)
    assert (~sure).mean() <= 0.15                   # the accumulated exclusion stays a small part of the model
    assert g.ctx.get_step() == o.step == cfg["rounds"] * k
    g.close()


def test_full_size_config_single_rounds_at_late_states():
    """One round from the oracle's own state at rounds 10, 20 and 30 of the C4 trajectory (oracle ->
    device only), compared at the full bar: the states a long run visits are checked without the
    drift of the rounds before them."""
    cfg = synth_inputs.CONFIGS["C4_mlp"]
    W, shape, batch, k = cfg["W"], cfg["mlp"], cfg["batch"], cfg["k"][0]
    hyper = dict(lr=cfg["lr"], momentum=cfg["momentum"], weight_decay=cfg["weight_decay"], seed=cfg["seed"])
    theta0 = synth_inputs.mlp_he_init(cfg["seed"], *shape)
    W = 4                                                           # four workers carry the trajectory, on both sides
    g = GpuMlp(W, shape, batch, theta0, **hyper)
    o = mlp.MlpOracle(theta0, W, *shape, batch, **hyper)
    for r in range(cfg["rounds"]):
        if r % 10 != 9:
            o.round(k)
            continue
        g.ctx.sync()
        live = g.xA if g.ctx.live_model() == g.xA.data_ptr() else g.xB
        live[:, :g.d] = torch.from_numpy(o.x.astype(np.float32)).to(g.dev)
        g.v[:, :g.d] = torch.from_numpy(o.v.astype(np.float32)).to(g.dev)
        torch.cuda.synchronize()
        g.ctx.set_step(o.step)
        o.clear_ambiguous()
        g.ctx.round(k); o.round(k)
        sure = o.certain_mask()
        gx, gv = g.x(), g.vel()
        ex, ev = rel_err(gx[sure], o.x[sure]), rel_err(gv[sure], o.v[sure])
        loose = rel_err(gx[~sure], o.x[~sure]) if (~sure).any() else 0.0
        print("C4 round %d from the oracle's state: rel err x %.3g v %.3g; borderline-relu columns: %d params, x err %.3g"
              % (r + 1, ex, ev, int((~sure).sum()), loose), flush=True)
        assert ex <= TOL and ev <= 10 * TOL, (r, ex, ev)
        assert loose <= 5e-3, (r, loose)
    g.close()
