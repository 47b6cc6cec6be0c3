"""Pins for the MLP-gradient oracle (CPU only): the gradient against finite differences and against
an autograd library on the same network, textbook identities, and the round structure."""
import numpy as np
import pytest
import torch

import synth_inputs
from oracle import cocod_oracle as orc
from oracle import mlp_oracle as mlp

SHAPE = (12, 8, 3)


def small_problem(seed=0, batch=4, shape=SHAPE):
    n_in, n_hidden, n_out = shape
    theta = synth_inputs.mlp_he_init(seed, n_in, n_hidden, n_out).astype(np.float64)
    theta += 0.1 * np.random.default_rng(seed).standard_normal(theta.size)       # non-zero biases too
    X, y = mlp.minibatch(seed, 1, 2, batch, n_in, n_out)
    return theta, X, y


def test_gradient_matches_central_differences():
    theta, X, y = small_problem()
    loss, grad = mlp.loss_and_gradient(theta, X, y, *SHAPE)
    eps = 1e-6
    for j in range(theta.size):
        e = np.zeros_like(theta); e[j] = eps
        lp, _ = mlp.loss_and_gradient(theta + e, X, y, *SHAPE)
        lm, _ = mlp.loss_and_gradient(theta - e, X, y, *SHAPE)
        assert abs((lp - lm) / (2 * eps) - grad[j]) < 1e-8, j


@pytest.mark.parametrize("shape,batch", [(SHAPE, 4), ((64, 32, 10), 16)])
def test_loss_and_gradient_match_autograd_library(shape, batch):
    n_in, n_hidden, n_out = shape
    theta, X, y = small_problem(seed=3, batch=batch, shape=shape)
    loss, grad = mlp.loss_and_gradient(theta, X, y, *shape)
    t = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    a = n_in * n_hidden; b = a + n_hidden; c = b + n_hidden * n_out
    W1, b1, W2, b2 = t[:a].view(n_in, n_hidden), t[a:b], t[b:c].view(n_hidden, n_out), t[c:]
    Z = torch.relu(torch.tensor(X) @ W1 + b1) @ W2 + b2
    ref = torch.nn.functional.cross_entropy(Z, torch.tensor(y))
    ref.backward()
    assert abs(loss - ref.item()) < 1e-13
    assert np.max(np.abs(grad - t.grad.numpy())) < 1e-13


def test_output_layer_identities():
    theta, X, y = small_problem(seed=5, batch=16)
    _, grad = mlp.loss_and_gradient(theta, X, y, *SHAPE)
    n_in, n_hidden, n_out = SHAPE
    db2 = grad[-n_out:]
    assert abs(db2.sum()) < 1e-15                     # softmax rows sum to 1, one-hot rows too
    dW2 = grad[n_in * n_hidden + n_hidden:-n_out].reshape(n_hidden, n_out)
    assert np.max(np.abs(dW2.sum(axis=1))) < 1e-15
    # uniform logits: loss is log(n_out) whatever the labels
    zero = np.zeros_like(theta)
    loss, g0 = mlp.loss_and_gradient(zero, X, y, *SHAPE)
    assert abs(loss - np.log(n_out)) < 1e-15
    counts = np.bincount(y, minlength=n_out)
    assert np.allclose(g0[-n_out:], (1.0 / n_out) - counts / y.size, rtol=0, atol=1e-15)


def test_minibatch_streams():
    seed, B, n_in, n_out = 0x5EED0004, 128, 3072, 10
    X, y = mlp.minibatch(seed, 7, 11, B, n_in, n_out)
    assert X.shape == (B, n_in) and y.shape == (B,)
    assert y.min() >= 0 and y.max() < n_out
    # element (b, f) is the normal at flat index b * n_in + f of stream 4
    for b, f in [(0, 0), (0, 5), (3, 17), (127, 3071)]:
        z = orc.normals(seed, orc.TAG_MLP_X, 7, 11, b * n_in + f, 1)[0]
        assert X[b, f] == float(np.float32(z))
    assert abs(X.mean()) < 0.01 and abs(X.std() - 1) < 0.01
    # labels: floor(u * n_out) with u = word / 2^32, roughly uniform over many batches
    w = orc.raw_words(seed, orc.TAG_MLP_Y, 7, 11, 0, B).astype(np.float64)
    assert np.array_equal(y, np.floor(w / 2**32 * n_out).astype(np.int64))
    ys = np.concatenate([mlp.minibatch(seed, i, s, B, 4, n_out)[1] for i in range(4) for s in range(20)])
    freq = np.bincount(ys, minlength=n_out) / ys.size
    assert np.max(np.abs(freq - 0.1)) < 0.015
    X2, y2 = mlp.minibatch(seed, 7, 12, B, n_in, n_out)      # fresh batch every step
    assert not np.array_equal(X, X2) and not np.array_equal(y, y2)


def test_borderline_relu_unit_touches_one_column_only():
    """Taking the other relu branch at a pre-activation of ~0 changes column n of dW1 and db1[n] and
    nothing else (H is ~0 either way); loss_and_gradient reports exactly those units."""
    n_in, n_hidden, n_out = SHAPE
    theta, X, y = small_problem(seed=8, batch=6)
    W1, b1, W2, b2 = mlp.split(theta, *SHAPE)
    b, n = 2, 5
    A = X @ W1 + b1
    grads = []
    for eps in (+1e-9, -1e-9):                       # put A[b][n] just above / just below zero
        th = theta.copy()
        th[n_in * n_hidden + n] += -A[b, n] + eps
        # other samples of unit n move too; keep them away from zero so only (b, n) is borderline
        loss, g, amb = mlp.loss_and_gradient(th, X, y, *SHAPE, margin=1e-6)
        assert list(amb) == [n]
        grads.append(g)
    diff = np.abs(grads[0] - grads[1])
    touched = np.zeros(theta.size, dtype=bool)
    touched[n:n_in * n_hidden:n_hidden] = True
    touched[n_in * n_hidden + n] = True
    assert diff[touched].max() > 1e-4 and diff[~touched].max() < 1e-9
    o = make(2)
    o.ambiguous[1].add(3)
    mask = o.certain_mask()
    assert mask[0].all() and (~mask[1]).sum() == 16 + 1 and not mask[1, 3] and not mask[1, 16 * 8 + 3]


def make(W, shape=(16, 8, 4), batch=8, **kw):
    theta0 = synth_inputs.mlp_he_init(1, *shape)
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=1e-3, seed=9)
    hyper.update(kw)
    return mlp.MlpOracle(theta0, W, *shape, batch, **hyper)


def test_single_worker_is_plain_momentum_sgd():
    o = make(1)
    ref = make(1)
    for _ in range(3):
        o.round(2)
    ref.local_steps(6)
    assert np.max(np.abs(o.x - ref.x)) < 1e-14 and np.array_equal(o.v, ref.v)
    # the loss goes down on the same batch distribution with a sane learning rate
    assert np.isfinite(o.last_loss).all()


def test_plain_sgd_step_formula():
    """One step, mu = 0, wd = 0: x' = x - lr G with G from the pinned gradient routine."""
    o = make(2, momentum=0.0, weight_decay=0.0)
    x_before = o.x.copy()
    o.local_steps(1)
    for i in range(2):
        X, y = mlp.minibatch(9, i, 0, 8, 16, 4)
        _, G = mlp.loss_and_gradient(x_before[i], X, y, 16, 8, 4)
        assert np.array_equal(o.x[i], x_before[i] - o.lr * G)


def test_line6_preserves_worker_mean_and_first_round_is_identity():
    o = make(4)
    ref = make(4)
    o.round(2); ref.local_steps(2)
    assert np.max(np.abs(o.x - ref.x)) < 1e-15       # all workers equal at the start: mean == stored model
    o.average_begin()
    assert np.allclose(o.mean, o.snap.mean(axis=0), rtol=0, atol=1e-16)
    o.local_steps(3)
    pre = o.x.copy()
    o.average_end_apply()
    assert np.allclose(o.x.mean(axis=0), pre.mean(axis=0), rtol=0, atol=1e-15)
    assert np.allclose(o.x - o.x.mean(axis=0), (pre - o.snap) - (pre - o.snap).mean(axis=0), rtol=0, atol=1e-15)
    assert o.step == 5
