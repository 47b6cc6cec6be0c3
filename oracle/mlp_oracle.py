"""CPU oracle for CoCoD-SGD rounds with MLP-gradient workers -- TEST INFRASTRUCTURE ONLY.

Same round as oracle/cocod_oracle.c (Algorithm 1: store, mean, k local steps, line 6), but the
stochastic gradient of Step II is a real mini-batch gradient: a two-layer perceptron
    A = X W1 + b1 ;  H = relu(A) ;  Z = H W2 + b2 ;  loss = mean_b CE(softmax(Z_b), y_b)
on a fresh seeded mini-batch per (worker, step).  Plain numpy in fp64, textbook backpropagation,
no blocking or fusion.  Shares no code with the HIP library.

Readings (the paper only says "mini-batch stochastic gradient"; the workload is the benchmark's):
  * parameters are one flat vector in the order W1 (row-major [n_in][n_hidden]) | b1 | W2
    (row-major [n_hidden][n_out]) | b2;
  * inputs X[b][f] = standard normal of generator stream 4 at flat index b*n_in + f, keyed by
    (seed, worker, step); stored as fp32 (they are data);
  * labels y_b = (word * n_out) >> 32 with the raw generator word of stream 5 at index b;
  * softmax is evaluated with the row maximum subtracted; relu'(0) = 0;
  * optimizer and line 6 as in the quadratic oracle: g = G + wd x; v = mu v + g; x = x - lr v;
    momentum buffers stay local.
Pins: tests/test_oracle_mlp.py (finite differences, an autograd library on the same net, softmax
and gradient-sum identities, the optimizer lines against a library optimizer and against hand values,
W = 1 reduces to plain SGD, mean preservation by line 6).

Diagnostic mirrors (never the reference): `state_dtype=np.float32` rounds x and v to fp32 after every
update while all arithmetic stays fp64; `compute_dtype=np.float32` runs every operation in fp32.
They measure how far ANY fp32 evaluation of this iteration drifts from the fp64 one.
"""
import numpy as np

from . import cocod_oracle as orc


def split(theta, n_in, n_hidden, n_out):
    """Views of a flat parameter vector: W1 [n_in][n_hidden], b1, W2 [n_hidden][n_out], b2."""
    a = n_in * n_hidden
    b = a + n_hidden
    c = b + n_hidden * n_out
    return (theta[:a].reshape(n_in, n_hidden), theta[a:b], theta[b:c].reshape(n_hidden, n_out), theta[c:c + n_out])


def minibatch(seed, worker, step, batch, n_in, n_out):
    X = orc.normals(seed, orc.TAG_MLP_X, worker, step, 0, batch * n_in).astype(np.float32).astype(np.float64)
    words = orc.raw_words(seed, orc.TAG_MLP_Y, worker, step, 0, batch).astype(np.uint64)
    y = ((words * np.uint64(n_out)) >> np.uint64(32)).astype(np.int64)
    return X.reshape(batch, n_in), y


def loss_and_gradient(theta, X, y, n_in, n_hidden, n_out, margin=None):
    """Mean softmax cross-entropy of the perceptron and its gradient w.r.t. the flat parameters.

    With margin set, also returns the hidden units n for which some sample's pre-activation has
    |A[b][n]| < margin: there the relu decision A > 0 depends on rounding, and an fp32 evaluation
    may legitimately take the other branch (which changes column n of dW1 and db1[n] only)."""
    W1, b1, W2, b2 = split(theta, n_in, n_hidden, n_out)
    B = X.shape[0]
    A = X @ W1 + b1
    H = np.maximum(A, 0.0)
    Z = H @ W2 + b2
    Zs = Z - Z.max(axis=1, keepdims=True)
    E = np.exp(Zs)
    P = E / E.sum(axis=1, keepdims=True)
    loss = float(np.mean(np.log(E.sum(axis=1)) - Zs[np.arange(B), y]))
    dZ = P.copy()
    dZ[np.arange(B), y] -= 1.0
    dZ /= B
    dW2 = H.T @ dZ
    db2 = dZ.sum(axis=0)
    dH = dZ @ W2.T
    dA = dH * (A > 0.0)
    dW1 = X.T @ dA
    db1 = dA.sum(axis=0)
    grad = np.concatenate([dW1.ravel(), db1, dW2.ravel(), db2])
    if margin is None:
        return loss, grad
    return loss, grad, np.unique(np.nonzero(np.abs(A) < margin)[1])


class MlpOracle:
    """W workers, each a copy of the perceptron; methods are the steps of Algorithm 1."""

    def __init__(self, theta0, W, n_in, n_hidden, n_out, batch, *, lr, momentum=0.0, weight_decay=0.0,
                 seed=0, weights=None, state_dtype=None, compute_dtype=np.float64):
        self.W, self.shape, self.batch = W, (n_in, n_hidden, n_out), batch
        self.real = np.dtype(compute_dtype).type   # np.float64: the oracle; np.float32: diagnostic mirror
        self.state_dtype = state_dtype             # diagnostic mirror: state rounded to this type after every update
        theta0 = np.asarray(theta0, dtype=self.real)
        self.d = theta0.shape[-1]
        assert self.d == n_in * n_hidden + n_hidden + n_hidden * n_out + n_out
        self.x = np.empty((W, self.d), dtype=self.real)
        self.x[...] = theta0                       # every worker starts from the same point
        self.v = np.zeros_like(self.x)
        self.snap = np.zeros_like(self.x)
        self.mean = np.zeros(self.d, dtype=self.real)
        self.lr, self.mu, self.wd = (self.real(orc.f32(a)) for a in (lr, momentum, weight_decay))
        self.seed = int(seed)
        self.p = (np.full(W, 1.0 / W) if weights is None else np.asarray(weights, dtype=np.float64)).astype(self.real)
        self.step = 0
        self.averaging = False
        self.last_loss = np.zeros(W)
        # see loss_and_gradient; an fp32 dot product of length 3072 with O(1) terms is good to a few 1e-6
        self.margin = 2e-5
        self.ambiguous = [set() for _ in range(W)]         # per worker: hidden units with a borderline relu

    def local_steps(self, k):
        n_in, n_hidden, n_out = self.shape
        for _ in range(k):
            for i in range(self.W):
                X, y = minibatch(self.seed, i, self.step, self.batch, n_in, n_out)
                self.last_loss[i], G, amb = loss_and_gradient(self.x[i], X.astype(self.real), y, n_in, n_hidden, n_out,
                                                              self.margin)
                self.ambiguous[i].update(int(n) for n in amb)
                g = G + self.wd * self.x[i]
                self.v[i] = self._stored(self.mu * self.v[i] + g)
                self.x[i] = self._stored(self.x[i] - self.lr * self.v[i])
            self.step += 1

    def _stored(self, a):
        return a if self.state_dtype is None else a.astype(self.state_dtype).astype(self.real)

    def certain_mask(self):
        """[W][d] bool: False on the parameters (column n of W1, b1[n]) fed by a borderline relu unit
        since the last clear_ambiguous()."""
        n_in, n_hidden, n_out = self.shape
        mask = np.ones((self.W, self.d), dtype=bool)
        for i, units in enumerate(self.ambiguous):
            for n in units:
                mask[i, n:n_in * n_hidden:n_hidden] = False
                mask[i, n_in * n_hidden + n] = False
        return mask

    def clear_ambiguous(self):
        self.ambiguous = [set() for _ in range(self.W)]

    def average_begin(self):
        assert not self.averaging
        self.snap[...] = self.x
        self.mean = self.p @ self.snap
        self.averaging = True

    def average_end_apply(self):
        assert self.averaging
        self.x = self._stored(self.mean[None, :] + (self.x - self.snap))
        self.averaging = False

    def round(self, k):
        self.average_begin()
        self.local_steps(k)
        self.average_end_apply()
