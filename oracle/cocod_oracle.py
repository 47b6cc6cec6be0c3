"""ctypes front end of the C oracle (oracle/cocod_oracle.c) -- TEST INFRASTRUCTURE ONLY.

`QuadraticOracle` holds the state of W simulated workers on a set of columns and
advances it by the steps of Algorithm 1 (CoCoD-SGD) in the paper's order.  The
arithmetic is all in the C file; this module only marshals numpy arrays.
"""
import ctypes as C
import os

import numpy as np

from . import build_oracle

TAG_NOISE, TAG_H, TAG_C, TAG_MLP_X, TAG_MLP_Y = 0, 1, 2, 4, 5

_libs = {}


def _lib(kind):
    if kind not in _libs:
        path = build_oracle.lib_path(kind)
        if not os.path.exists(path):
            build_oracle.build()
        lib = C.CDLL(path)
        u64, u32, i32, sz, dbl, ptr = C.c_uint64, C.c_uint32, C.c_int, C.c_size_t, C.c_double, C.c_void_p
        lib.oracle_philox4x32_10.argtypes = [ptr, ptr, ptr]
        lib.oracle_words.argtypes = [u64, u32, u32, u32, u64, ptr]
        lib.oracle_normal_quad.argtypes = [u64, u32, u32, u32, u64, ptr]
        lib.oracle_normals.argtypes = [u64, u32, u32, u32, u64, u64, ptr]
        lib.oracle_uniforms.argtypes = [u64, u32, u32, u32, u64, u64, ptr]
        lib.oracle_raw_words.argtypes = [u64, u32, u32, u32, u64, u64, ptr]
        lib.oracle_fill_quadratic.argtypes = [u64, i32, sz, ptr, ptr, ptr]
        lib.oracle_local_step.argtypes = [i32, sz, ptr, ptr, ptr, ptr, ptr, dbl, dbl, dbl, dbl, ptr, u64, u32, ptr]
        lib.oracle_mean.argtypes = [i32, sz, ptr, ptr, ptr]
        lib.oracle_correct.argtypes = [i32, sz, ptr, ptr, ptr]
        lib.oracle_round.argtypes = [i32, sz, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr,
                                     dbl, dbl, dbl, dbl, ptr, u64, u32, i32]
        for name in ("oracle_philox4x32_10", "oracle_words", "oracle_normal_quad", "oracle_normals",
                     "oracle_uniforms", "oracle_raw_words", "oracle_fill_quadratic", "oracle_local_step",
                     "oracle_mean", "oracle_correct", "oracle_round"):
            getattr(lib, name).restype = None
        lib.oracle_real_bytes.restype = C.c_int
        lib.oracle_num_threads.restype = C.c_int
        _libs[kind] = lib
    return _libs[kind]


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def philox4x32_10(ctr, key):
    ctr = np.asarray(ctr, dtype=np.uint32)
    key = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    _lib("f64").oracle_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def normals(seed, tag, worker, step, j0, n):
    out = np.zeros(n, dtype=np.float64)
    _lib("f64").oracle_normals(seed, tag, worker, step, j0, n, _p(out))
    return out


def uniforms(seed, tag, worker, step, j0, n):
    out = np.zeros(n, dtype=np.float64)
    _lib("f64").oracle_uniforms(seed, tag, worker, step, j0, n, _p(out))
    return out


def raw_words(seed, tag, worker, step, j0, n):
    out = np.zeros(n, dtype=np.uint32)
    _lib("f64").oracle_raw_words(seed, tag, worker, step, j0, n, _p(out))
    return out


def fill_quadratic(seed, W, n=None, idx=None):
    """h, c ([W][n] fp32) drawn by the counter-based generator at columns idx (or 0..n-1)."""
    if idx is not None:
        idx = np.ascontiguousarray(idx, dtype=np.uint64)
        n = idx.size
    h = np.zeros((W, n), dtype=np.float32)
    c = np.zeros((W, n), dtype=np.float32)
    _lib("f64").oracle_fill_quadratic(seed, W, n, _p(idx), _p(h), _p(c))
    return h, c


def num_threads():
    return _lib("f64").oracle_num_threads()


def f32(value):
    """The double that equals the fp32 rounding of value (hyper-parameters are fp32 inputs)."""
    return float(np.float32(value))


class QuadraticOracle:
    """State of W workers on n columns; methods are the steps of Algorithm 1.

    h, c: [W][n] fp32 objective data.  x0: [n] or [W][n] start (same point for every
    worker in Algorithm 1's initialisation).  idx: global indices of the columns
    (None = 0..n-1); only the noise generator looks at them.  weights: p_i of the
    weighted mean (None = uniform).  kind: "f64" reference or "f32" mirror.
    """

    def __init__(self, h, c, x0=None, *, lr, momentum=0.0, weight_decay=0.0, noise_sigma=0.0,
                 seed=0, idx=None, weights=None, noise_sigma_w=None, kind="f64"):
        self.lib = _lib(kind)
        self.real = np.float64 if kind == "f64" else np.float32
        assert self.lib.oracle_real_bytes() == np.dtype(self.real).itemsize
        self.h = np.ascontiguousarray(h, dtype=np.float32)
        self.c = np.ascontiguousarray(c, dtype=np.float32)
        self.W, self.n = self.h.shape
        assert self.c.shape == self.h.shape
        self.x = np.zeros((self.W, self.n), dtype=self.real)
        if x0 is not None:
            self.x[...] = np.asarray(x0, dtype=self.real)
        self.momentum = f32(momentum)
        self.v = np.zeros_like(self.x) if self.momentum != 0.0 else None
        self.snap = np.zeros_like(self.x)
        self.mean = np.zeros(self.n, dtype=self.real)
        self.lr, self.wd, self.sigma = f32(lr), f32(weight_decay), f32(noise_sigma)
        self.seed = int(seed)
        self.idx = None if idx is None else np.ascontiguousarray(idx, dtype=np.uint64)
        self.p = None if weights is None else np.ascontiguousarray(weights, dtype=np.float64)
        self.sigma_w = None if noise_sigma_w is None else np.ascontiguousarray(noise_sigma_w, dtype=np.float32)
        assert self.sigma_w is None or self.sigma_w.shape == (self.W,)
        self.step = 0
        self.averaging = False

    def local_steps(self, k, log_gradients=False):
        """k iterations of Step II; returns the list of G arrays if asked."""
        logged = []
        for _ in range(k):
            g = np.zeros_like(self.x) if log_gradients else None
            self.lib.oracle_local_step(self.W, self.n, _p(self.idx), _p(self.x), _p(self.v), _p(self.h),
                                       _p(self.c), self.lr, self.momentum, self.wd, self.sigma, _p(self.sigma_w),
                                       self.seed, self.step, _p(g))
            self.step += 1
            if log_gradients:
                logged.append(g)
        return logged

    def external_step(self, G):
        """One iteration of Step II with a given stochastic gradient G [W][n] (a real model's
        backward pass in the paper's experiments): g = G + wd x; v = mu v + g; x = x - lr v."""
        g = np.asarray(G, dtype=self.real) + self.real(self.wd) * self.x
        if self.v is not None:
            self.v[...] = self.real(self.momentum) * self.v + g
            g = self.v
        self.x[...] = self.x - self.real(self.lr) * g
        self.step += 1

    def average_begin(self):
        """Step I: store the models and take their (weighted) mean."""
        assert not self.averaging
        self.snap[...] = self.x
        self.lib.oracle_mean(self.W, self.n, _p(self.snap), _p(self.p), _p(self.mean))
        self.averaging = True

    def average_end_apply(self):
        """Line 6: x_i <- mean + (x_i - snap_i)."""
        assert self.averaging
        self.lib.oracle_correct(self.W, self.n, _p(self.x), _p(self.snap), _p(self.mean))
        self.averaging = False

    def consensus_distance(self):
        """sum_i p_i ||xbar - x_i||^2 with xbar = sum_i p_i x_i: the quantity bounded by Lemma 2."""
        p = np.full(self.W, 1.0 / self.W) if self.p is None else self.p
        x = self.x.astype(np.float64)
        xbar = p @ x
        return float(np.sum(p[:, None] * (x - xbar[None, :]) ** 2))

    def objective(self, x):
        """f(x) = sum_i p_i f_i(x), f_i(x) = 1/2 sum_j h_ij (x_j - c_ij)^2: the problem definition's
        objective for the quadratic workers, at one point x [n].  Returns (f, grad f [n])."""
        p = np.full(self.W, 1.0 / self.W) if self.p is None else self.p
        diff = np.asarray(x, dtype=np.float64)[None, :] - self.c.astype(np.float64)
        hd = self.h.astype(np.float64) * diff
        return float(0.5 * np.sum(p[:, None] * hd * diff)), p @ hd

    def objective_at_mean(self):
        """(f(xbar), ||grad f(xbar)||^2) at xbar = sum_i p_i x_i, the point Theorem 1 speaks about."""
        p = np.full(self.W, 1.0 / self.W) if self.p is None else self.p
        f, grad = self.objective(p @ self.x.astype(np.float64))
        return f, float(grad @ grad)

    def round(self, k):
        """One pass of the while-loop body through the single C routine."""
        self.lib.oracle_round(self.W, self.n, _p(self.idx), _p(self.x), _p(self.v), _p(self.snap),
                              _p(self.mean), _p(self.h), _p(self.c), _p(self.p), self.lr, self.momentum,
                              self.wd, self.sigma, _p(self.sigma_w), self.seed, self.step, k)
        self.step += k
