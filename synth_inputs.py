"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Holds workload descriptions and input data only -- none of the method's
arithmetic.  Both the HIP library and the CPU oracle are fed from here; neither
side's code lives here.

The paper (CoCoD-SGD) trains ResNet18 / VGG16 on CIFAR with 16 workers,
momentum 0.9 and a small communication period k.  None of that data is
available, so the workloads keep only its shape: worker count, parameter count,
optimizer hyper-parameters, k.  Each worker's loss is a separable quadratic with
per-worker curvature h and centre c, plus seeded gradient noise.
"""
import math

import numpy as np

# W workers, d fp32 parameters each; lr, momentum, weight decay, noise sigma; k; rounds
CONFIGS = {
    "C1_tiny": dict(W=4, d=65536, lr=0.1, momentum=0.0, weight_decay=0.0, noise_sigma=0.01,
                    k=(4,), rounds=10, seed=0x5EED0001),
    "C2_resnet18": dict(W=16, d=11_200_000, lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01,
                        k=(1, 2, 4), rounds=50, seed=0x5EED0002),
    "C3_vgg16": dict(W=16, d=138_000_000, lr=0.01, momentum=0.9, weight_decay=0.0, noise_sigma=0.01,
                     k=(2,), rounds=20, seed=0x5EED0003),
    "C4_mlp": dict(W=16, mlp=(3072, 1024, 10), batch=128, lr=0.05, momentum=0.9, weight_decay=0.0,
                   k=(2,), rounds=30, seed=0x5EED0004),
    "C5_bucketed": dict(W=64, d=11_200_000, n_tensors=62, tensor_lo=64, tensor_hi=2_400_000,
                        bucket_bytes=25 << 20, lr=0.05, momentum=0.9, weight_decay=5e-4,
                        noise_sigma=0.01, k=(1, 2, 4, 8), rounds=20, seed=0x5EED0005),
}


def quadratic_data(seed, W, n):
    """h ~ U[0.5, 2], c ~ N(0, 1) as fp32 arrays [W][n] (host-generated variant of the data)."""
    rng = np.random.default_rng(seed)
    h = rng.uniform(0.5, 2.0, size=(W, n)).astype(np.float32)
    c = rng.standard_normal(size=(W, n)).astype(np.float32)
    return h, c


def tensor_sizes(seed, n_tensors, total, lo, hi):
    """A ResNet18-like list of tensor sizes: log-uniform in [lo, hi], rescaled to sum to total."""
    rng = np.random.default_rng(seed)
    raw = np.exp(rng.uniform(math.log(lo), math.log(hi), size=n_tensors))
    sizes = np.maximum(1, np.floor(raw * (total / raw.sum()))).astype(np.int64)
    sizes[int(np.argmax(sizes))] += total - int(sizes.sum())
    assert int(sizes.sum()) == total and sizes.min() >= 1
    return [int(s) for s in sizes]


def mlp_param_count(n_in, n_hidden, n_out):
    return n_in * n_hidden + n_hidden + n_hidden * n_out + n_out


def mlp_he_init(seed, n_in, n_hidden, n_out):
    """He-normal weights, zero biases, flat fp32 vector in the order W1 | b1 | W2 | b2
    (W1 row-major [n_in][n_hidden], W2 row-major [n_hidden][n_out])."""
    rng = np.random.default_rng(seed)
    w1 = rng.standard_normal(n_in * n_hidden) * math.sqrt(2.0 / n_in)
    w2 = rng.standard_normal(n_hidden * n_out) * math.sqrt(2.0 / n_hidden)
    flat = np.concatenate([w1, np.zeros(n_hidden), w2, np.zeros(n_out)])
    return flat.astype(np.float32)


def sample_columns(seed, d, n_random, must_include=()):
    """Sorted unique global indices: n_random uniform draws plus the given boundary indices."""
    rng = np.random.default_rng(seed)
    picks = rng.integers(0, d, size=n_random, dtype=np.int64)
    extra = np.asarray([j for j in must_include if 0 <= j < d], dtype=np.int64)
    return np.unique(np.concatenate([picks, extra])).astype(np.uint64)
