"""Pins for the oracle's random streams (CPU only).

The generator is Philox4x32-10 of Salmon et al. (SC'11); the paper itself has no
generator, only "mini-batch stochastic gradient" in Step II of Algorithm 1.
"""
import os

import numpy as np
import pytest
from scipy import stats

from oracle import cocod_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def philox_bigint(ctr, key, rounds=10):
    """Independent implementation with Python integers, written from the published round function."""
    mask = 0xFFFFFFFF
    c = list(ctr)
    k = list(key)
    for _ in range(rounds):
        prod_a = 0xD2511F53 * c[0]
        prod_b = 0xCD9E8D57 * c[2]
        c = [((prod_b >> 32) ^ c[1] ^ k[0]) & mask, prod_b & mask,
             ((prod_a >> 32) ^ c[3] ^ k[1]) & mask, prod_a & mask]
        k = [(k[0] + 0x9E3779B9) & mask, (k[1] + 0xBB67AE85) & mask]
    return c


def read_kat():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_known_answers():
    rows = read_kat()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert list(orc.philox4x32_10(ctr, key)) == want
        assert philox_bigint(ctr, key) == want


def test_matches_bigint_on_random_counters():
    rng = np.random.default_rng(7)
    for _ in range(200):
        ctr = [int(t) for t in rng.integers(0, 2**32, size=4)]
        key = [int(t) for t in rng.integers(0, 2**32, size=2)]
        assert list(orc.philox4x32_10(ctr, key)) == philox_bigint(ctr, key)


def test_keying_layout():
    """word j&3 of block (j>>2, step, worker, tag) under key (seed lo, seed hi)."""
    seed = 0x0123456789ABCDEF
    words = orc.raw_words(seed, orc.TAG_C, worker=3, step=9, j0=5, n=7)
    for m, j in enumerate(range(5, 12)):
        block = philox_bigint([j >> 2, 9, 3, orc.TAG_C], [seed & 0xFFFFFFFF, seed >> 32])
        assert int(words[m]) == block[j & 3]


def test_streams_are_distinct():
    seed = 42
    base = orc.raw_words(seed, orc.TAG_NOISE, 0, 0, 0, 4096)
    for other in (orc.raw_words(seed, orc.TAG_H, 0, 0, 0, 4096),
                  orc.raw_words(seed, orc.TAG_NOISE, 1, 0, 0, 4096),
                  orc.raw_words(seed, orc.TAG_NOISE, 0, 1, 0, 4096),
                  orc.raw_words(seed + 1, orc.TAG_NOISE, 0, 0, 0, 4096),
                  orc.raw_words(seed + (1 << 32), orc.TAG_NOISE, 0, 0, 0, 4096)):
        assert np.count_nonzero(base == other) <= 1
    # counter -> output is a bijection for a fixed key: no repeated blocks
    blocks = orc.raw_words(seed, orc.TAG_NOISE, 0, 0, 0, 1 << 16).reshape(-1, 4)
    assert len({tuple(b) for b in blocks}) == blocks.shape[0]


def test_uniform_grid_and_distribution():
    u = orc.uniforms(11, orc.TAG_H, 2, 0, 0, 200_000)
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 2**24 == np.round(u * 2**24))           # 24-bit grid, exact in fp32
    assert stats.kstest(u, "uniform").pvalue > 1e-3
    w = orc.raw_words(11, orc.TAG_H, 2, 0, 0, 1000)
    assert np.array_equal(u[:1000], (w >> 8).astype(np.float64) / 2**24)


def test_normals_are_standard_normal():
    z = orc.normals(5, orc.TAG_NOISE, 1, 3, 0, 400_000)
    assert np.all(np.isfinite(z))
    assert abs(z.mean()) < 4 / np.sqrt(z.size)
    assert abs(z.var() - 1.0) < 0.01
    assert abs(stats.skew(z)) < 0.02
    assert abs(stats.kurtosis(z)) < 0.05
    assert stats.kstest(z, "norm").pvalue > 1e-3
    # the four normals of a block, and neighbouring blocks, are uncorrelated
    quad = z.reshape(-1, 4)
    corr = np.corrcoef(quad.T)
    assert np.max(np.abs(corr - np.eye(4))) < 0.01
    assert abs(np.corrcoef(z[:-4], z[4:])[0, 1]) < 0.01
    # each output of a pair is normal on its own (cosine and sine branches)
    for col in range(4):
        assert stats.kstest(quad[:, col], "norm").pvalue > 1e-3
    # radius^2 of a pair is chi-square with 2 degrees of freedom, angle is uniform
    r2 = quad[:, 0] ** 2 + quad[:, 1] ** 2
    assert stats.kstest(r2, "chi2", args=(2,)).pvalue > 1e-3
    ang = np.arctan2(quad[:, 3], quad[:, 2]) / (2 * np.pi) % 1.0
    assert stats.kstest(ang, "uniform").pvalue > 1e-3


def test_normal_tail_is_bounded():
    # U1 >= 2^-24 so |z| <= sqrt(2 * 24 * ln 2)
    z = orc.normals(1, orc.TAG_NOISE, 0, 0, 0, 100_000)
    assert np.max(np.abs(z)) <= np.sqrt(48 * np.log(2)) + 1e-12


def test_fill_quadratic_ranges_and_subset():
    seed, W, n = 99, 3, 4099
    h, c = orc.fill_quadratic(seed, W, n)
    assert h.dtype == np.float32 and c.dtype == np.float32
    assert h.min() >= 0.5 and h.max() < 2.0
    assert abs(h.mean() - 1.25) < 0.02 and abs(c.mean()) < 0.03 and abs(c.std() - 1) < 0.03
    idx = np.array([0, 1, 5, 4095, 4096, 4098], dtype=np.uint64)
    hs, cs = orc.fill_quadratic(seed, W, idx=idx)
    assert np.array_equal(hs, h[:, idx.astype(np.int64)])
    assert np.array_equal(cs, c[:, idx.astype(np.int64)])
    # h is the affine image of the tag-H uniforms; c is the tag-C normal stream
    u = orc.uniforms(seed, orc.TAG_H, 1, 0, 0, n)
    assert np.array_equal(h[1], (0.5 + 1.5 * u).astype(np.float32))
    assert np.array_equal(c[2], orc.normals(seed, orc.TAG_C, 2, 0, 0, n).astype(np.float32))


@pytest.mark.parametrize("kind", ["f64", "f32"])
def test_noise_enters_with_scale_sigma_and_right_key(kind):
    """h = 0, lr = 1: one step from x = 0 leaves x = -sigma z(seed, worker, step, j)."""
    seed, W, n, sigma = 1234, 3, 37, 0.25
    h = np.zeros((W, n), np.float32)
    c = np.zeros((W, n), np.float32)
    idx = (np.arange(n, dtype=np.uint64) * 3 + 2)
    o = orc.QuadraticOracle(h, c, lr=1.0, noise_sigma=sigma, seed=seed, idx=idx, kind=kind)
    o.step = 5
    o.local_steps(1)
    for i in range(W):
        want = np.array([-sigma * orc.normals(seed, orc.TAG_NOISE, i, 5, int(j), 1)[0] for j in idx])
        tol = 0 if kind == "f64" else 1e-6
        assert np.max(np.abs(o.x[i] - want)) <= tol
