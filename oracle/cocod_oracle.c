/*
 * CoCoD-SGD reference oracle (quadratic-gradient workers) -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, step-by-step CPU implementation of one round of the decoupled
 * update of Algorithm 1 (CoCoD-SGD): snapshot, cross-worker mean of the
 * snapshots (Step I), k local SGD steps (Step II), correction (line 6).
 * It exists to check the HIP library; nothing in the product path may call it.
 * It shares no code with the HIP sources.
 *
 * Arithmetic type: REAL (double unless the build says -DREAL=float).  The
 * paper fixes no precision, so the reference is the algorithm in fp64; the
 * float build is a diagnostic mirror of what an fp32 device computes.
 *
 * Everything that is not in the paper (the synthetic per-worker objective,
 * the noise generator and its keying, the optimizer details taken from the
 * experiment section) is a documented reading, repeated at each function.
 *
 * Pins (tests/test_oracle_*.py): Philox known answers and an independent
 * big-integer implementation; W=1 == plain SGD; identical workers == single
 * worker; mean preservation by the correction (proof of Lemma 2, the
 * representation of the averaged model); the representation of the local
 * model as averaged model minus gamma times the summed local gradients
 * (same proof); closed-form affine-map trajectory of the noiseless quadratic;
 * a hand-computed W=2, d=1 case; subset == full run; per-worker noise scale
 * against the generator's own normals; the bound of Theorem 1 on workers that
 * satisfy its assumptions (with a planted wrong-sign line 6 as negative control).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#ifndef REAL
#define REAL double
#endif

/* stream tags: 4th counter word, keeps the random streams disjoint */
enum { TAG_NOISE = 0, TAG_H = 1, TAG_C = 2, TAG_MLP_X = 4, TAG_MLP_Y = 5 };

/* ------------------------------------------------------------------------
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as
 * easy as 1, 2, 3", SC'11).  Ten rounds; each round multiplies counter words
 * 0 and 2 by two fixed constants, keeps the low halves as new words 3 and 1,
 * and xors the high halves with the other two words and the key; the key is
 * advanced by two Weyl constants between rounds.
 * ---------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * Keying (a reading; the paper has no generator): key = (seed low, seed high);
 * counter = (q, step, worker, tag) with q = j >> 2, so one block of four words
 * serves the four consecutive indices 4q .. 4q+3 (word j & 3 belongs to j).
 * Requires j < 2^34 and step < 2^32.
 */
void oracle_words(uint64_t seed, uint32_t tag, uint32_t worker, uint32_t step,
                  uint64_t q, uint32_t out[4])
{
    uint32_t ctr[4] = { (uint32_t)q, step, worker, tag };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    oracle_philox4x32_10(ctr, key, out);
}

/* uniform in [0,1) on a 2^-24 grid from the top 24 bits of a word */
static double u_half_open(uint32_t r) { return (double)(r >> 8) * (1.0 / 16777216.0); }
/* uniform in (0,1] on the same grid (safe argument for the logarithm) */
static double u_open_zero(uint32_t r) { return ((double)(r >> 8) + 1.0) * (1.0 / 16777216.0); }

/*
 * Four standard normals for indices 4q .. 4q+3 by the Box-Muller transform:
 * words (0,1) give normals 0 and 1, words (2,3) give normals 2 and 3;
 * radius from the first word of a pair, angle from the second;
 * even index takes the cosine, odd index the sine.
 */
void oracle_normal_quad(uint64_t seed, uint32_t tag, uint32_t worker, uint32_t step,
                        uint64_t q, double z[4])
{
    const double two_pi = 6.283185307179586476925286766559;
    uint32_t r[4];
    oracle_words(seed, tag, worker, step, q, r);
    for (int pair = 0; pair < 2; ++pair) {
        double radius = sqrt(-2.0 * log(u_open_zero(r[2 * pair])));
        double angle  = two_pi * u_half_open(r[2 * pair + 1]);
        z[2 * pair]     = radius * cos(angle);
        z[2 * pair + 1] = radius * sin(angle);
    }
}

/* n normals / uniforms / raw words for flat indices j0 .. j0+n-1 of one (tag, worker, step) */
void oracle_normals(uint64_t seed, uint32_t tag, uint32_t worker, uint32_t step,
                    uint64_t j0, uint64_t n, double *out)
{
    #pragma omp parallel for schedule(static) if (n > 4096)
    for (uint64_t m = 0; m < n; ++m) {
        uint64_t j = j0 + m;
        double z[4];
        oracle_normal_quad(seed, tag, worker, step, j >> 2, z);
        out[m] = z[j & 3];
    }
}

void oracle_uniforms(uint64_t seed, uint32_t tag, uint32_t worker, uint32_t step,
                     uint64_t j0, uint64_t n, double *out)
{
    for (uint64_t m = 0; m < n; ++m) {
        uint64_t j = j0 + m;
        uint32_t r[4];
        oracle_words(seed, tag, worker, step, j >> 2, r);
        out[m] = u_half_open(r[j & 3]);
    }
}

void oracle_raw_words(uint64_t seed, uint32_t tag, uint32_t worker, uint32_t step,
                      uint64_t j0, uint64_t n, uint32_t *out)
{
    for (uint64_t m = 0; m < n; ++m) {
        uint64_t j = j0 + m;
        uint32_t r[4];
        oracle_words(seed, tag, worker, step, j >> 2, r);
        out[m] = r[j & 3];
    }
}

/* global index of column m: idx[m], or m itself when no subset is given */
static uint64_t column_index(const uint64_t *idx, size_t m) { return idx ? idx[m] : (uint64_t)m; }

/*
 * Synthetic per-worker objective f_i(x) = 1/2 sum_j h_ij (x_j - c_ij)^2 when
 * the data is drawn on the device instead of being handed in:
 * h_ij = 0.5 + 1.5 U (tag H), c_ij = standard normal (tag C), step word 0,
 * both stored as fp32 (they are data, so they are rounded once here).
 * Arrays are [W][n] over the columns idx[0..n).
 */
void oracle_fill_quadratic(uint64_t seed, int W, size_t n, const uint64_t *idx, float *h, float *c)
{
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < W; ++i) {
        for (size_t m = 0; m < n; ++m) {
            uint64_t j = column_index(idx, m);
            uint32_t r[4];
            double z[4];
            oracle_words(seed, TAG_H, (uint32_t)i, 0, j >> 2, r);
            oracle_normal_quad(seed, TAG_C, (uint32_t)i, 0, j >> 2, z);
            h[(size_t)i * n + m] = (float)(0.5 + 1.5 * u_half_open(r[j & 3]));
            c[(size_t)i * n + m] = (float)z[j & 3];
        }
    }
}

/*
 * One local step of Step II of Algorithm 1 for every worker, with the
 * stochastic gradient of the synthetic objective
 *     G = h (x - c) + sigma z(seed, worker, step, j)
 * and the optimizer of the experiment section (momentum, weight decay; a
 * reading: classic heavy-ball as in the framework the authors used, no
 * dampening, no Nesterov, v starts at 0):
 *     g = G + wd x ;  v = mu v + g ;  x = x - lr v .
 * mu = 0 and wd = 0 give the update of Algorithm 1 exactly.
 * x, v: [W][n]; h, c: [W][n] fp32 data; g_out (may be NULL): [W][n] receives G.
 * v may be NULL when mu == 0.
 */
void oracle_local_step(int W, size_t n, const uint64_t *idx, REAL *x, REAL *v,
                       const float *h, const float *c, double lr, double mu, double wd,
                       double sigma_all, const float *sigma_w, uint64_t seed, uint32_t step, REAL *g_out)
{
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < W; ++i) {
        uint64_t cached_q = UINT64_MAX;
        double z[4] = { 0, 0, 0, 0 };
        /* heterogeneous workers: the variance of worker i's mini-batch gradient falls with its
           batch size M_i, so each worker may carry its own standard deviation */
        const double sigma = sigma_w ? (double)sigma_w[i] : sigma_all;
        for (size_t m = 0; m < n; ++m) {
            size_t at = (size_t)i * n + m;
            uint64_t j = column_index(idx, m);
            if (sigma != 0.0 && (j >> 2) != cached_q) {       /* same block serves 4 neighbours */
                cached_q = j >> 2;
                oracle_normal_quad(seed, TAG_NOISE, (uint32_t)i, step, cached_q, z);
            }
            REAL noise = (sigma != 0.0) ? (REAL)((REAL)sigma * (REAL)z[j & 3]) : (REAL)0;
            REAL diff = x[at] - (REAL)c[at];
            REAL G = (REAL)h[at] * diff;
            G = G + noise;
            if (g_out) g_out[at] = G;
            REAL g = G + (REAL)wd * x[at];
            if (v) {
                REAL vel = (REAL)mu * v[at];
                vel = vel + g;
                v[at] = vel;
                g = vel;
            }
            x[at] = x[at] - (REAL)lr * g;
        }
    }
}

/*
 * Step I of Algorithm 1: weighted mean of the stored models,
 * mean_j = sum_i p_i snap_ij with p_i = M_i / sum_l M_l; p == NULL means the
 * homogeneous case p_i = 1/W.  Accumulated in fp64 in worker order.
 */
void oracle_mean(int W, size_t n, const REAL *snap, const double *p, REAL *mean)
{
    #pragma omp parallel for schedule(static)
    for (size_t m = 0; m < n; ++m) {
        double acc = 0.0;
        for (int i = 0; i < W; ++i) {
            double weight = p ? p[i] : 1.0;
            acc += weight * (double)snap[(size_t)i * n + m];
        }
        if (!p) acc = acc / (double)W;
        mean[m] = (REAL)acc;
    }
}

/* Line 6 of Algorithm 1: x_i <- mean + (x_i - snap_i), in that order of operations. */
void oracle_correct(int W, size_t n, REAL *x, const REAL *snap, const REAL *mean)
{
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < W; ++i)
        for (size_t m = 0; m < n; ++m) {
            size_t at = (size_t)i * n + m;
            REAL delta = x[at] - snap[at];
            x[at] = mean[m] + delta;
        }
}

/*
 * One full round (the body of the while loop of Algorithm 1): store the
 * models, average the stored models, take k local steps, apply line 6.
 * Steps I and II are independent (one reads only the snapshot, the other never
 * touches it), so running them one after the other is the same computation.
 * snap [W][n] and mean [n] are caller-provided work arrays and hold the
 * round's snapshot and average on return.  step0 is the global step counter
 * t at the start of the round; the caller advances it by k.
 */
void oracle_round(int W, size_t n, const uint64_t *idx, REAL *x, REAL *v, REAL *snap, REAL *mean,
                  const float *h, const float *c, const double *p, double lr, double mu,
                  double wd, double sigma, const float *sigma_w, uint64_t seed, uint32_t step0, int k)
{
    for (size_t at = 0; at < (size_t)W * n; ++at) snap[at] = x[at];
    oracle_mean(W, n, snap, p, mean);
    for (int s = 0; s < k; ++s)
        oracle_local_step(W, n, idx, x, v, h, c, lr, mu, wd, sigma, sigma_w, seed, step0 + (uint32_t)s, NULL);
    oracle_correct(W, n, x, snap, mean);
}

int oracle_real_bytes(void) { return (int)sizeof(REAL); }

/* number of threads the parallel loops above use (for reporting the CPU baseline) */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
