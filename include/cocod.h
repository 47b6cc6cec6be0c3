/*
 * libcocod -- one round of CoCoD-SGD (computation and communication decoupled
 * SGD) for W simulated workers resident in one GPU's memory.
 *
 * The round is the body of the while loop of Algorithm 1 of the paper:
 *   Step I   store every worker's model x_t^i and form the weighted mean of the
 *            stored models, x^_t = sum_i p_i x_t^i           (cocod_average_begin)
 *   Step II  k local stochastic-gradient steps on the live model, concurrently
 *            with Step I                                     (cocod_local_steps)
 *   line 6   x_{t+k}^i = x^_t + (x_{t+k}^i - x_t^i)         (cocod_average_end_apply)
 *   line 7   t = t + k                                       (the step counter)
 * The paper's all-reduce between workers is, on one GPU, a reduction over the
 * worker axis on a second stream that overlaps the local steps.
 *
 * Conventions
 *   - plain C ABI; every function returns a cocod_status (0 = ok, < 0 = error)
 *     unless stated otherwise; no exception crosses the boundary.
 *   - "device" pointers are HIP device memory, "host" pointers ordinary memory.
 *   - every call only ENQUEUES work on the caller's streams; nothing waits for
 *     the GPU except cocod_sync, cocod_step_timing_read and cocod_destroy
 *     (cocod_create copies its small tables synchronously).
 *   - the caller owns all large device buffers and both streams; they must
 *     outlive the context.  The context owns its small tables (chunk table, weight and
 *     noise-scale vectors), two events, the MLP work space, the scratch of the
 *     diagnostics, and the recorded graphs with their step-counter word.
 *   - argument errors are detected before any GPU call is made.
 *   - a context is not thread safe; use it from one host thread at a time.
 */
#ifndef COCOD_H
#define COCOD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cocod_ctx cocod_ctx;

typedef enum cocod_status {
    COCOD_OK = 0,
    COCOD_ERR_INVALID = -1,      /* bad argument (null, misaligned, out of range, inconsistent) */
    COCOD_ERR_STATE = -2,        /* call not legal in the current state of the round */
    COCOD_ERR_HIP = -3,          /* a HIP runtime call failed; see cocod_last_error */
    COCOD_ERR_NOMEM = -4,        /* host or device allocation failed */
    COCOD_ERR_UNSUPPORTED = -5   /* valid request this build does not implement */
} cocod_status;

/* Where the stochastic gradient G of Step II comes from. */
typedef enum cocod_grad_kind {
    /* G_j = h_ij (x_j - c_ij) + sigma z(seed, i, t, j): separable quadratic with seeded noise
       standing in for the mini-batch gradient of Step II. */
    COCOD_GRAD_QUADRATIC = 0,
    /* G = gradient of the mean softmax cross-entropy of a two-layer ReLU perceptron on a fresh
       seeded mini-batch per (worker, step): a real mini-batch gradient, dense contractions. */
    COCOD_GRAD_MLP = 1,
    /* G is computed by the caller (a real model's backward pass) and handed to cocod_external_step;
       h, c and the MLP fields are unused. */
    COCOD_GRAD_EXTERNAL = 2
} cocod_grad_kind;

/* How Step I is scheduled relative to Step II (the arithmetic is the same in all of them). */
typedef enum cocod_schedule {
    COCOD_SCHED_OVERLAP = 0,   /* mean on avg_stream, concurrent with the local steps (the paper's scheme) */
    COCOD_SCHED_SERIAL = 1,    /* mean on compute_stream after the local steps, then line 6 (sequential, as
                                  the paper's Local-SGD timeline) */
    COCOD_SCHED_FUSED = 2,     /* mean and line 6 in one kernel after the local steps */
    COCOD_SCHED_HEAD = 3       /* mean formed inside the first local step of the round, which reads every
                                  stored model anyway: Step I costs one 4/W-byte store per parameter and no
                                  pass of its own; with k = 1 through cocod_local_steps_end_apply the mean,
                                  the step and line 6 are ONE kernel (built-in quadratic gradient, W <= 131
                                  workers, d < 2^30; whenever the round's first step is not such a step, the
                                  mean is formed on compute_stream just before line 6 needs it) */
} cocod_schedule;

enum {
    COCOD_FLAG_DRY_RUN = 1u    /* validate, plan and track state but make no GPU call at all (host tests) */
};

/*
 * Memory layout.  Every per-worker array is worker-major: element e of worker i
 * lives at base[i * stride + e], 0 <= e < padded_d.  A flat model (n_tensors <= 1)
 * has padded_d = d rounded up to 4.  A parameter list of n_tensors tensors is
 * packed in list order, each tensor starting on a 4 KiB boundary (offset multiple
 * of 1024 elements) and the end of the list rounded up to 4; see
 * cocod_plan_layout.  The elements in the gaps are pads: the local step and line 6
 * never touch them, the mean kernels may carry them along, and they never
 * influence real elements (their contents are unspecified).  For full memory
 * bandwidth choose stride as a multiple of 1024 elements, so that every
 * worker's row starts on a 4 KiB boundary as well (any multiple of 4 is legal).
 */
typedef struct cocod_config {
    uint32_t struct_size;          /* sizeof(cocod_config); checked */
    uint32_t W;                    /* number of workers N of Algorithm 1, >= 1 */
    uint64_t d;                    /* parameters per worker (sum of tensor sizes), >= 1, < 2^34; and
                                      W * ceil(d / 1024) <= 2^31 - 1 (blocks of one launch; tensors of a
                                      list each round up on their own); the padded extent (every tensor
                                      of a list starts on a 1024-element boundary) must not exceed 2^34 - 1024 */
    uint32_t n_tensors;            /* 0 or 1: one flat vector; else length of tensor_numel */
    uint32_t grad;                 /* cocod_grad_kind */
    const uint64_t *tensor_numel;  /* host, [n_tensors], each >= 1, sum == d; copied */
    uint64_t bucket_bytes;         /* averaging granularity: tensors are grouped, in order, into buckets of
                                      at most this many bytes (a larger tensor gets its own); 0 = one bucket */
    float lr;                      /* gamma */
    float momentum;                /* mu of the experiments' optimizer; 0 = the update of Algorithm 1 */
    float weight_decay;            /* lambda, added to the gradient as lambda x */
    float noise_sigma;             /* sigma of the gradient noise (quadratic kind) */
    uint64_t seed;                 /* key of the counter-based generator */
    const float *weights;          /* host, [W], p_i = M_i / sum M_l, must sum to 1 within 1e-4; NULL = 1/W */
    const float *noise_sigma_w;    /* host, [W], copied; NULL = noise_sigma for every worker.  Heterogeneous
                                      workers (quadratic kind): worker i's mini-batch of M_i samples has
                                      gradient variance sigma^2 / M_i (bounded-variance assumption), so the
                                      caller passes sigma / sqrt(M_i); each finite and >= 0 */
    float *xA;                     /* device [W][stride]: holds the models at create time (the live buffer) */
    float *xB;                     /* device [W][stride]: second model buffer; need not be initialised */
    float *v;                      /* device [W][stride]: momentum buffer, caller-initialised (0 for a fresh
                                      run); may be NULL when momentum == 0 */
    float *mean;                   /* device [stride]: receives x^_t */
    const float *h;                /* device [W][stride]: curvatures (quadratic kind) */
    const float *c;                /* device [W][stride]: centres (quadratic kind) */
    uint64_t stride;               /* elements between consecutive workers; >= padded_d, multiple of 4 */
    void *compute_stream;          /* hipStream_t for Step II and line 6 (NULL = the null stream) */
    void *avg_stream;              /* hipStream_t for Step I; equal to compute_stream = no overlap.
                                      The share of the device that the averaging may occupy (the fraction a% of
                                      the paper's time-speedup analysis) is a property of THIS stream and
                                      therefore the caller's: create it with a compute-unit mask if the
                                      platform allows.  The library offers no field for it: it never creates
                                      streams, and on the machines this was built on the runtime refused
                                      masked streams, so the setting could not be tested. */
    uint32_t mlp_in, mlp_hidden, mlp_out, mlp_batch;   /* MLP kind: layer widths and mini-batch size.  Supported
                                      shapes (else COCOD_ERR_UNSUPPORTED): mlp_in and mlp_batch multiples of 128,
                                      mlp_batch <= 1024, mlp_hidden a multiple of 64, 1 <= mlp_out <= 16,
                                      mlp_hidden * (mlp_out rounded up to odd) <= 32768 */
    uint32_t flags;                /* COCOD_FLAG_* */
} cocod_config;

/*
 * Plan the packed layout of a parameter list (pure host arithmetic, no GPU).
 *   d, n_tensors, tensor_numel, bucket_bytes: as in cocod_config.
 *   padded_d      out: elements per worker including alignment pads.
 *   tensor_offset out, may be NULL: [n_tensors] element offset of each tensor inside a worker.
 *   n_buckets     out, may be NULL.
 *   bucket_begin  out, may be NULL: [n_tensors + 1] capacity; bucket b covers elements
 *                 [bucket_begin[b], bucket_begin[b+1]) of a worker; n_buckets + 1 entries written.
 * Follows the packed-buffer practice of the communication library the paper used
 * (tensor fusion); Algorithm 1 itself treats the model as one vector.
 */
int cocod_plan_layout(uint64_t d, uint32_t n_tensors, const uint64_t *tensor_numel,
                      uint64_t bucket_bytes, uint64_t *padded_d, uint64_t *tensor_offset,
                      uint32_t *n_buckets, uint64_t *bucket_begin);

/*
 * Initialisation of Algorithm 1: validates cfg, plans the layout, builds the
 * device chunk table and creates the events.  xA must already hold x_0^i for
 * every worker (the paper starts all workers from the same point; the library
 * does not require it).  On success *out receives the context (state IDLE,
 * step counter t = 0, live buffer xA).  On failure *out is NULL and
 * cocod_last_error(NULL) describes the reason.
 */
int cocod_create(const cocod_config *cfg, cocod_ctx **out);

/* Waits for both streams, frees what the context owns.  NULL is accepted. */
int cocod_destroy(cocod_ctx *ctx);

/*
 * Step II: enqueue k >= 0 local steps on compute_stream.  Each step computes the
 * stochastic gradient G_t^i at the live model and applies
 *     g = G + lambda x ;  v = mu v + g ;  x = x - gamma v          (mu = 0: x = x - gamma g)
 * and advances the step counter t by one.  Legal in both states; outside a round
 * it is plain local SGD.  The first step after cocod_average_begin reads the
 * stored model and writes the other model buffer, so storing x_t^i costs no copy.
 */
int cocod_local_steps(cocod_ctx *ctx, int k);

/*
 * Step I: marks the live models as the stored models x_t^i and (OVERLAP schedule)
 * enqueues the weighted mean on avg_stream, ordered after all work already on
 * compute_stream.  IDLE -> AVERAGING; COCOD_ERR_STATE if already averaging.
 */
int cocod_average_begin(cocod_ctx *ctx);

/*
 * Join and line 6: compute_stream waits for the mean and then applies
 * x^i = x^_t + (x^i - x_t^i) to every worker (with zero local steps since begin this
 * leaves every worker at x^_t).  AVERAGING -> IDLE; COCOD_ERR_STATE if not averaging.
 */
int cocod_average_end_apply(cocod_ctx *ctx);

/*
 * Step I and line 6 in ONE pass over the models, with nothing overlapped: the weighted mean of the
 * stored models is formed and x^i = x^_t + (x^i - x_t^i) applied by the same kernel (read x_t^i, read
 * x^i, write x^i: 12 + 4/W bytes per parameter; the mean is still written to `mean`).  This is the
 * sequential timeline that the paper's time-speedup analysis sets against the decoupled one
 * (communication AFTER the k local steps instead of beside them); it exists to measure what the
 * overlap buys.  Whatever schedule is set:
 *   - while a round is open (after cocod_average_begin and any local steps) it closes the round;
 *     if the overlapped schedule has already started the mean on avg_stream, compute_stream first
 *     waits for it (same values, so the result does not change);
 *   - while IDLE it is the blocking average of Local SGD: every worker is set to the weighted mean
 *     of the live models (a round with zero local steps).
 * Same bits as cocod_average_end_apply under any schedule.  Always ends IDLE.
 */
int cocod_average_apply_fused(cocod_ctx *ctx);

/*
 * Step II and line 6 together: k local steps of which the LAST one applies line 6 to the model it
 * has just computed, before storing it (x = x^_t + ((x - gamma v) - x_t^i) in the step kernel's
 * registers), and closes the round.  Same arithmetic, in the same order, as
 * cocod_local_steps(k) followed by cocod_average_end_apply, but the separate pass of line 6 over
 * the models (read x, read x_t, write x) disappears: 8 bytes per parameter less per round (24 at
 * k = 1, where the step reads the stored models anyway).  The join moves in front of the last
 * step, so the mean overlaps the first k-1 steps only.  k = 0 is cocod_average_end_apply.
 * AVERAGING -> IDLE; COCOD_ERR_STATE if no round is open.
 */
int cocod_local_steps_end_apply(cocod_ctx *ctx, int k);

/*
 * Step II with the caller's stochastic gradient: one local step x = x - gamma v,
 * v = mu v + (g + lambda x), with g [W][stride] in device memory in the same packed layout as the
 * models (pads ignored), ordered after the work already on compute_stream; the caller makes sure g
 * is complete on that stream and stays untouched until the step has run.  Advances t by one.  Legal
 * for every gradient kind.  close_round != 0 also applies line 6 inside this step and closes the
 * open round (as cocod_local_steps_end_apply does); COCOD_ERR_STATE if no round is open then.
 * Reads x, v, g and writes x, v: 20 bytes per parameter.
 */
int cocod_external_step(cocod_ctx *ctx, const float *g, int close_round);

/*
 * The same step of Step II with g stored as 16-bit brain floats (the upper 16 bits of an fp32, as
 * mixed-precision training produces): g is [W][stride] 16-bit elements, element (i, j) at
 * g[i * stride + j], device memory, 8-byte aligned.  Each value is widened exactly to fp32 and the
 * step then proceeds as cocod_external_step does.  18 bytes per parameter.  Same state rules and
 * error behaviour.
 */
int cocod_external_step_bf16(cocod_ctx *ctx, const uint16_t *g, int close_round);

/*
 * One whole pass of the while-loop body of Algorithm 1 (Step I and Step II side by side, then line
 * 6 and line 7) replayed from a HIP graph: the same kernels, in the same order and on the same two
 * branches, as cocod_average_begin + cocod_local_steps(k) + cocod_average_end_apply (fused_tail == 0)
 * or cocod_average_begin + cocod_local_steps_end_apply(k) (fused_tail != 0), with bit-identical
 * results, but submitted with ONE call instead of one per kernel and event: for small models, where
 * the launches and not the memory traffic bound a round.  The first call for a given (k, fused_tail,
 * schedule, live buffer) records and instantiates the graph (this allocates, and is the only slow
 * call); later calls only launch it on compute_stream.  The averaging branch runs inside the graph,
 * not on avg_stream.  Kernels in the graph read the step counter t from a device word the library
 * owns, so a replay continues the noise stream exactly where eager calls would.  Graph rounds and
 * the eager calls may be mixed freely between rounds.  cocod_set_lr drops the recorded graphs (it
 * then waits for compute_stream).  Launches inside a graph are not seen by cocod_step_timing.
 * Only legal while IDLE (COCOD_ERR_STATE otherwise); k >= 0; needs a built-in gradient when k > 0.
 * compute_stream must be a stream of the caller's own: the null stream cannot be captured, and a
 * context created on it gets COCOD_ERR_INVALID here, before any GPU call.
 */
int cocod_graph_round(cocod_ctx *ctx, int k, int fused_tail);

/* Choose how Step I is scheduled; only legal while IDLE.  Default COCOD_SCHED_OVERLAP. */
int cocod_set_schedule(cocod_ctx *ctx, int schedule);

/* Learning-rate schedules live in the caller: set gamma between steps. */
int cocod_set_lr(cocod_ctx *ctx, float lr);

/* The global step counter t (line 7).  It keys the noise / mini-batch streams, so a run that is
   saved (models, momentum, t) and restored continues bit-identically.  t < 2^32. */
int cocod_get_step(const cocod_ctx *ctx, uint64_t *step);
int cocod_set_step(cocod_ctx *ctx, uint64_t step);

/* Which of xA / xB currently holds the models (device pointer, [W][stride]). */
int cocod_live_model(const cocod_ctx *ctx, float **x_live);

/* 1 while a round is open (between begin and end_apply), else 0; < 0 on error. */
int cocod_is_averaging(const cocod_ctx *ctx);

/* Number of chunks of the step kernel's chunk table and number of buckets (for inspection). */
int cocod_get_plan(const cocod_ctx *ctx, uint64_t *padded_d, uint32_t *n_chunks, uint32_t *n_buckets);

/*
 * Measurement aid.  cocod_step_timing(ctx, n) with n > 0 makes the next n local-step kernel
 * launches carry the runtime's own start/stop timestamps (events on compute_stream, owned by the
 * context); n = 0 switches it off.  cocod_step_timing_read waits for compute_stream, returns the
 * summed kernel durations and the number of launches measured since the last read, and rearms.
 * A local step of the MLP kind is several kernels: its duration runs from the start of the first
 * to the end of the last.
 * Index 0 of both arrays: plain local steps; index 1: steps that carry line 6
 * (cocod_local_steps_end_apply's last step, the one-pass k = 1 step included); index 2: first steps
 * of a round that also form the mean (COCOD_SCHED_HEAD).
 */
int cocod_step_timing(cocod_ctx *ctx, int max_launches);
int cocod_step_timing_read(cocod_ctx *ctx, double total_ms[3], uint32_t launches[3]);

/*
 * Diagnostic: the weighted consensus distance sum_i p_i || x^ - x^i ||^2 of the live models, with
 * x^ = sum_i p_i x^i (the quantity that Lemma 2 of the paper bounds), over the real parameters
 * (alignment pads excluded).  Runs a reduction on compute_stream after the work already queued
 * there, WAITS for it and writes the scalar to *result (host).  The first call allocates a small
 * scratch buffer owned by the context.
 */
int cocod_consensus_distance(cocod_ctx *ctx, double *result);

/*
 * cocod_consensus_distance for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same kernels and same bits, but
 *   - the block partials live in a static device array of the library (2 MiB per GPU, held until the
 *     process ends) instead of a buffer allocated on first use;
 *   - the scalar goes to *result_device, DEVICE memory of the caller (one double, 8-byte aligned);
 *   - the call only enqueues on compute_stream and returns: no wait, no copy, no allocation of any
 *     kind (cocod_create has looked up the array's device address once for its GPU).
 * Limit: at most 2^18 chunks of 1024 parameters per worker (tensors of a list round up each on their
 * own), i.e. d up to 268 M for a flat model; beyond that COCOD_ERR_UNSUPPORTED.  All contexts on one
 * GPU share the array: calls that overlap in time on one GPU (two streams, two threads) race on it and
 * must be ordered by the caller; calls on one stream are ordered by the stream.  Nothing in the array
 * has to be cleared between calls.
 */
int cocod_consensus_distance_noalloc(cocod_ctx *ctx, double *result_device);

/*
 * Diagnostic (quadratic kind only): the objective of the paper's problem definition,
 * f(x) = sum_i p_i f_i(x) with f_i(x) = 1/2 sum_j h_ij (x_j - c_ij)^2, evaluated at the averaged
 * model x^ = sum_i p_i x^i of the live models, and || grad f(x^) ||^2, the quantity whose running
 * mean Theorem 1 bounds.  Real parameters only.  Same scheduling, waiting and scratch behaviour as
 * cocod_consensus_distance; both results are host doubles.  COCOD_ERR_INVALID for other kinds.
 */
int cocod_quadratic_objective(cocod_ctx *ctx, double *f_at_mean, double *grad_norm_sq_at_mean);

/* Block the host until both streams have drained. */
int cocod_sync(cocod_ctx *ctx);

/*
 * Draw the synthetic objective on the device (quadratic kind): fills the buffers
 * behind cfg.h and cfg.c on compute_stream with h_ij = 0.5 + 1.5 U and c_ij ~ N(0,1)
 * from the counter-based generator (streams 1 and 2 of the seed), pads set to 0.
 * For models too large to generate on the host.
 */
int cocod_fill_quadratic(cocod_ctx *ctx);

/*
 * Inspection of the MLP kind's work space after a local step (device pointers owned by the
 * context, valid until cocod_destroy; any output pointer may be NULL):
 *   X [W][batch][mlp_in] last mini-batch, H [W][batch][mlp_hidden] relu output,
 *   dA [W][batch][mlp_hidden] gradient at the hidden pre-activation,
 *   dZ [W][batch][*dz_pitch] gradient at the logits (first mlp_out entries of each row),
 *   y [W][batch] labels.
 * X and y are those of the most recent local step: the context keeps two mini-batch buffers (a step
 * draws the next step's batch into the other one while its output layer runs), so the two pointers
 * change from step to step - ask again after each.
 */
int cocod_mlp_workspace(const cocod_ctx *ctx, float **X, float **H, float **dA, float **dZ, int32_t **y,
                        uint32_t *dz_pitch);

/*
 * Generator check: n standard normals of stream `tag` for (worker, step) at flat
 * indices j0 .. j0+n-1, written to device memory `out` on `stream`, produced by the
 * same device routine as the local step's noise (fast = 1) or by the accurate routine
 * used for the objective data (fast = 0).  No context needed.
 */
int cocod_debug_normals(void *stream, uint64_t seed, uint32_t tag, uint32_t worker, uint32_t step,
                        uint64_t j0, uint64_t n, int fast, float *out);

/*
 * Measurement aid: plain streaming copy of n fp32 elements (n multiple of 4, both pointers device,
 * 16-byte aligned, not overlapping) on `stream`.  A kernel of exactly known traffic (4n bytes read,
 * 4n written) against which hardware memory counters are calibrated.  No context needed.
 */
int cocod_debug_copy(void *stream, const float *src, float *dst, uint64_t n);

/* Last error text of ctx, or of the last failed cocod_create / context-free call when ctx is NULL.
   Never NULL; owned by the library; valid until the next call on the same context / thread. */
const char *cocod_last_error(const cocod_ctx *ctx);

/* Library version, major * 1000 + minor. */
int cocod_version(void);

#ifdef __cplusplus
}
#endif
#endif /* COCOD_H */
