// Internal declarations shared by the host side of libcocod and its kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cocod {

// One block of the local-step kernel serves one chunk: up to kChunkElems
// consecutive elements of ONE tensor of one worker, one 16-byte quad per thread.
constexpr uint32_t kStepThreads = 256;
constexpr uint32_t kChunkElems = kStepThreads * 4;

// Stream tags: fourth counter word of the generator, keeps random streams disjoint.
enum : uint32_t { kTagNoise = 0, kTagH = 1, kTagC = 2, kTagMlpX = 4, kTagMlpY = 5 };

struct Chunk {
    uint64_t glob_off;  // unpadded global parameter index of the chunk's first element
    uint32_t mem_quad;  // 16-byte quad offset inside a worker's padded row (element offset / 4)
    uint32_t n;         // real elements in the chunk (1 .. kChunkElems)
};
static_assert(sizeof(Chunk) == 16, "one 16-byte scalar load per block");

struct StepParams {
    const Chunk *table;
    uint32_t n_chunks;
    uint32_t W;
    uint64_t stride;
    const float *x_in;   // models read by the step
    float *x_out;        // models written by the step (== x_in for an in-place step)
    float *v;            // momentum, unused when momentum == 0
    const float *h;
    const float *c;
    const float *g;      // non-null: the stochastic gradient is read from here ([W][stride]) instead of h, c, noise
    uint32_t g_bf16;     // g holds 16-bit brain floats (same element layout, half the bytes)
    const float *snap;   // non-null: this is the last step of a round and line 6 is applied to its result
    const float *mean;   //           x = mean + (x_new - snap); mean is [stride], valid when snap is set
    float lr, momentum, weight_decay, sigma;
    const float *sigma_w; // non-null: device [W], worker i's noise standard deviation instead of sigma
    uint32_t key0, key1; // generator key (seed low, seed high)
    uint32_t step;       // global step counter t (relative to *step_base when that is set)
    const uint32_t *step_base;   // non-null inside a replayable graph: device word holding t at the start of the replay
    uint32_t panel_tiles;      // line-6 step only, non-zero: blocks run in panels of this many tiles, worker by worker
                               // inside a panel (for a mean larger than the cache); 0 = grid (tiles, workers)
    float *mean_out;           // non-null: first step of a round that also forms the mean of the models it reads
    const float *weights;      //           (Step I inside Step II's first pass); p_i, nullptr = 1/W
};

// One local step of all W workers (local_step.hip).  The kind of step follows from the parameters:
//   snap == nullptr, mean_out == nullptr   plain step
//   snap set                               last step of a round, line 6 applied to its result
//   mean_out set                           first step of a round that also forms the mean of the models it reads
//   mean_out and snap (== x_in) set        k = 1: mean, step and line 6 in one pass
// start / stop: optional events that receive the kernel's own begin / end timestamps.
hipError_t launch_local_step(hipStream_t stream, const StepParams &p, hipEvent_t start = nullptr,
                             hipEvent_t stop = nullptr);
// Line 6 alone, in place on p.x_out (== p.x_in): x = mean + (x - snap), one launch for the whole parameter list
// (uses table, n_chunks, W, stride, x_in, x_out, snap, mean, panel_tiles of p).
hipError_t launch_line6(hipStream_t stream, const StepParams &p);
// Column quads per lane (1 or 2) with which the mean-forming steps hold the W rows of a tile in LDS;
// 0 = W is too large for them (the mean is then formed by a pass of its own).
int local_step_mean_quads_per_lane(uint32_t W, bool one_pass);

// mean[e] = sum_i p_i snap[i][e] for e in [begin, end) (both multiples of 4);
// weights == nullptr means p_i = 1/W.  max_blocks != 0 caps the grid (single-wave blocks that stride over
// the columns): a mean that runs beside a kernel it should not starve.
hipError_t launch_wmean(hipStream_t stream, const float *snap, uint64_t stride, uint32_t W,
                        uint64_t begin, uint64_t end, const float *weights, float *mean, uint32_t max_blocks);

// the mean and line 6, x[i][e] = mean[e] + (x[i][e] - snap[i][e]), in one pass; mean is still written
hipError_t launch_mean_correct(hipStream_t stream, float *x, const float *snap, uint64_t stride,
                               uint32_t W, uint64_t begin, uint64_t end, const float *weights,
                               float *mean);

// out[0] = sum_i p_i || xbar - x_i ||^2 over the real (unpadded) elements; partial: n_chunks doubles of scratch
hipError_t launch_consensus_distance(hipStream_t stream, const Chunk *table, uint32_t n_chunks, const float *x,
                                     uint64_t stride, uint32_t W, const float *weights, double *partial, double *out);

// out[0] = f(xbar) = sum_i p_i 1/2 sum_j h_ij (xbar_j - c_ij)^2, out[1] = || grad f(xbar) ||^2, xbar = sum_i p_i x_i;
// partial: 2 * n_chunks doubles of scratch
hipError_t launch_quadratic_objective(hipStream_t stream, const Chunk *table, uint32_t n_chunks, const float *x,
                                      const float *h, const float *c, uint64_t stride, uint32_t W, const float *weights,
                                      double *partial, double *out);

hipError_t launch_fill_quadratic(hipStream_t stream, const Chunk *table, uint32_t n_chunks, uint32_t W,
                                 uint64_t stride, uint64_t padded_d, float *h, float *c,
                                 uint32_t key0, uint32_t key1);

// One local step of W perceptron workers (MLP gradient kind).
struct MlpParams {
    uint32_t W, n_in, n_hid, n_out, batch;
    uint64_t stride;          // elements between workers in x_in / x_out / v
    const float *x_in;        // flat parameters W1 | b1 | W2 | b2 per worker
    float *x_out;             // == x_in for an in-place step
    float *v;                 // momentum, unused when momentum == 0
    float lr, momentum, weight_decay;
    uint32_t key0, key1, step;
    const uint32_t *step_base;   // as in StepParams
    const float *snap;        // non-null: last step of a round; line 6 is applied to every updated parameter
    const float *mean;        //           before it is stored: x = mean + (x_new - snap)   (mean is [stride])
    // work space owned by the context
    float *X;                 // [W][batch][n_in]   this step's mini-batch
    float *X_next;            // same shape, the other batch buffer: the step also draws the NEXT step's
    int32_t *y_next;          //   mini-batch and labels into these (null: it does not)
    bool have_batch;          // X and y already hold this step's mini-batch (drawn by the previous step)
    float *H;                 // [W][batch][n_hid]  relu output
    float *dA;                // [W][batch][n_hid]  gradient at the hidden pre-activation
    float *dZ;                // [W][batch][mlp_dz_pitch()]  gradient at the logits
    int32_t *y;               // [W][batch] labels
};

bool mlp_shape_supported(uint32_t n_in, uint32_t n_hid, uint32_t n_out, uint32_t batch);
size_t mlp_dz_pitch();
// start / stop (may be null) receive the start timestamp of the step's first kernel and the end timestamp of its last
hipError_t launch_mlp_step(hipStream_t stream, const MlpParams &p, hipEvent_t start, hipEvent_t stop);

hipError_t launch_copy(hipStream_t stream, const float *src, float *dst, uint64_t n_quads);

// *word = value  /  *word += inc : the device copy of the step counter that graph replays read
hipError_t launch_set_word(hipStream_t stream, uint32_t *word, uint32_t value);
hipError_t launch_add_word(hipStream_t stream, uint32_t *word, uint32_t inc);

hipError_t launch_debug_normals(hipStream_t stream, uint32_t key0, uint32_t key1, uint32_t tag,
                                uint32_t worker, uint32_t step, uint64_t j0, uint64_t n, int fast,
                                float *out);

}  // namespace cocod
