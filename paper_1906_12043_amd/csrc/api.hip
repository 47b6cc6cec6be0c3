// Host side of libcocod: argument validation, layout planning, the state machine of
// one CoCoD-SGD round (Algorithm 1: Step I and Step II in parallel, then line 6)
// and the stream/event choreography that makes the two steps overlap on one GPU.
// No arithmetic on model data happens here; every step of the round is a kernel.
#include "../../include/cocod.h"
#include "internal.hpp"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using cocod::Chunk;

struct cocod_ctx {
    cocod_config cfg{};                 // copy of the caller's config (host array pointers cleared)
    std::vector<uint64_t> tensor_numel, tensor_offset, bucket_begin;
    uint64_t padded_d = 0;
    std::vector<Chunk> chunks;
    Chunk *d_chunks = nullptr;          // device copy of the chunk table (owned)
    float *d_weights = nullptr;         // device copy of p_i (owned), nullptr = uniform
    float *d_sigma_w = nullptr;         // device copy of the per-worker noise scale (owned), nullptr = cfg.noise_sigma
    double *d_reduce = nullptr;         // scratch of the consensus-distance reduction (owned, allocated on first use)
    double *static_scratch = nullptr;   // this GPU's copy of the library's static scratch array (not owned)
    float *mlp_ws = nullptr;            // MLP kind: work space (owned); mlp holds the pointers carved from it
    cocod::MlpParams mlp{};
    // MLP kind: two mini-batch buffers.  A local step draws the NEXT step's batch into the other one while
    // its output layer runs, so that only the first step after anything else draws its own up front.
    float *mlp_X[2] = {nullptr, nullptr};
    int32_t *mlp_y[2] = {nullptr, nullptr};
    uint32_t compute_units = 0;         // of the device the context was created on
    uint32_t batch_buf = 0;             // buffer the next eager step takes its batch from
    uint32_t batch_last = 0;            // buffer the most recent step took its batch from
    uint64_t batch_ready_step = ~0ull;  // mlp_X[batch_buf] holds the batch of this step index (~0: of none)
    hipEvent_t ev_snap = nullptr;       // compute stream reached the point where the models are stored
    hipEvent_t ev_mean = nullptr;       // mean of the stored models is complete
    hipStream_t s_compute = nullptr, s_avg = nullptr;
    float *live = nullptr;              // buffer holding the current models
    float *spare = nullptr;             // the other model buffer
    const float *snap = nullptr;        // stored models x_t^i of the open round (aliases one of the two)
    bool averaging = false;             // a round is open
    bool store_pending = false;         // next local step must write out of place (keeps the stored models intact)
    bool mean_pending = false;          // the open round's mean has not been enqueued yet (every schedule but OVERLAP)
    int schedule = COCOD_SCHED_OVERLAP;
    uint64_t step = 0;                  // global step counter t
    bool dry = false;
    bool timing = false;                // bracket step launches with start/stop events
    std::vector<hipEvent_t> t_start, t_stop;   // event pool for step timing (owned)
    std::vector<char> t_kind;           // per timed launch: 0 plain step, 1 step with line 6
    size_t t_used = 0;
    // replayable rounds: one instantiated graph per (k, variant, schedule, which buffer is live)
    struct RoundGraph { int k; int fused_tail; int schedule; bool live_is_A; uint32_t batch_buf; bool batch_ready; hipGraphExec_t exec; };
    std::vector<RoundGraph> graphs;     // owned
    uint32_t *d_step = nullptr;         // device copy of t that captured kernels read (owned)
    uint64_t d_step_value = ~0ull;      // what *d_step holds once the work queued on the compute stream has run
    bool capturing = false;             // enqueue_step runs under stream capture: step relative to *d_step
    uint64_t capture_base = 0;          // value of `step` when the capture began
    std::string err;
};

namespace {

// Scratch of cocod_consensus_distance_noalloc: block partials of the reduction, in device memory that
// exists from the moment the library is loaded, so the call never allocates.  One copy per GPU, held
// until the process ends; every call on a GPU shares that GPU's copy.  In host code the array's name
// is only a handle: the device address comes from hipGetSymbolAddress (scratch_for_current_device).
constexpr uint32_t kNoAllocMaxChunks = 1u << 18;                       // 2^18 chunks of 1024 = 268 M parameters per worker
static __device__ __align__(256) double scratch[2 + kNoAllocMaxChunks];   // result words, then one partial per chunk (2 MiB)

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double *g_scratch_ptr[kMaxDevices] = {};                               // device address of `scratch`, per device

// Device address of this GPU's copy of `scratch`; looked up once per device, with that device current.
hipError_t scratch_for_current_device(double **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        double *ptr = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

thread_local std::string g_err;         // errors that have no context to live in

int fail(cocod_ctx *ctx, int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf; else g_err = buf;
    return code;
}

int hip_fail(cocod_ctx *ctx, hipError_t e, const char *what)
{
    return fail(ctx, COCOD_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define COCOD_HIP(ctx, call)                                             \
    do {                                                                 \
        hipError_t e_ = (call);                                          \
        if (e_ != hipSuccess) return hip_fail((ctx), e_, #call);         \
    } while (0)

// Block order of a line-6 step whose mean exceeds the cache: panels of this many tiles (4 MiB of the mean;
// every worker streams 4 MiB of each of its arrays per panel).  Measured at W = 16, d = 138 M: 9.9 ms per
// launch, against 10.6 ms with the worker fastest for every single tile and 11.4 ms on the (tiles, workers)
// grid, where the mean comes from memory once per worker.
constexpr uint32_t kPanelTiles = 16384;

// A mean vector up to this size is expected to stay in the 256 MB last-level cache while the W
// workers of a line-6 step read it one after the other.
constexpr uint64_t kMeanCacheBytes = 128ull << 20;
// one grid dimension holds fewer than 2^32 threads
constexpr uint64_t kMaxThreadsPerGridDim = 1ull << 32;
// the mean-forming steps launch up to four 1024-thread blocks per chunk in one grid dimension
constexpr uint64_t kMaxChunksMeanStep = 1ull << 20;

inline uint64_t round_up4(uint64_t n) { return (n + 3u) & ~static_cast<uint64_t>(3u); }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Layout of a parameter list: tensors in order, each start rounded up to a chunk (1024 elements =
// 4 KiB: measured 10 % faster streaming than 16-byte alignment, because every full chunk of the step
// kernel then covers whole 4 KiB blocks of memory); the end of the list rounded up to 4 elements.
// Buckets are maximal runs of tensors whose padded extent fits bucket_bytes.
int plan(uint64_t d, uint32_t n_tensors, const uint64_t *numel, uint64_t bucket_bytes,
         std::vector<uint64_t> &sizes, std::vector<uint64_t> &offsets, std::vector<uint64_t> &bucket_begin,
         uint64_t &padded_d)
{
    if (d == 0) return fail(nullptr, COCOD_ERR_INVALID, "d must be >= 1");
    if (d >= (1ull << 34)) return fail(nullptr, COCOD_ERR_INVALID, "d must be < 2^34 (generator counter width)");
    sizes.clear(); offsets.clear(); bucket_begin.clear();
    if (n_tensors <= 1) {
        if (n_tensors == 1 && numel && numel[0] != d)
            return fail(nullptr, COCOD_ERR_INVALID, "tensor_numel[0] != d");
        sizes.push_back(d);
    } else {
        if (!numel) return fail(nullptr, COCOD_ERR_INVALID, "tensor_numel is NULL with n_tensors > 1");
        uint64_t sum = 0;
        for (uint32_t t = 0; t < n_tensors; ++t) {
            if (numel[t] == 0) return fail(nullptr, COCOD_ERR_INVALID, "tensor %u is empty", t);
            if (numel[t] > d) return fail(nullptr, COCOD_ERR_INVALID, "tensor %u larger than d", t);
            sum += numel[t];
            sizes.push_back(numel[t]);
        }
        if (sum != d) return fail(nullptr, COCOD_ERR_INVALID, "tensor sizes sum to %llu, d is %llu",
                                  (unsigned long long)sum, (unsigned long long)d);
    }
    uint64_t at = 0;
    for (uint64_t n : sizes) {
        at = (at + cocod::kChunkElems - 1) / cocod::kChunkElems * cocod::kChunkElems;
        offsets.push_back(at);
        at += n;
    }
    padded_d = round_up4(at);
    // fewer than 2^24 chunks: the chunk table addresses memory in 32-bit quad offsets, and four single-wave
    // blocks (or one 256-thread block) per chunk must stay below 2^32 threads in one grid dimension
    if (padded_d > (1ull << 34) - cocod::kChunkElems)
        return fail(nullptr, COCOD_ERR_INVALID, "the padded parameter list holds %llu elements, more than 2^34 - 1024",
                    (unsigned long long)padded_d);
    const uint64_t cap = bucket_bytes / sizeof(float);
    bucket_begin.push_back(0);
    uint64_t bucket_start = 0;
    for (size_t t = 1; t < sizes.size(); ++t) {
        const uint64_t end_with_t = round_up4(offsets[t] + sizes[t]);
        if (cap != 0 && end_with_t - bucket_start > cap) {   // tensor t does not fit: it opens a new bucket
            bucket_begin.push_back(offsets[t]);
            bucket_start = offsets[t];
        }
    }
    bucket_begin.push_back(padded_d);
    return COCOD_OK;
}

bool overlap(const void *a, uint64_t a_bytes, const void *b, uint64_t b_bytes)
{
    if (!a || !b) return false;
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + b_bytes && b0 < a0 + a_bytes;
}

int validate(const cocod_config *cfg, uint64_t padded_d)
{
    const unsigned known_flags = COCOD_FLAG_DRY_RUN;
    if (cfg->flags & ~known_flags) return fail(nullptr, COCOD_ERR_INVALID, "unknown flag bits 0x%x", cfg->flags & ~known_flags);
    if (cfg->W == 0 || cfg->W > 65535u) return fail(nullptr, COCOD_ERR_INVALID, "W must be in 1..65535");
    if (cfg->grad != COCOD_GRAD_QUADRATIC && cfg->grad != COCOD_GRAD_MLP && cfg->grad != COCOD_GRAD_EXTERNAL)
        return fail(nullptr, COCOD_ERR_INVALID, "unknown gradient kind %u", cfg->grad);
    if (cfg->stride < padded_d || (cfg->stride & 3u))
        return fail(nullptr, COCOD_ERR_INVALID, "stride %llu must be a multiple of 4 and >= padded size %llu",
                    (unsigned long long)cfg->stride, (unsigned long long)padded_d);
    if (!std::isfinite(cfg->lr)) return fail(nullptr, COCOD_ERR_INVALID, "lr is not finite");
    if (!(cfg->momentum >= 0.0f && cfg->momentum < 1.0f)) return fail(nullptr, COCOD_ERR_INVALID, "momentum must be in [0,1)");
    if (!(cfg->weight_decay >= 0.0f) || !std::isfinite(cfg->weight_decay)) return fail(nullptr, COCOD_ERR_INVALID, "weight_decay must be finite and >= 0");
    if (!(cfg->noise_sigma >= 0.0f) || !std::isfinite(cfg->noise_sigma)) return fail(nullptr, COCOD_ERR_INVALID, "noise_sigma must be finite and >= 0");
    if (!cfg->xA || !cfg->xB || !cfg->mean) return fail(nullptr, COCOD_ERR_INVALID, "xA, xB and mean must not be NULL");
    if (cfg->momentum != 0.0f && !cfg->v) return fail(nullptr, COCOD_ERR_INVALID, "v must not be NULL when momentum != 0");
    if (cfg->grad == COCOD_GRAD_QUADRATIC && (!cfg->h || !cfg->c))
        return fail(nullptr, COCOD_ERR_INVALID, "h and c must not be NULL for the quadratic gradient");
    const void *ptrs[] = { cfg->xA, cfg->xB, cfg->v, cfg->mean, cfg->h, cfg->c };
    const char *names[] = { "xA", "xB", "v", "mean", "h", "c" };
    for (int i = 0; i < 6; ++i)
        if (!aligned16(ptrs[i])) return fail(nullptr, COCOD_ERR_INVALID, "%s is not 16-byte aligned", names[i]);
    const uint64_t big = static_cast<uint64_t>(cfg->W) * cfg->stride * sizeof(float);
    const uint64_t sizes[] = { big, big, big, cfg->stride * sizeof(float), big, big };
    for (int i = 0; i < 6; ++i)
        for (int j = i + 1; j < 6; ++j)
            if (overlap(ptrs[i], sizes[i], ptrs[j], sizes[j]))
                return fail(nullptr, COCOD_ERR_INVALID, "%s and %s overlap", names[i], names[j]);
    if (cfg->weights) {
        double sum = 0.0;
        for (uint32_t i = 0; i < cfg->W; ++i) {
            if (!(cfg->weights[i] >= 0.0f) || !std::isfinite(cfg->weights[i]))
                return fail(nullptr, COCOD_ERR_INVALID, "weights[%u] must be finite and >= 0", i);
            sum += cfg->weights[i];
        }
        if (std::fabs(sum - 1.0) > 1e-4) return fail(nullptr, COCOD_ERR_INVALID, "weights sum to %g, not 1", sum);
    }
    if (cfg->noise_sigma_w)
        for (uint32_t i = 0; i < cfg->W; ++i)
            if (!(cfg->noise_sigma_w[i] >= 0.0f) || !std::isfinite(cfg->noise_sigma_w[i]))
                return fail(nullptr, COCOD_ERR_INVALID, "noise_sigma_w[%u] must be finite and >= 0", i);
    if (cfg->grad == COCOD_GRAD_MLP) {
        const uint64_t want = static_cast<uint64_t>(cfg->mlp_in) * cfg->mlp_hidden + cfg->mlp_hidden +
                              static_cast<uint64_t>(cfg->mlp_hidden) * cfg->mlp_out + cfg->mlp_out;
        if (cfg->d != want)
            return fail(nullptr, COCOD_ERR_INVALID, "d is %llu but the MLP has %llu parameters",
                        (unsigned long long)cfg->d, (unsigned long long)want);
        if (cfg->n_tensors > 1) return fail(nullptr, COCOD_ERR_INVALID, "the MLP parameters are one flat tensor");
        if (!cocod::mlp_shape_supported(cfg->mlp_in, cfg->mlp_hidden, cfg->mlp_out, cfg->mlp_batch))
            return fail(nullptr, COCOD_ERR_UNSUPPORTED,
                        "MLP shape: mlp_in and mlp_batch must be multiples of 128 (batch <= 1024), mlp_hidden a "
                        "multiple of 64, 1 <= mlp_out <= 16, mlp_hidden * (mlp_out rounded up to odd) <= 32768");
    }
    return COCOD_OK;
}

void release(cocod_ctx *ctx)
{
    if (!ctx->dry) {
        if (ctx->d_chunks) (void)hipFree(ctx->d_chunks);
        if (ctx->d_weights) (void)hipFree(ctx->d_weights);
        if (ctx->d_sigma_w) (void)hipFree(ctx->d_sigma_w);
        if (ctx->mlp_ws) (void)hipFree(ctx->mlp_ws);
        if (ctx->d_reduce) (void)hipFree(ctx->d_reduce);
        if (ctx->d_step) (void)hipFree(ctx->d_step);
        for (auto &g : ctx->graphs) (void)hipGraphExecDestroy(g.exec);
        if (ctx->ev_snap) (void)hipEventDestroy(ctx->ev_snap);
        if (ctx->ev_mean) (void)hipEventDestroy(ctx->ev_mean);
        for (hipEvent_t e : ctx->t_start) (void)hipEventDestroy(e);
        for (hipEvent_t e : ctx->t_stop) (void)hipEventDestroy(e);
    }
    delete ctx;
}

// Step I arithmetic on `stream`, one launch per bucket.
int enqueue_mean(cocod_ctx *ctx, hipStream_t stream)
{
    // Perceptron workers, mean on the averaging stream: the kernel beside it is the forward contraction, which
    // needs a steady trickle of its weight stream and little bandwidth.  At full width the mean takes the memory
    // system for its 43 us and the contraction loses 36 of them; in four single-wave blocks per compute unit it
    // takes longer and the round is 15 us shorter (W = 16, 3072-1024-10, k = 2: 0.705 -> 0.690 ms; two blocks per
    // unit: 0.700, one or eight: 0.709; k = 1, where the step waits for the mean: unchanged, 0.392 ms).
    const uint32_t cap = ctx->cfg.grad == COCOD_GRAD_MLP && stream == ctx->s_avg && ctx->s_avg != ctx->s_compute
                             ? 4u * ctx->compute_units : 0u;
    for (size_t b = 0; b + 1 < ctx->bucket_begin.size(); ++b)
        COCOD_HIP(ctx, cocod::launch_wmean(stream, ctx->snap, ctx->cfg.stride, ctx->cfg.W, ctx->bucket_begin[b],
                                           ctx->bucket_begin[b + 1], ctx->d_weights, ctx->cfg.mean, cap));
    return COCOD_OK;
}

// Make the open round's mean available to line 6 on the compute stream: enqueue it there if no
// earlier call has (sequential schedules), or join the averaging stream (overlapped schedule).
int mean_before_line6(cocod_ctx *ctx)
{
    if (ctx->mean_pending) {
        const int rc = enqueue_mean(ctx, ctx->s_compute);
        if (rc != COCOD_OK) return rc;
        ctx->mean_pending = false;
    } else if (ctx->schedule == COCOD_SCHED_OVERLAP && ctx->s_avg != ctx->s_compute) {
        COCOD_HIP(ctx, hipStreamWaitEvent(ctx->s_compute, ctx->ev_mean, 0));
    }
    return COCOD_OK;
}

}  // namespace

extern "C" {

int cocod_version(void) { return 1000; }

const char *cocod_last_error(const cocod_ctx *ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

int cocod_plan_layout(uint64_t d, uint32_t n_tensors, const uint64_t *tensor_numel, uint64_t bucket_bytes,
                      uint64_t *padded_d, uint64_t *tensor_offset, uint32_t *n_buckets, uint64_t *bucket_begin)
{
    if (!padded_d) return fail(nullptr, COCOD_ERR_INVALID, "padded_d is NULL");
    std::vector<uint64_t> sizes, offsets, buckets;
    uint64_t pd = 0;
    const int rc = plan(d, n_tensors, tensor_numel, bucket_bytes, sizes, offsets, buckets, pd);
    if (rc != COCOD_OK) return rc;
    *padded_d = pd;
    if (tensor_offset) std::memcpy(tensor_offset, offsets.data(), offsets.size() * sizeof(uint64_t));
    if (n_buckets) *n_buckets = static_cast<uint32_t>(buckets.size() - 1);
    if (bucket_begin) std::memcpy(bucket_begin, buckets.data(), buckets.size() * sizeof(uint64_t));
    return COCOD_OK;
}

int cocod_create(const cocod_config *cfg, cocod_ctx **out)
{
    if (out) *out = nullptr;
    if (!cfg || !out) return fail(nullptr, COCOD_ERR_INVALID, "cfg and out must not be NULL");
    if (cfg->struct_size != sizeof(cocod_config))
        return fail(nullptr, COCOD_ERR_INVALID, "struct_size %u does not match this library (%zu)", cfg->struct_size,
                    sizeof(cocod_config));
    cocod_ctx *ctx = new (std::nothrow) cocod_ctx;
    if (!ctx) return fail(nullptr, COCOD_ERR_NOMEM, "out of host memory");
    int rc = plan(cfg->d, cfg->n_tensors, cfg->tensor_numel, cfg->bucket_bytes, ctx->tensor_numel, ctx->tensor_offset,
                  ctx->bucket_begin, ctx->padded_d);
    if (rc == COCOD_OK) rc = validate(cfg, ctx->padded_d);
    if (rc != COCOD_OK) { delete ctx; return rc; }

    ctx->cfg = *cfg;
    ctx->cfg.tensor_numel = nullptr;
    ctx->dry = (cfg->flags & COCOD_FLAG_DRY_RUN) != 0;
    ctx->s_compute = static_cast<hipStream_t>(cfg->compute_stream);
    ctx->s_avg = static_cast<hipStream_t>(cfg->avg_stream);
    ctx->live = cfg->xA;
    ctx->spare = cfg->xB;

    uint64_t global = 0;
    for (size_t t = 0; t < ctx->tensor_numel.size(); ++t) {
        const uint64_t span = cocod::kChunkElems;
        for (uint64_t off = 0; off < ctx->tensor_numel[t]; off += span) {
            const uint64_t left = ctx->tensor_numel[t] - off;
            Chunk ck{};
            ck.mem_quad = static_cast<uint32_t>((ctx->tensor_offset[t] + off) / 4);
            ck.glob_off = global + off;
            ck.n = static_cast<uint32_t>(left < span ? left : span);
            ctx->chunks.push_back(ck);
        }
        global += ctx->tensor_numel[t];
    }
    // Launch limits.  A grid dimension holds fewer than 2^32 THREADS.  The (tiles, workers) grid of the local
    // step has up to four single-wave blocks per chunk in x (fewer than 2^24 chunks: checked with the layout) and W <= 65535
    // in y (checked above); the orders that put more into ONE dimension (panels of a line-6 step, 1024-thread
    // blocks of the mean-forming steps) are only used below that limit (see enqueue_step).  The total is capped
    // as well, so that block counts stay inside 32-bit arithmetic everywhere.
    if (ctx->chunks.size() * static_cast<uint64_t>(cfg->W) > 0x7fffffffull) {
        delete ctx;
        return fail(nullptr, COCOD_ERR_INVALID, "W * d is too large for one launch (more than 2^31 chunks of 1024 elements)");
    }

    std::vector<float> weights;
    if (cfg->weights) weights.assign(cfg->weights, cfg->weights + cfg->W);
    ctx->cfg.weights = nullptr;
    std::vector<float> sigma_w;
    if (cfg->noise_sigma_w && cfg->grad == COCOD_GRAD_QUADRATIC) sigma_w.assign(cfg->noise_sigma_w, cfg->noise_sigma_w + cfg->W);
    ctx->cfg.noise_sigma_w = nullptr;

    if (!ctx->dry) {
        hipError_t e = hipMalloc(reinterpret_cast<void **>(&ctx->d_chunks), ctx->chunks.size() * sizeof(Chunk));
        if (e == hipSuccess)
            e = hipMemcpy(ctx->d_chunks, ctx->chunks.data(), ctx->chunks.size() * sizeof(Chunk), hipMemcpyHostToDevice);
        if (e == hipSuccess && !weights.empty()) {
            e = hipMalloc(reinterpret_cast<void **>(&ctx->d_weights), weights.size() * sizeof(float));
            if (e == hipSuccess)
                e = hipMemcpy(ctx->d_weights, weights.data(), weights.size() * sizeof(float), hipMemcpyHostToDevice);
        }
        if (e == hipSuccess && !sigma_w.empty()) {
            e = hipMalloc(reinterpret_cast<void **>(&ctx->d_sigma_w), sigma_w.size() * sizeof(float));
            if (e == hipSuccess)
                e = hipMemcpy(ctx->d_sigma_w, sigma_w.data(), sigma_w.size() * sizeof(float), hipMemcpyHostToDevice);
        }
        if (e == hipSuccess && cfg->grad == COCOD_GRAD_MLP) {      // one work-space block, carved below
            const size_t wb = static_cast<size_t>(cfg->W) * cfg->mlp_batch;
            const size_t n_x = wb * cfg->mlp_in, n_h = wb * cfg->mlp_hidden, n_z = wb * cocod::mlp_dz_pitch();
            e = hipMalloc(reinterpret_cast<void **>(&ctx->mlp_ws), (2 * n_x + 2 * n_h + n_z + 2 * wb) * sizeof(float));
            if (e == hipSuccess) {
                float *at = ctx->mlp_ws;
                ctx->mlp_X[0] = at; at += n_x;
                ctx->mlp_X[1] = at; at += n_x;
                ctx->mlp.H = at;  at += n_h;
                ctx->mlp.dA = at; at += n_h;
                ctx->mlp.dZ = at; at += n_z;
                ctx->mlp_y[0] = reinterpret_cast<int32_t *>(at); at += wb;
                ctx->mlp_y[1] = reinterpret_cast<int32_t *>(at);
                ctx->mlp.X = ctx->mlp_X[0];
                ctx->mlp.y = ctx->mlp_y[0];
            }
        }
        if (e == hipSuccess) {
            int dev = 0, cus = 0;
            e = hipGetDevice(&dev);
            if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
            ctx->compute_units = cus > 0 ? static_cast<uint32_t>(cus) : 0u;
        }
        if (e == hipSuccess) e = scratch_for_current_device(&ctx->static_scratch);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_snap, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_mean, hipEventDisableTiming);
        if (e != hipSuccess) {
            const int code = (e == hipErrorOutOfMemory) ? COCOD_ERR_NOMEM : COCOD_ERR_HIP;
            fail(nullptr, code, "cocod_create: %s", hipGetErrorString(e));
            release(ctx);
            return code;
        }
    }
    *out = ctx;
    return COCOD_OK;
}

int cocod_destroy(cocod_ctx *ctx)
{
    if (!ctx) return COCOD_OK;
    int rc = COCOD_OK;
    if (!ctx->dry) {
        hipError_t e = hipStreamSynchronize(ctx->s_avg);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->s_compute);
        if (e != hipSuccess) rc = hip_fail(nullptr, e, "cocod_destroy");
    }
    release(ctx);
    return rc;
}

int cocod_sync(cocod_ctx *ctx)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (ctx->dry) return COCOD_OK;
    COCOD_HIP(ctx, hipStreamSynchronize(ctx->s_avg));
    COCOD_HIP(ctx, hipStreamSynchronize(ctx->s_compute));
    return COCOD_OK;
}

// Panel order of the kernels that apply line 6 (see kPanelTiles): 4 * chunks * W single-wave blocks plus the
// padding of the last panel must fit one grid dimension.
static uint32_t panel_tiles_for(const cocod_ctx *ctx)
{
    return ctx->padded_d * sizeof(float) > kMeanCacheBytes &&
           (4 * ctx->chunks.size() + kPanelTiles) * static_cast<uint64_t>(ctx->cfg.W) * 64 < kMaxThreadsPerGridDim
               ? kPanelTiles : 0u;
}

// The next step, if it carries line 6, can also form the round's mean itself (k = 1 under the schedule
// that folds Step I into Step II: the step reads exactly the stored models).
static bool one_pass_applies(const cocod_ctx *ctx)
{
    return ctx->schedule == COCOD_SCHED_HEAD && ctx->mean_pending && ctx->store_pending &&
           ctx->cfg.grad == COCOD_GRAD_QUADRATIC && cocod::local_step_mean_quads_per_lane(ctx->cfg.W, true) != 0 &&
           ctx->chunks.size() < kMaxChunksMeanStep;
}

// One local step on the compute stream; with_line6 fuses line 6 into it (last step of a round).
static int enqueue_step(cocod_ctx *ctx, bool with_line6, const void *g_ext = nullptr, bool g_bf16 = false)
{
    // Keep the stored models intact: the first step of an open round reads them and
    // writes the spare buffer, which then becomes the live one.
    float *dst = ctx->store_pending ? ctx->spare : ctx->live;
    if (!ctx->dry && ctx->cfg.grad == COCOD_GRAD_MLP && !g_ext) {
        cocod::MlpParams p = ctx->mlp;             // work-space pointers
        // Mini-batch buffers: steps alternate between the two, and the context remembers for which step
        // index the next one is already filled (a captured round is keyed by both facts as they stand at
        // its first step, and leaves them as the same eager calls would).
        const uint32_t buf = ctx->batch_buf;
        p.X = ctx->mlp_X[buf];
        p.y = ctx->mlp_y[buf];
        p.X_next = ctx->mlp_X[buf ^ 1u];
        p.y_next = ctx->mlp_y[buf ^ 1u];
        p.have_batch = ctx->batch_ready_step == ctx->step;
        p.W = ctx->cfg.W;
        p.n_in = ctx->cfg.mlp_in; p.n_hid = ctx->cfg.mlp_hidden; p.n_out = ctx->cfg.mlp_out; p.batch = ctx->cfg.mlp_batch;
        p.stride = ctx->cfg.stride;
        p.x_in = ctx->live;
        p.x_out = dst;
        p.v = ctx->cfg.v;
        p.lr = ctx->cfg.lr;
        p.momentum = ctx->cfg.momentum;
        p.weight_decay = ctx->cfg.weight_decay;
        p.key0 = static_cast<uint32_t>(ctx->cfg.seed);
        p.key1 = static_cast<uint32_t>(ctx->cfg.seed >> 32);
        p.step = static_cast<uint32_t>(ctx->capturing ? ctx->step - ctx->capture_base : ctx->step);
        p.step_base = ctx->capturing ? ctx->d_step : nullptr;
        p.snap = with_line6 ? ctx->snap : nullptr;
        p.mean = ctx->cfg.mean;
        const bool timed = ctx->timing && ctx->t_used < ctx->t_start.size();
        COCOD_HIP(ctx, cocod::launch_mlp_step(ctx->s_compute, p, timed ? ctx->t_start[ctx->t_used] : nullptr,
                                              timed ? ctx->t_stop[ctx->t_used] : nullptr));
        ctx->batch_last = buf;
        ctx->batch_buf = buf ^ 1u;
        ctx->batch_ready_step = ctx->step + 1;
        if (timed) {
            ctx->t_kind[ctx->t_used] = with_line6 ? 1 : 0;
            ctx->t_used += 1;
        }
    } else if (!ctx->dry) {
        cocod::StepParams p{};
        p.table = ctx->d_chunks;
        p.n_chunks = static_cast<uint32_t>(ctx->chunks.size());
        p.W = ctx->cfg.W;
        p.stride = ctx->cfg.stride;
        p.x_in = ctx->live;
        p.x_out = dst;
        p.v = ctx->cfg.v;
        p.h = ctx->cfg.h;
        p.c = ctx->cfg.c;
        p.g = static_cast<const float *>(g_ext);
        p.g_bf16 = g_bf16 ? 1u : 0u;
        p.snap = with_line6 ? ctx->snap : nullptr;
        p.mean = ctx->cfg.mean;
        p.lr = ctx->cfg.lr;
        p.momentum = ctx->cfg.momentum;
        p.weight_decay = ctx->cfg.weight_decay;
        p.sigma = ctx->cfg.noise_sigma;
        p.sigma_w = ctx->d_sigma_w;
        p.key0 = static_cast<uint32_t>(ctx->cfg.seed);
        p.key1 = static_cast<uint32_t>(ctx->cfg.seed >> 32);
        p.step = static_cast<uint32_t>(ctx->capturing ? ctx->step - ctx->capture_base : ctx->step);
        p.step_base = ctx->capturing ? ctx->d_step : nullptr;
        p.panel_tiles = panel_tiles_for(ctx);
        // Step I inside the round's first step: that step reads exactly the stored models (when there are
        // too many workers for its LDS tile, the mean stays pending and is formed just before line 6)
        const bool head = ctx->schedule == COCOD_SCHED_HEAD && ctx->mean_pending && ctx->store_pending && !g_ext &&
                          !with_line6 && ctx->cfg.grad == COCOD_GRAD_QUADRATIC &&
                          cocod::local_step_mean_quads_per_lane(ctx->cfg.W, false) != 0 &&
                          ctx->chunks.size() < kMaxChunksMeanStep;
        // k = 1 under the same schedule: mean, step and line 6 in one pass over the stored models
        const bool one_pass = with_line6 && !g_ext && one_pass_applies(ctx);
        if (head || one_pass) {
            p.mean_out = ctx->cfg.mean;
            p.weights = ctx->d_weights;
            ctx->mean_pending = false;
        }
        hipEvent_t t0 = nullptr, t1 = nullptr;
        if (ctx->timing && ctx->t_used < ctx->t_start.size()) {
            t0 = ctx->t_start[ctx->t_used];
            t1 = ctx->t_stop[ctx->t_used];
            ctx->t_kind[ctx->t_used] = head ? 2 : (with_line6 ? 1 : 0);
            ctx->t_used += 1;
        }
        COCOD_HIP(ctx, cocod::launch_local_step(ctx->s_compute, p, t0, t1));
    }
    if (ctx->store_pending) {
        ctx->spare = ctx->live;
        ctx->live = dst;
        ctx->store_pending = false;
    }
    ctx->step += 1;
    return COCOD_OK;
}

static int check_steps(cocod_ctx *ctx, int k)
{
    if (k < 0) return fail(ctx, COCOD_ERR_INVALID, "k must be >= 0, got %d", k);
    if (ctx->step + static_cast<uint64_t>(k) > 0xffffffffull)
        return fail(ctx, COCOD_ERR_INVALID, "step counter would exceed 2^32 - 1");
    return COCOD_OK;
}

static int need_builtin_gradient(cocod_ctx *ctx)
{
    if (ctx->cfg.grad == COCOD_GRAD_EXTERNAL)
        return fail(ctx, COCOD_ERR_INVALID, "this context has no built-in gradient: use cocod_external_step");
    return COCOD_OK;
}

static int external_step(cocod_ctx *ctx, const void *g, bool bf16, int close_round)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (!g || (bf16 ? reinterpret_cast<uintptr_t>(g) % 8 != 0 : !aligned16(g)))
        return fail(ctx, COCOD_ERR_INVALID, "g must be a device pointer aligned to %d bytes", bf16 ? 8 : 16);
    if (close_round && !ctx->averaging) return fail(ctx, COCOD_ERR_STATE, "cocod_external_step: no round is open to close");
    int rc = check_steps(ctx, 1);
    if (rc != COCOD_OK) return rc;
    if (close_round && !ctx->dry) {      // the mean is consumed inside this step
        rc = mean_before_line6(ctx);
        if (rc != COCOD_OK) return rc;
    }
    rc = enqueue_step(ctx, close_round != 0, g, bf16);
    if (rc == COCOD_OK && close_round) {
        ctx->averaging = false;
        ctx->mean_pending = false;
        ctx->snap = nullptr;
    }
    return rc;
}

int cocod_external_step(cocod_ctx *ctx, const float *g, int close_round)
{
    return external_step(ctx, g, false, close_round);
}

int cocod_external_step_bf16(cocod_ctx *ctx, const uint16_t *g, int close_round)
{
    return external_step(ctx, g, true, close_round);
}

int cocod_local_steps(cocod_ctx *ctx, int k)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    int rc = check_steps(ctx, k);
    if (rc == COCOD_OK && k > 0) rc = need_builtin_gradient(ctx);
    for (int s = 0; s < k && rc == COCOD_OK; ++s) rc = enqueue_step(ctx, false);
    return rc;
}

int cocod_local_steps_end_apply(cocod_ctx *ctx, int k)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (!ctx->averaging) return fail(ctx, COCOD_ERR_STATE, "cocod_local_steps_end_apply: no round is open");
    int rc = check_steps(ctx, k);
    if (rc != COCOD_OK) return rc;
    if (k == 0) return cocod_average_end_apply(ctx);
    rc = need_builtin_gradient(ctx);
    if (rc != COCOD_OK) return rc;
    for (int s = 0; s + 1 < k && rc == COCOD_OK; ++s) rc = enqueue_step(ctx, false);
    if (rc != COCOD_OK) return rc;
    if (!ctx->dry && !one_pass_applies(ctx)) {
        // the mean must be complete before the last step starts: it is consumed inside it
        rc = mean_before_line6(ctx);
        if (rc != COCOD_OK) return rc;
    }
    rc = enqueue_step(ctx, true);
    if (rc != COCOD_OK) return rc;
    ctx->averaging = false;
    ctx->mean_pending = false;
    ctx->snap = nullptr;
    return COCOD_OK;
}

int cocod_average_begin(cocod_ctx *ctx)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (ctx->averaging) return fail(ctx, COCOD_ERR_STATE, "cocod_average_begin: a round is already open");
    ctx->snap = ctx->live;
    if (!ctx->dry && ctx->schedule == COCOD_SCHED_OVERLAP) {
        const bool two_streams = ctx->s_avg != ctx->s_compute;
        if (two_streams) {
            COCOD_HIP(ctx, hipEventRecord(ctx->ev_snap, ctx->s_compute));
            COCOD_HIP(ctx, hipStreamWaitEvent(ctx->s_avg, ctx->ev_snap, 0));
        }
        const int rc = enqueue_mean(ctx, ctx->s_avg);
        if (rc != COCOD_OK) return rc;
        if (two_streams) COCOD_HIP(ctx, hipEventRecord(ctx->ev_mean, ctx->s_avg));
    }
    ctx->averaging = true;
    ctx->store_pending = true;
    ctx->mean_pending = ctx->schedule != COCOD_SCHED_OVERLAP;
    return COCOD_OK;
}

int cocod_average_end_apply(cocod_ctx *ctx)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (!ctx->averaging) return fail(ctx, COCOD_ERR_STATE, "cocod_average_end_apply: no round is open");
    if (!ctx->dry) {
        const size_t n_buckets = ctx->bucket_begin.size() - 1;
        if (ctx->mean_pending && ctx->schedule != COCOD_SCHED_SERIAL) {     // FUSED, or HEAD with no step to ride on
            for (size_t b = 0; b < n_buckets; ++b)
                COCOD_HIP(ctx, cocod::launch_mean_correct(ctx->s_compute, ctx->live, ctx->snap, ctx->cfg.stride, ctx->cfg.W,
                                                          ctx->bucket_begin[b], ctx->bucket_begin[b + 1], ctx->d_weights,
                                                          ctx->cfg.mean));
        } else {
            const int rc = mean_before_line6(ctx);                                // SERIAL: the mean; OVERLAP: the join
            if (rc != COCOD_OK) return rc;
            {                                                                      // line 6, one launch for the whole list
                cocod::StepParams p{};
                p.table = ctx->d_chunks;
                p.n_chunks = static_cast<uint32_t>(ctx->chunks.size());
                p.W = ctx->cfg.W;
                p.stride = ctx->cfg.stride;
                p.x_in = ctx->live;
                p.x_out = ctx->live;
                p.snap = ctx->snap;
                p.mean = ctx->cfg.mean;
                p.panel_tiles = panel_tiles_for(ctx);
                COCOD_HIP(ctx, cocod::launch_line6(ctx->s_compute, p));
            }
        }
    }
    ctx->averaging = false;
    ctx->store_pending = false;
    ctx->mean_pending = false;
    ctx->snap = nullptr;
    return COCOD_OK;
}

int cocod_average_apply_fused(cocod_ctx *ctx)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    const bool opened_here = !ctx->averaging;
    if (opened_here) {                   // blocking average of the live models: the stored models ARE the live ones
        ctx->snap = ctx->live;
        ctx->averaging = true;
        ctx->mean_pending = true;
    }
    if (!ctx->dry) {
        // a mean already running on the averaging stream (overlapped schedule) writes the same values to
        // `mean`: let it finish first so that the two writers never overlap
        if (!ctx->mean_pending && ctx->schedule == COCOD_SCHED_OVERLAP && ctx->s_avg != ctx->s_compute)
            COCOD_HIP(ctx, hipStreamWaitEvent(ctx->s_compute, ctx->ev_mean, 0));
        for (size_t b = 0; b + 1 < ctx->bucket_begin.size(); ++b)
            COCOD_HIP(ctx, cocod::launch_mean_correct(ctx->s_compute, ctx->live, ctx->snap, ctx->cfg.stride, ctx->cfg.W,
                                                      ctx->bucket_begin[b], ctx->bucket_begin[b + 1], ctx->d_weights,
                                                      ctx->cfg.mean));
    }
    ctx->averaging = false;
    ctx->store_pending = false;
    ctx->mean_pending = false;
    ctx->snap = nullptr;
    return COCOD_OK;
}

// Record one round into a graph.  Nothing executes; the context's state is put back afterwards.
static int capture_round(cocod_ctx *ctx, int k, int fused_tail, hipGraphExec_t *exec)
{
    float *const live = ctx->live, *const spare = ctx->spare;
    const uint64_t step = ctx->step;
    const bool timing = ctx->timing;
    const uint32_t batch_buf = ctx->batch_buf, batch_last = ctx->batch_last;
    const uint64_t batch_ready_step = ctx->batch_ready_step;
    ctx->timing = false;
    ctx->capturing = true;
    ctx->capture_base = step;
    hipError_t e = hipStreamBeginCapture(ctx->s_compute, hipStreamCaptureModeThreadLocal);
    int rc = e == hipSuccess ? COCOD_OK : hip_fail(ctx, e, "hipStreamBeginCapture");
    hipGraph_t graph = nullptr;
    if (rc == COCOD_OK) {
        rc = cocod_average_begin(ctx);
        if (rc == COCOD_OK) {
            if (fused_tail) {
                rc = cocod_local_steps_end_apply(ctx, k);
            } else {
                rc = cocod_local_steps(ctx, k);
                if (rc == COCOD_OK) rc = cocod_average_end_apply(ctx);
            }
        }
        if (rc == COCOD_OK && k > 0) {
            e = cocod::launch_add_word(ctx->s_compute, ctx->d_step, static_cast<uint32_t>(k));
            if (e != hipSuccess) rc = hip_fail(ctx, e, "launch_add_word");
        }
        e = hipStreamEndCapture(ctx->s_compute, &graph);          // always: leaves the stream usable
        if (rc == COCOD_OK && e != hipSuccess) rc = hip_fail(ctx, e, "hipStreamEndCapture");
    }
    ctx->live = live; ctx->spare = spare; ctx->snap = nullptr;
    ctx->averaging = false; ctx->store_pending = false; ctx->mean_pending = false;
    ctx->step = step;
    ctx->batch_buf = batch_buf; ctx->batch_last = batch_last; ctx->batch_ready_step = batch_ready_step;
    ctx->timing = timing;
    ctx->capturing = false;
    if (rc == COCOD_OK) {
        e = hipGraphInstantiate(exec, graph, nullptr, nullptr, 0);
        if (e != hipSuccess) rc = hip_fail(ctx, e, "hipGraphInstantiate");
    }
    if (graph) (void)hipGraphDestroy(graph);
    return rc;
}

int cocod_graph_round(cocod_ctx *ctx, int k, int fused_tail)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (ctx->averaging) return fail(ctx, COCOD_ERR_STATE, "cocod_graph_round: a round is already open");
    int rc = check_steps(ctx, k);
    if (rc == COCOD_OK && k > 0) rc = need_builtin_gradient(ctx);
    if (rc != COCOD_OK) return rc;
    // stream capture cannot record the null stream (nor the legacy default stream handle)
    if (!ctx->s_compute || ctx->s_compute == hipStreamLegacy)
        return fail(ctx, COCOD_ERR_INVALID, "cocod_graph_round needs a compute stream of its own: the null stream cannot be captured");
    fused_tail = fused_tail != 0;
    if (ctx->dry) {                                  // state transitions only
        rc = cocod_average_begin(ctx);
        if (rc == COCOD_OK) rc = fused_tail ? cocod_local_steps_end_apply(ctx, k) : cocod_local_steps(ctx, k);
        if (rc == COCOD_OK && !fused_tail) rc = cocod_average_end_apply(ctx);
        return rc;
    }
    if (!ctx->d_step) COCOD_HIP(ctx, hipMalloc(reinterpret_cast<void **>(&ctx->d_step), sizeof(uint32_t)));
    const bool live_is_A = ctx->live == ctx->cfg.xA;
    const bool mlp = ctx->cfg.grad == COCOD_GRAD_MLP && k > 0;
    const uint32_t batch_buf = mlp ? ctx->batch_buf : 0u;                    // which mini-batch buffer the first step reads,
    const bool batch_ready = mlp && ctx->batch_ready_step == ctx->step;      // and whether its batch is already there
    hipGraphExec_t exec = nullptr;
    for (const auto &g : ctx->graphs)
        if (g.k == k && g.fused_tail == fused_tail && g.schedule == ctx->schedule && g.live_is_A == live_is_A &&
            g.batch_buf == batch_buf && g.batch_ready == batch_ready) exec = g.exec;
    if (!exec) {
        rc = capture_round(ctx, k, fused_tail, &exec);
        if (rc != COCOD_OK) return rc;
        ctx->graphs.push_back({k, fused_tail, ctx->schedule, live_is_A, batch_buf, batch_ready, exec});
    }
    if (ctx->d_step_value != ctx->step) {            // eager calls since the last replay moved t
        COCOD_HIP(ctx, cocod::launch_set_word(ctx->s_compute, ctx->d_step, static_cast<uint32_t>(ctx->step)));
        ctx->d_step_value = ctx->step;
    }
    COCOD_HIP(ctx, hipGraphLaunch(exec, ctx->s_compute));
    if (k > 0) {                                     // what the round's calls would have done to the host state
        float *t = ctx->live; ctx->live = ctx->spare; ctx->spare = t;
        ctx->step += static_cast<uint64_t>(k);
        ctx->d_step_value = ctx->step;
        if (mlp) {                                   // k steps alternated the batch buffers; the last drew the next batch
            ctx->batch_last = (batch_buf + static_cast<uint32_t>(k - 1)) & 1u;
            ctx->batch_buf = ctx->batch_last ^ 1u;
            ctx->batch_ready_step = ctx->step;
        }
    }
    return COCOD_OK;
}

int cocod_set_schedule(cocod_ctx *ctx, int schedule)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (schedule != COCOD_SCHED_OVERLAP && schedule != COCOD_SCHED_SERIAL && schedule != COCOD_SCHED_FUSED &&
        schedule != COCOD_SCHED_HEAD)
        return fail(ctx, COCOD_ERR_INVALID, "unknown schedule %d", schedule);
    if (ctx->averaging) return fail(ctx, COCOD_ERR_STATE, "cocod_set_schedule: not while a round is open");
    ctx->schedule = schedule;
    return COCOD_OK;                     // graphs are keyed by schedule: nothing to drop
}

int cocod_set_lr(cocod_ctx *ctx, float lr)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (!std::isfinite(lr)) return fail(ctx, COCOD_ERR_INVALID, "lr is not finite");
    if (lr != ctx->cfg.lr && !ctx->graphs.empty()) {     // captured kernels carry the old step size
        COCOD_HIP(ctx, hipStreamSynchronize(ctx->s_compute));
        for (auto &g : ctx->graphs) (void)hipGraphExecDestroy(g.exec);
        ctx->graphs.clear();
    }
    ctx->cfg.lr = lr;
    return COCOD_OK;
}

int cocod_get_step(const cocod_ctx *ctx, uint64_t *step)
{
    if (!ctx || !step) return fail(nullptr, COCOD_ERR_INVALID, "ctx and step must not be NULL");
    *step = ctx->step;
    return COCOD_OK;
}

int cocod_set_step(cocod_ctx *ctx, uint64_t step)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (step > 0xffffffffull) return fail(ctx, COCOD_ERR_INVALID, "step must be < 2^32");
    ctx->step = step;
    return COCOD_OK;
}

int cocod_live_model(const cocod_ctx *ctx, float **x_live)
{
    if (!ctx || !x_live) return fail(nullptr, COCOD_ERR_INVALID, "ctx and x_live must not be NULL");
    *x_live = ctx->live;
    return COCOD_OK;
}

int cocod_is_averaging(const cocod_ctx *ctx)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    return ctx->averaging ? 1 : 0;
}

int cocod_get_plan(const cocod_ctx *ctx, uint64_t *padded_d, uint32_t *n_chunks, uint32_t *n_buckets)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (padded_d) *padded_d = ctx->padded_d;
    if (n_chunks) *n_chunks = static_cast<uint32_t>(ctx->chunks.size());
    if (n_buckets) *n_buckets = static_cast<uint32_t>(ctx->bucket_begin.size() - 1);
    return COCOD_OK;
}

int cocod_step_timing(cocod_ctx *ctx, int max_launches)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (max_launches < 0 || max_launches > (1 << 20)) return fail(ctx, COCOD_ERR_INVALID, "max_launches out of range");
    ctx->timing = max_launches > 0;
    ctx->t_used = 0;
    if (ctx->dry) return COCOD_OK;
    while (ctx->t_start.size() < static_cast<size_t>(max_launches)) {
        hipEvent_t a = nullptr, b = nullptr;
        COCOD_HIP(ctx, hipEventCreate(&a));
        ctx->t_start.push_back(a);
        COCOD_HIP(ctx, hipEventCreate(&b));
        ctx->t_stop.push_back(b);
        ctx->t_kind.push_back(0);
    }
    return COCOD_OK;
}

int cocod_step_timing_read(cocod_ctx *ctx, double total_ms[3], uint32_t launches[3])
{
    if (!ctx || !total_ms || !launches) return fail(nullptr, COCOD_ERR_INVALID, "ctx, total_ms and launches must not be NULL");
    total_ms[0] = total_ms[1] = total_ms[2] = 0.0;
    launches[0] = launches[1] = launches[2] = 0;
    if (ctx->dry) return COCOD_OK;
    COCOD_HIP(ctx, hipStreamSynchronize(ctx->s_compute));
    for (size_t i = 0; i < ctx->t_used && i < ctx->t_stop.size(); ++i) {
        float ms = 0.0f;
        COCOD_HIP(ctx, hipEventElapsedTime(&ms, ctx->t_start[i], ctx->t_stop[i]));
        const int kind = ctx->t_kind[i];
        total_ms[kind] += ms;
        launches[kind] += 1;
    }
    ctx->t_used = 0;
    return COCOD_OK;
}

int cocod_consensus_distance(cocod_ctx *ctx, double *result)
{
    if (!ctx || !result) return fail(nullptr, COCOD_ERR_INVALID, "ctx and result must not be NULL");
    *result = 0.0;
    if (ctx->dry) return COCOD_OK;
    const uint32_t n_chunks = static_cast<uint32_t>(ctx->chunks.size());
    if (!ctx->d_reduce)     // two results, then two runs of block partials
        COCOD_HIP(ctx, hipMalloc(reinterpret_cast<void **>(&ctx->d_reduce), (static_cast<size_t>(n_chunks) + 1) * 2 * sizeof(double)));
    COCOD_HIP(ctx, cocod::launch_consensus_distance(ctx->s_compute, ctx->d_chunks, n_chunks, ctx->live, ctx->cfg.stride,
                                                    ctx->cfg.W, ctx->d_weights, ctx->d_reduce + 2, ctx->d_reduce));
    COCOD_HIP(ctx, hipMemcpyAsync(result, ctx->d_reduce, sizeof(double), hipMemcpyDeviceToHost, ctx->s_compute));
    COCOD_HIP(ctx, hipStreamSynchronize(ctx->s_compute));
    return COCOD_OK;
}

int cocod_consensus_distance_noalloc(cocod_ctx *ctx, double *result_device)
{
    if (!ctx || !result_device) return fail(nullptr, COCOD_ERR_INVALID, "ctx and result_device must not be NULL");
    if (reinterpret_cast<uintptr_t>(result_device) % sizeof(double) != 0)
        return fail(ctx, COCOD_ERR_INVALID, "result_device must be 8-byte aligned");
    const uint64_t n_chunks = ctx->chunks.size();
    if (n_chunks > kNoAllocMaxChunks)
        return fail(ctx, COCOD_ERR_UNSUPPORTED,
                    "cocod_consensus_distance_noalloc: %llu chunks of 1024 parameters exceed the static scratch (%u chunks); "
                    "use cocod_consensus_distance", (unsigned long long)n_chunks, kNoAllocMaxChunks);
    if (ctx->dry) return COCOD_OK;
    // Every partial the final pass reads is written by this call's first pass: nothing has to start at zero.
    double *const partial = ctx->static_scratch + 2;
    COCOD_HIP(ctx, cocod::launch_consensus_distance(ctx->s_compute, ctx->d_chunks, static_cast<uint32_t>(n_chunks), ctx->live,
                                                    ctx->cfg.stride, ctx->cfg.W, ctx->d_weights, partial, result_device));
    return COCOD_OK;
}

int cocod_quadratic_objective(cocod_ctx *ctx, double *f_at_mean, double *grad_norm_sq_at_mean)
{
    if (!ctx || !f_at_mean || !grad_norm_sq_at_mean)
        return fail(nullptr, COCOD_ERR_INVALID, "ctx, f_at_mean and grad_norm_sq_at_mean must not be NULL");
    *f_at_mean = *grad_norm_sq_at_mean = 0.0;
    if (ctx->cfg.grad != COCOD_GRAD_QUADRATIC) return fail(ctx, COCOD_ERR_INVALID, "not a quadratic-gradient context");
    if (ctx->dry) return COCOD_OK;
    const uint32_t n_chunks = static_cast<uint32_t>(ctx->chunks.size());
    if (!ctx->d_reduce)
        COCOD_HIP(ctx, hipMalloc(reinterpret_cast<void **>(&ctx->d_reduce), (static_cast<size_t>(n_chunks) + 1) * 2 * sizeof(double)));
    COCOD_HIP(ctx, cocod::launch_quadratic_objective(ctx->s_compute, ctx->d_chunks, n_chunks, ctx->live, ctx->cfg.h, ctx->cfg.c,
                                                     ctx->cfg.stride, ctx->cfg.W, ctx->d_weights, ctx->d_reduce + 2,
                                                     ctx->d_reduce));
    double both[2] = {0.0, 0.0};
    COCOD_HIP(ctx, hipMemcpyAsync(both, ctx->d_reduce, sizeof both, hipMemcpyDeviceToHost, ctx->s_compute));
    COCOD_HIP(ctx, hipStreamSynchronize(ctx->s_compute));
    *f_at_mean = both[0];
    *grad_norm_sq_at_mean = both[1];
    return COCOD_OK;
}

int cocod_mlp_workspace(const cocod_ctx *ctx, float **X, float **H, float **dA, float **dZ, int32_t **y, uint32_t *dz_pitch)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (ctx->cfg.grad != COCOD_GRAD_MLP) return fail(nullptr, COCOD_ERR_INVALID, "not an MLP-gradient context");
    if (X) *X = ctx->mlp_X[ctx->batch_last];
    if (H) *H = ctx->mlp.H;
    if (dA) *dA = ctx->mlp.dA;
    if (dZ) *dZ = ctx->mlp.dZ;
    if (y) *y = ctx->mlp_y[ctx->batch_last];
    if (dz_pitch) *dz_pitch = static_cast<uint32_t>(cocod::mlp_dz_pitch());
    return COCOD_OK;
}

int cocod_fill_quadratic(cocod_ctx *ctx)
{
    if (!ctx) return fail(nullptr, COCOD_ERR_INVALID, "ctx is NULL");
    if (ctx->cfg.grad != COCOD_GRAD_QUADRATIC) return fail(ctx, COCOD_ERR_INVALID, "not a quadratic-gradient context");
    if (ctx->dry) return COCOD_OK;
    COCOD_HIP(ctx, cocod::launch_fill_quadratic(ctx->s_compute, ctx->d_chunks, static_cast<uint32_t>(ctx->chunks.size()),
                                                ctx->cfg.W, ctx->cfg.stride, ctx->padded_d,
                                                const_cast<float *>(ctx->cfg.h), const_cast<float *>(ctx->cfg.c),
                                                static_cast<uint32_t>(ctx->cfg.seed),
                                                static_cast<uint32_t>(ctx->cfg.seed >> 32)));
    return COCOD_OK;
}

int cocod_debug_copy(void *stream, const float *src, float *dst, uint64_t n)
{
    if (n == 0) return COCOD_OK;
    if (!src || !dst) return fail(nullptr, COCOD_ERR_INVALID, "src and dst must not be NULL");
    if ((n & 3u) || !aligned16(src) || !aligned16(dst))
        return fail(nullptr, COCOD_ERR_INVALID, "n must be a multiple of 4 and the pointers 16-byte aligned");
    const hipError_t e = cocod::launch_copy(static_cast<hipStream_t>(stream), src, dst, n / 4);
    if (e != hipSuccess) return hip_fail(nullptr, e, "cocod_debug_copy");
    return COCOD_OK;
}

int cocod_debug_normals(void *stream, uint64_t seed, uint32_t tag, uint32_t worker, uint32_t step, uint64_t j0,
                        uint64_t n, int fast, float *out)
{
    if (n == 0) return COCOD_OK;
    if (!out) return fail(nullptr, COCOD_ERR_INVALID, "out is NULL");
    if (j0 + n > (1ull << 34)) return fail(nullptr, COCOD_ERR_INVALID, "index range exceeds 2^34");
    const hipError_t e = cocod::launch_debug_normals(static_cast<hipStream_t>(stream), static_cast<uint32_t>(seed),
                                                     static_cast<uint32_t>(seed >> 32), tag, worker, step, j0, n, fast, out);
    if (e != hipSuccess) return hip_fail(nullptr, e, "cocod_debug_normals");
    return COCOD_OK;
}

}  // extern "C"
