// Step I and line 6 of Algorithm 1 (CoCoD-SGD) on one GPU.
//
//   wmean         mean_j = sum_i p_i snap_ij           (the paper's all-reduce between workers)
//   mean_correct  the mean and line 6, x_ij = mean_j + (x_ij - snap_ij), in one pass (sequential
//                 schedule, nothing to overlap)
// (Line 6 on its own is a mode of the local-step kernel: a row-wise stream like the step itself.)
//
// Models are worker-major [W][stride], so the reduction runs along the SLOW axis:
// a thread owns one 16-byte column quad and walks the W rows with independent
// 16-byte loads; consecutive lanes own consecutive quads, so every wave load is
// 1 KiB contiguous.  The sum is taken in worker order 0..W-1 in fp32, which fixes
// the result bit for bit regardless of launch shape or schedule.
// In mean_correct the same thread then serves all W workers of its column for line 6, so each stored
// model is read once (12 + 4/W bytes per parameter).
#include "internal.hpp"
#include "mean_sum.hpp"

namespace cocod {
namespace {

// Single-wave blocks.  Beside a local step made of single-wave blocks the workgroup dispatcher then gives
// the mean a fair share of the chip: measured at W = 16, d = 11.2 M the mean takes 0.20 ms next to the
// step with 64-thread blocks, 0.33 ms with 128 and 0.79 ms (the whole step) with 256 or 1024.  Alone the
// averaging kernels run at the same rate for every block size.
constexpr uint32_t kAvgThreads = 64;
constexpr int kRowBatch = 8;   // independent row loads in flight per thread

typedef float f4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ void st4(float *p, const float4 &a) { *reinterpret_cast<float4 *>(p) = a; }
// models are streamed once per kernel and exceed the caches: non-temporal hint
__device__ __forceinline__ float4 ld4_stream(const float *p)
{
    const f4v t = __builtin_nontemporal_load(reinterpret_cast<const f4v *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void st4_stream(float *p, const float4 &a)
{
    __builtin_nontemporal_store(f4v{a.x, a.y, a.z, a.w}, reinterpret_cast<f4v *>(p));
}

// Ordered weighted sum over the rows of one column quad.
template <bool WEIGHTED>
__device__ __forceinline__ float4 column_mean(const float *col, uint64_t stride, uint32_t W, const float *weights)
{
    MeanSum acc;
    acc.clear();
    uint32_t i = 0;
    for (; i + kRowBatch <= W; i += kRowBatch) {
        float4 r[kRowBatch];
        #pragma unroll
        for (int b = 0; b < kRowBatch; ++b) r[b] = ld4_stream(col + static_cast<uint64_t>(i + b) * stride);
        #pragma unroll
        for (int b = 0; b < kRowBatch; ++b)
            acc.add<WEIGHTED>(WEIGHTED ? weights[i + b] : 1.0f, r[b].x, r[b].y, r[b].z, r[b].w);
    }
    for (; i < W; ++i) {
        const float4 r = ld4_stream(col + static_cast<uint64_t>(i) * stride);
        acc.add<WEIGHTED>(WEIGHTED ? weights[i] : 1.0f, r.x, r.y, r.z, r.w);
    }
    acc.finish<WEIGHTED>(W);
    return make_float4(acc.s[0], acc.s[1], acc.s[2], acc.s[3]);
}

template <bool WEIGHTED>
__global__ __launch_bounds__(kAvgThreads) void wmean_kernel(const float *snap, uint64_t stride, uint32_t W,
                                                            uint64_t begin, uint64_t n_quads,
                                                            const float *weights, float *mean)
{
    // Line 6 waits for this kernel while the local step beside it has no one waiting: its waves issue first
    // (0.20 -> 0.18 ms next to the step; the round's time does not change).
    __builtin_amdgcn_s_setprio(3);
    for (uint64_t quad = static_cast<uint64_t>(blockIdx.x) * kAvgThreads + threadIdx.x; quad < n_quads;
         quad += static_cast<uint64_t>(gridDim.x) * kAvgThreads) {
        const uint64_t e = begin + quad * 4;
        st4(mean + e, column_mean<WEIGHTED>(snap + e, stride, W, weights));
    }
}

__device__ __forceinline__ void correct_column(float *xcol, const float *scol, const float4 m, uint64_t stride, uint32_t W)
{
    constexpr int B = 4;
    uint32_t i = 0;
    for (; i + B <= W; i += B) {
        float4 xr[B], sr[B];
        #pragma unroll
        for (int b = 0; b < B; ++b) {
            xr[b] = ld4_stream(xcol + static_cast<uint64_t>(i + b) * stride);
            sr[b] = ld4_stream(scol + static_cast<uint64_t>(i + b) * stride);
        }
        #pragma unroll
        for (int b = 0; b < B; ++b) {
            float4 o;
            o.x = m.x + (xr[b].x - sr[b].x); o.y = m.y + (xr[b].y - sr[b].y);
            o.z = m.z + (xr[b].z - sr[b].z); o.w = m.w + (xr[b].w - sr[b].w);
            st4_stream(xcol + static_cast<uint64_t>(i + b) * stride, o);
        }
    }
    for (; i < W; ++i) {
        const float4 xr = ld4_stream(xcol + static_cast<uint64_t>(i) * stride);
        const float4 sr = ld4_stream(scol + static_cast<uint64_t>(i) * stride);
        float4 o;
        o.x = m.x + (xr.x - sr.x); o.y = m.y + (xr.y - sr.y);
        o.z = m.z + (xr.z - sr.z); o.w = m.w + (xr.w - sr.w);
        st4_stream(xcol + static_cast<uint64_t>(i) * stride, o);
    }
}

// WREG > 0: W <= WREG and the column's stored models stay in registers between the two passes, so
// each is read from memory once (12 + 4/W bytes per parameter).  WREG == 0: any W, the stored models
// are read a second time for line 6.
template <bool WEIGHTED, int WREG>
__global__ __launch_bounds__(kAvgThreads) void mean_correct_kernel(float *x, const float *snap, uint64_t stride,
                                                                   uint32_t W, uint64_t begin, uint64_t n_quads,
                                                                   const float *weights, float *mean)
{
    const uint64_t quad = static_cast<uint64_t>(blockIdx.x) * kAvgThreads + threadIdx.x;
    if (quad >= n_quads) return;
    const uint64_t e = begin + quad * 4;
    if (WREG == 0) {
        const float4 m = column_mean<WEIGHTED>(snap + e, stride, W, weights);
        st4(mean + e, m);
        correct_column(x + e, snap + e, m, stride, W);
        return;
    }
    constexpr int R = WREG > 0 ? WREG : 1;
    float4 s[R];
    #pragma unroll
    for (int i = 0; i < R; ++i)
        if (static_cast<uint32_t>(i) < W) s[i] = ld4_stream(snap + e + static_cast<uint64_t>(i) * stride);
    MeanSum acc;
    acc.clear();
    #pragma unroll
    for (int i = 0; i < R; ++i) {                          // same order and operations as column_mean
        if (static_cast<uint32_t>(i) < W)                  // guard, not break: the loop must unroll fully or s[] goes to scratch
            acc.add<WEIGHTED>(WEIGHTED ? weights[i] : 1.0f, s[i].x, s[i].y, s[i].z, s[i].w);
    }
    acc.finish<WEIGHTED>(W);
    const float4 m = make_float4(acc.s[0], acc.s[1], acc.s[2], acc.s[3]);
    st4(mean + e, m);
    #pragma unroll
    for (int i = 0; i < R; ++i) {
        if (static_cast<uint32_t>(i) < W) {
            float *xp = x + e + static_cast<uint64_t>(i) * stride;
            const float4 xr = ld4_stream(xp);
            float4 o;
            o.x = m.x + (xr.x - s[i].x); o.y = m.y + (xr.y - s[i].y);
            o.z = m.z + (xr.z - s[i].z); o.w = m.w + (xr.w - s[i].w);
            st4_stream(xp, o);
        }
    }
}

// ---- consensus distance: sum_i p_i || xbar - x_i ||^2 with xbar = sum_i p_i x_i ---------------------
// (the quantity bounded by Lemma 2 of the paper).  A scalar, so this is where wave and LDS reductions
// belong: per thread a column quad (its W rows held in registers up to 16 workers; above, two passes
// over the rows, the second one from cache), then a butterfly over the wave, the four wave sums through LDS, one double per block; a second one-block
// kernel adds the block partials in a fixed order, so the result is deterministic.
// the same mean with ordinary (cached) loads, for the kernels that read the models a second time
template <bool WEIGHTED>
__device__ __forceinline__ float4 column_mean_cached(const float *col, uint64_t stride, uint32_t W, const float *weights)
{
    MeanSum acc;
    acc.clear();
    uint32_t i = 0;
    for (; i + kRowBatch <= W; i += kRowBatch) {
        float4 r[kRowBatch];
        #pragma unroll
        for (int b = 0; b < kRowBatch; ++b) r[b] = ld4(col + static_cast<uint64_t>(i + b) * stride);
        #pragma unroll
        for (int b = 0; b < kRowBatch; ++b)
            acc.add<WEIGHTED>(WEIGHTED ? weights[i + b] : 1.0f, r[b].x, r[b].y, r[b].z, r[b].w);
    }
    for (; i < W; ++i) {
        const float4 r = ld4(col + static_cast<uint64_t>(i) * stride);
        acc.add<WEIGHTED>(WEIGHTED ? weights[i] : 1.0f, r.x, r.y, r.z, r.w);
    }
    acc.finish<WEIGHTED>(W);
    return make_float4(acc.s[0], acc.s[1], acc.s[2], acc.s[3]);
}

constexpr uint32_t kRowsInRegisters = 16;   // up to this many workers a thread keeps its whole column quad in registers

__device__ __forceinline__ double wave_sum_f64(double v)
{
    #pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

template <bool WEIGHTED>
__global__ __launch_bounds__(kStepThreads) void consensus_partial_kernel(const Chunk *table, const float *x, uint64_t stride,
                                                                         uint32_t W, const float *weights, double *partial)
{
    __shared__ double wave_part[kStepThreads / 64];
    const Chunk ck = table[blockIdx.x];
    const uint32_t e = threadIdx.x * 4;
    double local = 0.0;
    if (e < ck.n) {
        const float *col = x + static_cast<uint64_t>(ck.mem_quad) * 4 + e;
        const float uniform = 1.0f / static_cast<float>(W);
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        auto add_row = [&](uint32_t i, const float4 &r, const float4 &m) {
            const float pw = WEIGHTED ? weights[i] : uniform;
            acc.x += pw * (r.x - m.x) * (r.x - m.x); acc.y += pw * (r.y - m.y) * (r.y - m.y);
            acc.z += pw * (r.z - m.z) * (r.z - m.z); acc.w += pw * (r.w - m.w) * (r.w - m.w);
        };
        if (W <= kRowsInRegisters) {
            // one pass: every row of the column quad is requested at once and stays in registers for the
            // squared distances (the guards are uniform over the grid)
            float4 r[kRowsInRegisters];
            #pragma unroll
            for (uint32_t i = 0; i < kRowsInRegisters; ++i)
                if (i < W) r[i] = ld4_stream(col + static_cast<uint64_t>(i) * stride);
            MeanSum ms;
            ms.clear();
            #pragma unroll
            for (uint32_t i = 0; i < kRowsInRegisters; ++i)
                if (i < W) ms.add<WEIGHTED>(WEIGHTED ? weights[i] : 1.0f, r[i].x, r[i].y, r[i].z, r[i].w);
            ms.finish<WEIGHTED>(W);
            const float4 m = make_float4(ms.s[0], ms.s[1], ms.s[2], ms.s[3]);
            #pragma unroll
            for (uint32_t i = 0; i < kRowsInRegisters; ++i)
                if (i < W) add_row(i, r[i], m);
        } else {
            // two passes over the W rows, the second one from cache
            const float4 m = column_mean_cached<WEIGHTED>(col, stride, W, weights);
            uint32_t i = 0;
            for (; i + kRowBatch <= W; i += kRowBatch) {
                float4 r[kRowBatch];
                #pragma unroll
                for (int b = 0; b < kRowBatch; ++b) r[b] = ld4(col + static_cast<uint64_t>(i + b) * stride);
                #pragma unroll
                for (int b = 0; b < kRowBatch; ++b) add_row(i + b, r[b], m);
            }
            for (; i < W; ++i) add_row(i, ld4(col + static_cast<uint64_t>(i) * stride), m);
        }
        const uint32_t keep = ck.n - e;                   // alignment pads of a tensor's tail quad do not count
        local = static_cast<double>(acc.x);
        if (keep > 1) local += static_cast<double>(acc.y);
        if (keep > 2) local += static_cast<double>(acc.z);
        if (keep > 3) local += static_cast<double>(acc.w);
    }
    local = wave_sum_f64(local);
    if (threadIdx.x % 64 == 0) wave_part[threadIdx.x / 64] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (uint32_t w = 0; w < kStepThreads / 64; ++w) s += wave_part[w];
        partial[blockIdx.x] = s;
    }
}

// block b adds the b-th run of n block partials into out[b]
__global__ __launch_bounds__(256) void consensus_final_kernel(const double *partial, uint32_t n, double *out)
{
    __shared__ double wave_part[4];
    partial += static_cast<uint64_t>(blockIdx.x) * n;
    double local = 0.0;
    for (uint32_t i = threadIdx.x; i < n; i += 256) local += partial[i];
    local = wave_sum_f64(local);
    if (threadIdx.x % 64 == 0) wave_part[threadIdx.x / 64] = local;
    __syncthreads();
    if (threadIdx.x == 0) out[blockIdx.x] = (wave_part[0] + wave_part[1]) + (wave_part[2] + wave_part[3]);
}

// ---- the objective of the paper's problem definition at the averaged model ------------------------
// f(xbar) = sum_i p_i f_i(xbar) with the workers' quadratics f_i(x) = 1/2 sum_j h_ij (x_j - c_ij)^2 and
// xbar = sum_i p_i x_i, and || grad f(xbar) ||^2 (the quantity whose running mean Theorem 1 bounds),
// grad f(xbar)_j = sum_i p_i h_ij (xbar_j - c_ij).  Same reduction structure as the consensus distance;
// partial holds two runs of gridDim.x doubles (objective, squared gradient norm).
template <bool WEIGHTED>
__global__ __launch_bounds__(kStepThreads) void objective_partial_kernel(const Chunk *table, const float *x, const float *h,
                                                                         const float *c, uint64_t stride, uint32_t W,
                                                                         const float *weights, double *partial)
{
    __shared__ double wave_part[2][kStepThreads / 64];
    const Chunk ck = table[blockIdx.x];
    const uint32_t e = threadIdx.x * 4;
    double f_local = 0.0, g_local = 0.0;
    if (e < ck.n) {
        const uint64_t at = static_cast<uint64_t>(ck.mem_quad) * 4 + e;
        const float uniform = 1.0f / static_cast<float>(W);
        const float4 m = column_mean_cached<WEIGHTED>(x + at, stride, W, weights);
        float4 f = make_float4(0.f, 0.f, 0.f, 0.f), g = make_float4(0.f, 0.f, 0.f, 0.f);
        auto add_row = [&](uint32_t i, const float4 &hr, const float4 &cr) {
            const float pw = WEIGHTED ? weights[i] : uniform;
            const float4 dl = make_float4(m.x - cr.x, m.y - cr.y, m.z - cr.z, m.w - cr.w);
            g.x += pw * hr.x * dl.x; g.y += pw * hr.y * dl.y; g.z += pw * hr.z * dl.z; g.w += pw * hr.w * dl.w;
            f.x += pw * hr.x * dl.x * dl.x; f.y += pw * hr.y * dl.y * dl.y;
            f.z += pw * hr.z * dl.z * dl.z; f.w += pw * hr.w * dl.w * dl.w;
        };
        uint32_t i = 0;
        for (; i + kRowBatch <= W; i += kRowBatch) {              // h and c are read once: streamed, a batch of rows in flight
            float4 hr[kRowBatch], cr[kRowBatch];
            #pragma unroll
            for (int b = 0; b < kRowBatch; ++b) {
                hr[b] = ld4_stream(h + at + static_cast<uint64_t>(i + b) * stride);
                cr[b] = ld4_stream(c + at + static_cast<uint64_t>(i + b) * stride);
            }
            #pragma unroll
            for (int b = 0; b < kRowBatch; ++b) add_row(i + b, hr[b], cr[b]);
        }
        for (; i < W; ++i)
            add_row(i, ld4_stream(h + at + static_cast<uint64_t>(i) * stride), ld4_stream(c + at + static_cast<uint64_t>(i) * stride));
        const uint32_t keep = ck.n - e;                   // alignment pads of a tensor's tail quad do not count
        f_local = static_cast<double>(f.x);              g_local = static_cast<double>(g.x) * g.x;
        if (keep > 1) { f_local += static_cast<double>(f.y); g_local += static_cast<double>(g.y) * g.y; }
        if (keep > 2) { f_local += static_cast<double>(f.z); g_local += static_cast<double>(g.z) * g.z; }
        if (keep > 3) { f_local += static_cast<double>(f.w); g_local += static_cast<double>(g.w) * g.w; }
        f_local *= 0.5;
    }
    f_local = wave_sum_f64(f_local);
    g_local = wave_sum_f64(g_local);
    if (threadIdx.x % 64 == 0) { wave_part[0][threadIdx.x / 64] = f_local; wave_part[1][threadIdx.x / 64] = g_local; }
    __syncthreads();
    if (threadIdx.x < 2) {
        double s = 0.0;
        for (uint32_t w = 0; w < kStepThreads / 64; ++w) s += wave_part[threadIdx.x][w];
        partial[static_cast<uint64_t>(threadIdx.x) * gridDim.x + blockIdx.x] = s;
    }
}

inline uint32_t blocks_for(uint64_t n_quads) { return static_cast<uint32_t>((n_quads + kAvgThreads - 1) / kAvgThreads); }

}  // namespace

hipError_t launch_wmean(hipStream_t stream, const float *snap, uint64_t stride, uint32_t W, uint64_t begin,
                        uint64_t end, const float *weights, float *mean, uint32_t max_blocks)
{
    const uint64_t n_quads = (end - begin) / 4;
    if (n_quads == 0) return hipSuccess;
    uint32_t blocks = blocks_for(n_quads);
    if (max_blocks != 0 && max_blocks < blocks) blocks = max_blocks;     // the kernel strides over the rest
    const dim3 grid(blocks), block(kAvgThreads);
    if (weights) hipLaunchKernelGGL((wmean_kernel<true>), grid, block, 0, stream, snap, stride, W, begin, n_quads, weights, mean);
    else         hipLaunchKernelGGL((wmean_kernel<false>), grid, block, 0, stream, snap, stride, W, begin, n_quads, weights, mean);
    return hipGetLastError();
}

hipError_t launch_mean_correct(hipStream_t stream, float *x, const float *snap, uint64_t stride, uint32_t W,
                               uint64_t begin, uint64_t end, const float *weights, float *mean)
{
    const uint64_t n_quads = (end - begin) / 4;
    if (n_quads == 0) return hipSuccess;
    const dim3 grid(blocks_for(n_quads)), block(kAvgThreads);
    if (W <= 8) {
        if (weights) hipLaunchKernelGGL((mean_correct_kernel<true, 8>), grid, block, 0, stream, x, snap, stride, W, begin, n_quads, weights, mean);
        else         hipLaunchKernelGGL((mean_correct_kernel<false, 8>), grid, block, 0, stream, x, snap, stride, W, begin, n_quads, weights, mean);
        return hipGetLastError();
    }
    if (W <= 16) {
        if (weights) hipLaunchKernelGGL((mean_correct_kernel<true, 16>), grid, block, 0, stream, x, snap, stride, W, begin, n_quads, weights, mean);
        else         hipLaunchKernelGGL((mean_correct_kernel<false, 16>), grid, block, 0, stream, x, snap, stride, W, begin, n_quads, weights, mean);
        return hipGetLastError();
    }
    if (weights) hipLaunchKernelGGL((mean_correct_kernel<true, 0>), grid, block, 0, stream, x, snap, stride, W, begin, n_quads, weights, mean);
    else         hipLaunchKernelGGL((mean_correct_kernel<false, 0>), grid, block, 0, stream, x, snap, stride, W, begin, n_quads, weights, mean);
    return hipGetLastError();
}

hipError_t launch_consensus_distance(hipStream_t stream, const Chunk *table, uint32_t n_chunks, const float *x,
                                     uint64_t stride, uint32_t W, const float *weights, double *partial, double *out)
{
    if (weights) hipLaunchKernelGGL((consensus_partial_kernel<true>), dim3(n_chunks), dim3(kStepThreads), 0, stream, table, x, stride, W, weights, partial);
    else         hipLaunchKernelGGL((consensus_partial_kernel<false>), dim3(n_chunks), dim3(kStepThreads), 0, stream, table, x, stride, W, weights, partial);
    hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(256), 0, stream, partial, n_chunks, out);
    return hipGetLastError();
}

hipError_t launch_quadratic_objective(hipStream_t stream, const Chunk *table, uint32_t n_chunks, const float *x,
                                      const float *h, const float *c, uint64_t stride, uint32_t W, const float *weights,
                                      double *partial, double *out)
{
    if (weights) hipLaunchKernelGGL((objective_partial_kernel<true>), dim3(n_chunks), dim3(kStepThreads), 0, stream, table, x, h, c, stride, W, weights, partial);
    else         hipLaunchKernelGGL((objective_partial_kernel<false>), dim3(n_chunks), dim3(kStepThreads), 0, stream, table, x, h, c, stride, W, weights, partial);
    hipLaunchKernelGGL(consensus_final_kernel, dim3(2), dim3(256), 0, stream, partial, n_chunks, out);
    return hipGetLastError();
}

}  // namespace cocod
