// Step II of Algorithm 1 (CoCoD-SGD) for the synthetic quadratic workers: one
// fused local step.  Per parameter j of worker i at global step t
//     G = h_ij (x_j - c_ij) + sigma z(seed, i, t, j)        stochastic gradient
//     g = G + lambda x ;  v = mu v + g ;  x = x - gamma v    momentum SGD of the experiments
// The gradient is never written to memory: the kernel reads x, v, h, c and writes
// x, v (24 bytes per parameter; 16 when mu = 0 and v is untouched).
//
// Work decomposition: grid = (chunks, workers).  A chunk is up to 1024 consecutive
// elements of one tensor (multi-tensor apply: the chunk table maps a block to its
// tensor slice, so one launch covers a whole parameter list).  A thread owns one
// 16-byte quad; a wave moves 1 KiB contiguous per array.  Small blocks with one
// quad per thread measured faster on MI355X than fewer, longer-running blocks.
//
// Memory path: every array is streamed exactly once per step and is far larger
// than the caches, so all accesses carry the non-temporal hint.  Accesses go
// through buffer instructions whose descriptor covers exactly the chunk: lanes
// past the chunk's end read zeros and their stores are dropped by the hardware
// range check, so there is no divergent tail code.
//
// The generator's 128-bit block is keyed by the UNPADDED global parameter index, so
// results do not depend on how tensors are packed; when a tensor starts at a global
// index that is not a multiple of 4, a thread's memory quad straddles two generator blocks.
// Threads own consecutive blocks, so the missing normals are the right-hand neighbour's: three
// cross-lane moves (one LDS word across a wave boundary) instead of a second generator call.
#include "internal.hpp"
#include "step_common.hpp"
#include "philox.hpp"
#include "mean_sum.hpp"

#include <hip/hip_ext.h>

namespace cocod {
namespace {

// Four normals for a thread's memory quad whose first element has global index 4*q + shift.
// shift == 0: the quad is one generator block.  Otherwise the quad takes the last 4 - shift normals
// of block q and the first `shift` normals of block q + 1.  Threads own consecutive blocks, so block
// q + 1 is the right-hand neighbour's own block: a cross-lane move inside a wave, a word of LDS
// across a wave boundary, and one extra generator call by the block's very last thread.
// Must be called by all threads of the block (it synchronises when shift != 0).  A kernel that calls
// it in a loop alternates `parity` so that the LDS words of one call are not overwritten by the next
// call while a slower wave still reads them (one barrier per call then suffices).
__device__ __forceinline__ f4 noise_for_quad(uint64_t q, uint32_t shift, const StepParams &p, uint32_t worker,
                                             uint32_t parity = 0)
{
    const uint32_t step = p.step_base ? *p.step_base + p.step : p.step;      // wave-uniform

    const Normals4 a = box_muller_fast(
        philox4x32_10(static_cast<uint32_t>(q), step, worker, kTagNoise, p.key0, p.key1));
    if (shift == 0) return f4{a.z[0], a.z[1], a.z[2], a.z[3]};          // block-uniform branch
    __shared__ float both[2][kStepThreads / 64][3];
    float (*first_of_wave)[3] = both[parity & 1u];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    if (lane == 0) { first_of_wave[wave][0] = a.z[0]; first_of_wave[wave][1] = a.z[1]; first_of_wave[wave][2] = a.z[2]; }
    __syncthreads();
    float b0 = __shfl_down(a.z[0], 1, 64), b1 = __shfl_down(a.z[1], 1, 64), b2 = __shfl_down(a.z[2], 1, 64);
    if (lane == 63u) {
        if (wave + 1 < kStepThreads / 64) {
            b0 = first_of_wave[wave + 1][0]; b1 = first_of_wave[wave + 1][1]; b2 = first_of_wave[wave + 1][2];
        } else {                                                        // one lane of one wave per block
            const Normals4 nb = box_muller_fast(
                philox4x32_10(static_cast<uint32_t>(q + 1), step, worker, kTagNoise, p.key0, p.key1));
            b0 = nb.z[0]; b1 = nb.z[1]; b2 = nb.z[2];
        }
    }
    if (shift == 1) return f4{a.z[1], a.z[2], a.z[3], b0};
    if (shift == 2) return f4{a.z[2], a.z[3], b0, b1};
    return f4{a.z[3], b0, b1, b2};
}

// TAIL: 0 = plain local step; 1 = last step of a round with line 6 applied to the fresh model
// before it is stored, x = mean + ((x - gamma v) - snap); 2 = the same when the step reads the
// stored models themselves (k = 1: snap is x_in, no extra read).
// GRAD: where the stochastic gradient G comes from (step_common.hpp).

template <bool HAS_V, int GRAD, int TAIL>
__global__ __launch_bounds__(kStepThreads) void quad_step_kernel(const StepParams p)
{
    // Default: grid (chunks, workers), chunk fastest, so neighbouring blocks stream one worker's rows.
    // A step with line 6 whose mean (4 d bytes) does not fit the last-level cache runs on a 1-D grid
    // with the WORKER fastest instead: the W blocks that need the same chunk of the mean then run
    // together and it comes from memory once instead of W times (measured: +11 % at d = 138 M, but
    // 2-10 % slower when the mean does fit, hence the switch).
    const bool worker_fastest = TAIL != 0 && p.worker_fastest;
    const uint32_t chunk_id = worker_fastest ? blockIdx.x / p.W : blockIdx.x;
    const uint32_t worker = worker_fastest ? blockIdx.x % p.W : blockIdx.y;
    const Chunk ck = p.table[chunk_id];
    const uint64_t col = static_cast<uint64_t>(ck.mem_quad) * 4;
    const uint64_t row = static_cast<uint64_t>(worker) * p.stride + col;
    const uint32_t bytes = ((ck.n + 3u) & ~3u) * 4u;      // whole quads: a tensor's tail quad ends in pads
    const __amdgpu_buffer_rsrc_t rx_in = make_rsrc(p.x_in + row, bytes);
    const __amdgpu_buffer_rsrc_t rx_out = make_rsrc(p.x_out + row, bytes);
    const __amdgpu_buffer_rsrc_t rv = make_rsrc(HAS_V ? p.v + row : p.x_in + row, bytes);

    const uint32_t shift = static_cast<uint32_t>(ck.glob_off & 3u);
    const uint32_t e = threadIdx.x * 4;                   // first element of this thread's quad
    const uint32_t off = e * 4;
    const f4 x0 = load_quad(rx_in, off);
    const f4 v0 = HAS_V ? load_quad(rv, off) : f4{0.f, 0.f, 0.f, 0.f};
    constexpr bool QUADRATIC = GRAD == kGradQuadNoisy || GRAD == kGradQuadExact;
    f4 a, c = f4{0.f, 0.f, 0.f, 0.f};                     // a: curvature h, or the caller's gradient
    if (GRAD == kGradExternal) {                          // caller's gradient: read x, v, g; write x, v (20 B)
        a = load_quad(make_rsrc(p.g + row, bytes), off);
    } else if (GRAD == kGradExternalBf16) {               // the same with 16-bit gradients (18 B): a brain float
        const uint16_t *gb = reinterpret_cast<const uint16_t *>(p.g) + row;     // is the upper half of an fp32
        const __amdgpu_buffer_rsrc_t rg =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(gb), 0, static_cast<int>(bytes / 2), 0x00020000);
        const u2 w = __builtin_amdgcn_raw_buffer_load_b64(rg, static_cast<int>(off / 2), 0, kAuxNonTemporal);
        a = f4{__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u),
               __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xffff0000u)};
    } else {
        a = load_quad(make_rsrc(p.h + row, bytes), off);
        c = load_quad(make_rsrc(p.c + row, bytes), off);
    }
    f4 snap = x0, mean = f4{0.f, 0.f, 0.f, 0.f};
    if (TAIL == 1) snap = load_quad(make_rsrc(p.snap + row, bytes), off);
    if (TAIL != 0) {
        // the mean is shared by the W workers of a column: ordinary cached load
        const __amdgpu_buffer_rsrc_t rm = make_rsrc(p.mean + col, bytes);
        mean = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rm, static_cast<int>(off), 0, 0));
    }

    f4 z = f4{0.f, 0.f, 0.f, 0.f};
    if (GRAD == kGradQuadNoisy) z = noise_for_quad((ck.glob_off >> 2) + threadIdx.x, shift, p, worker);
    const float sigma = GRAD == kGradQuadNoisy ? (p.sigma_w ? p.sigma_w[worker] : p.sigma) : 0.0f;
    f4 x, v;
    local_step_quad<HAS_V, QUADRATIC, GRAD == kGradQuadNoisy, TAIL != 0>(x, v, x0, v0, a, c, z, sigma, p.lr, p.momentum,
                                                                          p.weight_decay, snap, mean);

    if (e + 4 > ck.n && e < ck.n) {                       // tensor tail: alignment pads keep their old values
        const uint32_t keep = ck.n - e;                   // 1..3 real elements
        if (keep < 2) { x.y = x0.y; v.y = v0.y; }
        if (keep < 3) { x.z = x0.z; v.z = v0.z; }
        x.w = x0.w; v.w = v0.w;
    }
    store_quad(rx_out, off, x);
    if (HAS_V) store_quad(rv, off, v);
}

// First local step of a round with Step I folded in: the step reads every worker's stored model
// anyway, so a thread that serves one column quad for ALL W workers (as the averaging kernels do)
// gets the weighted mean of the stored models for one extra 4/W-byte store per parameter instead of a
// second pass over them.  The sum runs over the workers in order 0..W-1 with the same expressions as the
// stand-alone mean kernel, so the mean has the same bits.  Loads of workers i+1 .. i+DEPTH are in flight
// during the arithmetic of worker i.  Grid = chunks.  Walking W rows of four arrays per block streams less
// well than the row-per-block step (measured 5.4 against 6.05 TB/s at W = 16, insensitive to prefetch depth
// and to the row stride), which eats about half of the bytes saved.
template <bool HAS_V, int GRAD, bool WEIGHTED, int DEPTH>
__global__ __launch_bounds__(kStepThreads) void quad_step_head_kernel(const StepParams p)
{
    const Chunk ck = p.table[blockIdx.x];
    const uint64_t col = static_cast<uint64_t>(ck.mem_quad) * 4;
    const uint32_t bytes = ((ck.n + 3u) & ~3u) * 4u;
    const uint32_t shift = static_cast<uint32_t>(ck.glob_off & 3u);
    const uint32_t e = threadIdx.x * 4;
    const uint32_t off = e * 4;
    const uint64_t q = (ck.glob_off >> 2) + threadIdx.x;

    struct Row { f4 x, v, h, c; };
    auto load_row = [&](uint32_t w) {
        const uint64_t row = static_cast<uint64_t>(w) * p.stride + col;
        Row r;
        r.x = load_quad(make_rsrc(p.x_in + row, bytes), off);
        r.v = HAS_V ? load_quad(make_rsrc(p.v + row, bytes), off) : f4{0.f, 0.f, 0.f, 0.f};
        r.h = load_quad(make_rsrc(p.h + row, bytes), off);
        r.c = load_quad(make_rsrc(p.c + row, bytes), off);
        return r;
    };

    MeanSum acc;
    acc.clear();
    Row ring[DEPTH];
    #pragma unroll
    for (int j = 0; j < DEPTH; ++j) ring[j] = load_row(static_cast<uint32_t>(j) < p.W ? j : 0);
    for (uint32_t w0 = 0; w0 < p.W; w0 += DEPTH) {
      #pragma unroll
      for (int j = 0; j < DEPTH; ++j) {
        const uint32_t w = w0 + j;
        if (w >= p.W) break;
        const Row cur = ring[j];
        if (w + DEPTH < p.W) ring[j] = load_row(w + DEPTH);
        acc.add<WEIGHTED>(WEIGHTED ? p.weights[w] : 1.0f, cur.x.x, cur.x.y, cur.x.z, cur.x.w);

        f4 z = f4{0.f, 0.f, 0.f, 0.f};
        if (GRAD == kGradQuadNoisy) z = noise_for_quad(q, shift, p, w, w);
        const float sigma = GRAD == kGradQuadNoisy ? (p.sigma_w ? p.sigma_w[w] : p.sigma) : 0.0f;
        f4 x, v;
        local_step_quad<HAS_V, true, GRAD == kGradQuadNoisy, false>(x, v, cur.x, cur.v, cur.h, cur.c, z, sigma, p.lr, p.momentum,
                                                                   p.weight_decay, cur.x, cur.x);
        if (e + 4 > ck.n && e < ck.n) {                   // tensor tail: alignment pads keep their old values
            const uint32_t keep = ck.n - e;
            if (keep < 2) { x.y = cur.x.y; v.y = cur.v.y; }
            if (keep < 3) { x.z = cur.x.z; v.z = cur.v.z; }
            x.w = cur.x.w; v.w = cur.v.w;
        }
        const uint64_t row = static_cast<uint64_t>(w) * p.stride + col;
        store_quad(make_rsrc(p.x_out + row, bytes), off, x);
        if (HAS_V) store_quad(make_rsrc(p.v + row, bytes), off, v);
      }
    }
    acc.finish<WEIGHTED>(p.W);
    // the mean is read again by line 6: ordinary (cached) store
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, f4{acc.s[0], acc.s[1], acc.s[2], acc.s[3]}),
                                           make_rsrc(p.mean_out + col, bytes),
                                           static_cast<int>(off), 0, 0);
}

void launch_head(hipStream_t stream, const StepParams &p, hipEvent_t start, hipEvent_t stop)
{
    const dim3 grid(p.n_chunks), block(kStepThreads);
    const bool has_v = p.momentum != 0.0f, noisy = p.sigma != 0.0f || p.sigma_w, weighted = p.weights != nullptr;
    // rows in flight per thread: 2 measured best (1: 1 % slower, 3 and 4: more registers, no gain)
#define COCOD_LAUNCH_HEAD_D(V, G, Wt, D)                                                                          \
    do {                                                                                                          \
        if (start || stop)                                                                                        \
            hipExtLaunchKernelGGL((quad_step_head_kernel<V, G, Wt, D>), grid, block, 0, stream, start, stop, 0, p);  \
        else                                                                                                      \
            hipLaunchKernelGGL((quad_step_head_kernel<V, G, Wt, D>), grid, block, 0, stream, p);                     \
    } while (0)
#define COCOD_LAUNCH_HEAD(V, G, Wt) COCOD_LAUNCH_HEAD_D(V, G, Wt, 2)
    if (has_v) {
        if (noisy) { if (weighted) COCOD_LAUNCH_HEAD(true, kGradQuadNoisy, true); else COCOD_LAUNCH_HEAD(true, kGradQuadNoisy, false); }
        else       { if (weighted) COCOD_LAUNCH_HEAD(true, kGradQuadExact, true); else COCOD_LAUNCH_HEAD(true, kGradQuadExact, false); }
    } else {
        if (noisy) { if (weighted) COCOD_LAUNCH_HEAD(false, kGradQuadNoisy, true); else COCOD_LAUNCH_HEAD(false, kGradQuadNoisy, false); }
        else       { if (weighted) COCOD_LAUNCH_HEAD(false, kGradQuadExact, true); else COCOD_LAUNCH_HEAD(false, kGradQuadExact, false); }
    }
#undef COCOD_LAUNCH_HEAD
}

template <int TAIL>
void launch_tail(hipStream_t stream, const StepParams &p, hipEvent_t start, hipEvent_t stop)
{
    const dim3 grid = (TAIL != 0 && p.worker_fastest) ? dim3(p.n_chunks * p.W) : dim3(p.n_chunks, p.W), block(kStepThreads);
    const bool has_v = p.momentum != 0.0f;
    const int grad = p.g ? (p.g_bf16 ? kGradExternalBf16 : kGradExternal) : (p.sigma != 0.0f || p.sigma_w ? kGradQuadNoisy : kGradQuadExact);
    // start/stop receive the kernel's own begin and end timestamps; without them an ordinary launch
    // (the only kind a stream capture records)
#define COCOD_LAUNCH_STEP(V, G)                                                                                   \
    do {                                                                                                          \
        if (start || stop)                                                                                        \
            hipExtLaunchKernelGGL((quad_step_kernel<V, G, TAIL>), grid, block, 0, stream, start, stop, 0, p);     \
        else                                                                                                      \
            hipLaunchKernelGGL((quad_step_kernel<V, G, TAIL>), grid, block, 0, stream, p);                        \
    } while (0)
    if (has_v) {
        if (grad == kGradExternal)       COCOD_LAUNCH_STEP(true, kGradExternal);
        else if (grad == kGradExternalBf16) COCOD_LAUNCH_STEP(true, kGradExternalBf16);
        else if (grad == kGradQuadNoisy) COCOD_LAUNCH_STEP(true, kGradQuadNoisy);
        else                             COCOD_LAUNCH_STEP(true, kGradQuadExact);
    } else {
        if (grad == kGradExternal)       COCOD_LAUNCH_STEP(false, kGradExternal);
        else if (grad == kGradExternalBf16) COCOD_LAUNCH_STEP(false, kGradExternalBf16);
        else if (grad == kGradQuadNoisy) COCOD_LAUNCH_STEP(false, kGradQuadNoisy);
        else                             COCOD_LAUNCH_STEP(false, kGradQuadExact);
    }
#undef COCOD_LAUNCH_STEP
}

}  // namespace

hipError_t launch_quad_step(hipStream_t stream, const StepParams &p, hipEvent_t start, hipEvent_t stop)
{
    if (p.mean_out)              launch_head(stream, p, start, stop);     // never with line 6 or a caller's gradient
    else if (!p.snap)            launch_tail<0>(stream, p, start, stop);
    else if (p.snap != p.x_in)   launch_tail<1>(stream, p, start, stop);
    else                         launch_tail<2>(stream, p, start, stop);
    return hipGetLastError();
}

}  // namespace cocod
