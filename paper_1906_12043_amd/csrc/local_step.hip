// Step II of Algorithm 1 (CoCoD-SGD) for the synthetic quadratic workers and for a caller's gradient:
// one fused local step.  Per parameter j of worker i at global step t
//     G = h_ij (x_j - c_ij) + sigma z(seed, i, t, j)        stochastic gradient (or the caller's g)
//     g = G + lambda x ;  v = mu v + g ;  x = x - gamma v    momentum SGD of the experiments
// The gradient is never written to memory: the kernel reads x, v, h, c and writes x, v (24 bytes per
// parameter; 16 when mu = 0 and v is untouched; 20 / 18 with a caller's fp32 / 16-bit gradient).
//
// Work decomposition.  A tile is Q x 64 consecutive 16-byte quads of one tensor (Q = 1 or 2: four or
// two tiles per 1024-element chunk of the chunk table, which maps a block to its tensor slice, so one
// launch covers a whole parameter list); a WAVE serves one tile of one worker row and moves Q
// contiguous KiB per array.  Every wave is self-contained (its noise too: the generator block of the
// right-hand neighbour, needed when a tensor starts at a global index that is not a multiple of 4,
// comes from the next lane or the wave's own next pass), so block shape is free:
//   PLAIN / TAIL   single-wave blocks, grid (tiles, workers).  Measured on MI355X at W = 16, d = 11.2 M:
//             6.6 TB/s against 6.05 TB/s for the same step in 4-wave blocks and 5.8 in 16-wave blocks;
//             small independent blocks stream best on this chip.  TAIL is the round's last step
//             with line 6 applied to the fresh model before it is stored, x = mean + (x_new - x_stored).
//   HEAD      the round's first step also forms Step I's weighted mean of the models it reads.  One
//             block = one tile of ALL W workers, one wave per worker row (16 rows at a time): every wave
//             puts its row's tile into LDS, the block sums the tile's columns over the workers in order
//             0..W-1 (the one compensated sum of mean_sum.hpp, so the bits equal those of the stand-alone
//             mean kernel) and stores the mean: 4/W bytes per parameter instead of a pass of its own.
//   ONE_PASS  k = 1: Step I, the local step and line 6 in a single sweep (24 + 4/W bytes per
//             parameter): as HEAD, and line 6 is applied with the tile's mean before anything is stored.
//
// Memory path: every model array is streamed exactly once per step and is far larger than the caches,
// so all accesses carry the non-temporal hint and go through buffer instructions whose descriptor
// covers exactly the tile (step_common.hpp).  The mean is shared by the W workers of a column and is
// read with an ordinary cached load.
#include "internal.hpp"
#include "step_common.hpp"
#include "philox.hpp"
#include "mean_sum.hpp"

#include <hip/hip_ext.h>

namespace cocod {
namespace {

enum { kModePlain = 0, kModeTail = 1, kModeTailIn = 2, kModeHead = 3, kModeOnePass = 4, kModeLine6 = 5 };

// Normals for the Q memory quads of one lane.  Quad u of lane l covers global indices
// 4 (q0 + 64 u + l) + shift .. + 3: with shift == 0 exactly generator block q0 + 64 u + l, else the
// last 4 - shift normals of that block and the first `shift` of the next one.
template <int Q>
__device__ __forceinline__ void noise_for_lane(f4 (&z)[Q], uint64_t q0, uint32_t shift, uint32_t lane, uint32_t worker,
                                               uint32_t step, const StepParams &p)
{
    Normals4 a[Q];
    #pragma unroll
    for (int u = 0; u < Q; ++u)
        a[u] = box_muller_fast(philox4x32_10(static_cast<uint32_t>(q0 + 64u * u + lane), step, worker, kTagNoise, p.key0, p.key1));
    if (shift == 0) {                                                   // block-uniform
        #pragma unroll
        for (int u = 0; u < Q; ++u) z[u] = f4{a[u].z[0], a[u].z[1], a[u].z[2], a[u].z[3]};
        return;
    }
    #pragma unroll
    for (int u = 0; u < Q; ++u) {
        float b0 = __shfl_down(a[u].z[0], 1, 64), b1 = __shfl_down(a[u].z[1], 1, 64), b2 = __shfl_down(a[u].z[2], 1, 64);
        if (u + 1 < Q) {                                                // lane 63's neighbour is lane 0 of the next pass
            const int nu = u + 1 < Q ? u + 1 : u;
            const float n0 = __shfl(a[nu].z[0], 0, 64), n1 = __shfl(a[nu].z[1], 0, 64), n2 = __shfl(a[nu].z[2], 0, 64);
            if (lane == 63u) { b0 = n0; b1 = n1; b2 = n2; }
        } else if (lane == 63u) {                                       // one lane per wave: the block behind the tile
            const Normals4 nb = box_muller_fast(
                philox4x32_10(static_cast<uint32_t>(q0 + 64u * Q), step, worker, kTagNoise, p.key0, p.key1));
            b0 = nb.z[0]; b1 = nb.z[1]; b2 = nb.z[2];
        }
        if (shift == 1)      z[u] = f4{a[u].z[1], a[u].z[2], a[u].z[3], b0};
        else if (shift == 2) z[u] = f4{a[u].z[2], a[u].z[3], b0, b1};
        else                 z[u] = f4{a[u].z[3], b0, b1, b2};
    }
}

// blockDim.x = 64 * (waves per block); NWMAX bounds it for the register allocator.
// Grid: x = tiles (chunks * 4 / Q); y = groups of workers (modes without a mean: ceil(W / waves);
// mean-forming modes: 1, the block loops over its worker groups itself).
// Dynamic LDS (mean-forming modes only): W rows of the tile, then (ONE_PASS) the tile of the mean.
template <bool HAS_V, int GRAD, int MODE, bool WEIGHTED, int NWMAX, int Q>
__global__ __launch_bounds__(64 * NWMAX) void local_step_kernel(const StepParams p)
{
    constexpr bool FORMS_MEAN = MODE == kModeHead || MODE == kModeOnePass;
    constexpr bool LINE6 = MODE == kModeTail || MODE == kModeTailIn || MODE == kModeOnePass || MODE == kModeLine6;
    constexpr uint32_t PARTS = 4 / Q, TILE_ELEMS = Q * 256;
    extern __shared__ __attribute__((aligned(16))) float lds[];

    // Grid: x = tiles, y = worker groups.  A step with line 6 whose mean does not fit the last-level
    // cache runs on a 1-D grid in PANELS of p.panel_tiles tiles instead: inside a panel the blocks
    // go worker by worker, so every worker still streams a contiguous run of its row, and the W readers
    // of a panel of the mean run close enough together for it to come from memory once.
    const uint32_t panel_tiles = (!FORMS_MEAN && LINE6) ? p.panel_tiles : 0u;
    uint32_t tile_id = blockIdx.x, group = blockIdx.y;
    if (panel_tiles != 0) {
        const uint32_t n_groups = (p.W + (blockDim.x >> 6) - 1) / (blockDim.x >> 6);
        const uint32_t n_tiles = p.n_chunks * PARTS;
        const uint32_t per_panel = panel_tiles * n_groups;
        const uint32_t panel = blockIdx.x / per_panel, r = blockIdx.x % per_panel;
        const uint32_t first_tile = panel * panel_tiles;
        const uint32_t here = n_tiles - first_tile < panel_tiles ? n_tiles - first_tile : panel_tiles;   // the last panel is short
        group = r / here;
        tile_id = first_tile + r % here;
        if (group >= n_groups) return;                       // block-uniform: padding of the short last panel
    }
    const uint32_t chunk_id = tile_id / PARTS, part = tile_id % PARTS;
    const Chunk ck = p.table[chunk_id];
    const uint32_t first = part * TILE_ELEMS;                 // first element of the tile inside its chunk
    if (first >= ck.n) return;                                // block-uniform: the tensor ends before this tile
    const uint32_t n = ck.n - first < TILE_ELEMS ? ck.n - first : TILE_ELEMS;     // real elements in the tile
    const uint32_t n4 = (n + 3u) & ~3u;                       // whole quads: a tensor's tail quad ends in pads
    const uint32_t bytes = n4 * 4u;
    const uint64_t col = static_cast<uint64_t>(ck.mem_quad) * 4 + first;
    const uint32_t shift = static_cast<uint32_t>(ck.glob_off & 3u);
    const uint64_t q0 = ((ck.glob_off + first) >> 2);         // generator block of lane 0's first quad
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const uint32_t step = p.step_base ? *p.step_base + p.step : p.step;      // wave-uniform

    struct Row { f4 v[Q], h[Q], c[Q]; };                      // what a step needs beside the model itself
    auto load_row = [&](uint32_t w) {
        const uint64_t row = static_cast<uint64_t>(w) * p.stride + col;
        Row r;
        #pragma unroll
        for (int u = 0; u < Q; ++u) {
            const uint32_t off = (64u * u + lane) * 16u;
            r.v[u] = HAS_V ? load_quad(make_rsrc(p.v + row, bytes), off) : f4{0.f, 0.f, 0.f, 0.f};
            r.c[u] = f4{0.f, 0.f, 0.f, 0.f};
            if (GRAD == kGradQuadNoisy || GRAD == kGradQuadExact) {
                r.h[u] = load_quad(make_rsrc(p.h + row, bytes), off);
                r.c[u] = load_quad(make_rsrc(p.c + row, bytes), off);
            } else if (GRAD == kGradExternal) {
                r.h[u] = load_quad(make_rsrc(p.g + row, bytes), off);         // the caller's gradient
            } else {                                                          // 16-bit gradients: the upper halves of fp32
                const uint16_t *gb = reinterpret_cast<const uint16_t *>(p.g) + row;
                const __amdgpu_buffer_rsrc_t rg =
                    __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(gb), 0, static_cast<int>(bytes / 2), 0x00020000);
                const u2 t = __builtin_amdgcn_raw_buffer_load_b64(rg, static_cast<int>(off / 2), 0, kAuxNonTemporal);
                r.h[u] = f4{__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xffff0000u),
                            __uint_as_float(t.y << 16), __uint_as_float(t.y & 0xffff0000u)};
            }
        }
        return r;
    };
    auto load_x = [&](f4 (&x)[Q], uint32_t w) {
        const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x_in + static_cast<uint64_t>(w) * p.stride + col, bytes);
        #pragma unroll
        for (int u = 0; u < Q; ++u) x[u] = load_quad(rx, (64u * u + lane) * 16u);
    };
    // the step itself for worker w: x0 = model read, r = its other streams, m = mean quads (line 6)
    auto step_row = [&](uint32_t w, const f4 (&x0)[Q], const Row &r, const f4 (&snap)[Q], const f4 (&m)[Q]) {
        const uint64_t row = static_cast<uint64_t>(w) * p.stride + col;
        const __amdgpu_buffer_rsrc_t rx_out = make_rsrc(p.x_out + row, bytes);
        const __amdgpu_buffer_rsrc_t rv = make_rsrc(HAS_V ? p.v + row : p.x_out + row, bytes);
        f4 z[Q];
        #pragma unroll
        for (int u = 0; u < Q; ++u) z[u] = f4{0.f, 0.f, 0.f, 0.f};
        if (GRAD == kGradQuadNoisy) noise_for_lane<Q>(z, q0, shift, lane, w, step, p);
        const float sigma = GRAD == kGradQuadNoisy ? (p.sigma_w ? p.sigma_w[w] : p.sigma) : 0.0f;
        #pragma unroll
        for (int u = 0; u < Q; ++u) {
            const uint32_t e = (64u * u + lane) * 4u, off = e * 4u;
            f4 x, v;
            local_step_quad<HAS_V, GRAD == kGradQuadNoisy || GRAD == kGradQuadExact, GRAD == kGradQuadNoisy, LINE6>(
                x, v, x0[u], r.v[u], r.h[u], r.c[u], z[u], sigma, p.lr, p.momentum, p.weight_decay, snap[u], m[u]);
            if (e + 4 > n && e < n) {                     // tensor tail: alignment pads keep their old values
                const uint32_t keep = n - e;              // 1..3 real elements
                if (keep < 2) { x.y = x0[u].y; v.y = r.v[u].y; }
                if (keep < 3) { x.z = x0[u].z; v.z = r.v[u].z; }
                x.w = x0[u].w; v.w = r.v[u].w;
            }
            store_quad(rx_out, off, x);
            if (HAS_V) store_quad(rv, off, v);
        }
    };

    if (!FORMS_MEAN) {
        const uint32_t w = group * nw + wave;
        if (w >= p.W) return;                              // no barrier in these modes
        f4 x0[Q], snap[Q], m[Q];
        load_x(x0, w);
        if constexpr (MODE == kModeLine6) {                // line 6 alone, in place: x = mean + (x - stored model)
            const uint64_t row = static_cast<uint64_t>(w) * p.stride + col;
            const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.snap + row, bytes), rm = make_rsrc(p.mean + col, bytes);
            const __amdgpu_buffer_rsrc_t rx_out = make_rsrc(p.x_out + row, bytes);
            #pragma unroll
            for (int u = 0; u < Q; ++u) {
                const uint32_t e = (64u * u + lane) * 4u, off = e * 4u;
                snap[u] = load_quad(rs, off);
                m[u] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rm, static_cast<int>(off), 0, 0));
            }
            #pragma unroll
            for (int u = 0; u < Q; ++u) {
                const uint32_t e = (64u * u + lane) * 4u;
                f4 x = line6_quad(m[u], x0[u], snap[u]);
                if (e + 4 > n && e < n) {                  // tensor tail: alignment pads keep their old values
                    const uint32_t keep = n - e;
                    if (keep < 2) x.y = x0[u].y;
                    if (keep < 3) x.z = x0[u].z;
                    x.w = x0[u].w;
                }
                store_quad(rx_out, e * 4u, x);
            }
            return;
        }
        const Row r = load_row(w);
        #pragma unroll
        for (int u = 0; u < Q; ++u) { snap[u] = x0[u]; m[u] = f4{0.f, 0.f, 0.f, 0.f}; }
        if (MODE == kModeTail) {
            const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.snap + static_cast<uint64_t>(w) * p.stride + col, bytes);
            #pragma unroll
            for (int u = 0; u < Q; ++u) snap[u] = load_quad(rs, (64u * u + lane) * 16u);
        }
        if (LINE6) {                                       // shared by the block's waves: ordinary cached load
            const __amdgpu_buffer_rsrc_t rm = make_rsrc(p.mean + col, bytes);
            #pragma unroll
            for (int u = 0; u < Q; ++u)
                m[u] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rm, static_cast<int>((64u * u + lane) * 16u), 0, 0));
        }
        step_row(w, x0, r, snap, m);
        return;
    }

    // ---- mean-forming modes: the tile of every worker passes through LDS -----------------------------
    float *xs = lds;                                          // [W][TILE_ELEMS]
    float *ms = lds + static_cast<size_t>(p.W) * TILE_ELEMS;  // [TILE_ELEMS], ONE_PASS only
    // the first group's other streams start now, so that they are in flight across the barriers
    Row cur;
    if (wave < p.W) cur = load_row(wave);
    // rows of the block's worker groups into LDS, four groups' loads in flight at a time (a block with
    // fewer waves than workers would otherwise pay one memory round trip per group)
    for (uint32_t w0 = wave; w0 < p.W; w0 += 4 * nw) {
        f4 x[4][Q];
        #pragma unroll
        for (int b = 0; b < 4; ++b)
            if (w0 + b * nw < p.W) load_x(x[b], w0 + b * nw);        // wave-uniform
        #pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t w = w0 + b * nw;
            if (w < p.W) {
                #pragma unroll
                for (int u = 0; u < Q; ++u)
                    *reinterpret_cast<f4 *>(xs + static_cast<size_t>(w) * TILE_ELEMS + (64u * u + lane) * 4u) = x[b][u];
            }
        }
    }
    __syncthreads();
    // Step I for this tile: thread t owns element columns t, t + blockDim, ...; workers in order.
    for (uint32_t e = threadIdx.x; e < n4; e += blockDim.x) {
        MeanSumN<1> acc;
        acc.clear();
        uint32_t w = 0;
        for (; w + 8 <= p.W; w += 8) {
            float r[8];
            #pragma unroll
            for (int b = 0; b < 8; ++b) r[b] = xs[static_cast<size_t>(w + b) * TILE_ELEMS + e];
            #pragma unroll
            for (int b = 0; b < 8; ++b) acc.add_one<WEIGHTED>(0, WEIGHTED ? p.weights[w + b] : 1.0f, r[b]);
        }
        for (; w < p.W; ++w) acc.add_one<WEIGHTED>(0, WEIGHTED ? p.weights[w] : 1.0f, xs[static_cast<size_t>(w) * TILE_ELEMS + e]);
        acc.finish<WEIGHTED>(p.W);
        p.mean_out[col + e] = acc.s[0];                    // read again by line 6: ordinary (cached) store
        if (MODE == kModeOnePass) ms[e] = acc.s[0];
    }
    if (MODE == kModeOnePass) __syncthreads();
    for (uint32_t w = wave; w < p.W; w += nw) {
        Row next = cur;
        if (w + nw < p.W) next = load_row(w + nw);           // the next group's streams run under this group's arithmetic
        f4 x0[Q], m[Q];
        #pragma unroll
        for (int u = 0; u < Q; ++u) {
            x0[u] = *reinterpret_cast<const f4 *>(xs + static_cast<size_t>(w) * TILE_ELEMS + (64u * u + lane) * 4u);
            m[u] = MODE == kModeOnePass ? *reinterpret_cast<const f4 *>(ms + (64u * u + lane) * 4u) : f4{0.f, 0.f, 0.f, 0.f};
        }
        step_row(w, x0, cur, x0, m);
        cur = next;
    }
}

// More than the default 64 KB of dynamic LDS, once per kernel instantiation.
template <typename K>
hipError_t allow_big_lds(K kernel, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
}

constexpr size_t kTileLdsMax = 132u << 10;      // of the 160 KB per compute unit

template <bool HAS_V, int GRAD, int MODE, bool WEIGHTED, int NWMAX, int Q>
hipError_t launch_one(hipStream_t stream, const StepParams &p, uint32_t waves, hipEvent_t start, hipEvent_t stop)
{
    constexpr bool FORMS_MEAN = MODE == kModeHead || MODE == kModeOnePass;
    auto kernel = local_step_kernel<HAS_V, GRAD, MODE, WEIGHTED, NWMAX, Q>;
    size_t lds = 0;
    if (FORMS_MEAN) {
        lds = (static_cast<size_t>(p.W) + (MODE == kModeOnePass ? 1 : 0)) * Q * 256 * sizeof(float);
        static const hipError_t lds_ok = allow_big_lds(kernel, kTileLdsMax);
        if (lds_ok != hipSuccess) return lds_ok;
    }
    constexpr bool LINE6 = MODE == kModeTail || MODE == kModeTailIn || MODE == kModeLine6;
    const uint32_t groups = FORMS_MEAN ? 1u : (p.W + waves - 1) / waves;
    const uint32_t tiles = p.n_chunks * (4 / Q);
    // panels: every panel takes panel_tiles * groups block ids, the short last one included
    const uint32_t panels = p.panel_tiles ? (tiles + p.panel_tiles - 1) / p.panel_tiles : 0;
    const dim3 grid = (LINE6 && p.panel_tiles) ? dim3(panels * p.panel_tiles * groups) : dim3(tiles, groups), block(64 * waves);
    if (start || stop) hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, start, stop, 0, p);
    else               hipLaunchKernelGGL(kernel, grid, block, lds, stream, p);
    return hipGetLastError();
}

template <int MODE, bool WEIGHTED, int NWMAX, int Q>
hipError_t launch_grad(hipStream_t stream, const StepParams &p, uint32_t waves, hipEvent_t start, hipEvent_t stop)
{
    const bool has_v = p.momentum != 0.0f;
    const int grad = p.g ? (p.g_bf16 ? kGradExternalBf16 : kGradExternal) : (p.sigma != 0.0f || p.sigma_w ? kGradQuadNoisy : kGradQuadExact);
    constexpr bool FORMS_MEAN = MODE == kModeHead || MODE == kModeOnePass;
    if (!FORMS_MEAN) {                      // the caller's gradient: plain steps and steps that carry line 6
        if (grad == kGradExternal)
            return has_v ? launch_one<true, kGradExternal, MODE, false, NWMAX, Q>(stream, p, waves, start, stop)
                         : launch_one<false, kGradExternal, MODE, false, NWMAX, Q>(stream, p, waves, start, stop);
        if (grad == kGradExternalBf16)
            return has_v ? launch_one<true, kGradExternalBf16, MODE, false, NWMAX, Q>(stream, p, waves, start, stop)
                         : launch_one<false, kGradExternalBf16, MODE, false, NWMAX, Q>(stream, p, waves, start, stop);
    } else if (grad != kGradQuadNoisy && grad != kGradQuadExact) {
        return hipErrorInvalidValue;
    }
    if (grad == kGradQuadNoisy)
        return has_v ? launch_one<true, kGradQuadNoisy, MODE, WEIGHTED, NWMAX, Q>(stream, p, waves, start, stop)
                     : launch_one<false, kGradQuadNoisy, MODE, WEIGHTED, NWMAX, Q>(stream, p, waves, start, stop);
    return has_v ? launch_one<true, kGradQuadExact, MODE, WEIGHTED, NWMAX, Q>(stream, p, waves, start, stop)
                 : launch_one<false, kGradQuadExact, MODE, WEIGHTED, NWMAX, Q>(stream, p, waves, start, stop);
}

// Launch shapes (measured on MI355X, see the file header): single-wave blocks with one quad per lane
// for the steps whose waves are independent; for the mean-forming steps sixteen worker rows per block,
// one quad per lane up to W = 16 and two above (fewer, larger blocks when every wave serves several rows).
template <int MODE>
hipError_t launch_mode(hipStream_t stream, const StepParams &p, hipEvent_t start, hipEvent_t stop)
{
    constexpr bool FORMS_MEAN = MODE == kModeHead || MODE == kModeOnePass;
    if constexpr (!FORMS_MEAN) {
        return launch_grad<MODE, false, 1, 1>(stream, p, 1, start, stop);
    } else {
        const uint32_t waves = p.W < 16u ? p.W : 16u;
        const int q = local_step_mean_quads_per_lane(p.W, MODE == kModeOnePass);
        if (q == 0) return hipErrorInvalidValue;
        if (p.weights) return q == 2 ? launch_grad<MODE, true, 16, 2>(stream, p, waves, start, stop)
                                     : launch_grad<MODE, true, 16, 1>(stream, p, waves, start, stop);
        return q == 2 ? launch_grad<MODE, false, 16, 2>(stream, p, waves, start, stop)
                      : launch_grad<MODE, false, 16, 1>(stream, p, waves, start, stop);
    }
}

}  // namespace

int local_step_mean_quads_per_lane(uint32_t W, bool one_pass)
{
    const size_t rows = static_cast<size_t>(W) + (one_pass ? 1 : 0);       // the W model rows, and the mean's in one-pass mode
    if (W > 16 && rows * 2 * 256 * sizeof(float) <= kTileLdsMax) return 2;
    if (rows * 256 * sizeof(float) <= kTileLdsMax) return 1;
    return 0;
}

hipError_t launch_line6(hipStream_t stream, const StepParams &p)
{
    return launch_one<false, kGradQuadExact, kModeLine6, false, 1, 1>(stream, p, 1, nullptr, nullptr);
}

hipError_t launch_local_step(hipStream_t stream, const StepParams &p, hipEvent_t start, hipEvent_t stop)
{
    if (p.mean_out) return p.snap ? launch_mode<kModeOnePass>(stream, p, start, stop) : launch_mode<kModeHead>(stream, p, start, stop);
    if (!p.snap) return launch_mode<kModePlain>(stream, p, start, stop);
    if (p.snap != p.x_in) return launch_mode<kModeTail>(stream, p, start, stop);
    return launch_mode<kModeTailIn>(stream, p, start, stop);
}

}  // namespace cocod
