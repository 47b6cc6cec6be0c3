// Step II of Algorithm 1 (CoCoD-SGD) for the synthetic quadratic workers: one
// fused local step.  Per parameter j of worker i at global step t
//     G = h_ij (x_j - c_ij) + sigma z(seed, i, t, j)        stochastic gradient
//     g = G + lambda x ;  v = mu v + g ;  x = x - gamma v    momentum SGD of the experiments
// The gradient is never written to memory: the kernel reads x, v, h, c and writes
// x, v (24 bytes per parameter; 16 when mu = 0 and v is untouched).
//
// Work decomposition: grid = (chunks, workers).  A chunk is up to 4096 consecutive
// elements of one tensor (multi-tensor apply: the chunk table maps a block to its
// tensor slice, so one launch covers a whole parameter list).  A thread owns one
// 16-byte quad per unrolled pass; a wave reads 1 KiB contiguous per array per pass.
// The generator's 128-bit block is keyed by the UNPADDED global parameter index, so
// results do not depend on how tensors are packed; when a tensor starts at a global
// index that is not a multiple of 4, a thread's quad straddles two generator blocks
// (block-uniform case, second block computed only then).
#include "internal.hpp"
#include "philox.hpp"

namespace cocod {
namespace {

constexpr int kUnroll = kChunkElems / (kStepThreads * 4);   // quads per thread
static_assert(kUnroll * kStepThreads * 4 == kChunkElems, "chunk must split evenly");

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ void st4(float *p, const float4 &a) { *reinterpret_cast<float4 *>(p) = a; }

// Four normals for the thread's quad whose first element has global index 4*q + shift.
__device__ __forceinline__ Normals4 noise_for_quad(uint64_t q, uint32_t shift, const StepParams &p, uint32_t worker)
{
    const Normals4 a = box_muller_fast(
        philox4x32_10(static_cast<uint32_t>(q), p.step, worker, kTagNoise, p.key0, p.key1));
    if (shift == 0) return a;                               // block-uniform branch
    const Normals4 b = box_muller_fast(
        philox4x32_10(static_cast<uint32_t>(q + 1), p.step, worker, kTagNoise, p.key0, p.key1));
    Normals4 out;
    if (shift == 1)      { out.z[0] = a.z[1]; out.z[1] = a.z[2]; out.z[2] = a.z[3]; out.z[3] = b.z[0]; }
    else if (shift == 2) { out.z[0] = a.z[2]; out.z[1] = a.z[3]; out.z[2] = b.z[0]; out.z[3] = b.z[1]; }
    else                 { out.z[0] = a.z[3]; out.z[1] = b.z[0]; out.z[2] = b.z[1]; out.z[3] = b.z[2]; }
    return out;
}

template <bool HAS_V>
__device__ __forceinline__ void update_one(float &x, float &v, float h, float c, float noise, const StepParams &p)
{
    float g = h * (x - c) + noise;
    g = g + p.weight_decay * x;
    if (HAS_V) {
        v = p.momentum * v + g;
        g = v;
    }
    x = x - p.lr * g;
}

template <bool HAS_V, bool NOISE, bool FULL>
__device__ __forceinline__ void process_chunk(const StepParams &p, const Chunk &ck, uint32_t worker)
{
    const uint64_t row = static_cast<uint64_t>(worker) * p.stride + ck.mem_off;
    const float *xin = p.x_in + row;
    float *xout = p.x_out + row;
    float *vp = HAS_V ? p.v + row : nullptr;
    const float *hp = p.h + row;
    const float *cp = p.c + row;
    const uint32_t shift = static_cast<uint32_t>(ck.glob_off & 3u);
    const uint64_t q_base = ck.glob_off >> 2;

    float4 X[kUnroll], V[kUnroll], H[kUnroll], Cc[kUnroll];
    bool live[kUnroll];
    #pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const uint32_t e = (u * kStepThreads + threadIdx.x) * 4;
        live[u] = FULL || e < ck.n;
        if (live[u]) {
            X[u] = ld4(xin + e);
            if (HAS_V) V[u] = ld4(vp + e);
            H[u] = ld4(hp + e);
            Cc[u] = ld4(cp + e);
        }
    }
    #pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        if (!live[u]) continue;
        const uint32_t e = (u * kStepThreads + threadIdx.x) * 4;
        Normals4 nz;
        if (NOISE) {
            nz = noise_for_quad(q_base + (e >> 2), shift, p, worker);
            #pragma unroll
            for (int i = 0; i < 4; ++i) nz.z[i] *= p.sigma;
        } else {
            nz.z[0] = nz.z[1] = nz.z[2] = nz.z[3] = 0.0f;
        }
        float4 x = X[u];
        float4 v = HAS_V ? V[u] : make_float4(0.f, 0.f, 0.f, 0.f);
        update_one<HAS_V>(x.x, v.x, H[u].x, Cc[u].x, nz.z[0], p);
        update_one<HAS_V>(x.y, v.y, H[u].y, Cc[u].y, nz.z[1], p);
        update_one<HAS_V>(x.z, v.z, H[u].z, Cc[u].z, nz.z[2], p);
        update_one<HAS_V>(x.w, v.w, H[u].w, Cc[u].w, nz.z[3], p);
        if (!FULL && e + 4 > ck.n) {          // tensor tail: alignment pads keep their old values
            const uint32_t keep = ck.n - e;   // 1..3 real elements
            if (keep < 2) { x.y = X[u].y; if (HAS_V) v.y = V[u].y; }
            if (keep < 3) { x.z = X[u].z; if (HAS_V) v.z = V[u].z; }
            x.w = X[u].w; if (HAS_V) v.w = V[u].w;
        }
        st4(xout + e, x);
        if (HAS_V) st4(vp + e, v);
    }
}

template <bool HAS_V, bool NOISE>
__global__ __launch_bounds__(kStepThreads) void quad_step_kernel(const StepParams p)
{
    const Chunk ck = p.table[blockIdx.x];
    if (ck.n == kChunkElems) process_chunk<HAS_V, NOISE, true>(p, ck, blockIdx.y);
    else                     process_chunk<HAS_V, NOISE, false>(p, ck, blockIdx.y);
}

}  // namespace

hipError_t launch_quad_step(hipStream_t stream, const StepParams &p)
{
    const dim3 grid(p.n_chunks, p.W), block(kStepThreads);
    const bool has_v = p.momentum != 0.0f, noise = p.sigma != 0.0f;
    if (has_v && noise)       hipLaunchKernelGGL((quad_step_kernel<true, true>), grid, block, 0, stream, p);
    else if (has_v && !noise) hipLaunchKernelGGL((quad_step_kernel<true, false>), grid, block, 0, stream, p);
    else if (noise)           hipLaunchKernelGGL((quad_step_kernel<false, true>), grid, block, 0, stream, p);
    else                      hipLaunchKernelGGL((quad_step_kernel<false, false>), grid, block, 0, stream, p);
    return hipGetLastError();
}

}  // namespace cocod
