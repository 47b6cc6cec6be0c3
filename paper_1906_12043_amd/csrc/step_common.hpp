// Device helpers shared by the local-step kernels: 16-byte vector types and streaming accesses
// through raw buffer instructions.  Every model array is streamed once per step and is far larger
// than the caches, so the accesses carry the non-temporal hint; the buffer descriptor covers exactly
// the piece of the row a block (or wave) works on, so lanes past its end read zeros and their stores
// are dropped by the hardware range check: no divergent tail code.
#pragma once
#include "internal.hpp"

namespace cocod {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

constexpr int kAuxNonTemporal = 2;   // cache-policy bits of the buffer instructions: nt

// Raw buffer descriptor over `bytes` bytes starting at p (stride 0, 32-bit data format).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const float *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p), 0, static_cast<int>(bytes), 0x00020000);
}
__device__ __forceinline__ f4 load_quad(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    return __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(r, static_cast<int>(byte_off), 0, kAuxNonTemporal));
}
__device__ __forceinline__ void store_quad(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, f4 a)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, a), r, static_cast<int>(byte_off), 0, kAuxNonTemporal);
}

// Where the stochastic gradient G of a step comes from.
enum { kGradQuadNoisy = 0, kGradQuadExact = 1, kGradExternal = 2, kGradExternalBf16 = 3 };

// Line 6 of Algorithm 1 on a quad: x = mean + (x - stored model), the parenthesis first.
__device__ __forceinline__ f4 line6_quad(const f4 mean, const f4 x, const f4 snap)
{
    #pragma clang fp contract(off)
    return mean + (x - snap);
}

// One local step of Algorithm 1's Step II on a quad of parameters, with the experiments' optimizer,
// and optionally line 6 on the result:
//     G = h (x - c) + sigma z      (QUADRATIC; else G = a, the caller's gradient)
//     g = G + lambda x ;  v = mu v + g ;  x = x - gamma v      (mu = 0: x = x - gamma g)
//     x = mean + (x - snap)                                      (LINE6)
// ONE definition for every kernel that takes a step, with every fused multiply-add written out and
// contraction switched off: left to the compiler, which products get fused depends on the code around
// them (h (x - c) + sigma z can become fma(sigma, z, .) or fma(h, x - c, .)), and kernels that must
// agree bit for bit (every mode and launch shape of the step) would differ in the last place.
template <bool HAS_V, bool QUADRATIC, bool NOISY, bool LINE6>
__device__ __forceinline__ void local_step_quad(f4 &x, f4 &v, const f4 x0, const f4 v0, const f4 a, const f4 c, const f4 z,
                                                float sigma, float lr, float momentum, float weight_decay,
                                                const f4 snap, const f4 mean)
{
    #pragma clang fp contract(off)
    #pragma unroll
    for (int j = 0; j < 4; ++j) {
        float g = QUADRATIC ? a[j] * (x0[j] - c[j]) : a[j];
        if (NOISY) g = __builtin_fmaf(sigma, z[j], g);
        g = __builtin_fmaf(weight_decay, x0[j], g);
        float vj = v0[j];
        if (HAS_V) { vj = __builtin_fmaf(momentum, v0[j], g); g = vj; }
        float xj = __builtin_fmaf(-lr, g, x0[j]);
        if (LINE6) xj = mean[j] + (xj - snap[j]);
        x[j] = xj;
        v[j] = vj;
    }
}

}  // namespace cocod
