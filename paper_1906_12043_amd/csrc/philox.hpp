// Device-side counter-based random numbers for the local step and the data fill.
//
// Generator: Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).
// Keying: key = (seed low, seed high); counter = (j >> 2, step, worker, tag), so
// one 128-bit block serves the four consecutive parameters 4q .. 4q+3.  Step II
// of Algorithm 1 only requires some stochastic gradient of a mini-batch; the
// seeded noise stands in for the sampling of that mini-batch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cocod {

struct Words4 { uint32_t w[4]; };

__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1)
{
    #pragma unroll
    for (int r = 0; r < 10; ++r) {
        // 32x32 -> 64 products; the compiler emits one wide multiply each
        const uint64_t pa = static_cast<uint64_t>(0xD2511F53u) * c0;
        const uint64_t pb = static_cast<uint64_t>(0xCD9E8D57u) * c2;
        const uint32_t n0 = static_cast<uint32_t>(pb >> 32) ^ c1 ^ k0;
        const uint32_t n2 = static_cast<uint32_t>(pa >> 32) ^ c3 ^ k1;
        c1 = static_cast<uint32_t>(pb);
        c3 = static_cast<uint32_t>(pa);
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;   // key schedule is wave-uniform: scalar ALU
        k1 += 0xBB67AE85u;
    }
    Words4 out;
    out.w[0] = c0; out.w[1] = c1; out.w[2] = c2; out.w[3] = c3;
    return out;
}

// top 24 bits -> [0,1) on a 2^-24 grid (exact in fp32)
__device__ __forceinline__ float u_half_open(uint32_t r) { return static_cast<float>(r >> 8) * 0x1p-24f; }
// top 24 bits -> (0,1]
__device__ __forceinline__ float u_open_zero(uint32_t r) { return static_cast<float>((r >> 8) + 1u) * 0x1p-24f; }

struct Normals4 { float z[4]; };

// Box-Muller on word pairs (0,1) and (2,3): radius from the first word, angle from
// the second, cosine to the even output and sine to the odd one.
// Fast variant for the hot loop: hardware log2 / sqrt / sin / cos (the sine and
// cosine units take their argument in revolutions, which is exactly U2).
__device__ __forceinline__ Normals4 box_muller_fast(const Words4 &r)
{
    Normals4 out;
    #pragma unroll
    for (int pair = 0; pair < 2; ++pair) {
        const float u1 = u_open_zero(r.w[2 * pair]);
        const float u2 = u_half_open(r.w[2 * pair + 1]);
        // -2 ln u1 = (-2 ln 2) log2 u1
        const float radius = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(u1));
        out.z[2 * pair]     = radius * __builtin_amdgcn_cosf(u2);
        out.z[2 * pair + 1] = radius * __builtin_amdgcn_sinf(u2);
    }
    return out;
}

// Accurate variant (library log / sincospi) for data that is generated once.
__device__ __forceinline__ Normals4 box_muller_accurate(const Words4 &r)
{
    Normals4 out;
    #pragma unroll
    for (int pair = 0; pair < 2; ++pair) {
        const float u1 = u_open_zero(r.w[2 * pair]);
        const float u2 = u_half_open(r.w[2 * pair + 1]);
        const float radius = sqrtf(-2.0f * logf(u1));
        float s, co;
        sincospif(2.0f * u2, &s, &co);
        out.z[2 * pair]     = radius * co;
        out.z[2 * pair + 1] = radius * s;
    }
    return out;
}

}  // namespace cocod
