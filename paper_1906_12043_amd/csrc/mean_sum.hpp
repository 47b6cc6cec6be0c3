// The weighted mean of Step I of Algorithm 1 (x^_t = sum_i p_i x_t^i) for one column quad, as every
// kernel that forms it computes it: workers in order 0..W-1, fp32, with a compensated (Kahan) running
// sum.  One definition shared by the mean kernel, the fused mean + line 6 kernel, the step kernel
// that forms the mean on its way and the diagnostics, so that all of them produce the same bits.
//
// Why compensated: a plain running sum commits one rounding per worker relative to the PARTIAL SUM,
// and the models of this method are close to each other (that is what the averaging is for), so the
// roundings do not cancel: the mean loses about W/2 ulp (measured 8e-4 relative at W = 65535).
// With the error term the result is accurate to a rounding or two for any W; the four extra
// additions per element hide under the memory time of these kernels.
#pragma once

#include <hip/hip_runtime.h>

namespace cocod {

// N independent element columns per thread: 4 for a thread that owns a 16-byte column quad, 1 for a
// thread that owns a single element column.  The operations on one element are the same either way.
template <int N>
struct MeanSumN {
    float s[N], c[N];

    __device__ __forceinline__ void clear()
    {
        #pragma unroll
        for (int j = 0; j < N; ++j) { s[j] = 0.0f; c[j] = 0.0f; }
    }

    // add p * r to element column j; WEIGHTED == false means p == 1 and no multiply
    template <bool WEIGHTED>
    __device__ __forceinline__ void add_one(int j, float p, float r)
    {
        // No contraction in here: where the compiler knows c == 0 (first worker of an unrolled loop) it
        // turns the fused multiply-add into a plain product and would then fuse that product into the
        // subtraction below, which changes the bits of c from one kernel to the next.
        #pragma clang fp contract(off)
        const float y = WEIGHTED ? __builtin_fmaf(p, r, -c[j]) : r - c[j];
        const float t = s[j] + y;
        c[j] = (t - s[j]) - y;          // what the addition lost, with opposite sign
        s[j] = t;
    }

    // add p * (r0, r1, r2, r3) to a column quad
    template <bool WEIGHTED>
    __device__ __forceinline__ void add(float p, float r0, float r1, float r2, float r3)
    {
        static_assert(N == 4, "quad form");
        add_one<WEIGHTED>(0, p, r0);
        add_one<WEIGHTED>(1, p, r1);
        add_one<WEIGHTED>(2, p, r2);
        add_one<WEIGHTED>(3, p, r3);
    }

    // the mean: the weights already sum to one, or the sum is divided by W
    template <bool WEIGHTED>
    __device__ __forceinline__ void finish(uint32_t W)
    {
        if (!WEIGHTED) {
            const float inv = 1.0f / static_cast<float>(W);
            #pragma unroll
            for (int j = 0; j < N; ++j) s[j] *= inv;
        }
    }
};

using MeanSum = MeanSumN<4>;

}  // namespace cocod
