// On-device draw of the synthetic per-worker objective f_i(x) = 1/2 sum_j h_ij (x_j - c_ij)^2
// (h_ij = 0.5 + 1.5 U, c_ij standard normal) and a generator check kernel.
// The objective is a stand-in for the local loss f_i of the paper's problem
// definition; it is drawn here only because the large models do not fit a host
// round trip.  Not on the hot path: accurate library math, one element per lane.
#include "internal.hpp"
#include "philox.hpp"

namespace cocod {
namespace {

constexpr uint32_t kFillThreads = 256;

__global__ __launch_bounds__(kFillThreads) void fill_quadratic_kernel(const Chunk *table, uint32_t W, uint64_t stride,
                                                                      float *h, float *c, uint32_t key0, uint32_t key1)
{
    const Chunk ck = table[blockIdx.x];
    const uint32_t worker = blockIdx.y;
    const uint64_t row = static_cast<uint64_t>(worker) * stride + static_cast<uint64_t>(ck.mem_quad) * 4;
    const uint32_t n_padded = (ck.n + 3u) & ~3u;       // a tensor's tail quad ends in alignment pads
    for (uint32_t e = threadIdx.x; e < n_padded; e += kFillThreads) {
        if (e >= ck.n) { h[row + e] = 0.0f; c[row + e] = 0.0f; continue; }
        const uint64_t j = ck.glob_off + e;
        const Words4 rh = philox4x32_10(static_cast<uint32_t>(j >> 2), 0u, worker, kTagH, key0, key1);
        const Normals4 zc = box_muller_accurate(
            philox4x32_10(static_cast<uint32_t>(j >> 2), 0u, worker, kTagC, key0, key1));
        const uint32_t lane = static_cast<uint32_t>(j & 3u);
        // 1.5 U has at most 26 significant bits: evaluate in fp64 and round once
        h[row + e] = static_cast<float>(0.5 + 1.5 * static_cast<double>(u_half_open(rh.w[lane])));
        c[row + e] = zc.z[lane];
    }
}

__global__ __launch_bounds__(kFillThreads) void debug_normals_kernel(uint32_t key0, uint32_t key1, uint32_t tag,
                                                                     uint32_t worker, uint32_t step, uint64_t j0,
                                                                     uint64_t n, int fast, float *out)
{
    const uint64_t m = static_cast<uint64_t>(blockIdx.x) * kFillThreads + threadIdx.x;
    if (m >= n) return;
    const uint64_t j = j0 + m;
    const Words4 r = philox4x32_10(static_cast<uint32_t>(j >> 2), step, worker, tag, key0, key1);
    const Normals4 z = fast ? box_muller_fast(r) : box_muller_accurate(r);
    out[m] = z.z[j & 3u];
}

// Plain streaming copy of n_quads 16-byte quads: the known-size reference that hardware traffic
// counters are calibrated against.
__global__ __launch_bounds__(kFillThreads) void copy_kernel(const float *src, float *dst, uint64_t n_quads)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const uint64_t q = static_cast<uint64_t>(blockIdx.x) * kFillThreads + threadIdx.x;
    if (q >= n_quads) return;
    const f4 t = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(src) + q);
    __builtin_nontemporal_store(t, reinterpret_cast<f4 *>(dst) + q);
}

__global__ void set_word_kernel(uint32_t *word, uint32_t value) { *word = value; }
__global__ void add_word_kernel(uint32_t *word, uint32_t inc) { *word += inc; }

}  // namespace

hipError_t launch_set_word(hipStream_t stream, uint32_t *word, uint32_t value)
{
    hipLaunchKernelGGL(set_word_kernel, dim3(1), dim3(1), 0, stream, word, value);
    return hipGetLastError();
}

hipError_t launch_add_word(hipStream_t stream, uint32_t *word, uint32_t inc)
{
    hipLaunchKernelGGL(add_word_kernel, dim3(1), dim3(1), 0, stream, word, inc);
    return hipGetLastError();
}

hipError_t launch_copy(hipStream_t stream, const float *src, float *dst, uint64_t n_quads)
{
    if (n_quads == 0) return hipSuccess;
    const uint64_t blocks = (n_quads + kFillThreads - 1) / kFillThreads;
    if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(copy_kernel, dim3(static_cast<uint32_t>(blocks)), dim3(kFillThreads), 0, stream, src, dst, n_quads);
    return hipGetLastError();
}

hipError_t launch_fill_quadratic(hipStream_t stream, const Chunk *table, uint32_t n_chunks, uint32_t W,
                                 uint64_t stride, uint64_t padded_d, float *h, float *c, uint32_t key0,
                                 uint32_t key1)
{
    (void)padded_d;
    hipLaunchKernelGGL(fill_quadratic_kernel, dim3(n_chunks, W), dim3(kFillThreads), 0, stream, table, W, stride,
                       h, c, key0, key1);
    return hipGetLastError();
}

hipError_t launch_debug_normals(hipStream_t stream, uint32_t key0, uint32_t key1, uint32_t tag, uint32_t worker,
                                uint32_t step, uint64_t j0, uint64_t n, int fast, float *out)
{
    if (n == 0) return hipSuccess;
    const uint32_t blocks = static_cast<uint32_t>((n + kFillThreads - 1) / kFillThreads);
    hipLaunchKernelGGL(debug_normals_kernel, dim3(blocks), dim3(kFillThreads), 0, stream, key0, key1, tag, worker,
                       step, j0, n, fast, out);
    return hipGetLastError();
}

}  // namespace cocod
