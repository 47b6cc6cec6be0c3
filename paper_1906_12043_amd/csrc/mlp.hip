// Step II of Algorithm 1 (CoCoD-SGD) with a REAL mini-batch gradient: every worker is a two-layer
// perceptron  A = X W1 + b1, H = relu(A), Z = H W2 + b2, loss = mean softmax cross-entropy,
// on a fresh seeded mini-batch per (worker, step); all W workers advance in the same launches.
//
// One local step = six launches on the compute stream:
//   gen_batch      X, X^T, labels from the counter-based generator              (vector ALU)
//   gemm<FWD>      H = relu(X W1 + b1)                         [B x in] x [in x hid]   fp32 MFMA
//   head_logits    Z = H W2 + b2, softmax, dZ = (P - onehot)/B  (one wave per sample, wave reductions)
//   head_backprop  dA = (dZ W2^T) * [H > 0]
//   head_update    dW2 = H^T dZ, db2, db1 = colsum(dA); momentum-SGD update of W2, b2, b1
//   gemm<BWD>      dW1 = X^T dA with the momentum-SGD update of W1 fused into the epilogue
//                  (the 12.6 MB gradient of W1 never goes to memory)   [in x B] x [B x hid]  fp32 MFMA
// The two big contractions (98 % of the flops) run on the matrix cores; the output layer has
// 10 columns and stays on the vector units.
//
// GEMM kernel: 128 x 64 output tile per 256-thread block, K in slices of 16 staged through LDS with
// register prefetch (double buffered); each of the 4 waves owns 32 rows x 64 columns = two
// 32x32x2 fp32 MFMA accumulators.  Both GEMMs read A with K contiguous and B with N contiguous
// (that is why the generator also writes X^T), so one kernel serves both with two epilogues.
#include "internal.hpp"
#include "philox.hpp"

namespace cocod {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int kBM = 128, kBN = 64, kBK = 16, kGemmThreads = 256;
constexpr int kMaxOut = 16;

struct Offsets { uint64_t W1, b1, W2, b2; };
__host__ __device__ inline Offsets offsets_of(const MlpParams &p)
{
    Offsets o;
    o.W1 = 0;
    o.b1 = static_cast<uint64_t>(p.n_in) * p.n_hid;
    o.W2 = o.b1 + p.n_hid;
    o.b2 = o.W2 + static_cast<uint64_t>(p.n_hid) * p.n_out;
    return o;
}

// g = G + lambda x ; v = mu v + g ; x' = x - gamma v   (same update as the quadratic step)
__device__ __forceinline__ void sgd_update(const MlpParams &p, uint64_t at, float G)
{
    const float x = p.x_in[at];
    float g = G + p.weight_decay * x;
    if (p.momentum != 0.0f) {
        const float v = p.momentum * p.v[at] + g;
        p.v[at] = v;
        g = v;
    }
    p.x_out[at] = x - p.lr * g;
}

// ---- mini-batch ---------------------------------------------------------------------------------
// X[b][f] = normal(stream X, worker, step, flat index b*n_in + f); also stored transposed.
// y[b] = (word * n_out) >> 32 from stream Y at index b.
__global__ __launch_bounds__(256) void gen_batch_kernel(const MlpParams p)
{
    const uint32_t worker = blockIdx.y;
    const uint64_t n_quads = static_cast<uint64_t>(p.batch) * p.n_in / 4;
    const uint64_t q = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (q < n_quads) {
        const Normals4 z = box_muller_fast(philox4x32_10(static_cast<uint32_t>(q), p.step, worker, kTagMlpX, p.key0, p.key1));
        const uint64_t flat = q * 4;
        const uint32_t b = static_cast<uint32_t>(flat / p.n_in), f = static_cast<uint32_t>(flat % p.n_in);
        float *X = p.X + static_cast<uint64_t>(worker) * p.batch * p.n_in;
        float *XT = p.XT + static_cast<uint64_t>(worker) * p.batch * p.n_in;
        *reinterpret_cast<f4 *>(X + flat) = f4{z.z[0], z.z[1], z.z[2], z.z[3]};
        #pragma unroll
        for (int i = 0; i < 4; ++i) XT[static_cast<uint64_t>(f + i) * p.batch + b] = z.z[i];
    }
    if (blockIdx.x == 0 && threadIdx.x < p.batch / 4) {
        const Words4 r = philox4x32_10(threadIdx.x, p.step, worker, kTagMlpY, p.key0, p.key1);
        #pragma unroll
        for (int i = 0; i < 4; ++i)
            p.y[static_cast<uint64_t>(worker) * p.batch + threadIdx.x * 4 + i] =
                static_cast<int32_t>((static_cast<uint64_t>(r.w[i]) * p.n_out) >> 32);
    }
}

// ---- the two big contractions ---------------------------------------------------------------------
enum { kFwd = 0, kBwd = 1 };

template <int EPI>
__global__ __launch_bounds__(kGemmThreads) void mlp_gemm_kernel(const MlpParams p)
{
    __shared__ float As[2][kBM][kBK + 1];      // [m][k], odd row pitch: conflict-free fragment reads
    __shared__ __attribute__((aligned(16))) float Bs[2][kBK][kBN + 4];      // [k][n], rows stay 16-byte aligned

    const uint32_t worker = blockIdx.z;
    const uint32_t m0 = blockIdx.y * kBM, n0 = blockIdx.x * kBN;
    const Offsets o = offsets_of(p);
    const float *A, *B;
    uint32_t lda, K;
    const uint32_t ldb = p.n_hid;
    if (EPI == kFwd) {          // X [batch][n_in] times W1 [n_in][n_hid]
        A = p.X + static_cast<uint64_t>(worker) * p.batch * p.n_in;
        B = p.x_in + static_cast<uint64_t>(worker) * p.stride + o.W1;
        lda = p.n_in; K = p.n_in;
    } else {                    // X^T [n_in][batch] times dA [batch][n_hid]
        A = p.XT + static_cast<uint64_t>(worker) * p.batch * p.n_in;
        B = p.dA + static_cast<uint64_t>(worker) * p.batch * p.n_hid;
        lda = p.batch; K = p.batch;
    }

    const uint32_t t = threadIdx.x;
    // global -> register staging: A tile 128 x 16 = 512 quads (2 per thread), B tile 16 x 64 = 256 quads
    const uint32_t a_m = t / 4, a_k = (t % 4) * 4;
    const uint32_t b_k = t / 16, b_n = (t % 16) * 4;
    const float *a_src0 = A + static_cast<uint64_t>(m0 + a_m) * lda + a_k;
    const float *a_src1 = A + static_cast<uint64_t>(m0 + a_m + 64) * lda + a_k;
    const float *b_src = B + static_cast<uint64_t>(b_k) * ldb + n0 + b_n;

    f4 ra0 = *reinterpret_cast<const f4 *>(a_src0);
    f4 ra1 = *reinterpret_cast<const f4 *>(a_src1);
    f4 rb = *reinterpret_cast<const f4 *>(b_src);

    const uint32_t wave = t / 64, lane = t % 64;
    const uint32_t frag_m = wave * 32 + lane % 32, frag_k = lane / 32, frag_n = lane % 32;
    f16v acc0 = {0}, acc1 = {0};

    const uint32_t n_slices = K / kBK;
    for (uint32_t s = 0; s < n_slices; ++s) {
        const uint32_t cur = s & 1;
        #pragma unroll
        for (int i = 0; i < 4; ++i) {
            As[cur][a_m][a_k + i] = ra0[i];
            As[cur][a_m + 64][a_k + i] = ra1[i];
        }
        *reinterpret_cast<f4 *>(&Bs[cur][b_k][b_n]) = rb;
        __syncthreads();        // slice s visible; everyone is done reading buffer cur from slice s-2
        if (s + 1 < n_slices) { // prefetch the next slice while this one is multiplied
            ra0 = *reinterpret_cast<const f4 *>(a_src0 + static_cast<uint64_t>(s + 1) * kBK);
            ra1 = *reinterpret_cast<const f4 *>(a_src1 + static_cast<uint64_t>(s + 1) * kBK);
            rb = *reinterpret_cast<const f4 *>(b_src + static_cast<uint64_t>(s + 1) * kBK * ldb);
        }
        #pragma unroll
        for (int kk = 0; kk < kBK; kk += 2) {
            const float a = As[cur][frag_m][kk + frag_k];
            const float b0 = Bs[cur][kk + frag_k][frag_n];
            const float b1 = Bs[cur][kk + frag_k][frag_n + 32];
            acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc1, 0, 0, 0);
        }
        // no second barrier: the next iteration writes the OTHER buffer, and the barrier inside it
        // orders those writes against the reads of the iteration after
    }

    // accumulator layout of the 32x32 tile: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32
    #pragma unroll
    for (int r = 0; r < 16; ++r) {
        const uint32_t row = m0 + wave * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
        #pragma unroll
        for (int half = 0; half < 2; ++half) {
            const uint32_t col = n0 + 32 * half + lane % 32;
            const float val = half ? acc1[r] : acc0[r];
            if (EPI == kFwd) {
                const float bias = p.x_in[static_cast<uint64_t>(worker) * p.stride + o.b1 + col];
                p.H[(static_cast<uint64_t>(worker) * p.batch + row) * p.n_hid + col] = fmaxf(val + bias, 0.0f);
            } else {
                sgd_update(p, static_cast<uint64_t>(worker) * p.stride + o.W1 + static_cast<uint64_t>(row) * p.n_hid + col, val);
            }
        }
    }
}

// ---- output layer -----------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
    #pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// One wave per sample: logits by a strided dot product over the hidden units and a butterfly
// reduction, then softmax (row maximum subtracted) and dZ = (P - onehot(y)) / batch.
__global__ __launch_bounds__(256) void head_logits_kernel(const MlpParams p)
{
    const uint32_t worker = blockIdx.y;
    const uint32_t b = blockIdx.x * 4 + threadIdx.x / 64, lane = threadIdx.x % 64;
    if (b >= p.batch) return;
    const Offsets o = offsets_of(p);
    const float *theta = p.x_in + static_cast<uint64_t>(worker) * p.stride;
    const float *Hrow = p.H + (static_cast<uint64_t>(worker) * p.batch + b) * p.n_hid;
    float z[kMaxOut];
    #pragma unroll
    for (int c = 0; c < kMaxOut; ++c) z[c] = 0.0f;
    for (uint32_t n = lane; n < p.n_hid; n += 64) {
        const float hv = Hrow[n];
        const float *w2 = theta + o.W2 + static_cast<uint64_t>(n) * p.n_out;
        #pragma unroll
        for (int c = 0; c < kMaxOut; ++c)
            if (c < static_cast<int>(p.n_out)) z[c] += hv * w2[c];
    }
    float zmax = -INFINITY;
    #pragma unroll
    for (int c = 0; c < kMaxOut; ++c)
        if (c < static_cast<int>(p.n_out)) {
            z[c] = wave_sum(z[c]) + theta[o.b2 + c];
            zmax = fmaxf(zmax, z[c]);
        }
    float denom = 0.0f;
    #pragma unroll
    for (int c = 0; c < kMaxOut; ++c)
        if (c < static_cast<int>(p.n_out)) { z[c] = expf(z[c] - zmax); denom += z[c]; }
    const int label = p.y[static_cast<uint64_t>(worker) * p.batch + b];
    const float inv_b = 1.0f / static_cast<float>(p.batch);
    #pragma unroll
    for (int c = 0; c < kMaxOut; ++c)
        if (c < static_cast<int>(p.n_out) && lane == static_cast<uint32_t>(c))
            p.dZ[(static_cast<uint64_t>(worker) * p.batch + b) * kMaxOut + c] =
                (z[c] / denom - (label == c ? 1.0f : 0.0f)) * inv_b;
}

// dA[b][n] = (sum_c dZ[b][c] W2[n][c]) * [H[b][n] > 0]; a thread owns hidden unit n for 8 samples.
__global__ __launch_bounds__(256) void head_backprop_kernel(const MlpParams p)
{
    const uint32_t worker = blockIdx.z;
    const uint32_t n = blockIdx.x * 256 + threadIdx.x;
    if (n >= p.n_hid) return;
    const Offsets o = offsets_of(p);
    const float *w2 = p.x_in + static_cast<uint64_t>(worker) * p.stride + o.W2 + static_cast<uint64_t>(n) * p.n_out;
    float w[kMaxOut];
    #pragma unroll
    for (int c = 0; c < kMaxOut; ++c) w[c] = c < static_cast<int>(p.n_out) ? w2[c] : 0.0f;
    for (uint32_t b = blockIdx.y * 8; b < blockIdx.y * 8 + 8 && b < p.batch; ++b) {
        const uint64_t sample = static_cast<uint64_t>(worker) * p.batch + b;
        const float *dz = p.dZ + sample * kMaxOut;
        float dh = 0.0f;
        #pragma unroll
        for (int c = 0; c < kMaxOut; ++c)
            if (c < static_cast<int>(p.n_out)) dh += dz[c] * w[c];
        p.dA[sample * p.n_hid + n] = p.H[sample * p.n_hid + n] > 0.0f ? dh : 0.0f;
    }
}

// Gradients of the small parameters and their update: a thread owns hidden unit n
// (row n of W2 and b1[n]); block 0 of a worker also owns b2 and the alignment pads.
__global__ __launch_bounds__(64) void head_update_kernel(const MlpParams p)
{
    const uint32_t worker = blockIdx.y;
    const uint32_t n = blockIdx.x * 64 + threadIdx.x;
    const Offsets o = offsets_of(p);
    const uint64_t base = static_cast<uint64_t>(worker) * p.stride;
    if (n < p.n_hid) {
        float gw[kMaxOut];
        #pragma unroll
        for (int c = 0; c < kMaxOut; ++c) gw[c] = 0.0f;
        float gb = 0.0f;
        for (uint32_t b = 0; b < p.batch; ++b) {
            const uint64_t sample = static_cast<uint64_t>(worker) * p.batch + b;
            const float hv = p.H[sample * p.n_hid + n];
            gb += p.dA[sample * p.n_hid + n];
            const float *dz = p.dZ + sample * kMaxOut;
            #pragma unroll
            for (int c = 0; c < kMaxOut; ++c)
                if (c < static_cast<int>(p.n_out)) gw[c] += hv * dz[c];
        }
        #pragma unroll
        for (int c = 0; c < kMaxOut; ++c)
            if (c < static_cast<int>(p.n_out)) sgd_update(p, base + o.W2 + static_cast<uint64_t>(n) * p.n_out + c, gw[c]);
        sgd_update(p, base + o.b1 + n, gb);
    }
    if (blockIdx.x == 0) {
        if (threadIdx.x < p.n_out) {
            float g = 0.0f;
            for (uint32_t b = 0; b < p.batch; ++b)
                g += p.dZ[(static_cast<uint64_t>(worker) * p.batch + b) * kMaxOut + threadIdx.x];
            sgd_update(p, base + o.b2 + threadIdx.x, g);
        }
        const uint64_t d = o.b2 + p.n_out;                       // pads after the last parameter travel along
        if (p.x_out != p.x_in && threadIdx.x < ((d + 3) & ~3ull) - d) p.x_out[base + d + threadIdx.x] = p.x_in[base + d + threadIdx.x];
    }
}

}  // namespace

bool mlp_shape_supported(uint32_t n_in, uint32_t n_hid, uint32_t n_out, uint32_t batch)
{
    return n_in >= static_cast<uint32_t>(kBM) && n_in % kBM == 0 && n_hid >= static_cast<uint32_t>(kBN) && n_hid % kBN == 0 &&
           n_out >= 1 && n_out <= static_cast<uint32_t>(kMaxOut) && batch >= static_cast<uint32_t>(kBM) && batch % kBM == 0 &&
           batch <= 1024;
}

size_t mlp_dz_pitch() { return kMaxOut; }

hipError_t launch_mlp_step(hipStream_t stream, const MlpParams &p)
{
    const uint64_t n_quads = static_cast<uint64_t>(p.batch) * p.n_in / 4;
    hipLaunchKernelGGL(gen_batch_kernel, dim3(static_cast<uint32_t>((n_quads + 255) / 256), p.W), dim3(256), 0, stream, p);
    hipLaunchKernelGGL((mlp_gemm_kernel<kFwd>), dim3(p.n_hid / kBN, p.batch / kBM, p.W), dim3(kGemmThreads), 0, stream, p);
    hipLaunchKernelGGL(head_logits_kernel, dim3((p.batch + 3) / 4, p.W), dim3(256), 0, stream, p);
    hipLaunchKernelGGL(head_backprop_kernel, dim3((p.n_hid + 255) / 256, (p.batch + 7) / 8, p.W), dim3(256), 0, stream, p);
    hipLaunchKernelGGL(head_update_kernel, dim3((p.n_hid + 63) / 64, p.W), dim3(64), 0, stream, p);
    hipLaunchKernelGGL((mlp_gemm_kernel<kBwd>), dim3(p.n_hid / kBN, p.n_in / kBM, p.W), dim3(kGemmThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace cocod
