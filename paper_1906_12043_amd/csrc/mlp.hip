// Step II of Algorithm 1 (CoCoD-SGD) with a REAL mini-batch gradient: every worker is a two-layer
// perceptron  A = X W1 + b1, H = relu(A), Z = H W2 + b2, loss = mean softmax cross-entropy,
// on a fresh seeded mini-batch per (worker, step); all W workers advance in the same launches.
//
// One local step = four launches on the compute stream (five for a step whose mini-batch no earlier
// step has drawn: gen_batch in front):
//   gemm<FWD>      H = relu(X W1 + b1)                         [B x in] x [in x hid]   fp32 MFMA
//   head           Z = H W2 + b2, softmax, dZ = (P - onehot)/B, dA = (dZ W2^T) * [H > 0]
//                  (one wave per sample, wave reductions, W2 in LDS)
//   head_update    dW2 = H^T dZ, db2, db1 = colsum(dA); momentum-SGD update of W2, b2, b1;
//                  further blocks of the same launch draw the NEXT step's X and labels from the
//                  counter-based generator into the other of two batch buffers (vector ALU work
//                  beside a kernel that is a short chain of dependent loads)
//   gemm<BWD>      dW1 = X^T dA with the momentum-SGD update of W1 fused into the epilogue
//                  (the 12.6 MB gradient of W1 never goes to memory)   [in x B] x [B x hid]  fp32 MFMA
// The two big contractions (98 % of the flops) run on the matrix cores; the output layer has
// 10 columns and stays on the vector units.
//
// GEMM kernel: 64 x 128 output tile per 512-thread block (8 waves, one 32x32 accumulator each; 64 x 64
// with 4 waves when the hidden width is not a multiple of 128).  K goes through LDS in slices
// of 32 with register prefetch and two buffers (one barrier per slice); a wave reads all fragments
// of a slice before it starts the slice's chain of 16 MFMAs.  The forward product reads
// its A operand K-contiguous; the backward product needs X^T and gets it by staging X through LDS
// transposed, so no transposed copy of the mini-batch is ever written.  After the K loop the
// accumulators pass through LDS once more so that the epilogue touches memory in 16-byte pieces
// along rows (256 contiguous bytes per row per wave) instead of 4-byte pieces along columns.
#include "internal.hpp"
#include "philox.hpp"

#include <hip/hip_ext.h>

#include <type_traits>
#include <utility>

namespace cocod {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int kBK = 32;               // K slice staged through LDS
constexpr int kAPitch = kBK + 1;      // odd pitch: conflict-free fragment reads
constexpr int kShapeM = 128, kShapeN = 64;   // shape contract: n_in, batch multiples of 128; n_hid of 64
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
    float x_new = x - p.lr * g;
    if (p.snap) x_new = p.mean[at % p.stride] + (x_new - p.snap[at]);     // line 6 (last step of a round)
    p.x_out[at] = x_new;
}

// ---- mini-batch ---------------------------------------------------------------------------------
// X[b][f] = normal(stream X, worker, step, flat index b*n_in + f);
// y[b] = (word * n_out) >> 32 from stream Y at index b.
// One 256-thread group's share (thread tid of group `block`) of a worker's mini-batch for local step
// `step`: 256 quads of X, and in group 0 the labels.
__device__ __forceinline__ void gen_batch_block(const MlpParams &p, uint32_t block, uint32_t tid, uint32_t worker, uint32_t step,
                                                float *X_all, int32_t *y_all)
{
    const uint64_t n_quads = static_cast<uint64_t>(p.batch) * p.n_in / 4;
    const uint64_t q = static_cast<uint64_t>(block) * 256 + tid;
    if (q < n_quads) {
        const Normals4 z = box_muller_fast(philox4x32_10(static_cast<uint32_t>(q), step, worker, kTagMlpX, p.key0, p.key1));
        float *X = X_all + static_cast<uint64_t>(worker) * p.batch * p.n_in;
        *reinterpret_cast<f4 *>(X + q * 4) = f4{z.z[0], z.z[1], z.z[2], z.z[3]};
    }
    if (block == 0 && tid < p.batch / 4) {
        const Words4 r = philox4x32_10(tid, step, worker, kTagMlpY, p.key0, p.key1);
        #pragma unroll
        for (int i = 0; i < 4; ++i)
            y_all[static_cast<uint64_t>(worker) * p.batch + tid * 4 + i] =
                static_cast<int32_t>((static_cast<uint64_t>(r.w[i]) * p.n_out) >> 32);
    }
}

__host__ __device__ inline uint32_t gen_batch_blocks(const MlpParams &p)
{
    return static_cast<uint32_t>((static_cast<uint64_t>(p.batch) * p.n_in / 4 + 255) / 256);
}

__global__ __launch_bounds__(256) void gen_batch_kernel(const MlpParams p)
{
    const uint32_t step = p.step_base ? *p.step_base + p.step : p.step;
    gen_batch_block(p, blockIdx.x, threadIdx.x, blockIdx.y, step, p.X, p.y);
}

// ---- the two big contractions ---------------------------------------------------------------------
enum { kFwd = 0, kBwd = 1, kBwdTail = 2 };   // kBwdTail: the backward product of a round's last step (line 6 in its epilogue)
constexpr uint32_t kXcds = 8;      // accelerator complex dies of the MI355X

// NWM x NWN waves per block, one 32x32 accumulator per wave: block tile (32 NWM) x (32 NWN).
template <int EPI, int NWM, int NWN>
__global__ __launch_bounds__(64 * NWM * NWN) void mlp_gemm_kernel(const MlpParams p)
{
    constexpr int BM = 32 * NWM, BN = 32 * NWN, THREADS = 64 * NWM * NWN;
    constexpr int BPITCH = BN + 4, CPITCH = BN + 4;            // rows stay 16-byte aligned
    constexpr int STAGE = 2 * BM * kAPitch + 2 * kBK * BPITCH, TILE = BM * CPITCH;
    __shared__ __attribute__((aligned(16))) float smem[STAGE > TILE ? STAGE : TILE];
    float (*As)[BM][kAPitch] = reinterpret_cast<float (*)[BM][kAPitch]>(smem);                    // [buf][m][k]
    float (*Bs)[kBK][BPITCH] = reinterpret_cast<float (*)[kBK][BPITCH]>(smem + 2 * BM * kAPitch);  // [buf][k][n]
    float (*Ct)[CPITCH] = reinterpret_cast<float (*)[CPITCH]>(smem);                               // epilogue tile

    // Workgroups go to the 8 XCDs (each with its own L2) round-robin by linear id.  Renumber them so
    // that every XCD owns a CONTIGUOUS run of tiles (n fastest, then m, then worker): the tiles that
    // share an operand panel (all n-tiles of an m-tile share its X panel, all m-tiles of an n-tile its
    // W1 / dA panel) then meet in one L2 instead of fetching the panel once per XCD.
    uint32_t bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    {
        const uint32_t total = gridDim.x * gridDim.y * gridDim.z;
        if (total % kXcds == 0) {
            const uint32_t linear = bx + gridDim.x * (by + gridDim.y * bz);
            const uint32_t logical = (linear % kXcds) * (total / kXcds) + linear / kXcds;
            bx = logical % gridDim.x;
            by = (logical / gridDim.x) % gridDim.y;
            bz = logical / (gridDim.x * gridDim.y);
        }
    }
    const uint32_t worker = bz;
    const uint32_t m0 = by * BM, n0 = bx * BN;
    const Offsets o = offsets_of(p);
    const uint32_t t = threadIdx.x;
    const uint32_t ldb = p.n_hid;
    const float *Xw = p.X + static_cast<uint64_t>(worker) * p.batch * p.n_in;

    // Global -> register staging of one K slice, in 16-byte quads.
    //   forward : A = X [batch][n_in], K-contiguous: a quad is 4 consecutive k of one row m
    //   backward: A = X^T, read from X M-contiguous: a quad is 4 consecutive rows m of one sample k
    //   B tile  : kBK x BN, N-contiguous (W1 rows, or dA rows)
    // (a tile with fewer A quads than threads is staged by the block's first A_QUADS threads: whole waves)
    constexpr int A_QUADS = BM * kBK / 4, PA = A_QUADS >= THREADS ? A_QUADS / THREADS : 1;
    constexpr int B_QUADS = kBK * BN / 4, PB = B_QUADS / THREADS;
    constexpr bool A_ALL = A_QUADS >= THREADS;
    static_assert((A_ALL ? PA * THREADS == A_QUADS : A_QUADS % 64 == 0) && PB * THREADS == B_QUADS, "tile must split evenly over the block");
    static_assert(EPI != kFwd || (PA <= 2 && PB <= 4), "the forward loop spreads the staging traffic over fixed slots of the MFMA chain");
    constexpr int A_MINOR = (EPI == kFwd) ? kBK / 4 : BM / 4;   // quads along the contiguous direction
    constexpr int A_MAJOR_PER_PASS = THREADS / A_MINOR;
    constexpr int B_K_PER_PASS = THREADS / (BN / 4);
    const uint32_t a_minor = (t % A_MINOR) * 4, a_major = t / A_MINOR;
    const uint32_t b_n = (t % (BN / 4)) * 4, b_k = t / (BN / 4);
    const float *a_src, *b_src;
    uint64_t a_slice, a_pass;    // element strides of A per K slice and per staging pass
    uint32_t K;
    if (EPI == kFwd) {
        a_src = Xw + static_cast<uint64_t>(m0 + a_major) * p.n_in + a_minor;
        a_slice = kBK; a_pass = static_cast<uint64_t>(A_MAJOR_PER_PASS) * p.n_in;
        K = p.n_in;
        b_src = p.x_in + static_cast<uint64_t>(worker) * p.stride + o.W1;                 // W1 [n_in][n_hid]
    } else {
        a_src = Xw + static_cast<uint64_t>(a_major) * p.n_in + m0 + a_minor;
        a_slice = static_cast<uint64_t>(kBK) * p.n_in; a_pass = static_cast<uint64_t>(A_MAJOR_PER_PASS) * p.n_in;
        K = p.batch;
        b_src = p.dA + static_cast<uint64_t>(worker) * p.batch * p.n_hid;                 // dA [batch][n_hid]
    }
    b_src += static_cast<uint64_t>(b_k) * ldb + n0 + b_n;

    // Forward product: four sets of staging registers, so global loads run four K slices ahead of their
    // use; that covers the HBM latency of the weight stream (one slice of MFMAs is shorter than it).
    // One block of 8 waves per CU leaves 256 registers per lane: the sets cost nothing in occupancy.
    // Backward product: K is only the batch (4 slices); one set keeps the registers, and with them
    // the number of resident blocks, where the memory-bound epilogue wants them.
    constexpr int NSETS = (EPI == kFwd) ? 4 : 1;
    f4 ra[NSETS][PA], rb[NSETS][PB];
    auto load_slice = [&](auto set, uint32_t slice) {
        constexpr int S = decltype(set)::value;
        if (A_ALL || t < A_QUADS) {
            #pragma unroll
            for (int i = 0; i < PA; ++i) ra[S][i] = *reinterpret_cast<const f4 *>(a_src + slice * a_slice + i * a_pass);
        }
        #pragma unroll
        for (int i = 0; i < PB; ++i)
            rb[S][i] = *reinterpret_cast<const f4 *>(b_src + (static_cast<uint64_t>(slice) * kBK + static_cast<uint64_t>(i) * B_K_PER_PASS) * ldb);
    };
    auto stage_to_lds = [&](auto set, uint32_t buf) {
        constexpr int S = decltype(set)::value;
        if (A_ALL || t < A_QUADS) {
            #pragma unroll
            for (int i = 0; i < PA; ++i) {
                const uint32_t major = a_major + i * A_MAJOR_PER_PASS;
                #pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (EPI == kFwd) As[buf][major][a_minor + j] = ra[S][i][j];      // (row, k)
                    else             As[buf][a_minor + j][major] = ra[S][i][j];      // transposed on the way in
                }
            }
        }
        #pragma unroll
        for (int i = 0; i < PB; ++i) *reinterpret_cast<f4 *>(&Bs[buf][b_k + i * B_K_PER_PASS][b_n]) = rb[S][i];
    };
    using Set0 = std::integral_constant<int, 0>;
    using Set1 = std::integral_constant<int, 1>;

    const uint32_t wave = t / 64, lane = t % 64;
    const uint32_t wm = wave % NWM, wn = wave / NWM;             // wave owns rows 32 wm .., columns 32 wn ..
    const uint32_t frag_m = wm * 32 + lane % 32, frag_k = lane / 32, frag_n = wn * 32 + lane % 32;
    f16v acc = {0};

    // Backward product: the epilogue updates this block's tile of W1 and its momentum.  Vector loads
    // return in order, so these 64 KB must be the YOUNGEST loads in flight or every operand slice
    // behind them would wait for them: they are issued right after the loads of the last K slice
    // and land under the remaining multiplies.
    constexpr int EPI_ITERS = (BM * BN / 4) / THREADS;
    f4 x_old[EPI_ITERS], v_old[EPI_ITERS], snap_old[EPI_ITERS];
    auto prefetch_tile = [&]() {
        #pragma unroll
        for (int it = 0; it < EPI_ITERS; ++it) {
            const uint32_t idx = it * THREADS + t;
            const uint64_t at = static_cast<uint64_t>(worker) * p.stride + o.W1 +
                                static_cast<uint64_t>(m0 + idx / (BN / 4)) * p.n_hid + n0 + (idx % (BN / 4)) * 4;
            x_old[it] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(p.x_in + at));
            v_old[it] = p.momentum != 0.0f ? __builtin_nontemporal_load(reinterpret_cast<const f4 *>(p.v + at)) : f4{0.f, 0.f, 0.f, 0.f};
            if (EPI == kBwdTail) snap_old[it] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(p.snap + at));
        }
    };

    // Software pipeline over the K slices (their number is a multiple of 4 by the shape contract).
    // At the top of iteration s: slice s sits in LDS buffer s&1, visible to all waves; slice s+1
    // sits in a register set; with two sets the loads of slice s+2 into the other set are in flight.
    // The iteration reads its fragments, pushes slice s+1 into the other LDS buffer and starts the
    // loads of the next slice to fetch BEFORE the chain of 16 MFMAs, so all of that runs under the
    // multiplies; one barrier per slice.
    const uint32_t n_slices = K / kBK;
    auto iteration = [&](auto next_set, uint32_t s, auto stage, auto load) {
        const uint32_t cur = s & 1;
        float af[kBK / 2], bf[kBK / 2];
        #pragma unroll
        for (int i = 0; i < kBK / 2; ++i) {
            af[i] = As[cur][frag_m][2 * i + frag_k];
            bf[i] = Bs[cur][2 * i + frag_k][frag_n];
        }
        // compile-time switches, not run-time conditions (see the forward loop)
        if constexpr (decltype(stage)::value) stage_to_lds(next_set, cur ^ 1);   // buffer last read in iteration s-1, before its barrier
        if constexpr (decltype(load)::value) load_slice(next_set, s + 2);
        #pragma unroll
        for (int i = 0; i < kBK / 2; ++i) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[i], acc, 0, 0, 0);
        __syncthreads();        // slice s+1 visible; everyone is done reading buffer cur
    };
    load_slice(Set0{}, 0);
    if constexpr (NSETS == 4) {
        // Forward product, one stage deeper: the fragments of slice s+1 are read from LDS during the MFMA
        // chain of slice s (two fragment sets), so the matrix pipe does not idle while both waves of a
        // SIMD sit in their LDS-read phase (there is one block of 8 waves per CU: nothing else to run).
        // Top of iteration s: fragments of slice s in set s&1; slice s+1 in LDS buffer (s+1)&1, visible;
        // slices s+2 .. s+5 in (or on their way into) the four staging sets.
        float af2[2][kBK / 2], bf2[2][kBK / 2];
        const uint32_t last = n_slices - 1;
        auto read_frags = [&](auto par, uint32_t buf) {
            constexpr int F = decltype(par)::value;
            #pragma unroll
            for (int i = 0; i < kBK / 2; ++i) {
                af2[F][i] = As[buf][frag_m][2 * i + frag_k];
                bf2[F][i] = Bs[buf][2 * i + frag_k][frag_n];
            }
        };
        // slice t lives in staging set t % 4; iteration s stages slice s+2 and refills that set with slice s+6
        auto deep_iteration = [&](auto par, auto other, auto set, uint32_t s) {
            constexpr int F = decltype(par)::value, O = decltype(other)::value, S = decltype(set)::value;
            // No run-time conditions in the loop body: past the end the same steps run on the last slice
            // again and their results are never used.  (With steps under `if`, the number of loads in
            // flight at a given point depends on the path taken, and the compiler must then wait for ALL
            // of them before the first use of any.)
            // Issue order: the 16 multiplies form a dependent chain (each waits 64 cycles for the one
            // before) and a wave issues in order, so the memory instructions go INTO the gaps of the
            // chain: after multiply i, element i of the next slice's fragments, and one piece of the
            // staging traffic.  A scheduling fence after every group pins that order; left to itself the
            // scheduler sinks each fragment read to its first use (which undoes the pipeline) or issues
            // the memory instructions in one lump (then both waves of a SIMD sit in that phase together,
            // right after the barrier, and the matrix pipe idles).
            const uint32_t nb = (s + 1) & 1, wb = s & 1;          // buffers: next fragments from nb, slice s+2 into wb
            const uint32_t refill = s + 6 < n_slices ? s + 6 : last;
            #pragma unroll
            for (int i = 0; i < kBK / 2; ++i) {
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af2[F][i], bf2[F][i], acc, 0, 0, 0);
                af2[O][i] = As[nb][frag_m][2 * i + frag_k];
                bf2[O][i] = Bs[nb][2 * i + frag_k][frag_n];
                if (i >= 2 && i < 2 + PA) {                       // A quad of slice s+2 -> LDS (buffer last read in iteration s-1)
                    const int a = i - 2;
                    const uint32_t major = a_major + a * A_MAJOR_PER_PASS;
                    #pragma unroll
                    for (int j = 0; j < 4; ++j) As[wb][major][a_minor + j] = ra[S][a][j];
                }
                if (i >= 4 && i < 4 + PB) {                       // B quads of slice s+2 -> LDS
                    const int bq = i - 4;
                    *reinterpret_cast<f4 *>(&Bs[wb][b_k + bq * B_K_PER_PASS][b_n]) = rb[S][bq];
                }
                if (i >= 8 && i < 8 + PA)                         // refill the staging set: slice s+6
                    ra[S][i - 8] = *reinterpret_cast<const f4 *>(a_src + refill * a_slice + (i - 8) * a_pass);
                if (i >= 10 && i < 10 + PB)
                    rb[S][i - 10] = *reinterpret_cast<const f4 *>(b_src + (static_cast<uint64_t>(refill) * kBK + static_cast<uint64_t>(i - 10) * B_K_PER_PASS) * ldb);
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();
        };
        using Set2 = std::integral_constant<int, 2>;
        using Set3 = std::integral_constant<int, 3>;
        load_slice(Set1{}, 1);
        load_slice(Set2{}, 2);
        load_slice(Set3{}, 3);
        // slices 4 and 5 do not exist when K = 128 (four slices): like the in-loop refill, the prefetch then
        // reads the last slice again (never used) instead of running past the operands
        stage_to_lds(Set0{}, 0);
        load_slice(Set0{}, 4 < n_slices ? 4 : last);
        __syncthreads();
        read_frags(Set0{}, 0);
        stage_to_lds(Set1{}, 1);
        load_slice(Set1{}, 5 < n_slices ? 5 : last);
        __syncthreads();
        for (uint32_t s = 0; s < n_slices; s += 4) {        // the slice count is a multiple of 4
            deep_iteration(Set0{}, Set1{}, Set2{}, s);
            deep_iteration(Set1{}, Set0{}, Set3{}, s + 1);
            deep_iteration(Set0{}, Set1{}, Set0{}, s + 2);
            deep_iteration(Set1{}, Set0{}, Set1{}, s + 3);
        }
    } else {
        stage_to_lds(Set0{}, 0);
        load_slice(Set0{}, 1);
        __syncthreads();
        uint32_t s = 0;
        for (; s + 2 < n_slices; ++s) iteration(Set0{}, s, std::true_type{}, std::true_type{});
        prefetch_tile();
        iteration(Set0{}, s, std::true_type{}, std::false_type{});
        iteration(Set0{}, s + 1, std::false_type{}, std::false_type{});
    }

    // accumulators -> LDS tile.  Register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32 of the 32x32 block.
    // (the loop's last barrier already guarantees that the staging buffers are dead)
    #pragma unroll
    for (int r = 0; r < 16; ++r)
        Ct[wm * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4)][wn * 32 + lane % 32] = acc[r];
    __syncthreads();

    // epilogue over the tile in row-major quads: BN/4 lanes cover one row
    #pragma unroll
    for (int it = 0; it < EPI_ITERS; ++it) {
        const uint32_t idx = it * THREADS + t;
        const uint32_t row = idx / (BN / 4), col = (idx % (BN / 4)) * 4;
        const f4 val = *reinterpret_cast<const f4 *>(&Ct[row][col]);
        if (EPI == kFwd) {
            const f4 bias = *reinterpret_cast<const f4 *>(p.x_in + static_cast<uint64_t>(worker) * p.stride + o.b1 + n0 + col);
            f4 h = val + bias;
            h.x = fmaxf(h.x, 0.f); h.y = fmaxf(h.y, 0.f); h.z = fmaxf(h.z, 0.f); h.w = fmaxf(h.w, 0.f);
            *reinterpret_cast<f4 *>(p.H + (static_cast<uint64_t>(worker) * p.batch + m0 + row) * p.n_hid + n0 + col) = h;
        } else {
            const uint64_t at = static_cast<uint64_t>(worker) * p.stride + o.W1 + static_cast<uint64_t>(m0 + row) * p.n_hid + n0 + col;
            f4 g = val + p.weight_decay * x_old[it];
            if (p.momentum != 0.0f) {
                g = p.momentum * v_old[it] + g;
                __builtin_nontemporal_store(g, reinterpret_cast<f4 *>(p.v + at));
            }
            f4 x_new = x_old[it] - p.lr * g;
            if (EPI == kBwdTail) {       // line 6 of Algorithm 1 on the fresh model, same operation order as the separate kernel
                const f4 mean = *reinterpret_cast<const f4 *>(p.mean + o.W1 + static_cast<uint64_t>(m0 + row) * p.n_hid + n0 + col);
                x_new = mean + (x_new - snap_old[it]);
            }
            __builtin_nontemporal_store(x_new, reinterpret_cast<f4 *>(p.x_out + at));
        }
    }
}

template <int EPI, int NWM, int NWN>
void launch_gemm(hipStream_t stream, const MlpParams &p, hipEvent_t start = nullptr, hipEvent_t stop = nullptr)
{
    const uint32_t M = (EPI == kFwd) ? p.batch : p.n_in;
    const dim3 grid(p.n_hid / (32 * NWN), M / (32 * NWM), p.W), block(64 * NWM * NWN);
    // the events, if any, take the kernel's own start / end timestamps (no marker of their own in the queue)
    if (start || stop) hipExtLaunchKernelGGL((mlp_gemm_kernel<EPI, NWM, NWN>), grid, block, 0, stream, start, stop, 0, p);
    else               hipLaunchKernelGGL((mlp_gemm_kernel<EPI, NWM, NWN>), grid, block, 0, stream, p);
}

// ---- output layer -----------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
    #pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Output layer, forward and backward, one wave per sample (eight waves and samples per block, so that two
// waves share a SIMD: a wave's loop is a chain of memory round trips and shuffles):
//   Z = H W2 + b2 by a strided dot product over the hidden units and a butterfly reduction, softmax
//   (row maximum subtracted), dZ = (P - onehot(y)) / batch, then dA = (dZ W2^T) * [H > 0] for the
//   wave's own hidden units.  W2 of the block's worker sits in LDS (row pitch n_out + 1 when n_out
//   is even, so the 64 lanes of a wave, which read 64 consecutive rows, spread over the banks).
//   The output width is a template parameter: with it known, the loops over the classes unroll into
//   straight-line code (as a run-time bound they became a branch per class and per hidden unit).
constexpr int kHeadSamples = 8;        // per block: one wave each
constexpr int kHeadBatch = 8;          // independent loads in flight per lane
constexpr int kHeadKeep = 2;           // head: batches of a sample's H row that stay in registers (1024 hidden units)
constexpr int kUpdateWaves = 8;                 // head_update: waves per block, each sums an eighth of the batch
constexpr int kDzGroup = 16, kDzBatch = 16;     //   samples per staged group of dZ rows, and per batch of H / dA loads
constexpr uint32_t kHeadLdsBytes = 128u << 10;
__host__ __device__ inline uint32_t head_w2_pitch(uint32_t n_out) { return n_out % 2 == 0 ? n_out + 1 : n_out; }
template <int NOUT>
__global__ __launch_bounds__(64 * kHeadSamples) void head_kernel(const MlpParams p)
{
    constexpr uint32_t THREADS = 64 * kHeadSamples;
    constexpr uint32_t w2_pitch = NOUT % 2 == 0 ? NOUT + 1 : NOUT;
    extern __shared__ float w2s[];     // [n_hid][w2_pitch]
    const uint32_t worker = blockIdx.y;
    const uint32_t lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const Offsets o = offsets_of(p);
    const float *theta = p.x_in + static_cast<uint64_t>(worker) * p.stride;
    // The wave's sample, and the first kHeadKeep batches of its H row: requested before anything else (they
    // arrive while W2 is staged) and kept in registers for the second pass.
    const uint32_t b = blockIdx.x * kHeadSamples + wave;
    const bool have_sample = b < p.batch;                              // wave-uniform
    const uint64_t sample = static_cast<uint64_t>(worker) * p.batch + (have_sample ? b : 0u);
    const float *Hrow = p.H + sample * p.n_hid;
    float hkeep[kHeadKeep][kHeadBatch];
    #pragma unroll
    for (int it = 0; it < kHeadKeep; ++it) {
        #pragma unroll
        for (int u = 0; u < kHeadBatch; ++u) {
            const uint32_t n = lane + 64u * (u + kHeadBatch * it);
            hkeep[it][u] = n < p.n_hid ? Hrow[n] : 0.0f;
        }
    }
    // W2 -> LDS in 16-byte pieces, four loads in flight per thread (the matrix starts on a 16-byte
    // boundary and holds a multiple of 4 elements, by the shape contract)
    const uint32_t n_quads = p.n_hid * NOUT / 4;
    for (uint32_t q0 = threadIdx.x; q0 < n_quads; q0 += THREADS * 4) {
        f4 r[4];
        #pragma unroll
        for (int u = 0; u < 4; ++u)
            r[u] = q0 + THREADS * u < n_quads ? *reinterpret_cast<const f4 *>(theta + o.W2 + 4ull * (q0 + THREADS * u)) : f4{0.f, 0.f, 0.f, 0.f};
        #pragma unroll
        for (int u = 0; u < 4; ++u)
            if (q0 + THREADS * u < n_quads) {
                #pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t i = 4 * (q0 + THREADS * u) + j;
                    w2s[(i / NOUT) * w2_pitch + i % NOUT] = r[u][j];
                }
            }
    }
    __syncthreads();
    const float inv_b = 1.0f / static_cast<float>(p.batch);
    {
        if (!have_sample) return;                                  // behind the only barrier
        float z[NOUT];
        #pragma unroll
        for (int c = 0; c < NOUT; ++c) z[c] = 0.0f;
        #pragma unroll
        for (int it = 0; it < kHeadKeep; ++it) {
            #pragma unroll
            for (int u = 0; u < kHeadBatch; ++u) {
                const uint32_t n = lane + 64u * (u + kHeadBatch * it);
                if (n < p.n_hid) {
                    const float *w2 = w2s + n * w2_pitch;
                    #pragma unroll
                    for (int c = 0; c < NOUT; ++c) z[c] += hkeep[it][u] * w2[c];
                }
            }
        }
        // hidden units beyond the kept ones in batches of kHeadBatch loads in flight (one load at a time
        // would make the loop a chain of memory latencies)
        for (uint32_t n0 = lane + 64u * kHeadBatch * kHeadKeep; n0 < p.n_hid; n0 += 64 * kHeadBatch) {
            float hv[kHeadBatch];
            #pragma unroll
            for (int u = 0; u < kHeadBatch; ++u) hv[u] = n0 + 64 * u < p.n_hid ? Hrow[n0 + 64 * u] : 0.0f;
            #pragma unroll
            for (int u = 0; u < kHeadBatch; ++u) {
                if (n0 + 64 * u < p.n_hid) {
                    const float *w2 = w2s + (n0 + 64 * u) * w2_pitch;
                    #pragma unroll
                    for (int c = 0; c < NOUT; ++c) z[c] += hv[u] * w2[c];
                }
            }
        }
        float zmax = -INFINITY;
        #pragma unroll
        for (int c = 0; c < NOUT; ++c) {
            z[c] = wave_sum(z[c]) + theta[o.b2 + c];
            zmax = fmaxf(zmax, z[c]);
        }
        float denom = 0.0f;
        #pragma unroll
        for (int c = 0; c < NOUT; ++c) { z[c] = expf(z[c] - zmax); denom += z[c]; }
        const int label = p.y[sample];
        #pragma unroll
        for (int c = 0; c < NOUT; ++c) {
            z[c] = (z[c] / denom - (label == c ? 1.0f : 0.0f)) * inv_b;                // dZ, the same in every lane
            if (lane == static_cast<uint32_t>(c)) p.dZ[sample * kMaxOut + c] = z[c];
        }
        #pragma unroll
        for (int it = 0; it < kHeadKeep; ++it) {
            #pragma unroll
            for (int u = 0; u < kHeadBatch; ++u) {
                const uint32_t n = lane + 64u * (u + kHeadBatch * it);
                if (n < p.n_hid) {
                    const float *w2 = w2s + n * w2_pitch;
                    float dh = 0.0f;
                    #pragma unroll
                    for (int c = 0; c < NOUT; ++c) dh += z[c] * w2[c];
                    p.dA[sample * p.n_hid + n] = hkeep[it][u] > 0.0f ? dh : 0.0f;
                }
            }
        }
        for (uint32_t n0 = lane + 64u * kHeadBatch * kHeadKeep; n0 < p.n_hid; n0 += 64 * kHeadBatch) {
            float hv[kHeadBatch];
            #pragma unroll
            for (int u = 0; u < kHeadBatch; ++u) hv[u] = n0 + 64 * u < p.n_hid ? Hrow[n0 + 64 * u] : 0.0f;
            #pragma unroll
            for (int u = 0; u < kHeadBatch; ++u) {
                if (n0 + 64 * u < p.n_hid) {
                    const float *w2 = w2s + (n0 + 64 * u) * w2_pitch;
                    float dh = 0.0f;
                    #pragma unroll
                    for (int c = 0; c < NOUT; ++c) dh += z[c] * w2[c];
                    p.dA[sample * p.n_hid + n0 + 64 * u] = hv[u] > 0.0f ? dh : 0.0f;
                }
            }
        }
    }
}

// Gradients of the small parameters and their update.  A block owns 64 hidden units (row n of W2 and
// b1[n]); its eight waves each sum an eighth of the batch and the partial sums meet in LDS in a fixed
// order.  Block 0 of a worker also owns b2 and the alignment pads.
template <int NOUT>
__global__ __launch_bounds__(64 * kUpdateWaves) void head_update_kernel(const MlpParams p)
{
    __shared__ float part[kUpdateWaves][64][NOUT + 1];
    __shared__ __attribute__((aligned(16))) float dzs[kUpdateWaves][kDzGroup][kMaxOut];     // per wave: dZ rows of the current group
    // The first W * ceil(n_hid / 64) blocks own hidden units.  The blocks behind them draw the NEXT local
    // step's mini-batch into the other batch buffer: the owners are a short chain of dependent loads on one
    // block per compute unit, and the generator is pure vector arithmetic that fills the rest of the chip
    // meanwhile.  Blocks are dispatched in the order of their index: the owners, whose chain decides when
    // the kernel ends, all start at once.
    const uint32_t own_blocks = (p.n_hid + 63) / 64;
    if (blockIdx.x >= own_blocks * p.W) {
        constexpr uint32_t GROUPS = kUpdateWaves / 4;                // 256-thread generator groups per block
        const uint32_t id = blockIdx.x - own_blocks * p.W, per_worker = (gen_batch_blocks(p) + GROUPS - 1) / GROUPS;
        const uint32_t step = p.step_base ? *p.step_base + p.step : p.step;
        gen_batch_block(p, (id % per_worker) * GROUPS + threadIdx.x / 256, threadIdx.x % 256, id / per_worker, step + 1, p.X_next, p.y_next);
        return;
    }
    const uint32_t worker = blockIdx.x / own_blocks, own = blockIdx.x % own_blocks;
    const uint32_t u = threadIdx.x % 64, slice = threadIdx.x / 64;
    const uint32_t n = own * 64 + u;
    const Offsets o = offsets_of(p);
    const uint64_t base = static_cast<uint64_t>(worker) * p.stride;
    float gw[NOUT];
    #pragma unroll
    for (int c = 0; c < NOUT; ++c) gw[c] = 0.0f;
    float gb = 0.0f;
    {
        // The wave's eighth of the batch in groups of 16 samples.  Every lane needs the same dZ rows: the wave
        // fetches a group's rows once (one quad per lane) into its own piece of LDS and reads them back as
        // broadcasts, instead of 10 same-address loads per sample and lane.
        const uint32_t per = p.batch / kUpdateWaves;                 // a multiple of 16 by the shape contract
        const bool mine = n < p.n_hid;
        for (uint32_t g0 = slice * per; g0 < (slice + 1) * per; g0 += kDzGroup) {
            const float *dz_rows = p.dZ + (static_cast<uint64_t>(worker) * p.batch + g0) * kMaxOut;
            static_assert(kDzGroup * kMaxOut == 4 * 64, "one quad of the group's dZ rows per lane");
            const f4 q0 = *reinterpret_cast<const f4 *>(dz_rows + 4 * u);
            #pragma unroll
            for (int half = 0; half < kDzGroup / kDzBatch; ++half) {
                float hv[kDzBatch], da[kDzBatch];                    // the batch's loads are all in flight together
                #pragma unroll
                for (int j = 0; j < kDzBatch; ++j) {
                    const uint64_t sample = static_cast<uint64_t>(worker) * p.batch + g0 + half * kDzBatch + j;
                    hv[j] = mine ? p.H[sample * p.n_hid + n] : 0.0f;
                    da[j] = mine ? p.dA[sample * p.n_hid + n] : 0.0f;
                }
                if (half == 0) {                                     // rows of the group -> LDS (this wave's piece only)
                    *reinterpret_cast<f4 *>(&dzs[slice][0][0] + 4 * u) = q0;
                }
                #pragma unroll
                for (int j = 0; j < kDzBatch; ++j) {
                    gb += da[j];
                    #pragma unroll
                    for (int c = 0; c < NOUT; ++c) gw[c] += hv[j] * dzs[slice][half * kDzBatch + j][c];
                }
            }
        }
    }
    #pragma unroll
    for (int c = 0; c < NOUT; ++c) part[slice][u][c] = gw[c];
    part[slice][u][NOUT] = gb;
    __syncthreads();
    if (slice == 0 && n < p.n_hid) {
        // row n of W2 and b1[n]: all old values first (independent loads), then the updates
        uint64_t at[NOUT + 1];
        float xo[NOUT + 1], vo[NOUT + 1];
        #pragma unroll
        for (int c = 0; c <= NOUT; ++c) {
            at[c] = c == NOUT ? base + o.b1 + n : base + o.W2 + static_cast<uint64_t>(n) * NOUT + c;
            xo[c] = p.x_in[at[c]];
            vo[c] = p.momentum != 0.0f ? p.v[at[c]] : 0.0f;
        }
        #pragma unroll
        for (int c = 0; c <= NOUT; ++c) {
            {
                float G = part[0][u][c];
                #pragma unroll
                for (int w = 1; w < kUpdateWaves; ++w) G += part[w][u][c];
                float g = G + p.weight_decay * xo[c];
                if (p.momentum != 0.0f) {
                    g = p.momentum * vo[c] + g;
                    p.v[at[c]] = g;
                }
                float x_new = xo[c] - p.lr * g;
                if (p.snap) x_new = p.mean[at[c] - base] + (x_new - p.snap[at[c]]);   // line 6 (last step of a round)
                p.x_out[at[c]] = x_new;
            }
        }
    }
    if (own == 0 && slice == 1) {
        // db2[c] = sum_b dZ[b][c]: lanes take the samples 64 apart, then a butterfly over the wave
        float col[NOUT];
        #pragma unroll
        for (int c = 0; c < NOUT; ++c) col[c] = 0.0f;
        for (uint32_t b = u; b < p.batch; b += 64) {
            const float *dz = p.dZ + (static_cast<uint64_t>(worker) * p.batch + b) * kMaxOut;
            #pragma unroll
            for (int c = 0; c < NOUT; ++c) col[c] += dz[c];
        }
        #pragma unroll
        for (int c = 0; c < NOUT; ++c) {
            const float g = wave_sum(col[c]);
            if (u == static_cast<uint32_t>(c)) sgd_update(p, base + o.b2 + u, g);
        }
        const uint64_t d = o.b2 + NOUT;                       // pads after the last parameter travel along
        if (p.x_out != p.x_in && u < ((d + 3) & ~3ull) - d) p.x_out[base + d + u] = p.x_in[base + d + u];
    }
}

// The two output-layer kernels, instantiated for every supported output width 1..kMaxOut.
template <int NOUT>
hipError_t launch_heads_for(hipStream_t stream, const MlpParams &p)
{
    // more than the default 64 KB of dynamic LDS for wide hidden layers
    static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void *>(head_kernel<NOUT>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, kHeadLdsBytes);
    if (lds_ok != hipSuccess) return lds_ok;
    hipLaunchKernelGGL(head_kernel<NOUT>, dim3((p.batch + kHeadSamples - 1) / kHeadSamples, p.W), dim3(64 * kHeadSamples),
                       static_cast<size_t>(p.n_hid) * head_w2_pitch(NOUT) * sizeof(float), stream, p);
    const uint32_t gen_blocks = p.X_next ? (gen_batch_blocks(p) + kUpdateWaves / 4 - 1) / (kUpdateWaves / 4) : 0u;
    const uint64_t update_blocks = (static_cast<uint64_t>((p.n_hid + 63) / 64) + gen_blocks) * p.W;
    if (update_blocks > 0x7fffffffull) return hipErrorInvalidValue;      // a mini-batch of terabytes: its work space was never allocated
    hipLaunchKernelGGL(head_update_kernel<NOUT>, dim3(static_cast<uint32_t>(update_blocks)), dim3(64 * kUpdateWaves), 0, stream, p);
    return hipSuccess;
}

template <int... I>
hipError_t launch_heads(hipStream_t stream, const MlpParams &p, std::integer_sequence<int, I...>)
{
    hipError_t rc = hipErrorInvalidValue;
    (void)((p.n_out == static_cast<uint32_t>(I + 1) ? (rc = launch_heads_for<I + 1>(stream, p), true) : false) || ...);
    return rc;
}

}  // namespace

bool mlp_shape_supported(uint32_t n_in, uint32_t n_hid, uint32_t n_out, uint32_t batch)
{
    return n_in >= static_cast<uint32_t>(kShapeM) && n_in % kShapeM == 0 && n_hid >= static_cast<uint32_t>(kShapeN) &&
           n_hid % kShapeN == 0 && n_out >= 1 && n_out <= static_cast<uint32_t>(kMaxOut) &&
           batch >= static_cast<uint32_t>(kShapeM) && batch % kShapeM == 0 && batch <= 1024 &&
           static_cast<uint64_t>(n_hid) * head_w2_pitch(n_out) * sizeof(float) <= kHeadLdsBytes;   // W2 lives in LDS
}

size_t mlp_dz_pitch() { return kMaxOut; }

hipError_t launch_mlp_step(hipStream_t stream, const MlpParams &p, hipEvent_t start, hipEvent_t stop)
{
    const bool wide = p.n_hid % 128 == 0;      // 64 x 128 block tiles (fastest measured), else 64 x 64
    if (!p.have_batch) {                       // the step then begins with this kernel
        if (start) hipExtLaunchKernelGGL(gen_batch_kernel, dim3(gen_batch_blocks(p), p.W), dim3(256), 0, stream, start, nullptr, 0, p);
        else       hipLaunchKernelGGL(gen_batch_kernel, dim3(gen_batch_blocks(p), p.W), dim3(256), 0, stream, p);
        start = nullptr;
    }
    if (wide) launch_gemm<kFwd, 2, 4>(stream, p, start); else launch_gemm<kFwd, 2, 2>(stream, p, start);
    const hipError_t head_rc = launch_heads(stream, p, std::make_integer_sequence<int, kMaxOut>{});
    if (head_rc != hipSuccess) return head_rc;
    if (p.snap) { if (wide) launch_gemm<kBwdTail, 2, 4>(stream, p, nullptr, stop); else launch_gemm<kBwdTail, 2, 2>(stream, p, nullptr, stop); }
    else        { if (wide) launch_gemm<kBwd, 2, 4>(stream, p, nullptr, stop); else launch_gemm<kBwd, 2, 2>(stream, p, nullptr, stop); }
    return hipGetLastError();
}

}  // namespace cocod
