// Batched per-worker minibatch gradient for the linear models (Algorithm 1,
// gradient step: g_k = gscale * sum_m grad F(x^_k; xi_{k,m}), evaluated at the
// stale read x^_k = row i_k of X at the round the planner chose).
//
//   least squares        grad F = a (a.x - b)
//   logistic regression  grad F = -y sigmoid(-y a.x) a + lambda x
//
// Wait-free variant (computation thread of the appendix on wait-free training): an operation
// may carry the slot of the worker's own pending gradient g_k'; the point of evaluation is then
// x^ = row - gamma_k' g_k' (two fp32 roundings, the same as the update itself).
//
// Three launches per group of gradient operations:
//   1. dots:     partial z[op][m][chunk] = A[idx_m, chunk] . x^[chunk]   (batched GEMV, HBM bound)
//   2. finalize: z -> per-sample coefficient c_m and the minibatch loss
//   3. combine:  g[chunk] = sum_m c_m A[idx_m, chunk] (+ reg * x^[chunk]) into the pending slot
// The gathered rows are read twice, both times from HBM (re-reading them from the
// memory-side cache is no faster, and a one-pass variant needs a chip-wide
// dependency that costs more than the second read).  Short models (d <= 2048)
// take the single-block kernel at the end of this file instead.  Partial sums
// are combined in a fixed order: results do not depend on scheduling.
#include "device_common.hpp"
#include "internal.hpp"

namespace adpsgd_impl {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
// tile shape of the two streaming kernels (8-32 rows per block and unrolls of 2-8 measure within 5 %)
constexpr int kDotUnroll = 4;                                 // float4 per thread per row
constexpr int64_t kDotChunk = kThreads * kDotUnroll * 4;     // floats of d per block
constexpr int kRowsPerBlock = 8;                              // minibatch rows per dots block

struct LinParams {
    int model;
    const float* X;
    int64_t ld;
    int64_t d;
    int64_t n_vec;
    int64_t n_chunks;   // dots chunks per row
    const GradOp* ops;
    int32_t M;
    const int32_t* batch_idx;
    float* slots;
    float gscale;
    float lambda;
    float* partial;     // [op][M + 1][n_chunks]
    float* coef;        // [op][M]
    float* loss;
    int factored;       // least squares: the coefficients go to the start of the operation's pending slot and
                        // stay there; the update kernel forms g = sum_m c_m a_m while it applies the event
};

__device__ __forceinline__ v4f zero_beyond(v4f v, int64_t e, int64_t d) {
    if (e + 4 > d) {
        if (e + 1 >= d) v.y = 0.0f;
        if (e + 2 >= d) v.z = 0.0f;
        if (e + 3 >= d) v.w = 0.0f;
        if (e >= d) v.x = 0.0f;
    }
    return v;
}
// the stale read of one operation, four elements at vector index v (v < n_vec)
__device__ __forceinline__ v4f read_xhat(const LinParams& p, const GradOp& op, int64_t v) {
#pragma clang fp contract(off)
    v4f x = *reinterpret_cast<const v4f*>(p.X + static_cast<int64_t>(op.worker) * p.ld + 4 * v);
    if (op.comp_slot >= 0) {
        const v4f g = *reinterpret_cast<const v4f*>(p.slots + static_cast<int64_t>(op.comp_slot) * p.ld + 4 * v);
        const v4f step = g * op.comp_gamma;
        x = x - step;
    }
    return x;
}
__device__ __forceinline__ float dot4(v4f a, v4f b) { return a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w; }

// grid = (n_chunks, ceil((M+1) / kRowsPerBlock), n_ops); "row" M is x^ itself (|x^|^2 for the regulariser)
// STREAM: the gathered rows exceed the L2 (they are read once per kernel): non-temporal loads,
// 7.0 instead of 6.2 TB/s on a read-only stream.
template <bool STREAM>
__global__ __launch_bounds__(kThreads) void linear_dots_kernel(const LinParams p) {
    __shared__ float red[kWaves][kRowsPerBlock];
    const GradOp op = p.ops[blockIdx.z];
    const float* __restrict__ A = static_cast<const float*>(op.features);
    const int32_t* __restrict__ idx = p.batch_idx + static_cast<int64_t>(op.event) * p.M;
    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * (kDotChunk / 4) + threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    v4f xh[kDotUnroll];
#pragma unroll
    for (int u = 0; u < kDotUnroll; ++u) {
        const int64_t v = v0 + static_cast<int64_t>(u) * kThreads;
        xh[u] = v < p.n_vec ? zero_beyond(read_xhat(p, op, v), 4 * v, p.d) : v4f{0, 0, 0, 0};
    }
    const int m_begin = blockIdx.y * kRowsPerBlock;
#pragma unroll 2
    for (int r = 0; r < kRowsPerBlock; ++r) {
        const int m = m_begin + r;
        if (m > p.M) break;
        if (m == p.M && p.model != ADPSGD_MODEL_LOGREG) break;
        float acc = 0.0f;
        if (m < p.M) {
            const float* __restrict__ row = A + static_cast<int64_t>(idx[m]) * op.ld;
#pragma unroll
            for (int u = 0; u < kDotUnroll; ++u) {
                const int64_t v = v0 + static_cast<int64_t>(u) * kThreads;
                if (v < p.n_vec) acc += dot4(zero_beyond(load4<STREAM>(row + 4 * v), 4 * v, p.d), xh[u]);
            }
        } else {   // |x^|^2 of this chunk
#pragma unroll
            for (int u = 0; u < kDotUnroll; ++u) acc += dot4(xh[u], xh[u]);
        }
        acc = wave_sum(acc);
        if (lane == 0) red[wave][r] = acc;
    }
    __syncthreads();
    if (threadIdx.x < kRowsPerBlock) {
        const int m = m_begin + threadIdx.x;
        if (m < p.M || (m == p.M && p.model == ADPSGD_MODEL_LOGREG)) {
            float s = red[0][threadIdx.x];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) s += red[w][threadIdx.x];
            p.partial[(static_cast<int64_t>(blockIdx.z) * (p.M + 1) + m) * p.n_chunks + blockIdx.x] = s;
        }
    }
}

// Sum of the n_chunks partials of one dot product by a group of L lanes (L a power of two):
// lane t adds the partials t, t + L, ... in order, 8 independent loads in flight, then the L lane
// sums are combined by a fixed butterfly.
__device__ __forceinline__ float sum_chunks(const float* __restrict__ part, int64_t n_chunks, int sub, int L) {
    float s = 0.0f;
    for (int64_t c0 = sub; c0 < n_chunks; c0 += 8 * L) {
        float vbuf[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int64_t c = c0 + static_cast<int64_t>(t) * L;
            vbuf[t] = c < n_chunks ? part[c] : 0.0f;
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) s += vbuf[t];
    }
    for (int off = L >> 1; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    return s;
}

// grid = n_ops; L = lanes_per_row lanes per minibatch sample (host: largest power of two with
// L * M <= 256, at most 64), so that M <= 256 is finished in one pass of the block
__global__ __launch_bounds__(kThreads) void linear_finalize_kernel(const LinParams p, const int L) {
    __shared__ float red[kWaves];
    const GradOp op = p.ops[blockIdx.x];
    const float* __restrict__ tg = static_cast<const float*>(op.targets);
    const int32_t* __restrict__ idx = p.batch_idx + static_cast<int64_t>(op.event) * p.M;
    const float* __restrict__ part = p.partial + static_cast<int64_t>(blockIdx.x) * (p.M + 1) * p.n_chunks;
    const int sub = threadIdx.x & (L - 1), grp = threadIdx.x / L, groups = kThreads / L;
    float reg_loss = 0.0f;
    if (p.model == ADPSGD_MODEL_LOGREG)
        reg_loss = 0.5f * p.lambda * sum_chunks(part + static_cast<int64_t>(p.M) * p.n_chunks, p.n_chunks, sub, L);
    float loss = 0.0f;
    for (int m0 = 0; m0 < p.M; m0 += groups) {     // uniform trip count: shuffles stay converged
        const int m = m0 + grp;
        const bool live = m < p.M;
        const float t = live ? tg[idx[m]] : 0.0f;   // issued before the partial sums are waited for
        const float z = sum_chunks(part + static_cast<int64_t>(live ? m : 0) * p.n_chunks, p.n_chunks, sub, L);
        if (live && sub == 0) {
            float c_m;
            if (p.model == ADPSGD_MODEL_LSQ) {
                const float r = z - t;              // a.x - b
                loss += 0.5f * r * r;
                c_m = r;
            } else {
                const float s = -t * z;             // F = log(1 + e^s) + reg
                loss += (s > 0.0f ? s + log1pf(expf(-s)) : log1pf(expf(s))) + reg_loss;
                c_m = -t / (1.0f + expf(-s));       // -y sigmoid(s)
            }
            float* __restrict__ dst = p.factored ? p.slots + static_cast<int64_t>(op.slot) * p.ld
                                                 : p.coef + static_cast<int64_t>(blockIdx.x) * p.M;
            dst[m] = c_m * p.gscale;
        }
    }
    loss = wave_sum(loss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = loss;
    __syncthreads();
    if (threadIdx.x == 0 && p.loss) {
        float s = red[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) s += red[w];
        p.loss[op.event] = s * p.gscale;
    }
}

// four elements of sum_m c_m a_m at vector index v (the one place this sum is written, so that the dense
// and the factored path produce the same bits)
template <bool STREAM>
__device__ __forceinline__ v4f combine_rows(const float* __restrict__ A, int64_t lda, const int32_t* __restrict__ idx,
                                            const float* __restrict__ cf, int M, int64_t v) {
    v4f acc = {0, 0, 0, 0};
#pragma unroll 8
    for (int m = 0; m < M; ++m) {
        const v4f a = load4<STREAM>(A + static_cast<int64_t>(idx[m]) * lda + 4 * v);
        acc += a * cf[m];
    }
    return acc;
}

// grid = (ceil(n_vec / kThreads), n_ops)
template <bool STREAM>
__global__ __launch_bounds__(kThreads) void linear_combine_kernel(const LinParams p) {
    const GradOp op = p.ops[blockIdx.y];
    const int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (v >= p.n_vec) return;
    const float* __restrict__ A = static_cast<const float*>(op.features);
    const int32_t* __restrict__ idx = p.batch_idx + static_cast<int64_t>(op.event) * p.M;
    const float* __restrict__ cf = p.coef + static_cast<int64_t>(blockIdx.y) * p.M;
    v4f acc = combine_rows<STREAM>(A, op.ld, idx, cf, p.M, v);
    if (p.model == ADPSGD_MODEL_LOGREG) {
        const v4f xh = read_xhat(p, op, v);
        acc += xh * (p.lambda * p.gscale * static_cast<float>(p.M));
    }
    acc = zero_beyond(acc, 4 * v, p.d);
    *reinterpret_cast<v4f*>(p.slots + static_cast<int64_t>(op.slot) * p.ld + 4 * v) = acc;
}

// ---- least squares, factored: the update of an event with g formed from its coefficients --------
//     avg = (x^i + x^j) / 2;  x^j <- avg;  x^i <- avg - gamma * sum_m c_m a_m
// The gradient of a linear model is a combination of its M minibatch rows, so the pending slot keeps
// the M coefficients and the rows are read when the event is applied: the dense gradient is never
// written to memory and read back (8 B per parameter and event less, and one launch per round less).
// grid = (ceil(n_vec / kThreads), events of the round)
struct LinApplyParams {
    float* X;
    int64_t ld;
    int64_t d;
    int64_t n_vec;
    const PairOp* ops;
    const float* slots;
    const int32_t* batch_idx;
    int32_t M;
    float* V;               // momentum buffers (MOM), else nullptr
    float momentum, weight_decay;
};

template <bool STREAM_ROWS, bool STREAM_X, bool MOM>
__global__ __launch_bounds__(kThreads) void linear_apply_factored_kernel(const LinApplyParams p) {
    const PairOp op = p.ops[blockIdx.y];
    const int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (v >= p.n_vec) return;
    float* __restrict__ xi = p.X + static_cast<int64_t>(op.i) * p.ld + 4 * v;
    float* __restrict__ xj = p.X + static_cast<int64_t>(op.j) * p.ld + 4 * v;
    const v4f a = load4<STREAM_X>(xi), b = load4<STREAM_X>(xj);
    const bool average_only = (op.flags & 1) != 0;      // extra pair of a general W_k: no gradient, no step
    v4f g = {0, 0, 0, 0};
    if (!average_only)
        g = zero_beyond(combine_rows<STREAM_ROWS>(static_cast<const float*>(op.features), op.feat_ld,
                                                  p.batch_idx + static_cast<int64_t>(op.event) * p.M,
                                                  p.slots + static_cast<int64_t>(op.slot) * p.ld, p.M, v), 4 * v, p.d);
    const float gamma = average_only ? 0.0f : op.gamma;
    const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w}, gv[4] = {g.x, g.y, g.z, g.w};
    float ni[4], nj[4];
    if (MOM && !average_only) {       // an averaging-only pair leaves the momentum buffers alone
        float* __restrict__ vi = p.V + static_cast<int64_t>(op.i) * p.ld + 4 * v;
        const v4f vo = load4<STREAM_X>(vi);
        const float vold[4] = {vo.x, vo.y, vo.z, vo.w};
        float vn[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            average_then_apply_momentum(av[c], bv[c], gv[c], vold[c], gamma, p.momentum, p.weight_decay, ni[c], nj[c], vn[c]);
        store4<STREAM_X>(vi, v4f{vn[0], vn[1], vn[2], vn[3]});   // zero in the padding, as x and g are
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) average_then_apply(av[c], bv[c], gv[c], gamma, ni[c], nj[c]);
    }
    store4<STREAM_X>(xi, v4f{ni[0], ni[1], ni[2], ni[3]});     // the padding beyond d stays zero: g is zero there
    if (op.i != op.j) store4<STREAM_X>(xj, v4f{nj[0], nj[1], nj[2], nj[3]});
}

template <bool MOM>
hipError_t launch_apply_variant(const LinApplyParams& p, dim3 grid, bool stream_rows, bool stream_x, hipStream_t st) {
    if (stream_rows && stream_x) hipLaunchKernelGGL((linear_apply_factored_kernel<true, true, MOM>), grid, dim3(kThreads), 0, st, p);
    else if (stream_rows) hipLaunchKernelGGL((linear_apply_factored_kernel<true, false, MOM>), grid, dim3(kThreads), 0, st, p);
    else if (stream_x) hipLaunchKernelGGL((linear_apply_factored_kernel<false, true, MOM>), grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((linear_apply_factored_kernel<false, false, MOM>), grid, dim3(kThreads), 0, st, p);
    return hipGetLastError();
}

// ---- short models: the whole gradient of one operation in one block, one launch -----------
// For d <= 2048 a round is a chain of launch-bound kernels, so the three steps above run in a
// single block of 1024 threads per gradient: wavefront w takes the minibatch rows w, w + 16, ...
// (lane l holds the float4 elements l, l + 64, ... of x^ in registers), the coefficients and the
// loss are finished by M threads, and the rows (read again, from the cache) are combined by
// 1024 / (64 U) thread groups that each take every G-th row of one float4 column and are added
// in group order through LDS.  U = float4 elements of x^ per lane, R = rows of a wavefront
// in flight (U (R + 1) float4 registers must fit the 128 a thread of a 1024-thread block has).
constexpr int kSmallT = 1024;
constexpr int kSmallWaves = kSmallT / 64;
constexpr int kSmallMaxM = 256;
constexpr int64_t kSmallMaxD = 2048;

template <int U, int R>
__global__ __launch_bounds__(kSmallT) void linear_small_kernel(const LinParams p) {
    __shared__ float z_s[kSmallMaxM + 1];
    __shared__ float coef_s[kSmallMaxM];
    __shared__ float loss_s[kSmallMaxM];
    __shared__ v4f part_s[kSmallT];        // [group][column]
    const GradOp op = p.ops[blockIdx.x];
    const float* __restrict__ A = static_cast<const float*>(op.features);
    const float* __restrict__ tg = static_cast<const float*>(op.targets);
    const int32_t* __restrict__ idx = p.batch_idx + static_cast<int64_t>(op.event) * p.M;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float target = 0.0f;
    if (static_cast<int>(threadIdx.x) < p.M) target = tg[idx[threadIdx.x]];      // requested now, used after the dots

    v4f xh[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t v = lane + 64 * u;
        xh[u] = v < p.n_vec ? zero_beyond(read_xhat(p, op, v), 4 * v, p.d) : v4f{0, 0, 0, 0};
    }
    const int n_rows = p.M + (p.model == ADPSGD_MODEL_LOGREG ? 1 : 0);   // row M: |x^|^2 for the regulariser
    for (int m0 = wave; m0 < n_rows; m0 += R * kSmallWaves) {
        float acc[R];
        v4f a[R][U];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            acc[r] = 0.0f;
            const int m = m0 + r * kSmallWaves;
            if (m < p.M) {
                const float* __restrict__ row = A + static_cast<int64_t>(idx[m]) * op.ld;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t v = lane + 64 * u;
                    a[r][u] = v < p.n_vec ? zero_beyond(*reinterpret_cast<const v4f*>(row + 4 * v), 4 * v, p.d) : v4f{0, 0, 0, 0};
                }
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) a[r][u] = xh[u];
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int u = 0; u < U; ++u) acc[r] += dot4(a[r][u], xh[u]);
            acc[r] = wave_sum(acc[r]);
            const int m = m0 + r * kSmallWaves;
            if (lane == 0 && m < n_rows) z_s[m] = acc[r];
        }
    }
    __syncthreads();
    if (static_cast<int>(threadIdx.x) < p.M) {
        const int m = threadIdx.x;
        const float z = z_s[m];
        float c_m, l_m;
        if (p.model == ADPSGD_MODEL_LSQ) {
            const float r = z - target;              // a.x - b
            l_m = 0.5f * r * r;
            c_m = r;
        } else {
            const float s = -target * z;             // F = log(1 + e^s) + reg
            l_m = (s > 0.0f ? s + log1pf(expf(-s)) : log1pf(expf(s))) + 0.5f * p.lambda * z_s[p.M];
            c_m = -target / (1.0f + expf(-s));       // -y sigmoid(s)
        }
        coef_s[m] = c_m * p.gscale;
        loss_s[m] = l_m;
    }
    __syncthreads();
    if (threadIdx.x == 0 && p.loss) {
        float sl = 0.0f;
        for (int m = 0; m < p.M; ++m) sl += loss_s[m];
        p.loss[op.event] = sl * p.gscale;
    }
    constexpr int kCols = 64 * U, kGroups = kSmallT / kCols;
    const int v = threadIdx.x % kCols, grp = threadIdx.x / kCols;
    {
        v4f acc = {0, 0, 0, 0};
        if (v < p.n_vec) {
#pragma unroll 8
            for (int m = grp; m < p.M; m += kGroups) {
                const v4f a = *reinterpret_cast<const v4f*>(A + static_cast<int64_t>(idx[m]) * op.ld + 4 * v);
                acc += a * coef_s[m];
            }
        }
        part_s[grp * kCols + v] = acc;
    }
    __syncthreads();
    if (grp == 0 && v < p.n_vec) {
        v4f acc = part_s[v];
#pragma unroll
        for (int g = 1; g < kGroups; ++g) acc += part_s[g * kCols + v];
        if (p.model == ADPSGD_MODEL_LOGREG) acc += read_xhat(p, op, v) * (p.lambda * p.gscale * static_cast<float>(p.M));
        acc = zero_beyond(acc, 4 * static_cast<int64_t>(v), p.d);
        *reinterpret_cast<v4f*>(p.slots + static_cast<int64_t>(op.slot) * p.ld + 4 * v) = acc;
    }
}

}  // namespace

int64_t linear_grad_chunks(int64_t d) { return (d + kDotChunk - 1) / kDotChunk; }

bool linear_can_factor(int model, int64_t d, int32_t M, int64_t ld) {
    // least squares only (the logistic gradient carries lambda x^, which needs the stale read itself);
    // long models only (short ones are bound by launches, not by bytes); the coefficients must fit a slot
    return model == ADPSGD_MODEL_LSQ && d > kSmallMaxD && M >= 1 && M <= ld;
}

hipError_t launch_linear_apply_factored(const LinearApplyArgs& a, hipStream_t st) {
    if (a.n_ops <= 0) return hipSuccess;
    LinApplyParams p;
    p.X = a.X;
    p.ld = a.ld;
    p.d = a.d;
    p.n_vec = (a.d + 3) / 4;
    p.ops = a.ops;
    p.slots = a.slots;
    p.batch_idx = a.batch_idx;
    p.M = a.M;
    p.V = a.V;
    p.momentum = a.momentum;
    p.weight_decay = a.weight_decay;
    const int64_t blocks = (p.n_vec + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFF || a.n_ops > 65535) return hipErrorInvalidValue;
    const dim3 grid(static_cast<uint32_t>(blocks), a.n_ops);
    const bool stream_rows = static_cast<int64_t>(a.M) * a.d * 4 > (8ll << 20);
    return a.V ? launch_apply_variant<true>(p, grid, stream_rows, a.streaming, st)
               : launch_apply_variant<false>(p, grid, stream_rows, a.streaming, st);
}

hipError_t launch_linear_gradient(const LinearGradArgs& a, hipStream_t st, int* n_launches) {
    if (a.n_ops <= 0) return hipSuccess;
    LinParams p;
    p.model = a.model;
    p.X = a.X;
    p.ld = a.ld;
    p.d = a.d;
    p.n_vec = (a.d + 3) / 4;
    p.n_chunks = linear_grad_chunks(a.d);
    p.ops = a.ops;
    p.M = a.M;
    p.batch_idx = a.batch_idx;
    p.slots = a.slots;
    p.gscale = a.gscale;
    p.lambda = a.lambda;
    p.partial = a.partial;
    p.coef = a.coef;
    p.loss = a.loss;
    p.factored = a.factored ? 1 : 0;
    if (a.factored && !linear_can_factor(a.model, a.d, a.M, a.ld)) return hipErrorInvalidValue;
    if (a.d <= kSmallMaxD && a.M <= kSmallMaxM && a.n_ops <= 0x7FFFFFFF) {
        const int lanes_vec = static_cast<int>((p.n_vec + 63) / 64);      // float4 elements of x^ per lane
        const dim3 grid(a.n_ops), block(kSmallT);
        if (lanes_vec <= 1) hipLaunchKernelGGL((linear_small_kernel<1, 2>), grid, block, 0, st, p);
        else if (lanes_vec <= 2) hipLaunchKernelGGL((linear_small_kernel<2, 2>), grid, block, 0, st, p);
        else if (lanes_vec <= 4) hipLaunchKernelGGL((linear_small_kernel<4, 2>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((linear_small_kernel<8, 1>), grid, block, 0, st, p);
        if (n_launches) *n_launches += 1;
        return hipGetLastError();
    }
    const int64_t out_blocks = (p.n_vec + kThreads - 1) / kThreads;
    if (p.n_chunks > 0x7FFFFFFF || out_blocks > 0x7FFFFFFF || a.n_ops > 65535) return hipErrorInvalidValue;
    const uint32_t row_groups = static_cast<uint32_t>((a.M + 1 + kRowsPerBlock - 1) / kRowsPerBlock);
    if (row_groups > 65535) return hipErrorInvalidValue;
    const bool stream_rows = static_cast<int64_t>(a.M) * a.d * 4 > (8ll << 20);
    const dim3 dots_grid(static_cast<uint32_t>(p.n_chunks), row_groups, a.n_ops);
    if (stream_rows) hipLaunchKernelGGL(linear_dots_kernel<true>, dots_grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL(linear_dots_kernel<false>, dots_grid, dim3(kThreads), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    int lanes_per_row = 64;
    while (lanes_per_row > 1 && lanes_per_row * a.M > kThreads) lanes_per_row >>= 1;
    hipLaunchKernelGGL(linear_finalize_kernel, dim3(a.n_ops), dim3(kThreads), 0, st, p, lanes_per_row);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.factored) {
        if (n_launches) *n_launches += 2;
        return hipSuccess;
    }
    const dim3 comb_grid(static_cast<uint32_t>(out_blocks), a.n_ops);
    if (stream_rows) hipLaunchKernelGGL(linear_combine_kernel<true>, comb_grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL(linear_combine_kernel<false>, comb_grid, dim3(kThreads), 0, st, p);
    if (n_launches) *n_launches += 3;
    return hipGetLastError();
}

}  // namespace adpsgd_impl
