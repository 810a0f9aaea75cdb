// Model initialisation and diagnostics: equal initial models (Algorithm 1's
// requirement), the bf16 shadow of the master weights, the mean model (the
// algorithm's output) and the consensus distance (1/n) sum_i |mean - x^i|^2
// (M_k of the proofs appendix with uniform p), reduced with wavefront shuffles.
#include <mutex>

#include "device_common.hpp"
#include "internal.hpp"

// Fixed device memory for adpsgd_consensus_distance_static (the entry point for callers that cannot allocate):
// [0, kStaticPartials) block partials, then a spare result, then kStaticWeights worker probabilities.  Every GPU the
// library runs on holds its own copy until the process ends; host code reaches it only through the address that
// hipGetSymbolAddress returns on that GPU (static_scratch below), never through this name.
static __device__ __align__(256) double scratch[adpsgd_impl::kStaticPartials + 8 + adpsgd_impl::kStaticWeights];

namespace adpsgd_impl {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kConsensusBlocksMax = kStaticPartials;
constexpr int64_t kStreamBytes = 256ll << 20;   // beyond this X cannot stay in the caches

// grid = (ceil(ld/4 / kThreads), n): every row <- x0 on [0, d), zero on [d, ld)
__global__ __launch_bounds__(kThreads) void broadcast_rows_kernel(float* X, int64_t ld, int64_t d, const float* x0) {
    const int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (4 * v >= ld) return;
    v4f val;
    float t[4];
    for (int c = 0; c < 4; ++c) t[c] = (4 * v + c < d) ? x0[4 * v + c] : 0.0f;
    val.x = t[0]; val.y = t[1]; val.z = t[2]; val.w = t[3];
    *reinterpret_cast<v4f*>(X + static_cast<int64_t>(blockIdx.y) * ld + 4 * v) = val;
}

__global__ __launch_bounds__(kThreads) void refresh_bf16_kernel(const float* X, uint16_t* Xb, int64_t ld) {
    const int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (4 * v >= ld) return;
    const int64_t off = static_cast<int64_t>(blockIdx.y) * ld + 4 * v;
    const v4f x = *reinterpret_cast<const v4f*>(X + off);
    v4h h = {bf16_rne(x.x), bf16_rne(x.y), bf16_rne(x.z), bf16_rne(x.w)};
    *reinterpret_cast<v4h*>(Xb + off) = h;
}

constexpr int kRowBatch = 8;   // rows whose loads are in flight together (4 and 16 measure the same)
constexpr int kMeanBlocksMax = 4096;

// column means over the n rows in a fixed order, fp64 accumulation; a thread takes one float4 of d at a time and
// the grid strides over d (a capped grid of 4096 blocks walks the rows in step and reads 6.25 TB/s at n = 128,
// d = 25.6 M, against 6.0 TB/s for one thread per float4 and 3.7 TB/s for dword accesses)
// STREAM: X does not fit the caches and is read once: non-temporal loads
// VEC_OUT: out is 16-byte aligned and takes 128-bit stores
template <bool STREAM, bool VEC_OUT>
__global__ __launch_bounds__(kThreads) void mean_model_kernel(const float* X, int64_t ld, int64_t d, int32_t n, float* out) {
    const int64_t n_vec = (d + 3) / 4;
    for (int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; v < n_vec;
         v += static_cast<int64_t>(gridDim.x) * kThreads) {
        double s[4] = {0, 0, 0, 0};
        for (int32_t i0 = 0; i0 < n; i0 += kRowBatch) {
            v4f x[kRowBatch];
#pragma unroll
            for (int r = 0; r < kRowBatch; ++r)
                x[r] = i0 + r < n ? load4<STREAM>(X + static_cast<int64_t>(i0 + r) * ld + 4 * v) : v4f{0, 0, 0, 0};
#pragma unroll
            for (int r = 0; r < kRowBatch; ++r) {
                s[0] += x[r].x; s[1] += x[r].y; s[2] += x[r].z; s[3] += x[r].w;
            }
        }
        const v4f mean = {static_cast<float>(s[0] / n), static_cast<float>(s[1] / n), static_cast<float>(s[2] / n),
                          static_cast<float>(s[3] / n)};
        if (4 * v + 4 <= d && VEC_OUT) {
            store4<STREAM>(out + 4 * v, mean);         // out is 16-byte aligned
        } else {
            const float m[4] = {mean.x, mean.y, mean.z, mean.w};
            for (int c = 0; c < 4; ++c)
                if (4 * v + c < d) out[4 * v + c] = m[c];
        }
    }
}

// Per column e: sum_i (x_i - mean)^2 = sum_i t_i^2 - (sum_i t_i)^2 / n with t_i = x_i - x_0
// (shifting by row 0 keeps the subtraction exact when the replicas are close).
// Grid-stride over float4 columns, fp64 accumulation, wavefront reduction, one
// partial per block; a second single-block launch sums the partials in order.
// WEIGHTED: sum_i p_i (x_i - mean)^2 with the workers' update probabilities p (device, n doubles, psum
// their sum): with tb = (sum_i t_i) / n it is  sum_i p_i t_i^2 - 2 tb sum_i p_i t_i + tb^2 psum.
template <bool STREAM, bool WEIGHTED>
__global__ __launch_bounds__(kThreads) void consensus_partial_kernel(const float* X, int64_t ld, int64_t d, int32_t n,
                                                                    double* partial, const double* __restrict__ p, double psum) {
    __shared__ double red[kWaves];
    const int64_t n_vec = (d + 3) / 4;
    double acc = 0.0;
    for (int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; v < n_vec;
         v += static_cast<int64_t>(gridDim.x) * kThreads) {
        const v4f x0 = *reinterpret_cast<const v4f*>(X + 4 * v);
        double s1[4] = {0, 0, 0, 0}, s2[4] = {0, 0, 0, 0}, sp1[4] = {0, 0, 0, 0};
        for (int32_t i0 = 1; i0 < n; i0 += kRowBatch) {
            v4f xr[kRowBatch];
#pragma unroll
            for (int r = 0; r < kRowBatch; ++r)      // rows beyond n repeat row 0: their t is zero
                xr[r] = i0 + r < n ? load4<STREAM>(X + static_cast<int64_t>(i0 + r) * ld + 4 * v) : x0;
#pragma unroll
            for (int r = 0; r < kRowBatch; ++r) {
                const v4f x = xr[r];
                const float t[4] = {x.x - x0.x, x.y - x0.y, x.z - x0.z, x.w - x0.w};
                const double pi = WEIGHTED && i0 + r < n ? p[i0 + r] : 0.0;       // uniform address: a scalar load
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    s1[c] += t[c];
                    if (WEIGHTED) {
                        const double pt = pi * t[c];
                        sp1[c] += pt;
                        s2[c] += pt * t[c];
                    } else {
                        s2[c] += static_cast<double>(t[c]) * t[c];
                    }
                }
            }
        }
        for (int c = 0; c < 4; ++c)
            if (4 * v + c < d) {
                const double tb = s1[c] / n;
                acc += WEIGHTED ? s2[c] - 2.0 * tb * sp1[c] + tb * tb * psum : s2[c] - s1[c] * s1[c] / n;
            }
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(kThreads) void consensus_final_kernel(const double* partial, int32_t count, int32_t divisor,
                                                                  double* result) {
    __shared__ double red[kWaves];
    double acc = 0.0;
    for (int32_t b = threadIdx.x; b < count; b += kThreads) acc += partial[b];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) *result = ((red[0] + red[1]) + (red[2] + red[3])) / divisor;
}

// ---- divergence check: number of entries of X that are NaN or infinite -----------------------
// grid-stride over float4 pieces of all rows; one count per block, summed by the host.
__global__ __launch_bounds__(kThreads) void count_nonfinite_kernel(const float* X, int64_t ld, int64_t d, int32_t n,
                                                                  unsigned long long* partial) {
    __shared__ unsigned long long red[kWaves];
    const int64_t n_vec = (d + 3) / 4, total = n_vec * n;
    unsigned long long bad = 0;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; t < total;
         t += static_cast<int64_t>(gridDim.x) * kThreads) {
        const int64_t row = t / n_vec, v = t % n_vec;
        const v4f x = *reinterpret_cast<const v4f*>(X + row * ld + 4 * v);     // the padding beyond d is zero
        bad += !isfinite(x.x);
        bad += !isfinite(x.y);
        bad += !isfinite(x.z);
        bad += !isfinite(x.w);
    }
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_xor(bad, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = bad;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

// ---- the objective at one point x: f(x) = (1/n) sum_i mean over worker i's rows of F(x; row) ----
// (the problem statement of Sec. 3.1 with uniform p; F as in the gradient kernels, so the logistic
// loss carries lambda |x|^2 / 2).  grid = (row groups, n): a wavefront takes one local row at a time,
// lanes stride over d with four float4 loads in flight, the dot product is reduced with shuffles
// and the loss terms are accumulated in fp64; one partial per block, summed in order by a second
// single-block launch that also adds the regulariser.
// count_errors: instead of the loss a row contributes 1 when its predicted label (+1 if a.x >= 0, else -1)
// differs from its target (logistic regression): the classification error behind the paper's accuracy tables.
// rows_per_wave: 4 when the workers hold many rows, 1 when they hold few long ones (every row then
// gets a wavefront of its own: 2.8 -> 5.9 TB/s at 64 rows of 4 M floats per worker)
__global__ __launch_bounds__(kThreads) void objective_partial_kernel(int model, const float* __restrict__ x, int64_t d,
                                                                    const ObjectiveWorker* __restrict__ workers, double* partial,
                                                                    int rows_per_wave, int count_errors) {
    __shared__ double red[kWaves];
    const ObjectiveWorker w = workers[blockIdx.y];
    const float* __restrict__ A = static_cast<const float*>(w.features);
    const float* __restrict__ tg = static_cast<const float*>(w.targets);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t n_vec = d >> 2;            // full float4 groups; the ragged tail is handled separately
    double acc = 0.0;
    for (int r = 0; r < rows_per_wave; ++r) {
        const int64_t row = (static_cast<int64_t>(blockIdx.x) * kWaves + wave) * rows_per_wave + r;
        if (row >= w.rows) break;            // uniform over the wavefront
        const float* __restrict__ a = A + row * w.ld;
        float z = 0.0f;
        for (int64_t v0 = lane; v0 < n_vec; v0 += 64 * 8) {
            v4f av[8], xv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t v = v0 + 64 * u;
                av[u] = v < n_vec ? load4<true>(a + 4 * v) : v4f{0, 0, 0, 0};      // the data rows are read once
                xv[u] = v < n_vec ? *reinterpret_cast<const v4f*>(x + 4 * v) : v4f{0, 0, 0, 0};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) z += av[u].x * xv[u].x + av[u].y * xv[u].y + av[u].z * xv[u].z + av[u].w * xv[u].w;
        }
        for (int64_t e = 4 * n_vec + lane; e < d; e += 64) z += a[e] * x[e];
        z = wave_sum(z);
        if (lane == 0) {
            const float t = tg[row];
            if (count_errors) {
                acc += (z >= 0.0f ? 1.0f : -1.0f) != t ? 1.0 : 0.0;
            } else if (model == ADPSGD_MODEL_LSQ) {
                const double res = static_cast<double>(z) - t;
                acc += 0.5 * res * res;
            } else {
                const double s = -static_cast<double>(t) * z;
                acc += s > 0.0 ? s + log1p(exp(-s)) : log1p(exp(s));
            }
        }
    }
    if (lane == 0) red[wave] = acc / static_cast<double>(w.rows);
    __syncthreads();
    if (threadIdx.x == 0) partial[static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// weights: the workers' probabilities p_i (device, n doubles) or nullptr for 1 / n; a worker's partials are
// the `groups` consecutive entries starting at worker * groups
__global__ __launch_bounds__(kThreads) void objective_final_kernel(const double* partial, int64_t count, int32_t n, const float* x,
                                                                  int64_t d, double half_lambda, double* result,
                                                                  const double* __restrict__ weights, int64_t groups) {
    __shared__ double red[kWaves], red2[kWaves];
    double acc = 0.0, sq = 0.0;
    for (int64_t b = threadIdx.x; b < count; b += kThreads) acc += weights ? partial[b] * (weights[b / groups] * n) : partial[b];
    if (half_lambda != 0.0)
        for (int64_t e = threadIdx.x; e < d; e += kThreads) sq += static_cast<double>(x[e]) * x[e];
    acc = wave_sum(acc);
    sq = wave_sum(sq);
    if ((threadIdx.x & 63) == 0) { red[threadIdx.x >> 6] = acc; red2[threadIdx.x >> 6] = sq; }
    __syncthreads();
    if (threadIdx.x == 0)
        *result = ((red[0] + red[1]) + (red[2] + red[3])) / n + half_lambda * ((red2[0] + red2[1]) + (red2[2] + red2[3]));
}

// Wait-free variant with caller-supplied gradients: the copy the caller's function evaluates at,
// out[t] = X[worker] - comp_gamma * slot[comp_slot] for the operations that are compensated (two
// roundings, as in the update itself); the others are skipped and read their row of X directly.
// grid = (ceil(ld / 4 / kThreads), n_ops)
__global__ __launch_bounds__(kThreads) void compensated_rows_kernel(const float* __restrict__ X, int64_t ld, const GradOp* __restrict__ ops,
                                                                   const float* __restrict__ slots, float* __restrict__ out) {
    const GradOp op = ops[blockIdx.y];
    if (op.comp_slot < 0) return;
    const int64_t e = 4 * (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x);
    if (e >= ld) return;
    const v4f x = *reinterpret_cast<const v4f*>(X + static_cast<int64_t>(op.worker) * ld + e);
    const v4f g = *reinterpret_cast<const v4f*>(slots + static_cast<int64_t>(op.comp_slot) * ld + e);
    v4f c;
    {
#pragma clang fp contract(off)
        const v4f step = g * op.comp_gamma;
        c = x - step;
    }
    *reinterpret_cast<v4f*>(out + static_cast<int64_t>(blockIdx.y) * ld + e) = c;
}

}  // namespace

// Grid of at most `cap` blocks striding over `work` block-sized pieces such that every block gets the same number of
// them (up to one): the last pass is then as full as the others.
static int64_t balanced_grid(int64_t work, int64_t cap) {
    if (work < 1) return 1;
    const int64_t passes = (work + cap - 1) / cap;
    return (work + passes - 1) / passes;
}

hipError_t launch_compensated_rows(const float* X, int64_t ld, const GradOp* ops, int32_t n_ops, const float* slots, float* out,
                                   hipStream_t st) {
    const int64_t blocks = (ld / 4 + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFF || n_ops > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(compensated_rows_kernel, dim3(static_cast<uint32_t>(blocks), n_ops), dim3(kThreads), 0, st, X, ld, ops, slots, out);
    return hipGetLastError();
}

hipError_t launch_count_nonfinite(const float* X, int64_t ld, int64_t d, int32_t n, unsigned long long* partial,
                                  int32_t blocks, hipStream_t st) {
    hipLaunchKernelGGL(count_nonfinite_kernel, dim3(blocks), dim3(kThreads), 0, st, X, ld, d, n, partial);
    return hipGetLastError();
}

int objective_rows_per_wave(int64_t max_rows) { return max_rows >= 4096 ? 4 : 1; }
int64_t objective_row_groups(int64_t max_rows) {
    const int64_t per_block = static_cast<int64_t>(kWaves) * objective_rows_per_wave(max_rows);
    return (max_rows + per_block - 1) / per_block;
}

hipError_t launch_objective(int model, const float* x, int64_t d, int32_t n, const ObjectiveWorker* workers, int64_t max_rows,
                            float lambda, double* partial, double* result, bool count_errors, const double* weights,
                            hipStream_t st) {
    const int64_t groups = objective_row_groups(max_rows);
    if (groups < 1 || groups > 0x7FFFFFFF || n > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(objective_partial_kernel, dim3(static_cast<uint32_t>(groups), n), dim3(kThreads), 0, st, model, x, d, workers, partial,
                       objective_rows_per_wave(max_rows), count_errors ? 1 : 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(objective_final_kernel, dim3(1), dim3(kThreads), 0, st, partial, groups * n, n, x, d,
                       model == ADPSGD_MODEL_LOGREG && !count_errors ? 0.5 * static_cast<double>(lambda) : 0.0, result, weights, groups);
    return hipGetLastError();
}

hipError_t launch_broadcast_rows(float* X, int64_t ld, int64_t d, int32_t n, const float* x0, hipStream_t st) {
    const int64_t blocks = (ld / 4 + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFF || n > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(broadcast_rows_kernel, dim3(static_cast<uint32_t>(blocks), n), dim3(kThreads), 0, st, X, ld, d, x0);
    return hipGetLastError();
}

hipError_t launch_refresh_bf16(const float* X, uint16_t* Xb, int64_t ld, int32_t n, hipStream_t st) {
    const int64_t blocks = (ld / 4 + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFF || n > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(refresh_bf16_kernel, dim3(static_cast<uint32_t>(blocks), n), dim3(kThreads), 0, st, X, Xb, ld);
    return hipGetLastError();
}

hipError_t launch_mean_model(const float* X, int64_t ld, int64_t d, int32_t n, float* out, hipStream_t st) {
    const int64_t blocks = balanced_grid(((d + 3) / 4 + kThreads - 1) / kThreads, kMeanBlocksMax);
    const bool stream = static_cast<int64_t>(n) * ld * 4 > kStreamBytes;
    const bool vec = (reinterpret_cast<uintptr_t>(out) & 15u) == 0;
    const dim3 grid(static_cast<uint32_t>(blocks)), block(kThreads);
    if (stream && vec) hipLaunchKernelGGL((mean_model_kernel<true, true>), grid, block, 0, st, X, ld, d, n, out);
    else if (stream) hipLaunchKernelGGL((mean_model_kernel<true, false>), grid, block, 0, st, X, ld, d, n, out);
    else if (vec) hipLaunchKernelGGL((mean_model_kernel<false, true>), grid, block, 0, st, X, ld, d, n, out);
    else hipLaunchKernelGGL((mean_model_kernel<false, false>), grid, block, 0, st, X, ld, d, n, out);
    return hipGetLastError();
}

int32_t consensus_blocks(int64_t d) {
    return static_cast<int32_t>(balanced_grid(((d + 3) / 4 + kThreads - 1) / kThreads, kConsensusBlocksMax));
}

// The device address of `scratch` on the current GPU, resolved once per device.
hipError_t static_scratch(double** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static double* address[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!address[dev]) {
        double* ptr = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        address[dev] = ptr;
    }
    *out = address[dev];
    return hipSuccess;
}

hipError_t launch_consensus(const float* X, int64_t ld, int64_t d, int32_t n, double* partial, double* result,
                            const double* p, double psum, hipStream_t st) {
    const int32_t blocks = consensus_blocks(d);
    const bool stream = static_cast<int64_t>(n) * ld * 4 > kStreamBytes;
    const dim3 grid(blocks), block(kThreads);
    if (p && stream) hipLaunchKernelGGL((consensus_partial_kernel<true, true>), grid, block, 0, st, X, ld, d, n, partial, p, psum);
    else if (p) hipLaunchKernelGGL((consensus_partial_kernel<false, true>), grid, block, 0, st, X, ld, d, n, partial, p, psum);
    else if (stream) hipLaunchKernelGGL((consensus_partial_kernel<true, false>), grid, block, 0, st, X, ld, d, n, partial, p, psum);
    else hipLaunchKernelGGL((consensus_partial_kernel<false, false>), grid, block, 0, st, X, ld, d, n, partial, p, psum);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(kThreads), 0, st, partial, blocks, p ? 1 : n, result);
    return hipGetLastError();
}

}  // namespace adpsgd_impl
